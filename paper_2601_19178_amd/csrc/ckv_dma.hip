// Matrix-core gather-concat-attend kernel with direct global->LDS gathers (bf16 storage, fp32
// accumulation, d_a = 64, 128 or 256, d_u even up to 16 (32 at 256 columns) or odd up to 7).
//
// Same mathematics and MFMA operand layouts as the register-staged kernel next to it
// (S^T = K Q^T, O^T += V^T P^T, one query per lane), but the final K and V rows of a tile are
// assembled in LDS without passing through registers:
//   * pool rows are gathered with global_load_lds_dwordx4 (16 bytes per lane straight into
//     LDS; the instruction puts lane l at M0 + 16*l, so one wavefront fills 1 KiB of
//     consecutive rows).  The row layout inside LDS is [pool columns | user columns],
//     unpadded, with the 16-byte chunks of row p stored at slot (chunk XOR f(p)) so that the
//     operand reads stay free of bank conflicts (64 banks); the lane chooses which chunk it
//     fetches, so the swizzle costs nothing on the way in.
//   * the pool indices of a tile and its user-specific slices are fetched the same way
//     (global_load_lds_dword) into small staging areas; the "concat" of the paper
//     (eq. "eq: K") is an LDS->LDS copy of the user columns into the tail of each row.
// Tiles are 32 positions; a ring of 4 stages keeps two to three tiles of gathers in flight
// per workgroup while one tile is computed (2 stages, one tile in flight, for workgroups of
// one wavefront).  The loads are issued from inline asm and waited for with explicit
// s_waitcnt vmcnt(N): every wavefront issues the same number of loads per iteration
// (positions past the end of the history are clamped to the last one), so N is a constant.
#include <cstdlib>

#include <type_traits>

#include "ckv_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) unsigned char lds_u8;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef __attribute__((address_space(3))) uint16_t lds_u16;
typedef __attribute__((address_space(3))) float lds_f32;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLazy = 8.f;
constexpr int TP = 32;  // positions per tile

__device__ __forceinline__ float other_half(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return threadIdx.x & 32 ? __uint_as_float(r[0]) : __uint_as_float(r[1]);
}
__device__ __forceinline__ uint16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
// Masks one score of a ragged last tile.  The empty volatile asm pins the select inside the (wavefront-
// uniform) branch that calls it; without it the compiler turns that branch into sixteen compares and
// selects that every whole tile executes as well.
__device__ __forceinline__ float mask_tail(float x, bool past_end, float fill) {
    float v = past_end ? fill : x;
    asm volatile("" : "+v"(v));
    return v;
}

// 16 bytes per lane, global -> LDS[lds_base + 16*lane].  lds_base is wavefront-uniform.
__device__ __forceinline__ void dma16(const void* g, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_base) : "memory");
}
// 4 bytes per lane, global -> LDS[lds_base + 4*lane].
__device__ __forceinline__ void dma4(const void* g, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(g), "s"(lds_base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// LDS swizzle: 16-byte chunk c of row p is stored at slot c ^ f(p).  The LDS has 64 banks of 4 bytes
// (256 bytes per clock), so an access is conflict free when the lanes served together cover sixteen
// different 16-byte slots modulo 16.
//   K rows (ds_read_b128, sixteen consecutive rows, same chunk): the low four bits of the row for
//   256-byte rows; for 128-byte rows two neighbouring rows already differ in bit 3 of the slot number, so
//   the next three bits of the row are used.
//   V rows (ds_read_b64_tr_b16, four consecutive rows x four consecutive chunks per clock): the row's low
//   two bits select one of the four 64-byte quarters of a 256-byte row; for 128-byte rows bit 1 of the row
//   selects one of the two halves.
//   512-byte rows (d_a = 256) start on the same bank as 256-byte rows and use the same functions.
template <int DA>
__device__ __forceinline__ int fk(int p) { return DA >= 128 ? (p & 15) : ((p >> 1) & 7); }
template <int DA>
__device__ __forceinline__ int fv(int p) { return DA >= 128 ? ((p & 3) << 2) : (((p >> 1) & 1) << 2); }

// WIDEU: user slices of 10 to 16 columns at 64 or 128 columns (a larger staging area; the 256-column geometry always has it)
template <int DA, int NW, bool WIDEU = false>
struct Geo {
    static constexpr int NT = NW * 64;
    // stages in the ring (a power of two).  Workgroups of one wavefront: two stages, so that LDS leaves room for twice
    // the workgroups on a CU (64 columns: eight, two wavefronts per SIMD; 128 columns: four, one on every SIMD instead
    // of on every other); measured faster than the deeper ring by 7.5 % (config 5) and 5.8 % (config 4 with 32 queries)
    static constexpr int NS = (DA <= 128 && NW == 1) ? 2 : 4;
    static constexpr int CH = DA / 8;            // 16-byte chunks per row
    static constexpr int ROWB = DA * 2;          // bytes per row
    static constexpr int RPI = 64 / CH;          // rows filled by one wavefront instruction
    static constexpr int NI = TP / RPI / NW;     // gather instructions per wavefront, K and V each
    static constexpr int NUI_MAX = (DA == 256 ? 16 : WIDEU ? 8 : 4) / NW;  // user-slice instructions per wavefront (d_u <= 8, <= 16, or <= 32 at 256 columns)
    static constexpr int KV = TP * ROWB;         // bytes of the K (or V) rows of a stage
    static constexpr int USER = NW * 64 * 4 * NUI_MAX;  // bytes of the user staging of a stage (1, 2 or 4 KiB)
    static constexpr int STAGE = 2 * KV + USER;
    static constexpr int IDX = 256;              // bytes of one index slot: 32 x I_k, 32 x I_v
    static constexpr int NIS = 4;                // index slots per wavefront (indices run 3 tiles ahead of the gathers)
    static constexpr int LDS = NS * STAGE + NW * NIS * IDX;
    // wavefronts per SIMD that LDS lets be resident; the register budget is sized for exactly that
    static constexpr int WG_PER_CU = 163840 / LDS;
    // (not below 2 for 64 columns, also where LDS leaves one wavefront per SIMD: with more than 256 registers the compiler puts
    // the accumulators into AGPRs and copies them back and forth for the weight arithmetic, over 100 moves per tile)
    // (the 128-column one-wavefront kernel needs more than 256 registers either way and keeps its budget of 512)
    static constexpr int WAVES_PER_EU =
        WG_PER_CU * NW / 4 < 2 ? (DA == 64 ? 2 : 1) : (WG_PER_CU * NW / 4 > 8 ? 8 : WG_PER_CU * NW / 4);
    static_assert(NI >= 1, "tile too small for this many wavefronts");
    static_assert((NS - 1) * (2 * NI + 1 + NUI_MAX) <= 63, "no more loads outstanding than the 6-bit counter holds");
    static_assert((NS - 2) * (2 * NI + 1 + NUI_MAX) <= 63, "the wait of the tile loop must fit the 6-bit counter");
};

// QG = groups of 32 queries owned by one wavefront.  With QG = 2 every K and V operand read
// from LDS feeds two MFMAs, and the weight arithmetic of one group can run while the matrix
// core works on the other.
// UK: kind of user slice. 0: d_u even, up to 8 (16 at 256 columns); 1: d_u odd, 1 or 3 (up to 7 at 256 columns), an
// instantiation of its own, so that the even case carries none of its code; 2: d_u even, 10 to 16, at 64 or 128 columns;
// 3: d_u odd, 5 or 7, at 64 or 128 columns.  2 and 3 have the larger staging area (an odd slice takes a lane per element);
// with it a 64-column kernel loses one of its four resident workgroups, which is why 1 and 3 are apart.
// Q16: sixteen queries per work item on v_mfma_f32_16x16x32_bf16 (one wavefront, 64 columns, even user slices of up to 8
// columns).  On the 32x32 instruction sixteen queries fill half of the query columns, so half of the matrix and weight
// arithmetic is spent on nothing; here a lane holds one query and eight positions of a tile, nothing is idle.
template <int DA, int NW, int QG, int MODE, int UK, bool Q16 = false>
__global__ __launch_bounds__(NW * 64)
__attribute__((amdgpu_waves_per_eu(Geo<DA, NW, (UK >= 2)>::WAVES_PER_EU, Geo<DA, NW, (UK >= 2)>::WAVES_PER_EU))) void ckv_dma_kernel(ckv_args a, int nui) {
    using G = Geo<DA, NW, (UK >= 2)>;
    static_assert(!Q16 || (DA == 64 && NW == 1 && QG == 1 && UK == 0), "sixteen-query organisation: one wavefront at 64 columns");
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    constexpr int NKK = DA / 16, NDT = DA / 32;
    constexpr bool kWide = DA > 128;  // operands of a whole tile no longer fit into registers beside the accumulators
    static_assert(!kWide || QG == 1, "one query group per wavefront at 256 columns");
    constexpr bool kAccInAgprs = G::WAVES_PER_EU == 1;  // a budget above 256 registers makes the compiler use the AGPR form of the MFMAs
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_u8*)smem;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // persistent workgroup: one list of work items per workgroup
    const int item_end = a.wg_begin[blockIdx.x + 1];
    for (int item = a.wg_begin[blockIdx.x]; item < item_end; ++item) {
    // The lane id is laundered once per item so that the many per-lane constants derived from it
    // are recomputed per item (a few dozen ALU operations) instead of being kept alive, and
    // spilled, across the whole kernel.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const ckv_item it = a.items[item];
    unsigned long long* tr = a.trace ? a.trace + (size_t)item * 8 : nullptr;
    if (tr && tid == 0) {
        tr[0] = wall_clock64();
        tr[4] = ((unsigned long long)__builtin_amdgcn_s_getreg((20 << 0) | (0 << 6) | (31 << 11)) << 32) |
                (unsigned)__builtin_amdgcn_s_getreg((4 << 0) | (0 << 6) | (31 << 11));
        tr[5] = (unsigned long long)it.n;
    }
    const int qn = lane & 31, hh = lane >> 5;
    const int d_g = a.d_g, d_u = a.d_u;
    constexpr bool uodd = UK == 1 || UK == 3;  // user and pool columns then change places at an odd column: no 32-bit shortcuts
    // A side that is not shared (only keys or only values gather from a pool) keeps whole d_a-wide rows in
    // its user array: its tile rows are fetched from there, position by position, with the same
    // instructions that fetch pool rows for a shared side, and it has no user slice to append.
    const bool ksh = a.d_gk > 0, vsh = a.d_gv > 0;
    const int dgk = ksh ? d_g : DA, duk = DA - dgk;  // pool and user columns of a K row in LDS
    const int dgv = vsh ? d_g : DA, duv = DA - dgv;
    const int n = it.n;

    const int64_t hT = (int64_t)it.h * a.T + it.t0;
    const int32_t* __restrict__ ik = a.idx_k + hT;
    const int32_t* __restrict__ iv = a.idx_v + hT;
    const uint32_t* __restrict__ uk32 = (const uint32_t*)((const uint16_t*)a.user_k + hT * d_u);
    const uint32_t* __restrict__ uv32 = (const uint32_t*)((const uint16_t*)a.user_v + hT * d_u);
    const unsigned char* __restrict__ pk = ksh ? (const unsigned char*)a.pool_k + (int64_t)it.h * a.P * a.pool_ld * 2
                                               : (const unsigned char*)a.user_k + hT * (DA * 2);
    const unsigned char* __restrict__ pv = vsh ? (const unsigned char*)a.pool_v + (int64_t)it.h * a.P * a.pool_ld * 2
                                               : (const unsigned char*)a.user_v + hT * (DA * 2);
    const uint32_t krow_bytes = ksh ? (uint32_t)a.pool_ld * 2 : (uint32_t)(DA * 2);
    const uint32_t vrow_bytes = vsh ? (uint32_t)a.pool_ld * 2 : (uint32_t)(DA * 2);

    // ---- the indices of the first three tiles are requested before the queries, so that the two round
    //      trips overlap (the index slots are private to the wavefront and apart from the query staging)
    const uint32_t idx_lds = lds0 + G::NS * G::STAGE + wave * G::NIS * G::IDX;
    // (with no pool at all, d_g = 0, there may be no index buffer: the load still has to be issued, because the
    // waits below count instructions, so it reads the work list instead and its value is never used)
    // (base and clamp are chosen once per item: a select inside the tile loop cost config 4 over 1 %)
    const bool any_pool = ksh || vsh;
    const int32_t* __restrict__ ibase = any_pool ? (hh ? iv : ik) : (const int32_t*)a.items;
    const int ilast = any_pool ? n - 1 : 7;
    auto issue_idx = [&](int tile) {
        const int pos = min(tile * TP + qn, ilast);
        dma4(ibase + pos, idx_lds + (tile & (G::NIS - 1)) * G::IDX);
    };
    if (n > 0) {
        issue_idx(0);
        issue_idx(1);
        issue_idx(2);
    }

    // ---- queries: the wavefront's 32*QG query rows are copied row-major into LDS with
    //      coalesced 16-byte loads, then every lane picks its B operands (kernel column order
    //      [pool | user], i.e. paper column + d_u for pool columns) out of LDS.
    constexpr int QS = DA * 2 + 16;  // bytes per staged row
    const int qfirst = it.q0 + wave * QG * 32;
    const int qrows = min(max(a.Nq - qfirst, 0), Q16 ? 16 : QG * 32);
    const int q16 = lane & 15, g4 = lane >> 4;  // Q16: the lane's query and its group of eight positions
    const int64_t qbyte0 = (((int64_t)it.b * a.H + it.h) * a.Nq + qfirst) * (DA * 2);
    const uint32_t qlds = lds0 + wave * (QG * 32 * QS);
    bf16x8 qreg[QG][NKK];
    {
        const unsigned char* qsrc = (const unsigned char*)a.q + qbyte0;
#pragma unroll
        for (int i = 0; i < QG * 32 * G::CH / 64; ++i) {
            const int e = i * 64 + lane, row = e / G::CH, c = e % G::CH;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (row < qrows) v = *reinterpret_cast<const u32x4*>(qsrc + (int64_t)row * (DA * 2) + c * 16);
            *(lds_u32x4*)(uintptr_t)(qlds + row * QS + c * 16) = v;
        }
#pragma unroll
        for (int g = 0; g < (Q16 ? 0 : QG); ++g)
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk) {
                u32x4 w;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int ci = 16 * kk + 8 * hh + 2 * j;
                    const int pc = ci < dgk ? ci + duk : ci - dgk;
                    if (!uodd) {
                        w[j] = *(const lds_u32*)(uintptr_t)(qlds + (g * 32 + qn) * QS + pc * 2);
                    } else {
                        const int pc1 = ci + 1 < dgk ? ci + 1 + duk : ci + 1 - dgk;
                        w[j] = (uint32_t) * (const lds_u16*)(uintptr_t)(qlds + (g * 32 + qn) * QS + pc * 2) |
                               ((uint32_t) * (const lds_u16*)(uintptr_t)(qlds + (g * 32 + qn) * QS + pc1 * 2) << 16);
                    }
                }
                qreg[g][kk] = __builtin_bit_cast(bf16x8, w);
            }
        if (Q16) {
            // B operands of the 16x16x32 instruction: query lane % 16, columns 32 ks + 8 (lane / 16) .. + 8 of the kernel's order
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                u32x4 w;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int ci = 32 * ks + 8 * g4 + 2 * j;
                    const int pc = ci < dgk ? ci + duk : ci - dgk;
                    w[j] = *(const lds_u32*)(uintptr_t)(qlds + q16 * QS + pc * 2);
                }
                qreg[0][ks] = __builtin_bit_cast(bf16x8, w);
            }
        }
        // everything above (global loads included) has to be complete here: a compiler-inserted
        // wait inside the tile loop would also drain the asynchronous gathers it cannot see, and
        // the gathers are about to overwrite the staging area
#pragma unroll
        for (int g = 0; g < QG; ++g)
#pragma unroll
            for (int kk = 0; kk < (Q16 ? 2 : NKK); ++kk) asm volatile("" : "+v"(qreg[g][kk]));
        lds_barrier();
    }

    f32x16 oacc[QG][NDT];
    float m_ref[QG], lsum[QG];
#pragma unroll
    for (int g = 0; g < QG; ++g) {
        m_ref[g] = -INFINITY;
        lsum[g] = 0.f;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[g][dt][r] = 0.f;
    }
    f32x4 o16[4];  // Q16: O^T blocks of 16 columns: query lane % 16, columns 16 dt + 4 (lane / 16) + r
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 4; ++r) o16[dt][r] = 0.f;
    const float sc = MODE == CKV_SOFTMAX ? a.scale * kLog2e : a.scale;
    const float nsc = -kLog2e * a.scale;    // SiLU: exponent of 2 per unit of raw score
    // SiLU: the weights are taken without the factor sc of their numerator (score / (1 + 2^(nsc score))); the output gets it
    const float osc = MODE == CKV_SOFTMAX ? 1.f : a.scale;

    const int ntiles = (n + TP - 1) / TP;
    if (ntiles > 0) {
        // ---- per-lane constants of the gather: instruction i of this wavefront fills rows
        //      (i*NW + wave)*RPI .. +RPI; this lane owns row gp[i] and LDS slot gslot of it.
        const int gslot = lane % G::CH;
        int gp[G::NI];
        uint32_t gk_off[G::NI], gv_off[G::NI];  // byte offset of the chunk this lane fetches, within a pool row
#pragma unroll
        for (int i = 0; i < G::NI; ++i) {
            gp[i] = (i * NW + wave) * G::RPI + lane / G::CH;
            int ck = gslot ^ fk<DA>(gp[i]);
            int cv = gslot ^ fv<DA>(gp[i]);
            if (ck * 8 >= dgk) ck = 0;  // a pure user chunk: fetch something valid, the concat overwrites it
            if (cv * 8 >= dgv) cv = 0;
            gk_off[i] = ck * 16;
            gv_off[i] = cv * 16;
        }
        // ---- per-lane constants of the user slices.  A wavefront fetches the user slices of
        //      exactly the rows it gathers, so that after its own wait it can copy them into the
        //      row tails (the concat) without depending on any other wavefront.  Dword jj of the
        //      wavefront's block is ((kv * ROWS_W + o) * hd + off): kv = K or V, o = ordinal of the
        //      own row, off = dword inside the d_u-wide slice (hd = d_u / 2 dwords).
        //      An odd d_u (1 to 7) cannot be moved in whole dwords: a lane then stands for one element, fetches
        //      the aligned dword that holds it and appends its half with a 16-bit LDS write.
        constexpr int ROWS_W = TP / NW;
        const int hd = d_u > 0 ? (uodd ? d_u : d_u >> 1) : 1;  // lanes per slice
        int up[G::NUI_MAX], uoff[G::NUI_MAX];
        bool uisv[G::NUI_MAX], uok[G::NUI_MAX];
        uint32_t cdst[G::NUI_MAX];
#pragma unroll
        for (int u = 0; u < G::NUI_MAX; ++u) {
            int jj = u * 64 + lane;
            uok[u] = u < nui && jj < 2 * ROWS_W * hd;
            if (!uok[u]) jj = 0;
            const int slice = jj / hd;            // kv * ROWS_W + o
            uoff[u] = jj - slice * hd;
            uisv[u] = slice >= ROWS_W;
            uok[u] = uok[u] && (uisv[u] ? vsh : ksh);  // nothing to append on a side that is not shared
            const int o = uisv[u] ? slice - ROWS_W : slice;
            up[u] = ((o / G::RPI) * NW + wave) * G::RPI + (o % G::RPI);
            const int col = d_g + (uodd ? uoff[u] : 2 * uoff[u]);
            const int slot = (col >> 3) ^ (uisv[u] ? fv<DA>(up[u]) : fk<DA>(up[u]));
            cdst[u] = (uisv[u] ? G::KV : 0) + up[u] * G::ROWB + slot * 16 + (col & 7) * 2;
        }
        // ---- per-lane constants of the operand reads
        const uint32_t krow = qn * G::ROWB;
        const int kx = fk<DA>(qn);
        const int g16 = lane >> 4, s16 = lane & 15;
        const uint32_t vrow = G::KV + (4 * hh + (s16 >> 2)) * G::ROWB + (s16 & 1) * 8;
        const int vc = 2 * (g16 & 1) + ((s16 & 3) >> 1), vx = fv<DA>(s16 >> 2);

        // (generic in the number NUI of user-slice loads per wavefront and tile, so that the tile loop, which is
        // instantiated per value below, carries no test of it)
        // rows of the tile that this wavefront's gather instructions fetch (pool index, or position for a side without pool)
        auto gather_rows = [&](auto both_c, int tile, int (&rk)[G::NI], int (&rv)[G::NI]) {
            constexpr bool kBoth = decltype(both_c)::value;  // both sides gather from their pool: the usual case
            const lds_u32* islot = (const lds_u32*)(uintptr_t)(idx_lds + (tile & (G::NIS - 1)) * G::IDX);
#pragma unroll
            for (int i = 0; i < G::NI; ++i) {
                const int jk = (int)islot[gp[i]], jv = (int)islot[32 + gp[i]];  // read in any case: a select, not a branch
                if (kBoth) {
                    rk[i] = jk;
                    rv[i] = jv;
                } else {
                    const int pos = min(tile * TP + gp[i], n - 1);
                    rk[i] = ksh ? jk : pos;
                    rv[i] = vsh ? jv : pos;
                }
            }
        };
        // load instruction number s of a tile: 2 * NI gathers (K and V alternating), then the user slices
        auto tile_dma = [&](int tile, int s, const int (&rk)[G::NI], const int (&rv)[G::NI]) {
            const uint32_t st = lds0 + (tile & (G::NS - 1)) * G::STAGE;
            if (s < 2 * G::NI) {
                const int i = s >> 1;
                const uint32_t dst = (i * NW + wave) * G::RPI * G::ROWB;
                if (!(s & 1)) dma16(pk + (uint64_t)(uint32_t)rk[i] * krow_bytes + gk_off[i], st + dst);
                else dma16(pv + (uint64_t)(uint32_t)rv[i] * vrow_bytes + gv_off[i], st + G::KV + dst);
            } else {
                const int u = s - 2 * G::NI;
                const int pos = min(tile * TP + up[u], n - 1);
                const uint32_t* g;
                if (uodd) g = (const uint32_t*)(uisv[u] ? a.user_v : a.user_k) + (((hT + pos) * d_u + uoff[u]) >> 1);
                else g = (uisv[u] ? uv32 : uk32) + (int64_t)pos * hd + uoff[u];
                dma4(g, st + 2 * G::KV + (wave * G::NUI_MAX + u) * 256);
            }
        };
        // the paper's concat: user columns behind the pool columns of the wavefront's own rows
        auto concat = [&](auto nui_c, int tile) {
            constexpr int NUI = decltype(nui_c)::value;
            const uint32_t st = lds0 + (tile & (G::NS - 1)) * G::STAGE;
            uint32_t x[G::NUI_MAX];
#pragma unroll
            for (int u = 0; u < G::NUI_MAX; ++u)
                if (u < NUI && uok[u]) x[u] = *(const lds_u32*)(uintptr_t)(st + 2 * G::KV + (wave * G::NUI_MAX + u) * 256 + lane * 4);
            if (uodd) {
#pragma unroll
                for (int u = 0; u < G::NUI_MAX; ++u)
                    if (u < NUI && uok[u]) {
                        const int pos = min(tile * TP + up[u], n - 1);
                        const bool upper = ((hT + pos) * d_u + uoff[u]) & 1;  // which half of the fetched dword
                        *(lds_u16*)(uintptr_t)(st + cdst[u]) = (uint16_t)(upper ? x[u] >> 16 : x[u]);
                    }
                return;
            }
#pragma unroll
            for (int u = 0; u < G::NUI_MAX; ++u)
                if (u < NUI && uok[u]) *(lds_u32*)(uintptr_t)(st + cdst[u]) = x[u];
        };

        // Order of the asynchronous loads of one wavefront, for NS stages (written out for NS = 4): iteration t
        // issues idx(t+NS+2) = idx(t+6), then the gathers of tile t+NS-1 = t+3 (whose rows were read from idx(t+3)
        // in LDS behind the previous iteration's wait).  The wait at the end of iteration t lets the loads of the
        // last NS-2 = two iterations stay outstanding, so it completes the wavefront's gathers of tile t+1 and,
        // being older, idx(t+4): NS-1 = three tiles of gathers are in flight while one is computed, and the
        // indices a gather needs landed at least one wait earlier.  After its wait the wavefront concatenates
        // its own rows of tile t+1; the barrier then publishes tile t+1 to the workgroup and retires tile t's
        // stage.  (At most NS-1 iterations' loads are ever outstanding, which the 6-bit counter holds.)
        wait_vm<0>();  // the indices of tiles 0..2, requested before the queries
        if (tr && tid == 0) tr[1] = wall_clock64();
        auto tile_loop = [&](auto nui_c, auto both_c) {
        constexpr int NUI = decltype(nui_c)::value;
        // (the rows a wavefront gathers for tile t+3 are looked up one iteration ahead, behind the previous iteration's
        // wait, so that the loads at the top of an iteration do not start with a round trip to LDS)
        // (measured: config 4 -1.4 %, config 5 -5.7 %; 256 columns +1.3 %, which therefore look their rows up in place)
        constexpr bool kAhead = !kWide;
        int rk[G::NI], rv[G::NI];
        if (kAhead) gather_rows(both_c, 0, rk, rv);
        constexpr int NS = G::NS;
        for (int t = -(NS - 1); t < ntiles; ++t) {
            issue_idx(t + NS + 2);
            if (!kAhead) gather_rows(both_c, t + NS - 1, rk, rv);
#pragma unroll
            for (int s = 0; s < 2 * G::NI + NUI; ++s) tile_dma(t + NS - 1, s, rk, rv);
            if (t >= 0) {
                const uint32_t st = lds0 + (t & (NS - 1)) * G::STAGE;
                const int nt = min(n - t * TP, TP);
                // S^T = K Q^T for every query group; each K operand is read once
                f32x16 sacc[QG];
#pragma unroll
                for (int g = 0; g < QG; ++g)
#pragma unroll
                    for (int r = 0; r < 16; ++r) sacc[g][r] = 0.f;
                bf16x8 ka[NKK];
#pragma unroll
                for (int kk = 0; kk < NKK; ++kk)
                    ka[kk] = *(const lds_bf16x8*)(uintptr_t)(st + krow + (((2 * kk + hh) ^ kx) << 4));
#pragma unroll
                for (int g = 0; g < QG; ++g)
#pragma unroll
                    for (int kk = 0; kk < NKK; ++kk)
                        sacc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk], qreg[g][kk], sacc[g], 0, 0, 0);
                if (!kWide) {
                    __builtin_amdgcn_sched_group_barrier(0x100, NKK, 0);       // all LDS reads ...
                    __builtin_amdgcn_sched_group_barrier(0x008, NKK * QG, 0);  // ... then the MFMAs
                } else {
                    // 256 columns: a window of eight operands, refilled four at a time under the MFMAs
                    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
                    for (int i = 0; i < (NKK - 8) / 4; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
                }
                // V^T operands of the whole tile: issued now, so that their LDS latency is hidden
                // behind the MFMAs above and the weight arithmetic below
                // (256 columns: the first sixteen positions now, the other sixteen under the first half's MFMAs)
                bf16x8 va[2][NDT];
                auto load_v = [&](int ks) {
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) {
                        const uint32_t ad = st + vrow + (16 * ks) * G::ROWB + (((4 * dt + vc) ^ vx) << 4);
                        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(uintptr_t)ad);
                        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(uintptr_t)(ad + 8 * G::ROWB));
                        va[ks][dt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    }
                };
                load_v(0);
                if (!kWide) load_v(1);
                __builtin_amdgcn_sched_group_barrier(0x100, (kWide ? 2 : 4) * NDT, 0);
                __builtin_amdgcn_sched_barrier(0);
                const bool ragged = nt < TP;
#pragma unroll
                for (int g = 0; g < QG; ++g) {
                    bf16x8 pb[2];
                    if (MODE == CKV_SOFTMAX) {
                        if (ragged) {  // see mask_tail: only the last tile of a history comes here
#pragma unroll
                            for (int r = 0; r < 16; ++r) sacc[g][r] = mask_tail(sacc[g][r], 8 * (r >> 2) + 4 * hh + (r & 3) >= nt, -INFINITY);
                        }
                        float tmax = sacc[g][0];
#pragma unroll
                        for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, sacc[g][r]);
                        tmax = fmaxf(tmax, other_half(tmax)) * sc;
                        if (__any(tmax > m_ref[g] + kLazy)) {
                            const float m_new = fmaxf(m_ref[g], tmax);
                            const float alpha = __builtin_amdgcn_exp2f(m_ref[g] - m_new);
                            lsum[g] *= alpha;
#pragma unroll
                            for (int dt = 0; dt < NDT; ++dt) {
                                // (accumulators in AGPRs: pinned there on both sides of the multiplication, so that
                                // their way through VGPRs stays inside this rare branch; otherwise every tile copies
                                // all of them out in case the branch is taken)
                                if (kAccInAgprs) asm volatile("" : "+a"(oacc[g][dt]));
#pragma unroll
                                for (int r = 0; r < 16; ++r) oacc[g][dt][r] *= alpha;
                                if (kAccInAgprs) asm volatile("" : "+a"(oacc[g][dt]));
                            }
                            m_ref[g] = m_new;
                        }
                        float psum = 0.f;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const float p = __builtin_amdgcn_exp2f(fmaf(sacc[g][r], sc, -m_ref[g]));
                            psum += p;
                            pb[r >> 3][r & 7] = (__bf16)p;
                        }
                        lsum[g] += psum;
                    } else {
                        if (ragged) {  // SiLU(0) = 0: positions past the end get a zero score
#pragma unroll
                            for (int r = 0; r < 16; ++r) sacc[g][r] = mask_tail(sacc[g][r], 8 * (r >> 2) + 4 * hh + (r & 3) >= nt, 0.f);
                        }
                        // p = x / (1 + 2^(-x log2 e)) with x = sc * score; the factor sc of the numerator is applied once, to the
                        // output (epilogue), instead of to every weight
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const float e = __builtin_amdgcn_exp2f(sacc[g][r] * nsc);
                            pb[r >> 3][r & 7] = (__bf16)(sacc[g][r] * __builtin_amdgcn_rcpf(1.f + e));
                        }
                    }
                    // O^T += V^T P^T
                    if (kWide) {
                        __builtin_amdgcn_sched_barrier(0);
                        load_v(1);
                    }
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int dt = 0; dt < NDT; ++dt)
                            oacc[g][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ks][dt], pb[ks], oacc[g][dt], 0, 0, 0);
                }
            }
            // own gathers of tile t+1 have landed once only the loads of this and the previous
            // iteration are outstanding
            wait_vm<(NS - 2) * (2 * G::NI + 1 + NUI)>();
            if (NUI > 0 && t + 1 >= 0 && t + 1 < ntiles) concat(nui_c, t + 1);
            if (kAhead) gather_rows(both_c, t + NS, rk, rv);  // (the indices of tile t+4 were requested two iterations ago: they have landed)
            lds_barrier();
        }
        };
        // The same loop with the scores one tile ahead (four wavefronts of one query group at 128 columns, the shape of the
        // long ragged configuration): iteration t takes the weights and the output of tile t from scores that the previous
        // iteration left in registers, and issues the score MFMAs of tile t + 1 between the exponentials of tile t, so that
        // the matrix pipe works under the vector arithmetic of the same wavefront instead of being waited for.  Tile t + 1
        // therefore has to be published one iteration earlier than above: the wait at the end of iteration t lets only that
        // iteration's loads stay outstanding (two tiles of gathers in flight instead of three), and the barrier publishes
        // tile t + 2.  The steady-state body (whole tiles) carries no test of the tile's length; the first score block and
        // the last, possibly ragged, tile are peeled.
        auto tile_loop_ahead = [&](auto nui_c, auto both_c) {
            constexpr int NUI = decltype(nui_c)::value;
            constexpr int NS = G::NS;
            constexpr int LPI = 2 * G::NI + 1 + NUI;  // loads per iteration and wavefront
            static_assert(QG == 1 && !kWide && NS == 4, "built for one query group on the four-stage ring");
            int rk[G::NI], rv[G::NI];
            gather_rows(both_c, 0, rk, rv);
            auto front = [&](int t) {
                issue_idx(t + NS + 2);
#pragma unroll
                for (int s = 0; s < 2 * G::NI + NUI; ++s) tile_dma(t + NS - 1, s, rk, rv);
            };
            auto back = [&](int t) {
                // (the scheduler had moved this wait up to the first score MFMA, ahead of the arithmetic that is to hide the latency)
                __builtin_amdgcn_sched_barrier(0);
                wait_vm<(NS - 3) * LPI>();  // own gathers of tile t + 2 have landed
                if (NUI > 0 && t + 2 >= 0 && t + 2 < ntiles) concat(nui_c, t + 2);
                gather_rows(both_c, t + NS, rk, rv);
                lds_barrier();  // tile t + 2 is published, the stage of tile t is retired
            };
            // (operand addresses: a per-lane part that is fixed for the item, tied to an empty asm statement at every use so
            // that the stage offset added to it stays an immediate of the LDS read instead of becoming a register per stage)
            uint32_t kb[NKK], vb[NDT];
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk) kb[kk] = lds0 + krow + (((2 * kk + hh) ^ kx) << 4);
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt) vb[dt] = lds0 + vrow + (((4 * dt + vc) ^ vx) << 4);
            auto read_k = [&](int tile, bf16x8 (&ka)[NKK]) {
                const uint32_t st = (tile & (NS - 1)) * G::STAGE;
#pragma unroll
                for (int kk = 0; kk < NKK; ++kk) {
                    asm volatile("" : "+v"(kb[kk]));
                    ka[kk] = *(const lds_bf16x8*)(uintptr_t)(kb[kk] + st);
                }
            };
            auto read_v = [&](int tile, bf16x8 (&va)[2][NDT]) {
                const uint32_t st = (tile & (NS - 1)) * G::STAGE;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) {
                        asm volatile("" : "+v"(vb[dt]));
                        const uint32_t ad = vb[dt] + st + (16 * ks) * G::ROWB;
                        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(uintptr_t)ad);
                        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(uintptr_t)(ad + 8 * G::ROWB));
                        va[ks][dt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    }
            };
            // weights of one tile from its scores s; kNext: the score MFMAs of the next tile (operands ka) go between the
            // exponentials and leave their result in s; then O^T += V^T P^T
            auto weights_and_output = [&](auto next_c, f32x16& s, const bf16x8 (&ka)[NKK], const bf16x8 (&va)[2][NDT], int nt) {
                constexpr bool kNext = decltype(next_c)::value;
                bf16x8 pb[2];
                f32x16 sn;
#pragma unroll
                for (int r = 0; r < 16; ++r) sn[r] = 0.f;
                if (MODE == CKV_SOFTMAX) {
                    if (!kNext && nt < TP) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) s[r] = mask_tail(s[r], 8 * (r >> 2) + 4 * hh + (r & 3) >= nt, -INFINITY);
                    }
                    float tmax = s[0];
#pragma unroll
                    for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, s[r]);
                    tmax = fmaxf(tmax, other_half(tmax)) * sc;
                    if (__any(tmax > m_ref[0] + kLazy)) {
                        const float m_new = fmaxf(m_ref[0], tmax);
                        const float alpha = __builtin_amdgcn_exp2f(m_ref[0] - m_new);
                        lsum[0] *= alpha;
#pragma unroll
                        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                            for (int r = 0; r < 16; ++r) oacc[0][dt][r] *= alpha;
                        m_ref[0] = m_new;
                    }
                    if (kNext) {
#pragma unroll
                        for (int kk = 0; kk < NKK; ++kk) sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk], qreg[0][kk], sn, 0, 0, 0);
                    }
                    float psum = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float p = __builtin_amdgcn_exp2f(fmaf(s[r], sc, -m_ref[0]));
                        psum += p;
                        pb[r >> 3][r & 7] = (__bf16)p;
                    }
                    lsum[0] += psum;
                } else {
                    if (!kNext && nt < TP) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) s[r] = mask_tail(s[r], 8 * (r >> 2) + 4 * hh + (r & 3) >= nt, 0.f);
                    }
                    if (kNext) {
#pragma unroll
                        for (int kk = 0; kk < NKK; ++kk) sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk], qreg[0][kk], sn, 0, 0, 0);
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float e = __builtin_amdgcn_exp2f(s[r] * nsc);
                        pb[r >> 3][r & 7] = (__bf16)(s[r] * __builtin_amdgcn_rcpf(1.f + e));
                    }
                }
                if (kNext) {
                    // one score MFMA of the next tile, then a share of this tile's weight arithmetic, eight times
#pragma unroll
                    for (int kk = 0; kk < NKK; ++kk) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
                    }
                }
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt)
                        oacc[0][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[ks][dt], pb[ks], oacc[0][dt], 0, 0, 0);
                if (kNext) s = sn;
            };
            f32x16 s_cur;
            bf16x8 ka[NKK], va[2][NDT];
            front(-(NS - 1));
            back(-(NS - 1));
            front(-(NS - 2));
            back(-(NS - 2));  // publishes tile 0
            front(-1);
            read_k(0, ka);
#pragma unroll
            for (int r = 0; r < 16; ++r) s_cur[r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk) s_cur = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk], qreg[0][kk], s_cur, 0, 0, 0);
            back(-1);
            auto steady = [&](int t) {
                front(t);
                read_k(t + 1, ka);
                read_v(t, va);
                weights_and_output(std::true_type{}, s_cur, ka, va, TP);
                back(t);
            };
            // four tiles per trip, the first a multiple of four: every stage is then a constant of its instruction
            const int nsteady = ntiles - 1;
            for (int j = 0; j < (nsteady >> 2); ++j) {
                const int t4 = j << 2;
                steady(t4);
                steady(t4 + 1);
                steady(t4 + 2);
                steady(t4 + 3);
            }
            for (int t = nsteady & ~3; t < nsteady; ++t) steady(t);
            front(ntiles - 1);
            read_v(ntiles - 1, va);
            weights_and_output(std::false_type{}, s_cur, ka, va, n - (ntiles - 1) * TP);
            back(ntiles - 1);
        };
        // The loop with the scores one tile ahead for 256 columns, where a SIMD holds one wavefront and nothing else hides its
        // vector work: the same schedule of loads, waits and publication as tile_loop_ahead.  Sixteen K operands and sixteen
        // V^T operands per tile do not fit in registers beside the queries, so the K operands of tile t + 1 come through the
        // window of eight that tile_loop uses, under the exponentials of tile t, and the V^T operands of tile t in two halves.
        auto tile_loop_ahead_wide = [&](auto nui_c, auto both_c) {
            constexpr int NUI = decltype(nui_c)::value;
            constexpr int NS = G::NS;
            constexpr int LPI = 2 * G::NI + 1 + NUI;
            static_assert(QG == 1 && NS == 4, "built for one query group on the four-stage ring");
            int rk[G::NI], rv[G::NI];
            gather_rows(both_c, 0, rk, rv);
            auto front = [&](int t) {
                issue_idx(t + NS + 2);
#pragma unroll
                for (int s = 0; s < 2 * G::NI + NUI; ++s) tile_dma(t + NS - 1, s, rk, rv);
            };
            auto back = [&](int t) {
                __builtin_amdgcn_sched_barrier(0);
                wait_vm<(NS - 3) * LPI>();
                if (NUI > 0 && t + 2 >= 0 && t + 2 < ntiles) concat(nui_c, t + 2);
                gather_rows(both_c, t + NS, rk, rv);
                lds_barrier();
            };
            // The same in two parts around the output MFMAs of a tile, whose matrix time then covers the LDS round trips
            // (slice staging -> registers, index slots -> registers) that back() waits out: the wait for the wavefront's loads
            // of tile t + 2, the staged slices and the row lookup in front of the MFMAs, the row tails and the barrier behind.
            // (measured: softmax weights -3 to -6 %; SiLU weights +1 % by itself and -2 % together with the loads that a step
            // then issues between its last MFMAs)
            constexpr bool kSplitBack = true;
            static_assert(!uodd, "slices in whole dwords");
            uint32_t cx[G::NUI_MAX];
            auto back_first = [&](int t) {
                __builtin_amdgcn_sched_barrier(0);
                wait_vm<(NS - 3) * LPI>();
                if (NUI > 0 && t + 2 < ntiles) {
                    const uint32_t st = lds0 + ((t + 2) & (NS - 1)) * G::STAGE;
#pragma unroll
                    for (int u = 0; u < NUI; ++u) cx[u] = *(const lds_u32*)(uintptr_t)(st + 2 * G::KV + (wave * G::NUI_MAX + u) * 256 + lane * 4);
                }
                gather_rows(both_c, t + NS, rk, rv);
                asm volatile("" ::: "memory");  // (the requests stay in front of the MFMAs)
            };
            auto back_second = [&](int t) {
                asm volatile("" ::: "memory");
                if (NUI > 0 && t + 2 < ntiles) {
                    const uint32_t st = lds0 + ((t + 2) & (NS - 1)) * G::STAGE;
#pragma unroll
                    for (int u = 0; u < NUI; ++u)
                        if (uok[u]) *(lds_u32*)(uintptr_t)(st + cdst[u]) = cx[u];
                }
                lds_barrier();
            };
            auto read_k = [&](int tile, int first, int count, bf16x8 (&ka)[NKK]) {
                const uint32_t st = lds0 + (tile & (NS - 1)) * G::STAGE;
#pragma unroll
                for (int kk = first; kk < first + count; ++kk) ka[kk] = *(const lds_bf16x8*)(uintptr_t)(st + krow + (((2 * kk + hh) ^ kx) << 4));
            };
            auto scores = [&](int tile, f32x16& sn) {
                bf16x8 ka[NKK];
                read_k(tile, 0, NKK, ka);
#pragma unroll
                for (int kk = 0; kk < NKK; ++kk) sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk], qreg[0][kk], sn, 0, 0, 0);
            };
            auto load_v = [&](int tile, int ks, bf16x8 (&va)[NDT]) {
                const uint32_t st = lds0 + (tile & (NS - 1)) * G::STAGE;
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) {
                    const uint32_t ad = st + vrow + (16 * ks) * G::ROWB + (((4 * dt + vc) ^ vx) << 4);
                    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(uintptr_t)ad);
                    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(uintptr_t)(ad + 8 * G::ROWB));
                    va[dt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
            };
            // Weights and output of tile t from its scores s; kNext: the sixteen score MFMAs of tile t + 1 go one in front of
            // each of the sixteen weights of a lane, in program order (a scheduling fence after every pair keeps them there:
            // a wavefront issues in order, so what is to run under a matrix instruction has to follow it directly).
            static_assert(NKK == 16, "one score MFMA per weight of a lane");
            auto step = [&](auto next_c, f32x16& s, int t, int nt) {
                constexpr bool kNext = decltype(next_c)::value;
                bf16x8 pb[2], va0[NDT], va1[NDT], ka[NKK];
                f32x16 sn;
#pragma unroll
                for (int r = 0; r < 16; ++r) sn[r] = 0.f;
                load_v(t, 0, va0);
                if (kNext) read_k(t + 1, 0, 8, ka);
                __builtin_amdgcn_sched_barrier(0);
                float psum = 0.f;
                if (MODE == CKV_SOFTMAX) {
                    if (!kNext && nt < TP) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) s[r] = mask_tail(s[r], 8 * (r >> 2) + 4 * hh + (r & 3) >= nt, -INFINITY);
                    }
                    float tmax = s[0];
#pragma unroll
                    for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, s[r]);
                    tmax = fmaxf(tmax, other_half(tmax)) * sc;
                    if (__any(tmax > m_ref[0] + kLazy)) {
                        const float m_new = fmaxf(m_ref[0], tmax);
                        const float alpha = __builtin_amdgcn_exp2f(m_ref[0] - m_new);
                        lsum[0] *= alpha;
#pragma unroll
                        for (int dt = 0; dt < NDT; ++dt) {
                            if (kAccInAgprs) asm volatile("" : "+a"(oacc[0][dt]));
#pragma unroll
                            for (int r = 0; r < 16; ++r) oacc[0][dt][r] *= alpha;
                            if (kAccInAgprs) asm volatile("" : "+a"(oacc[0][dt]));
                        }
                        m_ref[0] = m_new;
                    }
                } else if (!kNext && nt < TP) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[r] = mask_tail(s[r], 8 * (r >> 2) + 4 * hh + (r & 3) >= nt, 0.f);
                }
                __builtin_amdgcn_sched_barrier(0);
                // (values in flight between two MFMAs are tied to an empty asm statement: the compiler orders pure arithmetic
                // freely otherwise and had put all sixteen MFMAs in front of all the weights)
                float pprev = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float sr = s[r];
                    if (kNext) {
                        // the window of eight K operands is refilled four at a time, four MFMAs ahead of their use
                        if (r == 4) read_k(t + 1, 8, 4, ka);
                        if (r == 8) read_k(t + 1, 12, 4, ka);
                        // (the operands are tied group by group, as they were requested: one wait for LDS per group, not per MFMA)
                        if (r == 0) asm volatile("" : "+v"(ka[0]), "+v"(ka[1]), "+v"(ka[2]), "+v"(ka[3]), "+v"(ka[4]), "+v"(ka[5]), "+v"(ka[6]), "+v"(ka[7]));
                        if (r == 8) asm volatile("" : "+v"(ka[8]), "+v"(ka[9]), "+v"(ka[10]), "+v"(ka[11]));
                        if (r == 12) asm volatile("" : "+v"(ka[12]), "+v"(ka[13]), "+v"(ka[14]), "+v"(ka[15]));
                        asm volatile("" : "+v"(sr), "+v"(pprev));
                        sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[r], qreg[0][r], sn, 0, 0, 0);
                    }
                    if (r == 12) {
                        // the second half of the V^T operands, requested here (into the registers the first K operands have
                        // left) so that they have arrived when the first half's MFMAs are through; the fences keep the requests here
                        asm volatile("" ::: "memory");
                        load_v(t, 1, va1);
                        asm volatile("" ::: "memory");
                    }
                    if (r > 0) {
                        if (MODE == CKV_SOFTMAX) psum += pprev;
                        pb[(r - 1) >> 3][(r - 1) & 7] = (__bf16)pprev;
                    }
                    if (MODE == CKV_SOFTMAX) {
                        pprev = __builtin_amdgcn_exp2f(fmaf(sr, sc, -m_ref[0]));
                    } else {
                        const float e = __builtin_amdgcn_exp2f(sr * nsc);
                        pprev = sr * __builtin_amdgcn_rcpf(1.f + e);
                    }
                }
                if (MODE == CKV_SOFTMAX) psum += pprev;
                pb[1][7] = (__bf16)pprev;
                if (MODE == CKV_SOFTMAX) lsum[0] += psum;
                if (kSplitBack) back_first(t);
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) oacc[0][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va0[dt], pb[0], oacc[0][dt], 0, 0, 0);
                if (kSplitBack && kNext) {
                    // The barrier, then the loads of the next iteration with the second half of the output MFMAs between
                    // them, one behind each load (its operand tied to an asm statement there): issuing a tile's loads takes
                    // a wavefront as long as eight MFMAs take the matrix pipe.
                    static_assert(2 * G::NI >= NDT, "a load in front of every MFMA of the second half");
                    __builtin_amdgcn_sched_barrier(0);  // (the first half stays in front of the barrier, over the LDS round trips)
                    back_second(t);
                    issue_idx(t + 1 + NS + 2);
#pragma unroll
                    for (int i = 0; i < 2 * G::NI + NUI; ++i) {
                        tile_dma(t + NS, i, rk, rv);
                        if (i < NDT) {
                            asm volatile("" : "+v"(va1[i]));
                            oacc[0][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va1[i], pb[1], oacc[0][i], 0, 0, 0);
                            __builtin_amdgcn_sched_barrier(0);  // (or the scheduler gathers the MFMAs behind the last load)
                        }
                    }
                    s = sn;
                    return;
                }
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) oacc[0][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va1[dt], pb[1], oacc[0][dt], 0, 0, 0);
                if (kNext) s = sn;
                if (kSplitBack) back_second(t);
            };
            f32x16 s_cur;
            front(-(NS - 1));
            back(-(NS - 1));
            front(-(NS - 2));
            back(-(NS - 2));  // publishes tile 0
            front(-1);
#pragma unroll
            for (int r = 0; r < 16; ++r) s_cur[r] = 0.f;
            scores(0, s_cur);
            back(-1);
            if (kSplitBack) {
                // (a step ends with both parts of back(t) and with the loads that front(t + 1) issues)
                front(0);
                for (int t = 0; t < ntiles - 1; ++t) step(std::true_type{}, s_cur, t, TP);
                step(std::false_type{}, s_cur, ntiles - 1, n - (ntiles - 1) * TP);
            } else {
                for (int t = 0; t < ntiles - 1; ++t) {
                    front(t);
                    step(std::true_type{}, s_cur, t, TP);
                    back(t);
                }
                front(ntiles - 1);
                step(std::false_type{}, s_cur, ntiles - 1, n - (ntiles - 1) * TP);
                back(ntiles - 1);
            }
        };
        // Sixteen queries: the same ring, waits and publication as tile_loop; a tile is two score blocks of sixteen consecutive
        // positions (sixteen consecutive rows per K operand read: no LDS bank conflicts).  A lane ends up with the scores of
        // positions 16 b + 4 (lane / 16) + r (b = 0, 1; r = 0..3); the output instruction, 32 positions deep, takes them as its
        // k indices 8 (lane / 16) + 4 b + r, and the V^T operand is read in that order of positions.
        auto tile_loop_q16 = [&](auto nui_c, auto both_c) {
            constexpr int NUI = decltype(nui_c)::value;
            constexpr int NS = G::NS;
            int rk[G::NI], rv[G::NI];
            gather_rows(both_c, 0, rk, rv);
            // operand addresses within a stage: K rows of the two score blocks (16-byte chunk 4 ks + lane / 16), and the
            // transposed reads of V (the sixteen lanes of a group fetch four positions x sixteen columns, four columns each)
            uint32_t kad[2][2];
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int p = 16 * b + q16;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) kad[b][ks] = p * G::ROWB + (((4 * ks + g4) ^ fk<DA>(p)) << 4);
            }
            const int vp = 4 * g4 + (q16 >> 2);  // position row of the lane's transposed read (and that + 16)
            uint32_t vad[2][4];
#pragma unroll
            for (int hl = 0; hl < 2; ++hl)
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
                    const int p = vp + 16 * hl, col = 16 * dt + 4 * (q16 & 3);
                    vad[hl][dt] = G::KV + p * G::ROWB + (((col >> 3) ^ fv<DA>(p)) << 4) + (col & 7) * 2;
                }
            for (int t = -(NS - 1); t < ntiles; ++t) {
                issue_idx(t + NS + 2);
#pragma unroll
                for (int s = 0; s < 2 * G::NI + NUI; ++s) tile_dma(t + NS - 1, s, rk, rv);
                if (t >= 0) {
                    const uint32_t st = lds0 + (t & (NS - 1)) * G::STAGE;
                    const int nt = min(n - t * TP, TP);
                    bf16x8 ka[2][2], va[4];
#pragma unroll
                    for (int b = 0; b < 2; ++b)
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) ka[b][ks] = *(const lds_bf16x8*)(uintptr_t)(st + kad[b][ks]);
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt) {
                        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(uintptr_t)(st + vad[0][dt]));
                        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(uintptr_t)(st + vad[1][dt]));
                        va[dt] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    }
                    f32x4 sb[2];
#pragma unroll
                    for (int b = 0; b < 2; ++b) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) sb[b][r] = 0.f;
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) sb[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[b][ks], qreg[0][ks], sb[b], 0, 0, 0);
                    }
                    // the lane's eight scores, positions 16 (i / 4) + 4 (lane / 16) + i % 4 of the tile
                    float sv[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) sv[i] = sb[i >> 2][i & 3];
                    bf16x8 pb;
                    if (MODE == CKV_SOFTMAX) {
                        if (nt < TP) {
#pragma unroll
                            for (int i = 0; i < 8; ++i) sv[i] = mask_tail(sv[i], 16 * (i >> 2) + 4 * g4 + (i & 3) >= nt, -INFINITY);
                        }
                        float tmax = sv[0];
#pragma unroll
                        for (int i = 1; i < 8; ++i) tmax = fmaxf(tmax, sv[i]);
                        tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
                        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64)) * sc;
                        if (__any(tmax > m_ref[0] + kLazy)) {
                            const float m_new = fmaxf(m_ref[0], tmax);
                            const float alpha = __builtin_amdgcn_exp2f(m_ref[0] - m_new);
                            lsum[0] *= alpha;
#pragma unroll
                            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                                for (int r = 0; r < 4; ++r) o16[dt][r] *= alpha;
                            m_ref[0] = m_new;
                        }
                        float psum = 0.f;
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const float p = __builtin_amdgcn_exp2f(fmaf(sv[i], sc, -m_ref[0]));
                            psum += p;
                            pb[i] = (__bf16)p;
                        }
                        lsum[0] += psum;
                    } else {
                        if (nt < TP) {
#pragma unroll
                            for (int i = 0; i < 8; ++i) sv[i] = mask_tail(sv[i], 16 * (i >> 2) + 4 * g4 + (i & 3) >= nt, 0.f);
                        }
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const float e = __builtin_amdgcn_exp2f(sv[i] * nsc);
                            pb[i] = (__bf16)(sv[i] * __builtin_amdgcn_rcpf(1.f + e));
                        }
                    }
#pragma unroll
                    for (int dt = 0; dt < 4; ++dt) o16[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[dt], pb, o16[dt], 0, 0, 0);
                }
                wait_vm<(NS - 2) * (2 * G::NI + 1 + NUI)>();
                if (NUI > 0 && t + 1 >= 0 && t + 1 < ntiles) concat(nui_c, t + 1);
                gather_rows(both_c, t + NS, rk, rv);
                lds_barrier();
            }
        };
        constexpr bool kScoresAhead = (DA == 128 && NW == 4 && QG == 1 && UK == 0) || (DA == 256 && UK == 0);
        auto with_nui = [&](auto nui_c) {
            if constexpr (Q16) {
                if (ksh && vsh) tile_loop_q16(nui_c, std::true_type{});
                else tile_loop_q16(nui_c, std::false_type{});
                return;
            }
            if constexpr (kScoresAhead) {
                if (a.scores_ahead) {
                    if constexpr (kWide) {
                        if (ksh && vsh) tile_loop_ahead_wide(nui_c, std::true_type{});
                        else tile_loop_ahead_wide(nui_c, std::false_type{});
                    } else {
                        if (ksh && vsh) tile_loop_ahead(nui_c, std::true_type{});
                        else tile_loop_ahead(nui_c, std::false_type{});
                    }
                    return;
                }
            }
            if (ksh && vsh) tile_loop(nui_c, std::true_type{});
            else tile_loop(nui_c, std::false_type{});
        };
        if (nui == 0) with_nui(std::integral_constant<int, 0>{});
        else if (nui == 1) with_nui(std::integral_constant<int, 1>{});
        else if (G::NUI_MAX >= 2 && nui == 2) with_nui(std::integral_constant<int, G::NUI_MAX >= 2 ? 2 : 0>{});
        else if (G::NUI_MAX >= 4 && nui == 4) with_nui(std::integral_constant<int, G::NUI_MAX >= 4 ? 4 : 0>{});
        else if (G::NUI_MAX >= 8) with_nui(std::integral_constant<int, G::NUI_MAX >= 8 ? 8 : 0>{});
        // the clamped loads past the last tile must have landed, for every wavefront, before the
        // epilogue reuses the stages (and before the workgroup gives its LDS back)
        wait_vm<0>();
        lds_barrier();
        if (tr && tid == 0) tr[2] = wall_clock64();
    }

    // ---- epilogue.  Whole histories: normalise, transpose through LDS (the tile loop's last
    //      barrier has retired every stage) and write complete output rows, 16 bytes per lane.
    //      Pieces of a split history: unnormalised fp32 accumulators, maximum and sum.
    float l_tot[QG];
#pragma unroll
    for (int g = 0; g < QG; ++g) l_tot[g] = MODE == CKV_SOFTMAX ? lsum[g] + other_half(lsum[g]) : 0.f;
    if constexpr (Q16) {
        // a query's sum is spread over the four lanes that share it
        float l16 = 0.f;
        if (MODE == CKV_SOFTMAX) {
            l16 = lsum[0] + __shfl_xor(lsum[0], 16, 64);
            l16 += __shfl_xor(l16, 32, 64);
        }
        if (it.part < 0) {
            float inv;
            if (MODE == CKV_SOFTMAX) inv = l16 > 0.f ? 1.f / l16 : 0.f;
            else inv = it.n_total > 0 ? osc / (float)it.n_total : 0.f;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 4; r += 2) {
                    const int ci = 16 * dt + 4 * g4 + r;
                    const int pc = ci < dgv ? ci + duv : ci - dgv;
                    const uint32_t two = (uint32_t)f2bf(o16[dt][r] * inv) | ((uint32_t)f2bf(o16[dt][r + 1] * inv) << 16);
                    *(lds_u32*)(uintptr_t)(qlds + q16 * QS + pc * 2) = two;
                }
            unsigned char* odst = (unsigned char*)a.out + qbyte0;
#pragma unroll
            for (int i = 0; i < 16 * G::CH / 64; ++i) {
                const int e = i * 64 + lane, row = e / G::CH, c = e % G::CH;
                const u32x4 v = *(const lds_u32x4*)(uintptr_t)(qlds + row * QS + c * 16);
                if (row < qrows) *reinterpret_cast<u32x4*>(odst + (int64_t)row * (DA * 2) + c * 16) = v;
            }
        } else {
            float* ws = a.partial + (int64_t)it.part * a.QB * (DA + 2);
            constexpr int FS = DA * 4 + 16;  // bytes per staged row
            static_assert(16 * FS <= G::NS * G::STAGE, "the staged accumulators must fit in the retired stages");
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int ci = 16 * dt + 4 * g4 + r;
                    const int pc = ci < dgv ? ci + duv : ci - dgv;
                    *(lds_f32*)(uintptr_t)(lds0 + q16 * FS + pc * 4) = o16[dt][r] * osc;
                }
            if (g4 == 0) {
                ws[(int64_t)a.QB * DA + q16] = m_ref[0] * kLn2;
                ws[(int64_t)a.QB * DA + a.QB + q16] = l16;
            }
#pragma unroll
            for (int i = 0; i < 16 * (DA / 4) / 64; ++i) {
                const int e = i * 64 + lane, row = e / (DA / 4), c = e % (DA / 4);
                const u32x4 v = *(const lds_u32x4*)(uintptr_t)(lds0 + row * FS + c * 16);
                *reinterpret_cast<u32x4*>(ws + (int64_t)row * DA + c * 4) = v;
            }
            lds_barrier();
        }
    } else if (it.part < 0) {
#pragma unroll
        for (int g = 0; g < QG; ++g) {
            float inv;
            if (MODE == CKV_SOFTMAX) inv = l_tot[g] > 0.f ? 1.f / l_tot[g] : 0.f;
            else inv = it.n_total > 0 ? osc / (float)it.n_total : 0.f;
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const int ci = 32 * dt + 8 * (r >> 2) + 4 * hh + (r & 3);
                    const int pc = ci < dgv ? ci + duv : ci - dgv;
                    if (!uodd) {
                        const uint32_t two = (uint32_t)f2bf(oacc[g][dt][r] * inv) | ((uint32_t)f2bf(oacc[g][dt][r + 1] * inv) << 16);
                        *(lds_u32*)(uintptr_t)(qlds + (g * 32 + qn) * QS + pc * 2) = two;
                    } else {
                        const int pc1 = ci + 1 < dgv ? ci + 1 + duv : ci + 1 - dgv;
                        *(lds_u16*)(uintptr_t)(qlds + (g * 32 + qn) * QS + pc * 2) = f2bf(oacc[g][dt][r] * inv);
                        *(lds_u16*)(uintptr_t)(qlds + (g * 32 + qn) * QS + pc1 * 2) = f2bf(oacc[g][dt][r + 1] * inv);
                    }
                }
        }
        unsigned char* odst = (unsigned char*)a.out + qbyte0;
#pragma unroll
        for (int i = 0; i < QG * 32 * G::CH / 64; ++i) {
            const int e = i * 64 + lane, row = e / G::CH, c = e % G::CH;
            const u32x4 v = *(const lds_u32x4*)(uintptr_t)(qlds + row * QS + c * 16);
            if (row < qrows) *reinterpret_cast<u32x4*>(odst + (int64_t)row * (DA * 2) + c * 16) = v;
        }
    } else {
        // the fp32 accumulators go through LDS too (a lane holds one query's columns; written straight
        // to memory every store would touch 64 cache lines), then out as whole rows, 16 bytes per lane
        float* ws = a.partial + (int64_t)it.part * a.QB * (DA + 2);
        constexpr int FS = DA * 4 + 16;  // bytes per staged row
        static_assert(NW * QG * 32 * FS <= G::NS * G::STAGE, "the staged accumulators must fit in the retired stages");
        const uint32_t flds = lds0 + wave * (QG * 32 * FS);
#pragma unroll
        for (int g = 0; g < QG; ++g) {
            const int j = (wave * QG + g) * 32 + qn;
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ci = 32 * dt + 8 * (r >> 2) + 4 * hh + (r & 3);
                    const int pc = ci < dgv ? ci + duv : ci - dgv;
                    *(lds_f32*)(uintptr_t)(flds + (g * 32 + qn) * FS + pc * 4) = oacc[g][dt][r] * osc;
                }
            if (hh == 0) {
                ws[(int64_t)a.QB * DA + j] = m_ref[g] * kLn2;
                ws[(int64_t)a.QB * DA + a.QB + j] = l_tot[g];
            }
        }
        float* wdst = ws + (int64_t)(wave * QG * 32) * DA;
#pragma unroll
        for (int i = 0; i < QG * 32 * (DA / 4) / 64; ++i) {
            const int e = i * 64 + lane, row = e / (DA / 4), c = e % (DA / 4);
            const u32x4 v = *(const lds_u32x4*)(uintptr_t)(flds + row * FS + c * 16);
            *reinterpret_cast<u32x4*>(wdst + (int64_t)row * DA + c * 4) = v;
        }
        // this wavefront's staging rows lie where other wavefronts stage the next item's queries
        lds_barrier();
    }
    if (tr && tid == 0) tr[3] = wall_clock64();
    }  // items of this workgroup
}

template <int DA, int NW, int QG, int MODE, int UK, bool Q16 = false>
hipError_t prepare() {
    constexpr int lds = Geo<DA, NW, (UK >= 2)>::LDS;
    static hipError_t done =
        hipFuncSetAttribute((const void*)ckv_dma_kernel<DA, NW, QG, MODE, UK, Q16>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    return done;
}

template <int DA, int NW, int QG, int MODE, int UK, bool Q16 = false>
hipError_t launch(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    hipError_t e = prepare<DA, NW, QG, MODE, UK, Q16>();
    if (e != hipSuccess) return e;
    constexpr int lds = Geo<DA, NW, (UK >= 2)>::LDS;
    hipLaunchKernelGGL((ckv_dma_kernel<DA, NW, QG, MODE, UK, Q16>), dim3(c->n_wg), dim3(NW * 64), lds, s, a, c->nui);
    return hipGetLastError();
}

template <int DA, int NW, int QG, int MODE, int UK, bool Q16 = false>
int occupancy() {
    if (prepare<DA, NW, QG, MODE, UK, Q16>() != hipSuccess) return 0;
    int nb = 0;
    constexpr int lds = Geo<DA, NW, (UK >= 2)>::LDS;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, (const void*)ckv_dma_kernel<DA, NW, QG, MODE, UK, Q16>, NW * 64, lds) !=
        hipSuccess)
        return 0;
    return nb;
}

// (d_a, wavefronts per workgroup, query groups per wavefront)
#define CKV_DMA_SHAPES(X) \
    X(64, 1, 1) X(64, 1, 2) X(64, 2, 1) X(64, 2, 2) X(64, 4, 1) X(128, 1, 1) X(128, 1, 2) X(128, 2, 1) X(128, 2, 2) X(128, 4, 1) \
    X(256, 4, 1)
// (d_a, wavefronts) of the instantiations with one query group that exist for odd and for wide user slices
#define CKV_DMA_NARROW(X) X(64, 1) X(64, 2) X(64, 4) X(128, 1) X(128, 2) X(128, 4)

}  // namespace

bool ckv_dma_supported(int d_a, int nw, int qg) {
#define X(DA, NW, QG) \
    if (d_a == DA && nw == NW && qg == QG) return true;
    CKV_DMA_SHAPES(X)
#undef X
    return false;
}

// Number of user-slice load instructions per wavefront and tile, or -1 if the shape is not
// served by this kernel.
int ckv_dma_nui(int d_a, int nw, int d_u) {
    if ((d_a != 64 && d_a != 128 && d_a != 256) || (nw != 1 && nw != 2 && nw != 4)) return -1;
    if (d_a == 256 && nw != 4) return -1;  // (256 columns: four wavefronts only)
    if (d_u < 0 || d_u > (d_a == 256 ? 32 : 16) || ((d_u & 1) && d_u > 7)) return -1;
    // lanes that move the user slices of a tile: one per dword, or one per element when d_u is odd
    const int need = ((d_u & 1 ? 64 : 32) * d_u + nw * 64 - 1) / (nw * 64);
    return need <= 1 ? need : (need <= 2 ? 2 : (need <= 4 ? 4 : 8));  // (never above NUI_MAX of the geometry that serves the shape)
}

// (user slices of 10 to 16 columns, or of 5 or 7, at 64 or 128 columns: the instantiations with the larger staging area)
static bool wide_slices(int d_a, int d_u) { return d_a != 256 && (d_u & 1 ? d_u > 3 : d_u > 8); }

// Sixteen-query organisation (64 columns, one wavefront, even user slices of up to 8 columns).
bool ckv_dma_q16_supported(int d_a, int d_u, int d_g) { return d_a == 64 && (d_g == 0 || (!(d_u & 1) && d_u <= 8)); }
int ckv_dma_q16_occupancy(int mode) {
    return mode == CKV_SOFTMAX ? occupancy<64, 1, 1, CKV_SOFTMAX, 0, true>() : occupancy<64, 1, 1, CKV_SILU_OVER_N, 0, true>();
}

int ckv_dma_occupancy(int d_a, int nw, int qg, int mode, int d_u) {
    if ((d_u & 1) && !wide_slices(d_a, d_u)) {
#define X(DA, NW)                          \
    if (d_a == DA && nw == NW && qg == 1)  \
        return mode == CKV_SOFTMAX ? occupancy<DA, NW, 1, CKV_SOFTMAX, 1>() : occupancy<DA, NW, 1, CKV_SILU_OVER_N, 1>();
        CKV_DMA_NARROW(X) X(256, 4)
#undef X
        return 0;
    }
    if (d_u & 1) {
#define X(DA, NW)                          \
    if (d_a == DA && nw == NW && qg == 1)  \
        return mode == CKV_SOFTMAX ? occupancy<DA, NW, 1, CKV_SOFTMAX, 3>() : occupancy<DA, NW, 1, CKV_SILU_OVER_N, 3>();
        CKV_DMA_NARROW(X)
#undef X
        return 0;
    }
    if (wide_slices(d_a, d_u)) {
#define X(DA, NW)                          \
    if (d_a == DA && nw == NW && qg == 1)  \
        return mode == CKV_SOFTMAX ? occupancy<DA, NW, 1, CKV_SOFTMAX, 2>() : occupancy<DA, NW, 1, CKV_SILU_OVER_N, 2>();
        CKV_DMA_NARROW(X)
#undef X
        return 0;
    }
#define X(DA, NW, QG)                          \
    if (d_a == DA && nw == NW && qg == QG)     \
        return mode == CKV_SOFTMAX ? occupancy<DA, NW, QG, CKV_SOFTMAX, 0>() : occupancy<DA, NW, QG, CKV_SILU_OVER_N, 0>();
    CKV_DMA_SHAPES(X)
#undef X
    return 0;
}

hipError_t ckv_launch_dma(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    if (c->n_items == 0) return hipSuccess;
    const int d_a = a.d_a, nw = c->nw, qg = c->qg;
    if (c->q16)
        return c->shape.mode == CKV_SOFTMAX ? launch<64, 1, 1, CKV_SOFTMAX, 0, true>(c, a, s) : launch<64, 1, 1, CKV_SILU_OVER_N, 0, true>(c, a, s);
    if ((a.d_u & 1) && wide_slices(d_a, a.d_u)) {  // one query group per wavefront only
#define X(DA, NW)                                                                       \
    if (d_a == DA && nw == NW && qg == 1)                                               \
        return c->shape.mode == CKV_SOFTMAX ? launch<DA, NW, 1, CKV_SOFTMAX, 3>(c, a, s) \
                                            : launch<DA, NW, 1, CKV_SILU_OVER_N, 3>(c, a, s);
        CKV_DMA_NARROW(X)
#undef X
        return hipErrorInvalidValue;
    }
    if (a.d_u & 1) {  // one query group per wavefront only
#define X(DA, NW)                                                                          \
    if (d_a == DA && nw == NW && qg == 1)                                                  \
        return c->shape.mode == CKV_SOFTMAX ? launch<DA, NW, 1, CKV_SOFTMAX, 1>(c, a, s) \
                                            : launch<DA, NW, 1, CKV_SILU_OVER_N, 1>(c, a, s);
        CKV_DMA_NARROW(X) X(256, 4)
#undef X
        return hipErrorInvalidValue;
    }
    if (a.d_g > 0 && wide_slices(d_a, a.d_u)) {  // one query group per wavefront only
#define X(DA, NW)                                                                       \
    if (d_a == DA && nw == NW && qg == 1)                                               \
        return c->shape.mode == CKV_SOFTMAX ? launch<DA, NW, 1, CKV_SOFTMAX, 2>(c, a, s) \
                                            : launch<DA, NW, 1, CKV_SILU_OVER_N, 2>(c, a, s);
        CKV_DMA_NARROW(X)
#undef X
        return hipErrorInvalidValue;
    }
#define X(DA, NW, QG)                                                                           \
    if (d_a == DA && nw == NW && qg == QG)                                                      \
        return c->shape.mode == CKV_SOFTMAX ? launch<DA, NW, QG, CKV_SOFTMAX, 0>(c, a, s)    \
                                            : launch<DA, NW, QG, CKV_SILU_OVER_N, 0>(c, a, s);
    CKV_DMA_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}
