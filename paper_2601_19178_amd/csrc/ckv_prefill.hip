// Prefill stage of CollectiveKV (paper section 4.2 "In the prefill stage", section 4.3 router):
//   K_u = S W_k + b_k, V_u = S W_v + b_v            (projection to the d_u user-specific columns)
//   M = S W_r + b_r,  I[i] = argmax_j M[i][j]        (router; one for keys, one for values)
// written straight into the packed cache layout the attention kernels stream (indices
// [2][H][T], user slices [H][T][d_u]).  The routing map M (T x P per head and side) is never
// written anywhere: every workgroup keeps a block of positions in registers, streams the
// router weights through LDS in tiles of 32 pool entries and keeps a running (maximum, index)
// per position.
//
// Matrix-core kernel (d_e up to 256 in whole 16-byte chunks; built for 64, 128 and 256 columns, bf16 storage
// on v_mfma_f32_32x32x16_bf16, fp32 storage on v_mfma_f32_32x32x2_f32): M^T = W_r S^T,
// router rows as the A operand (read from LDS), positions as the B
// operand (registers), so that a lane owns one position and sixteen pool entries of the tile;
// the bias enters as the initial value of the accumulator (fp32, exact).  The maximum over the
// lane's sixteen entries costs eight v_max3; only when it beats the lane's running maximum
// (rare after the first tiles) is the entry that attains it located.  Equal scores keep the
// lowest pool entry: tiles are visited in increasing order and replaced only on a strict
// improvement, and inside a tile the lowest matching register wins.
// The projection is more tiles of the same kind whose 32 "pool entries" are rows of W_k (or W_v):
// one tile for the usual small d_u, d_a / 32 tiles for a side that is not shared.
//
// Scalar kernel: any other d_e (wider than 256, or rows that are not whole 16-byte chunks), either storage
// type, one thread per (position, head, side).
#include <algorithm>
#include <type_traits>

#include "ckv_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((address_space(3))) unsigned char lds_u8;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) f32x4 lds_f32x4;

constexpr int SR = 32;  // pool entries per MFMA row block

__device__ __forceinline__ void dma16(const void* g, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_base) : "memory");
}
// 16 bytes per lane from (wavefront-uniform base + per-lane 32-bit offset) to LDS[lds_base + 16*lane]
__device__ __forceinline__ void dma16_uniform(const void* base, uint32_t off, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_base) : "memory");
}
__device__ __forceinline__ void dma4(const void* g, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(g), "s"(lds_base) : "memory");
}
__device__ __forceinline__ void dma4_uniform(const void* base, uint32_t off, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(base), "s"(lds_base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
__device__ __forceinline__ uint32_t swap_halves(uint32_t x) {
    auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return threadIdx.x & 32 ? r[0] : r[1];
}
__device__ __forceinline__ uint16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

// One 16-byte chunk of a router row (A) against the same chunk of a position's embedding (B).  bf16: eight
// products per lane half in one v_mfma_f32_32x32x16_bf16.  fp32: four v_mfma_f32_32x32x2_f32; the
// instruction takes k = 0 from lanes 0-31 and k = 1 from lanes 32-63, and since the lane halves hold
// consecutive chunks, element e of both chunks is a valid (k = 0, k = 1) pair: the order in which the
// columns of a row are summed is permuted, which no result depends on beyond rounding.
template <typename U>
__device__ __forceinline__ f32x16 mma_chunk(u32x4 wa, u32x4 sb, f32x16 c);
template <>
__device__ __forceinline__ f32x16 mma_chunk<uint16_t>(u32x4 wa, u32x4 sb, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wa), __builtin_bit_cast(bf16x8, sb), c, 0, 0, 0);
}
template <>
__device__ __forceinline__ f32x16 mma_chunk<float>(u32x4 wa, u32x4 sb, f32x16 c) {
#pragma unroll
    for (int e = 0; e < 4; ++e) c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(wa[e]), __uint_as_float(sb[e]), c, 0, 0, 0);
    return c;
}
__device__ __forceinline__ void store_user(uint16_t* p, float x) { *p = __builtin_bit_cast(uint16_t, (__bf16)x); }
__device__ __forceinline__ void store_user(float* p, float x) { *p = x; }

// TR = pool entries per stage (one barrier per stage), NS = stages in the LDS ring.
template <int ES, int DE, int NW, int TR, int NS>
struct PGeo {
    static constexpr int ROWB = DE * ES;         // bytes per weight row (ES = bytes per stored element)
    static constexpr int CH = ROWB / 16;         // 16-byte chunks per weight row
    static constexpr int RPI = 64 / CH;          // rows filled by one wavefront load instruction
    static constexpr int NI = TR / RPI / NW;     // load instructions per wavefront and stage
    static constexpr int WT = TR * ROWB;         // bytes of the weight rows of a stage
    static constexpr int STAGE = WT + NW * 256;  // plus one private copy of the (up to 64) biases per wavefront
    static constexpr int LDS = NS * STAGE;
    static constexpr int NSUB = TR / SR;         // MFMA row blocks per stage
    // 16-byte chunk c of row p is stored at slot c ^ swz(p).  A 16-byte-per-lane LDS read is served sixteen
    // lanes at a time from 64 banks, so sixteen consecutive rows must land in sixteen different slots
    // modulo 16: rows of 256 bytes or more use the low four bits of the row, rows of 128 bytes (two rows
    // per 16 slots) the next three.
    __device__ static constexpr int swz(int p) { return CH >= 16 ? (p & 15) : ((p >> 1) & 7); }
    static_assert(NI >= 1 && (TR == 32 || TR == 64), "stage geometry");
};

// One workgroup: NW wavefronts x QG groups x 32 positions, one (head, side).
// WPE resident wavefronts per SIMD; with at most 256 registers per wavefront the accumulators live in
// ordinary vector registers, where the maximum search reads them without copies.  Three wavefronts per
// SIMD measured 10 % faster than two: while one searches its accumulators another feeds the matrix core.
template <typename U, int DE, int NW, int QG, int TR, int NS, int WPE>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(WPE, WPE))) void ckv_prefill_mfma_kernel(ckv_prefill_args a) {
    using G = PGeo<sizeof(U), DE, NW, TR, NS>;
    constexpr int NKK = G::CH / 2;  // k-steps: one 16-byte chunk per lane half each
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_u8*)smem;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int qn = lane & 31, hh = lane >> 5;
    const int ncls = 2 * a.H;
    // Blocks from split_first on are cut into split_s workgroups, each taking a share of the router tiles
    // (see launch_mfma); `part` of `nparts` is this workgroup's share.
    int64_t blk = blockIdx.x;
    int part = 0, nparts = 1;
    if (blk >= a.split_first) {
        const int64_t u = blk - a.split_first;
        blk = a.split_first + u / a.split_s;
        part = (int)(u % a.split_s);
        nparts = a.split_s;
    }
    const int cls = (int)(blk % ncls);
    const int64_t pblock = blk / ncls;
    const int h = cls >> 1, side = cls & 1;
    const int P = a.P[side], d_u = a.d_u[side];  // this side's pool entries (0: not shared) and projected columns

    // d_e may be smaller than the width DE the kernel is built for: rows in memory are `rs` bytes apart and
    // hold `nch` 16-byte chunks; the missing columns are zeros of the embedding (the weight chunk loaded
    // for them is a valid one of the same row, multiplied by zero)
    const int rs = a.d_e * (int)sizeof(U);
    const int nch = rs >> 4;
    const unsigned char* __restrict__ wr = (const unsigned char*)a.w_r[side] + (int64_t)h * P * rs;
    const float* __restrict__ br = a.b_r[side] + (int64_t)h * P;
    const unsigned char* __restrict__ wu = (const unsigned char*)a.w_u[side] + (int64_t)h * d_u * rs;
    const float* __restrict__ bu = a.b_u[side] + (int64_t)h * d_u;
    const int nfull = P / TR;                      // stages made of TR valid router rows
    const int nrt = (P + TR - 1) / TR;             // router stages
    const int npj = (d_u + SR - 1) / SR;           // projection stages: 32 columns of the user slice each
    // this workgroup's stages: router tiles [t_lo, t_hi), then (first part only) the projection tiles
    const int t_lo = (int)((int64_t)nrt * part / nparts), t_hi = (int)((int64_t)nrt * (part + 1) / nparts);
    const int nr_loc = t_hi - t_lo;
    const int n_loc = nr_loc + (part == 0 ? npj : 0);
    if (n_loc == 0) return;

    // ---- positions of this wavefront: B operands, 16 bytes per lane and k-step, straight from S
    const int64_t pos0 = pblock * (32 * QG * NW) + (int64_t)wave * QG * 32;
    u32x4 sreg[QG][NKK];
#pragma unroll
    for (int g = 0; g < QG; ++g) {
        const int64_t pos = pos0 + g * 32 + qn;
        const unsigned char* src = (const unsigned char*)a.S + pos * rs + hh * 16;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (pos < a.T && 2 * kk + hh < nch) v = *reinterpret_cast<const u32x4*>(src + kk * 32);
            sreg[g][kk] = v;
        }
    }
    // these loads have to be complete before the asynchronous loads below start: a wait the
    // compiler placed inside the tile loop would also drain the loads it cannot see
#pragma unroll
    for (int g = 0; g < QG; ++g)
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) asm volatile("" : "+v"(sreg[g][kk]));

    // ---- per-lane constants of the weight loads: instruction i of this wavefront fills rows
    //      (i*NW + wave)*RPI .. +RPI of the stage; chunk c of row p is stored at slot c ^ swz(p).
    //      For a stage of TR valid rows the per-lane byte offset inside the stage never changes and
    //      the stage base is wavefront-uniform, so issuing a load costs no vector arithmetic.
    int lrow[G::NI];
    uint32_t lchunk[G::NI], loff[G::NI];
#pragma unroll
    for (int i = 0; i < G::NI; ++i) {
        lrow[i] = (i * NW + wave) * G::RPI + lane / G::CH;
        lchunk[i] = (uint32_t)(min((lane % G::CH) ^ G::swz(lrow[i]), nch - 1) * 16);
        loff[i] = (uint32_t)lrow[i] * rs + lchunk[i];
    }
    const uint32_t boff = (uint32_t)(lane & (TR - 1)) * 4;
    // stage i of this workgroup when it is known to be a router tile of TR valid rows: no test, no vector arithmetic
    auto issue_full = [&](int i, auto slot_c) {
        constexpr int SLOT = decltype(slot_c)::value;  // ring slot of stage i when the caller knows it (-1: i % NS)
        const uint32_t st = __builtin_amdgcn_readfirstlane(lds0 + (SLOT >= 0 ? SLOT : i % NS) * G::STAGE);  // (uniform; kept in a scalar register)
        const int tile = __builtin_amdgcn_readfirstlane(t_lo + i);  // (uniform anyway; the loads take it in scalar registers)
        const unsigned char* base = wr + (int64_t)tile * (TR * rs);
#pragma unroll
        for (int k = 0; k < G::NI; ++k) dma16_uniform(base, loff[k], st + (k * NW + wave) * G::RPI * G::ROWB);
        dma4_uniform(br + (int64_t)tile * TR, boff, st + G::WT + wave * 256);
    };
    auto issue = [&](int i) {  // stage i of this workgroup (past the last one: a repeat nothing reads)
        const uint32_t st = __builtin_amdgcn_readfirstlane(lds0 + (i % NS) * G::STAGE);  // (uniform; kept in a scalar register)
        const int ic = min(i, n_loc - 1);
        int tile = ic < nr_loc ? t_lo + ic : nrt + (ic - nr_loc);
        if (i < nr_loc && tile < nfull) {
            const unsigned char* base = wr + (int64_t)tile * (TR * rs);
#pragma unroll
            for (int i = 0; i < G::NI; ++i) dma16_uniform(base, loff[i], st + (i * NW + wave) * G::RPI * G::ROWB);
            dma4_uniform(br + (int64_t)tile * TR, boff, st + G::WT + wave * 256);
            return;
        }
        // ragged last router stage, a projection stage, or a repeat of the last stage into a retired
        // slot (never read): rows are clamped to the last valid one
        const bool proj = tile >= nrt;
        const unsigned char* wbase = proj ? wu : wr;
        const float* bbase = proj ? bu : br;
        const int row0 = proj ? (tile - nrt) * SR : tile * TR;
        const int rmax = (proj ? d_u : P) - 1;
#pragma unroll
        for (int i = 0; i < G::NI; ++i) {
            const int row = min(row0 + lrow[i], rmax);
            dma16(wbase + (int64_t)row * rs + lchunk[i], st + (i * NW + wave) * G::RPI * G::ROWB);
        }
        dma4(bbase + min(row0 + (lane & (TR - 1)), rmax), st + G::WT + wave * 256);
    };

    float bv[QG];
    int bj[QG];
#pragma unroll
    for (int g = 0; g < QG; ++g) {
        bv[g] = -INFINITY;
        bj[g] = 0;
    }
    const uint32_t arow = qn * G::ROWB;
    const int ax = G::swz(qn);
    uint32_t waoff[NKK];  // this lane's sixteen-byte pieces of its router row within a stage, one per k-step
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) waoff[kk] = lds0 + arow + (((2 * kk + hh) ^ ax) << 4);
    const uint32_t boff_lane = lds0 + G::WT + wave * 256 + 16 * hh;  // this lane's biases within a stage

    // One stage: KIND 0 = TR valid router rows, 1 = last router stage with fewer, 2 = projection
    // (32 columns of the user slice).
    // The three are separate instantiations so that the loop over full stages stays free of their branches.
    // Iteration t issues the loads of stage t+NS-1 into the slot stage t-1 used (retired by the barrier at
    // the end of iteration t-1), computes stage t, then waits until only the loads of the last NS-2 issues
    // are outstanding, i.e. until its own part of stage t+1 has landed; the barrier publishes stage t+1.
    // SLOT: the ring slot of stage t when it is known at compile time (the loop over full stages is unrolled over the
    // ring, so that the stage's offset becomes an immediate of the LDS reads instead of a vector addition per read), else -1.
    auto stage = [&](auto kind, int t, auto full_ahead, auto slot_c) {
        constexpr int KIND = decltype(kind)::value;
        constexpr int SLOT = decltype(slot_c)::value;
        if (decltype(full_ahead)::value) issue_full(t + NS - 1, std::integral_constant<int, (SLOT >= 0 ? (SLOT + NS - 1) % NS : -1)>{});
        else issue(t + NS - 1);
        const uint32_t st = (SLOT >= 0 ? SLOT : t % NS) * G::STAGE;  // (offset of the stage; the lane's part of an address is loop-invariant)
        u32x4 wa[NKK];  // A operand: this lane's router row, all k-steps
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) wa[kk] = *(const lds_u32x4*)(uintptr_t)(waoff[kk] + st);
        f32x16 acc[QG];  // accumulators start from the biases of this lane's sixteen rows
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const f32x4 b4 = *(const lds_f32x4*)(uintptr_t)(boff_lane + (st + 32 * g4));
#pragma unroll
            for (int g = 0; g < QG; ++g)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[g][4 * g4 + j] = b4[j];
        }
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
            for (int g = 0; g < QG; ++g) acc[g] = mma_chunk<U>(wa[kk], sreg[g][kk], acc[g]);
        if (KIND == 2) {
            // projection: row c of the block is column c0 + c of the user slice
            const int c0 = (t - nr_loc) * SR;
#pragma unroll
            for (int g = 0; g < QG; ++g) {
                const int64_t pos = pos0 + g * 32 + qn;
                if (pos < a.T) {
                    U* dst = (U*)a.user[side] + ((int64_t)h * a.T + pos) * d_u;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int c = c0 + 8 * (r >> 2) + 4 * hh + (r & 3);
                        if (c < d_u) store_user(dst + c, acc[g][r]);
                    }
                }
            }
        } else {
            const int j0 = (t_lo + t) * TR;
            float tmax[QG];
#pragma unroll
            for (int g = 0; g < QG; ++g) {
                if (KIND == 1) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (j0 + 8 * (r >> 2) + 4 * hh + (r & 3) >= P) acc[g][r] = -INFINITY;
                }
                tmax[g] = acc[g][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) tmax[g] = fmaxf(tmax[g], acc[g][r]);
            }
            // the entry that attains a new maximum is located only when some lane of the wavefront has one
#pragma unroll
            for (int g = 0; g < QG; ++g) {
                if (__any(tmax[g] > bv[g])) {
                    int rr = 15;
#pragma unroll
                    for (int r = 14; r >= 0; --r) rr = acc[g][r] == tmax[g] ? r : rr;
                    if (tmax[g] > bv[g]) {
                        bv[g] = tmax[g];
                        bj[g] = j0 + 8 * (rr >> 2) + 4 * hh + (rr & 3);
                    }
                }
            }
        }
        wait_vm<(NS - 2) * (G::NI + 1)>();
        lds_barrier();
    };
    static_assert(G::NSUB == 1, "one row block per stage");
#pragma unroll
    for (int i = 0; i < NS - 1; ++i) issue(i);
    wait_vm<(NS - 2) * (G::NI + 1)>();
    lds_barrier();
    int t = 0;
    // while the stage issued NS-1 ahead is itself a full router tile the loop body has no branch for it
    const int t_ahead = min(nr_loc, nfull - t_lo) - (NS - 1);
    constexpr std::integral_constant<int, -1> any_slot{};
    // (t is a multiple of NS at the top of every round of this loop: stage t + k sits in ring slot k)
    for (; t + NS <= t_ahead; t += NS) {
        stage(std::integral_constant<int, 0>{}, t, std::true_type{}, std::integral_constant<int, 0>{});
        stage(std::integral_constant<int, 0>{}, t + 1, std::true_type{}, std::integral_constant<int, 1 % NS>{});
        if (NS > 2) stage(std::integral_constant<int, 0>{}, t + 2, std::true_type{}, std::integral_constant<int, 2 % NS>{});
        if (NS > 3) stage(std::integral_constant<int, 0>{}, t + 3, std::true_type{}, std::integral_constant<int, 3 % NS>{});
    }
    for (; t < t_ahead; ++t) stage(std::integral_constant<int, 0>{}, t, std::true_type{}, any_slot);
    for (; t < nr_loc && t_lo + t < nfull; ++t) stage(std::integral_constant<int, 0>{}, t, std::false_type{}, any_slot);
    if (t < nr_loc) stage(std::integral_constant<int, 1>{}, t++, std::false_type{}, any_slot);  // the part that owns the ragged last router tile
    for (; t < n_loc; ++t) stage(std::integral_constant<int, 2>{}, t, std::false_type{}, any_slot);
    wait_vm<0>();  // the repeated loads past the last stage must land before the workgroup gives its LDS back

    if (nr_loc > 0) {
#pragma unroll
        for (int g = 0; g < QG; ++g) {
            const float ov = __uint_as_float(swap_halves(__float_as_uint(bv[g])));
            const int oj = (int)swap_halves((uint32_t)bj[g]);
            const bool other = ov > bv[g] || (ov == bv[g] && oj < bj[g]);
            const int best = other ? oj : bj[g];
            const int64_t pos = pos0 + g * 32 + qn;
            if (hh == 0 && pos < a.T) {
                if (nparts == 1) {
                    a.idx[((int64_t)side * a.H + h) * a.T + pos] = best;
                } else {
                    // the parts of a block meet in one 64-bit maximum per position: score (as an ordered
                    // integer, -0 folded into +0) above, complement of the index below, so that of equal
                    // scores the lowest pool entry wins, as inside a workgroup
                    const uint32_t u = __float_as_uint((other ? ov : bv[g]) + 0.0f);
                    const uint32_t ord = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
                    const unsigned long long key = ((unsigned long long)ord << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)best);
                    atomicMax(a.ws + (blk - a.split_first) * (32 * QG * NW) + (wave * QG + g) * 32 + qn, key);
                }
            }
        }
    }
}

// Indices of the positions whose blocks were split: unpack the winning key, leave the workspace zeroed
// for the next call.
__global__ __launch_bounds__(256) void ckv_prefill_finish_kernel(ckv_prefill_args a, int per_wg, int64_t entries) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= entries) return;
    const int ncls = 2 * a.H;
    const int64_t blk = a.split_first + e / per_wg;
    const int cls = (int)(blk % ncls);
    const int h = cls >> 1, side = cls & 1;
    const int64_t pos = blk / ncls * per_wg + e % per_wg;
    const unsigned long long key = a.ws[e];
    a.ws[e] = 0ull;
    if (pos < a.T && a.P[side] > 0) a.idx[((int64_t)side * a.H + h) * a.T + pos] = (int32_t)(0xFFFFFFFFu - (uint32_t)key);
}

// Any d_e, fp32 or bf16 storage: one thread per (position, head, side); fp32 accumulation in
// column order, bias added last; the first maximum wins.
template <typename U>
__device__ __forceinline__ float widen(U x);
template <>
__device__ __forceinline__ float widen<float>(float x) { return x; }
template <>
__device__ __forceinline__ float widen<uint16_t>(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }
__device__ __forceinline__ void narrow(float* p, float x) { *p = x; }
__device__ __forceinline__ void narrow(uint16_t* p, float x) { *p = f2bf(x); }

template <typename U>
__global__ __launch_bounds__(256) void ckv_prefill_scalar_kernel(ckv_prefill_args a) {
    const int64_t total = a.T * a.H * 2;
    const int d_e = a.d_e;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        // consecutive threads take consecutive positions of one (head, side): the weight rows they
        // read are the same, the S rows are neighbours
        const int64_t pos = i % a.T;
        const int cls = (int)(i / a.T);
        const int h = cls >> 1, side = cls & 1;
        const U* __restrict__ s = (const U*)a.S + pos * d_e;
        const int P = a.P[side], d_u = a.d_u[side];
        if (P > 0) {
            const U* __restrict__ w = (const U*)a.w_r[side] + (int64_t)h * P * d_e;
            const float* __restrict__ b = a.b_r[side] + (int64_t)h * P;
            float best = -INFINITY;
            int bj = 0;
            for (int j = 0; j < P; ++j) {
                float m = 0.f;
                for (int c = 0; c < d_e; ++c) m = fmaf(widen<U>(s[c]), widen<U>(w[(int64_t)j * d_e + c]), m);
                m += b[j];
                if (m > best) {
                    best = m;
                    bj = j;
                }
            }
            a.idx[((int64_t)side * a.H + h) * a.T + pos] = bj;
        }
        if (d_u > 0) {
            const U* __restrict__ w = (const U*)a.w_u[side] + (int64_t)h * d_u * d_e;
            const float* __restrict__ b = a.b_u[side] + (int64_t)h * d_u;
            U* dst = (U*)a.user[side] + ((int64_t)h * a.T + pos) * d_u;
            for (int c0 = 0; c0 < d_u; ++c0) {
                float m = 0.f;
                for (int c = 0; c < d_e; ++c) m = fmaf(widen<U>(s[c]), widen<U>(w[(int64_t)c0 * d_e + c]), m);
                narrow(dst + c0, m + b[c0]);
            }
        }
    }
}

// Split policy.  All workgroups do the same amount of work, so a launch of nb blocks on `slots` resident
// workgroups runs in rounds and the last round is only partly full (or the only round, for a short batch).
// When it is less than 60 % full, each of its blocks is cut into s workgroups that take 1/s of the router
// tiles each and meet in a 64-bit atomic maximum per position (workspace of the handle), so that the round
// fills the chip: a batch of one or two users then uses all compute units instead of a handful.
struct SplitPlan {
    int64_t first;  // first split block (== nb: nothing is split)
    int s;
    int64_t entries;  // workspace entries needed
};
static SplitPlan plan_split(int64_t nb, int64_t slots, int per_wg, int max_router_tiles, size_t ws_entries) {
    SplitPlan p{nb, 1, 0};
    if (nb == 0 || slots <= 0) return p;
    const int64_t rem = nb % slots;
    if (rem == 0 || rem * 10 > slots * 6) return p;
    const int64_t s = std::min<int64_t>(std::min<int64_t>(slots / rem, max_router_tiles / 8), 64);
    if (s < 2 || (size_t)(rem * per_wg) > ws_entries) return p;
    p.first = nb - rem;
    p.s = (int)s;
    p.entries = rem * per_wg;
    return p;
}

template <typename U, int DE, int NW, int QG, int TR, int NS, int WPE>
int64_t resident_slots() {
    static const int64_t slots = [] {
        int dev = 0, cus = 0, per_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess) return (int64_t)0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return (int64_t)0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)ckv_prefill_mfma_kernel<U, DE, NW, QG, TR, NS, WPE>,
                                                         NW * 64, PGeo<sizeof(U), DE, NW, TR, NS>::LDS) != hipSuccess)
            return (int64_t)0;
        return (int64_t)cus * per_cu;
    }();
    return slots;
}

template <typename U, int DE, int NW, int QG, int TR, int NS, int WPE>
hipError_t launch_mfma(ckv_prefill_args a, hipStream_t s, bool plan_only, int64_t* entries) {
    constexpr int lds = PGeo<sizeof(U), DE, NW, TR, NS>::LDS;
    static_assert(lds <= 163840, "LDS of one compute unit");
    static hipError_t prepared = hipFuncSetAttribute((const void*)ckv_prefill_mfma_kernel<U, DE, NW, QG, TR, NS, WPE>,
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (prepared != hipSuccess) return prepared;
    constexpr int per_wg = 32 * QG * NW;
    const int64_t nb = (a.T + per_wg - 1) / per_wg * 2 * a.H;
    const int max_tiles = (std::max(a.P[0], a.P[1]) + TR - 1) / TR;
    const SplitPlan sp = plan_split(nb, resident_slots<U, DE, NW, QG, TR, NS, WPE>(), per_wg, max_tiles,
                                    plan_only ? (size_t)-1 : (a.ws ? a.ws_entries : 0));
    if (plan_only) {
        *entries = sp.entries;
        return hipSuccess;
    }
    a.split_first = sp.first;
    a.split_s = sp.s;
    const int64_t blocks = sp.first + (nb - sp.first) * sp.s;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL((ckv_prefill_mfma_kernel<U, DE, NW, QG, TR, NS, WPE>), dim3((unsigned)blocks), dim3(NW * 64), lds, s, a);
    if (sp.entries > 0)
        hipLaunchKernelGGL(ckv_prefill_finish_kernel, dim3((unsigned)((sp.entries + 255) / 256)), dim3(256), 0, s, a, per_wg, sp.entries);
    return hipGetLastError();
}

}  // namespace

// Rows of whole 16-byte chunks, up to 256 columns; the kernel is built for 64, 128 and 256 columns and a
// narrower row runs in the next wider one.
bool ckv_prefill_mfma_supported(int dtype, int d_e) {
    const int es = dtype == CKV_F32 ? 4 : 2;
    return (dtype == CKV_BF16 || dtype == CKV_F32) && d_e >= 1 && d_e <= 256 && (d_e * es) % 16 == 0;
}
static int prefill_width(int d_e) { return d_e <= 64 ? 64 : (d_e <= 128 ? 128 : 256); }

const char* ckv_prefill_variant(int dtype, int d_e) {
    if (ckv_prefill_mfma_supported(dtype, d_e)) {
        const int w = prefill_width(d_e);
        if (dtype == CKV_BF16) return w == 64 ? "prefill_mfma_bf16_e64" : (w == 128 ? "prefill_mfma_bf16_e128" : "prefill_mfma_bf16_e256");
        return w == 64 ? "prefill_mfma_f32_e64" : (w == 128 ? "prefill_mfma_f32_e128" : "prefill_mfma_f32_e256");
    }
    return dtype == CKV_F32 ? "prefill_scalar_f32" : "prefill_scalar_bf16";
}

// <storage type, d_e, wavefronts, position groups per wavefront, pool entries per stage, stages, wavefronts per SIMD>.
// fp32 rows are twice as long and the fp32 matrix instruction is sixteen times slower per product, so one
// position group per wavefront is enough to hide everything else behind it.
static hipError_t dispatch_mfma(const ckv_prefill_args& a, int dtype, hipStream_t s, bool plan_only, int64_t* entries) {
    const int w = prefill_width(a.d_e);
    if (dtype == CKV_BF16) {
        if (w == 64) return launch_mfma<uint16_t, 64, 4, 2, 32, 4, 3>(a, s, plan_only, entries);
        if (w == 128) return launch_mfma<uint16_t, 128, 4, 2, 32, 4, 3>(a, s, plan_only, entries);
        return launch_mfma<uint16_t, 256, 4, 1, 32, 4, 3>(a, s, plan_only, entries);
    }
    if (w == 64) return launch_mfma<float, 64, 4, 2, 32, 4, 3>(a, s, plan_only, entries);
    if (w == 128) return launch_mfma<float, 128, 4, 1, 32, 3, 3>(a, s, plan_only, entries);
    return launch_mfma<float, 256, 4, 1, 32, 2, 2>(a, s, plan_only, entries);
}

int64_t ckv_prefill_workspace_entries(const ckv_prefill_args& a, int dtype) {
    int64_t entries = 0;
    if (a.T == 0 || !ckv_prefill_mfma_supported(dtype, a.d_e)) return 0;
    if (dispatch_mfma(a, dtype, nullptr, true, &entries) != hipSuccess) return 0;
    return entries;
}

hipError_t ckv_launch_prefill(const ckv_prefill_args& a, int dtype, hipStream_t s) {
    if (a.T == 0) return hipSuccess;
    if (ckv_prefill_mfma_supported(dtype, a.d_e)) return dispatch_mfma(a, dtype, s, false, nullptr);
    const int64_t total = a.T * a.H * 2;
    const int blocks = (int)((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
    if (dtype == CKV_F32) hipLaunchKernelGGL(ckv_prefill_scalar_kernel<float>, dim3(blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(ckv_prefill_scalar_kernel<uint16_t>, dim3(blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}
