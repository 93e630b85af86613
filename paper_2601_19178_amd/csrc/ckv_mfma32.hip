// Matrix-core gather-concat-attend kernel for many candidate queries per user, fp32 storage
// (fp32 products and accumulation on v_mfma_f32_32x32x2_f32; built for rows of DA = 64, 128 or 256
// columns, a narrower d_a runs in the next wider kernel with zero columns; the 256-column kernel
// keeps one workgroup per compute unit, it needs most of the LDS).
//
// Same organisation as the bf16 register-staged kernel: a workgroup of four wavefronts serves one
// work item (a run of positions of one user and head, a block of 128 queries; wavefront w owns
// queries 32w .. 32w+31, a wavefront whose queries lie past Nq only helps with the gathers).
// The 256-column kernel splits the columns instead of the queries: a block of 64 queries, wavefronts
// w and w + 2 share queries 32(w & 1) .. +31; each sums S^T over one half of the columns of K, the
// two halves meet in LDS (a + b on one side, b + a on the other: the same bits), both form the same
// weights and each accumulates one half of the columns of O^T.  Queries and outputs then take 64
// registers each instead of 128, and 64 queries keep all four SIMDs busy.  Per
// tile of TP positions the workgroup gathers the final K and V rows into LDS, 16 bytes (four
// columns) per lane, in kernel column order [pool | user]; then per 32 positions each wavefront
// computes
//   S^T (32 pos x 32 q)  = K (A operand from LDS) * Q^T (B operand, registers)
//   O^T (d_a x 32 q)    += V^T (A operand, one LDS word per lane) * P^T (B operand = the weights
//                          as they sit in the accumulator registers of S^T)
// The instruction multiplies a 32 x 2 by a 2 x 32 block: k = 0 comes from lanes 0-31, k = 1 from
// lanes 32-63.  For S^T the lane halves hold consecutive 16-byte chunks of a row, so element e of
// both chunks forms a valid pair (the columns of a row are summed in a permuted order); for O^T
// register r of the two halves holds the weights of positions 8*(r/4) + r%4 and that + 4, and the
// V words are read from exactly those two rows.
#include "ckv_internal.h"

#include <type_traits>

namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLazy = 8.f;  // rescale only when the maximum grows by more than 2^8

__device__ __forceinline__ float other_half(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return threadIdx.x & 32 ? __uint_as_float(r[0]) : __uint_as_float(r[1]);
}

// One 16-byte chunk of a final row in kernel order [pool | user]: columns 4c .. 4c+3; columns past
// d_g + d_u (a row narrower than the kernel's) are zeros.
__device__ __forceinline__ u32x4 gather_chunk(const float* __restrict__ pool_h, int row, int64_t pool_ld,
                                              const float* __restrict__ user_pos, int c, int d_g, int d_u) {
    u32x4 v = {0u, 0u, 0u, 0u};
    const int c0 = 4 * c;
    if (c0 < d_g) v = *reinterpret_cast<const u32x4*>(pool_h + (int64_t)row * pool_ld + c0);
    if (c0 + 4 > d_g) {
        const int first = d_g > c0 ? d_g - c0 : 0;  // first element of the chunk that is not a pool column
        const float* u = user_pos + (c0 + first - d_g);
        if (first == 0 && c0 + 4 <= d_g + d_u && ((d_g | d_u) & 3) == 0) {
            v = *reinterpret_cast<const u32x4*>(u);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (e >= first) v[e] = c0 + e < d_g + d_u ? __float_as_uint(u[e - first]) : 0u;
        }
    }
    return v;
}

template <int DA, int TP, int MODE, bool SPLIT>
__global__ __launch_bounds__(256, (DA == 256 ? 1 : 2)) void ckv_mfma32_kernel(ckv_args a) {
    constexpr int NT = 256;            // threads: four wavefronts
    constexpr int CH = DA / 4;         // 16-byte chunks per row
    constexpr int RPP = NT / CH;       // rows gathered per pass
    constexpr int NL = TP / RPP;       // passes per tile (chunks per lane per tile, K and V each)
    constexpr int KS = DA * 4 + 16;    // LDS row stride of K: sixteen rows of one chunk column fall in sixteen bank groups
    constexpr int VS = DA * 4 + 32;    // LDS row stride of V: rows p and p + 4 are 32 banks apart (one word per lane, two rows per read)
    constexpr int BUF = TP * (KS + VS);
    // SPLIT: wavefront pairs split the columns (see above): always at 256 columns, and at 64 or 128 columns when a user
    // has 64 queries or fewer, which would leave two of the four wavefronts (two of the four SIMDs) without work
    constexpr int NKK = DA / 8 / (SPLIT ? 2 : 1);   // this wavefront's k-steps of S^T: one chunk per lane half each, four instructions
    constexpr int NDT = DA / 32 / (SPLIT ? 2 : 1);  // this wavefront's 32-row tiles of O^T
    static_assert(TP % RPP == 0 && TP % 32 == 0 && (!SPLIT || TP == 32), "tile shape");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const ckv_item it = a.items[blockIdx.x];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int qn = lane & 31, hh = lane >> 5;
    const int d_gk = a.d_gk, d_uk = a.d_uk, d_gv = a.d_gv, d_uv = a.d_uv;
    const int d_a = a.d_a;  // <= DA
    const int n = it.n;

    const int64_t hT = (int64_t)it.h * a.T + it.t0;
    const int32_t* __restrict__ ik = a.idx_k + hT;
    const int32_t* __restrict__ iv = a.idx_v + hT;
    const float* __restrict__ uk = (const float*)a.user_k + hT * d_uk;
    const float* __restrict__ uv = (const float*)a.user_v + hT * d_uv;
    const float* __restrict__ pk = (const float*)a.pool_k + (int64_t)it.h * a.P * a.pool_ld;
    const float* __restrict__ pv = (const float*)a.pool_v + (int64_t)it.h * a.P * a.pool_ld;

    // ---- queries of this lane, kernel column order, as B operands
    const int qblk = SPLIT ? (wave & 1) : wave;  // which 32 queries of the block
    const int half = SPLIT ? (wave >> 1) : 0;    // which half of the columns
    const int kk0 = half * NKK, dt0 = half * NDT;
    const bool wave_has_q = it.q0 + qblk * 32 < a.Nq;  // wavefront-uniform
    const int qj = it.q0 + qblk * 32 + qn;
    const bool qok = qj < a.Nq;
    const int64_t qo = (((int64_t)it.b * a.H + it.h) * a.Nq + (qok ? qj : 0)) * d_a;
    float qreg[NKK][4];
    {
        const float* qp = (const float*)a.q + qo;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int ci = 4 * (2 * (kk0 + kk) + hh) + e;
                const int pc = ci < d_gk ? ci + d_uk : ci - d_gk;  // kernel column of K -> column of q
                qreg[kk][e] = qok && ci < d_a ? qp[pc] : 0.f;
            }
        // the queries have to have arrived before the tile loop: a wait for them that the compiler placed inside
        // the loop would also wait for the row gathers of the next tile, which are meant to stay in flight
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk)
#pragma unroll
            for (int e = 0; e < 4; ++e) asm volatile("" : "+v"(qreg[kk][e]));
    }

    f32x16 oacc[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
    float m_ref = -INFINITY, lsum = 0.f;
    const float sc = MODE == CKV_SOFTMAX ? a.scale * kLog2e : a.scale;
    const float nsc = -kLog2e * a.scale;                     // SiLU: exponent of 2 per unit of raw score
    const float osc = MODE == CKV_SOFTMAX ? 1.f : a.scale;  // SiLU: the scale of the weights' numerator, applied to the output

    // ---- gather bookkeeping: this lane owns chunk c of rows p0 + i*RPP
    const int c = tid % CH, p0 = tid / CH;
    int rk[NL], rv[NL];
    u32x4 kreg[NL], vreg[NL];
    const int ntiles = (n + TP - 1) / TP;

    // (a side without pool columns keeps the zeros: nothing but loads may write these registers inside the tile
    // loop, or the compiler guards the write with a wait for every load in flight, the row gathers included)
#pragma unroll
    for (int i = 0; i < NL; ++i) rk[i] = rv[i] = 0;
    auto load_idx = [&](int tile) {
        if (d_gk > 0) {
#pragma unroll
            for (int i = 0; i < NL; ++i) rk[i] = ik[min(tile * TP + p0 + i * RPP, n - 1)];
        }
        if (d_gv > 0) {
#pragma unroll
            for (int i = 0; i < NL; ++i) rv[i] = iv[min(tile * TP + p0 + i * RPP, n - 1)];
        }
    };
    // When pool and user widths are multiples of four columns on both sides (workgroup-uniform), this lane's chunk
    // lies for every row in one and the same place: in the pool row, in the user row, or past d_a.  Where it comes
    // from is then settled once (source, column), and a row costs one address and one 16-byte load without a
    // branch.  A chunk past d_a fetches chunk 0 instead: for K it meets query columns that are zero, for V it
    // lands in rows of O^T that nobody stores (inputs are finite).
    const bool chunked = ((d_gk | d_uk | d_gv | d_uv) & 3) == 0 && a.pool_ld <= 0x7fffffff;
    const int ck = 4 * c < d_a ? 4 * c : 0, cv = ck;
    const bool k_pool = ck < d_gk, v_pool = cv < d_gv;
    // (source of this lane's chunk: first element of its column in row 0, and the distance between rows)
    const float* const k_src = k_pool ? pk + ck : uk + (ck - d_gk);
    const float* const v_src = v_pool ? pv + cv : uv + (cv - d_gv);
    const uint32_t k_ld = k_pool ? (uint32_t)a.pool_ld : (uint32_t)d_uk, v_ld = v_pool ? (uint32_t)a.pool_ld : (uint32_t)d_uv;
    auto load_rows = [&](int tile) {
        if (chunked) {
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int pos = min(tile * TP + p0 + i * RPP, n - 1);
                const uint32_t krow = (uint32_t)(k_pool ? rk[i] : pos), vrow = (uint32_t)(v_pool ? rv[i] : pos);
                kreg[i] = *reinterpret_cast<const u32x4*>(k_src + (uint64_t)krow * k_ld);
                vreg[i] = *reinterpret_cast<const u32x4*>(v_src + (uint64_t)vrow * v_ld);
            }
        } else {
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int pos = min(tile * TP + p0 + i * RPP, n - 1);
                kreg[i] = gather_chunk(pk, rk[i], a.pool_ld, uk + (int64_t)pos * d_uk, c, d_gk, d_uk);
                vreg[i] = gather_chunk(pv, rv[i], a.pool_ld, uv + (int64_t)pos * d_uv, c, d_gv, d_uv);
            }
        }
    };
    auto store_rows = [&](int buf) {
        unsigned char* kb = smem + buf * BUF;
        unsigned char* vb = kb + TP * KS;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int p = p0 + i * RPP;
            *reinterpret_cast<u32x4*>(kb + p * KS + c * 16) = kreg[i];
            *reinterpret_cast<u32x4*>(vb + p * VS + c * 16) = vreg[i];
        }
    };
    // The same work one row at a time, for a wavefront that multiplies (chunked widths only): with one or two wavefronts
    // per SIMD whatever is issued outside the matrix instructions is serial time, so the loads of row i of the next
    // tile go between the matrix instructions of S^T, the index loads of the tile after it behind them, and the LDS
    // writes between those of O^T.  No branch: past the last tile the last tile is fetched again (into the idle
    // buffer), and a side without pool columns reads one valid word (the first work item) that nothing uses.
    const int32_t* const ik1 = d_gk > 0 ? ik : (const int32_t*)a.items;
    const int32_t* const iv1 = d_gv > 0 ? iv : (const int32_t*)a.items;
    const int istep_k = d_gk > 0 ? 1 : 0, istep_v = d_gv > 0 ? 1 : 0;
    auto gather_piece = [&](int i, int tile) {
        const int pos = min(tile * TP + p0 + i * RPP, n - 1);
        const uint32_t krow = (uint32_t)(k_pool ? rk[i] : pos), vrow = (uint32_t)(v_pool ? rv[i] : pos);
        kreg[i] = *reinterpret_cast<const u32x4*>(k_src + (uint64_t)krow * k_ld);
        vreg[i] = *reinterpret_cast<const u32x4*>(v_src + (uint64_t)vrow * v_ld);
    };
    auto idx_piece = [&](int i, int tile) {
        const int pos = min(tile * TP + p0 + i * RPP, n - 1);
        rk[i] = ik1[pos * istep_k];
        rv[i] = iv1[pos * istep_v];
    };
    auto store_piece = [&](int i, int buf) {
        unsigned char* kb = smem + buf * BUF;
        unsigned char* vb = kb + TP * KS;
        const int p = p0 + i * RPP;
        *reinterpret_cast<u32x4*>(kb + p * KS + c * 16) = kreg[i];
        *reinterpret_cast<u32x4*>(vb + p * VS + c * 16) = vreg[i];
    };
    constexpr int GK = NKK / NL;  // k-steps of S^T per gathered row
    constexpr int RS = 16 / NL;   // weight registers of O^T per stored row
    static_assert(NKK % NL == 0 && GK >= 2 && 16 % NL == 0, "rows of the next tile are spread over the matrix instructions");

    if (ntiles > 0) {
        load_idx(0);
        load_rows(0);
        if (ntiles > 1) load_idx(1);
        store_rows(0);
        __syncthreads();
    }

    // WOVEN: this wavefront multiplies and the widths are chunked, so its share of the gather is woven into the matrix
    // instructions; otherwise (a wavefront without queries, or odd widths) it is issued before them and stored after.
    auto tile_loop = [&](auto woven_c) {
    constexpr bool WOVEN = decltype(woven_c)::value;
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        const int tnext = min(t + 1, ntiles - 1), tnext2 = min(t + 2, ntiles - 1);
        if (!WOVEN) {
            if (t + 1 < ntiles) load_rows(t + 1);
            if (t + 2 < ntiles) load_idx(t + 2);
        }

        const unsigned char* kb = smem + buf * BUF;
        const unsigned char* vb = kb + TP * KS;
        const int nt = min(n - t * TP, TP);
#pragma unroll
        for (int s = 0; s < TP / 32; ++s) {
            f32x16 sacc;
            if (SPLIT || (wave_has_q && 32 * s < nt)) {
                // S^T = K Q^T
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
                const unsigned char* krow = kb + (32 * s + qn) * KS + (2 * kk0 + hh) * 16;
                if (wave_has_q) {
                    // two chains of dependent instructions, and the K chunk of the next k-step on its way while
                    // this one is multiplied
                    f32x16 sodd;
#pragma unroll
                    for (int r = 0; r < 16; ++r) sodd[r] = 0.f;
                    u32x4 kn = *reinterpret_cast<const u32x4*>(krow);
#pragma unroll
                    for (int kk = 0; kk < NKK; ++kk) {
                        if (WOVEN && s == 0 && kk % GK == 0) gather_piece(kk / GK, tnext);
                        if (WOVEN && s == 0 && kk % GK == GK / 2) idx_piece(kk / GK, tnext2);
                        const u32x4 ka = kn;
                        if (kk + 1 < NKK) kn = *reinterpret_cast<const u32x4*>(krow + (kk + 1) * 32);
                        sacc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(ka[0]), qreg[kk][0], sacc, 0, 0, 0);
                        sodd = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(ka[1]), qreg[kk][1], sodd, 0, 0, 0);
                        sacc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(ka[2]), qreg[kk][2], sacc, 0, 0, 0);
                        sodd = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(ka[3]), qreg[kk][3], sodd, 0, 0, 0);
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) sacc[r] += sodd[r];
                }
            }
            if (SPLIT) {
                // the two halves of the sums meet: every wavefront leaves its sixteen registers in LDS (behind the
                // row buffers; one tile per barrier pair, so the slot is free again when the next tile writes it)
                float* xs = reinterpret_cast<float*>(smem + 2 * BUF);
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const u32x4 v = {__float_as_uint(sacc[4 * r4]), __float_as_uint(sacc[4 * r4 + 1]), __float_as_uint(sacc[4 * r4 + 2]),
                                     __float_as_uint(sacc[4 * r4 + 3])};
                    *reinterpret_cast<u32x4*>(xs + ((wave * 4 + r4) * 64 + lane) * 4) = v;
                }
                __syncthreads();
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const u32x4 v = *reinterpret_cast<const u32x4*>(xs + (((wave ^ 2) * 4 + r4) * 64 + lane) * 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) sacc[4 * r4 + e] += __uint_as_float(v[e]);
                }
            }
            if (wave_has_q && 32 * s < nt) {
                // weights
                const bool ragged = 32 * s + 32 > nt;
                float p[16];
                if (MODE == CKV_SOFTMAX) {
                    if (ragged) {
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (32 * s + 8 * (r >> 2) + 4 * hh + (r & 3) >= nt) sacc[r] = -INFINITY;
                    }
                    float tmax = sacc[0];
#pragma unroll
                    for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, sacc[r]);
                    tmax = fmaxf(tmax, other_half(tmax)) * sc;
                    if (__any(tmax > m_ref + kLazy)) {
                        const float m_new = fmaxf(m_ref, tmax);
                        const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
                        lsum *= alpha;
#pragma unroll
                        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                            for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
                        m_ref = m_new;
                    }
                    float psum = 0.f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        p[r] = __builtin_amdgcn_exp2f(fmaf(sacc[r], sc, -m_ref));
                        psum += p[r];
                    }
                    lsum += psum;
                } else {
                    // (sixteen independent chains, one kind of instruction at a time: the transcendental unit's
                    // latency is then covered by the other fifteen instead of being waited for sixteen times)
                    float e[16];
                    // (the weight without the factor scale of its numerator, which the output gets once: a multiplication less)
#pragma unroll
                    for (int r = 0; r < 16; ++r) e[r] = __builtin_amdgcn_exp2f(nsc * sacc[r]);
#pragma unroll
                    for (int r = 0; r < 16; ++r) e[r] = __builtin_amdgcn_rcpf(1.f + e[r]);
#pragma unroll
                    for (int r = 0; r < 16; ++r) p[r] = sacc[r] * e[r];
                    if (ragged) {
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (32 * s + 8 * (r >> 2) + 4 * hh + (r & 3) >= nt) p[r] = 0.f;
                    }
                }
                // O^T += V^T P^T: register r pairs position 8*(r/4) + r%4 (lanes 0-31) with that + 4 (lanes 32-63)
                const unsigned char* vcol = vb + (32 * s + 4 * hh) * VS + qn * 4;
                // (the V words of register r + 1 are on their way while those of r are multiplied)
                float vn[NDT];
#pragma unroll
                for (int dt = 0; dt < NDT; ++dt) vn[dt] = *reinterpret_cast<const float*>(vcol + (dt0 + dt) * 128);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    if (WOVEN && s == TP / 32 - 1 && r % RS == 0) store_piece(r / RS, (t + 1) & 1);
                    float va[NDT];
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) va[dt] = vn[dt];
                    if (r + 1 < 16) {
#pragma unroll
                        for (int dt = 0; dt < NDT; ++dt)
                            vn[dt] = *reinterpret_cast<const float*>(vcol + (8 * ((r + 1) >> 2) + ((r + 1) & 3)) * VS + (dt0 + dt) * 128);
                    }
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x2f32(va[dt], p[r], oacc[dt], 0, 0, 0);
                }
            }
        }

        if (!WOVEN && t + 1 < ntiles) store_rows((t + 1) & 1);
        __syncthreads();
    }
    };
    if (chunked && wave_has_q) tile_loop(std::true_type{});
    else tile_loop(std::false_type{});

    // ---- epilogue
    float l_tot = 0.f;
    if (MODE == CKV_SOFTMAX) l_tot = lsum + other_half(lsum);
    if (it.part < 0) {
        float inv;
        if (MODE == CKV_SOFTMAX) inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        else inv = it.n_total > 0 ? osc / (float)it.n_total : 0.f;
        if (qok) {
            float* op = (float*)a.out + qo;
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ci = 32 * (dt0 + dt) + 8 * (r >> 2) + 4 * hh + (r & 3);
                    const int pc = ci < d_gv ? ci + d_uv : ci - d_gv;  // kernel column of V -> column of out
                    if (ci < d_a) op[pc] = oacc[dt][r] * inv;
                }
        }
    } else {
        float* ws = a.partial + (int64_t)it.part * a.QB * (d_a + 2);
        const int j = qblk * 32 + qn;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ci = 32 * (dt0 + dt) + 8 * (r >> 2) + 4 * hh + (r & 3);
                const int pc = ci < d_gv ? ci + d_uv : ci - d_gv;
                if (ci < d_a) ws[(int64_t)j * d_a + pc] = oacc[dt][r] * osc;
            }
        if (hh == 0 && half == 0) {
            ws[(int64_t)a.QB * d_a + j] = m_ref * kLn2;  // natural-log units, as the merge expects
            ws[(int64_t)a.QB * d_a + a.QB + j] = l_tot;
        }
    }
}

template <int DA, int TP, bool SPLIT>
constexpr int lds_bytes() {
    return 2 * TP * ((DA * 4 + 16) + (DA * 4 + 32)) + (SPLIT ? 4 * 16 * 64 * 4 : 0);  // (+ the exchange of the column halves)
}

template <int DA, int TP, int MODE, bool SPLIT>
hipError_t prepare() {
    constexpr int lds = lds_bytes<DA, TP, SPLIT>();
    static_assert(lds <= 163840, "LDS of one compute unit");
    static hipError_t done =
        hipFuncSetAttribute((const void*)ckv_mfma32_kernel<DA, TP, MODE, SPLIT>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    return done;
}

template <int DA, int TP, int MODE, bool SPLIT>
hipError_t launch(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    hipError_t e = prepare<DA, TP, MODE, SPLIT>();
    if (e != hipSuccess) return e;
    constexpr int lds = lds_bytes<DA, TP, SPLIT>();
    hipLaunchKernelGGL((ckv_mfma32_kernel<DA, TP, MODE, SPLIT>), dim3(c->n_items), dim3(256), lds, s, a);
    return hipGetLastError();
}

template <int DA, int TP, int MODE, bool SPLIT>
int occupancy() {
    if (prepare<DA, TP, MODE, SPLIT>() != hipSuccess) return 0;
    int nb = 0;
    constexpr int lds = lds_bytes<DA, TP, SPLIT>();
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, (const void*)ckv_mfma32_kernel<DA, TP, MODE, SPLIT>, 256, lds) != hipSuccess) return 0;
    return nb;
}

// one call per built kernel: F<DA, TP, MODE, SPLIT>
#define CKV_MFMA32_DISPATCH(F, dak, split, softmax, ...)                                                                   \
    do {                                                                                                                  \
        if (dak == 64 && !split) return softmax ? F<64, 64, CKV_SOFTMAX, false>(__VA_ARGS__) : F<64, 64, CKV_SILU_OVER_N, false>(__VA_ARGS__);   \
        if (dak == 64) return softmax ? F<64, 32, CKV_SOFTMAX, true>(__VA_ARGS__) : F<64, 32, CKV_SILU_OVER_N, true>(__VA_ARGS__);               \
        if (dak == 128 && !split) return softmax ? F<128, 32, CKV_SOFTMAX, false>(__VA_ARGS__) : F<128, 32, CKV_SILU_OVER_N, false>(__VA_ARGS__); \
        if (dak == 128) return softmax ? F<128, 32, CKV_SOFTMAX, true>(__VA_ARGS__) : F<128, 32, CKV_SILU_OVER_N, true>(__VA_ARGS__);            \
        return softmax ? F<256, 32, CKV_SOFTMAX, true>(__VA_ARGS__) : F<256, 32, CKV_SILU_OVER_N, true>(__VA_ARGS__);                            \
    } while (0)

}  // namespace

// Wavefront pairs split the columns (64 queries per work item) at 256 columns, and at 64 or 128 columns for 64 queries or fewer.
bool ckv_mfma32_split(int dak, int Nq) { return dak == 256 || Nq <= 64; }
// positions per tile
int ckv_mfma32_tile(int dak, bool split) { return dak == 64 && !split ? 64 : 32; }
int ckv_mfma32_queries(bool split) { return split ? 64 : 128; }

int ckv_mfma32_occupancy(int dak, int mode, bool split) {
    const bool softmax = mode == CKV_SOFTMAX;
    CKV_MFMA32_DISPATCH(occupancy, dak, split, softmax);
}

hipError_t ckv_launch_mfma32(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    if (c->n_items == 0) return hipSuccess;
    const bool softmax = c->shape.mode == CKV_SOFTMAX;
    const int dak = a.d_a <= 64 ? 64 : (a.d_a <= 128 ? 128 : 256);
    const bool split = c->QB == 64;
    // the plan (queries per work item, positions per tile) must be the one the kernel is built for
    if (a.d_a > 256 || (dak == 256 && !split) || c->QB != ckv_mfma32_queries(split) || c->tp != ckv_mfma32_tile(dak, split))
        return hipErrorInvalidValue;
    CKV_MFMA32_DISPATCH(launch, dak, split, softmax, c, a, s);
}
