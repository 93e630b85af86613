// Streaming gather-concat-attend kernel for wide rows and for user slices of any width: target attention
// (one or two queries per user, section 2.1) over rows of up to 1024 bytes, such as the 256 columns behind
// the compression ratios of Table 1 (d_u = 1, 2, 3, 4, 6, 10 of d = 256) in bf16 or fp32.
//
// The final row of a position is [user slice | pool row] (eq. "eq: Kc", "eq: K").  The two parts sit in
// different arrays with different alignment: a pool row starts on a 16-byte boundary whatever d_u is, a
// user slice starts wherever position * d_u elements lands.  So the two parts are fetched separately:
//   * the wide part (the pool row, or the whole d_a-wide row of a side that is not shared) with one 16-byte
//     load per lane, G lanes per row, 64 / G rows per load instruction, eight instructions per side and batch;
//     elements past the row's width (the padding of the pool stride) are masked off after the load;
//   * the slice (d_u columns) element by element, by the lanes that end up holding that position's score.
// The concat is the column offset d_u at which the wide part's scores and outputs are placed.
// A batch is 8 * 64 / G positions.  The eight partial dot products a lane holds (one per instruction) are
// reduced over the G lanes of a row with a butterfly that halves the number of values at every step, so the
// score of batch position (i, g) (instruction i, row group g) ends up in the lanes g * G + o * 8 + i for
// every octet o of the group; the G / 8 lanes of the octets share the slice of that position column-wise and
// add their share before the last steps of the reduction.  Softmax is online per batch with one reference
// maximum per row group (a reduction over eight lanes); the groups, and the four (or two) wavefronts of a
// workgroup, which take the 64-position tiles of a work item in turn, are merged exactly at the end.
#include "ckv_internal.h"

namespace {

constexpr int kLanes = 64;
constexpr int NSL_MAX = 8;  // most slice columns per lane (a position's slice is shared by G / 8 lanes)
constexpr int NSL_SMALL = 2, NSL_MID = 4;  // slice columns per lane of the instantiations for narrower slices
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <typename T> struct Store;
template <> struct Store<float> {
    static constexpr int EPL = 4;  // elements per 16-byte lane
    static __device__ __forceinline__ float up(float x) { return x; }
    static __device__ __forceinline__ float down(float x) { return x; }
    static __device__ __forceinline__ void unpack(const u32x4& w, float (&f)[EPL]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(w[i]);
    }
    // AND mask of raw word i of a lane whose first column is c0, for a row of `width` valid columns
    static __device__ __forceinline__ uint32_t mask(int c0, int i, int width) { return c0 + i < width ? 0xFFFFFFFFu : 0u; }
};
template <> struct Store<uint16_t> {  // bfloat16 bit patterns
    static constexpr int EPL = 8;
    static __device__ __forceinline__ float up(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }
    static __device__ __forceinline__ uint16_t down(float f) {  // round to nearest even
        uint32_t u = __float_as_uint(f);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
    static __device__ __forceinline__ void unpack(const u32x4& w, float (&f)[EPL]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ uint32_t mask(int c0, int i, int width) {
        return (c0 + 2 * i < width ? 0x0000FFFFu : 0u) | (c0 + 2 * i + 1 < width ? 0xFFFF0000u : 0u);
    }
};

// G = lanes per row (8, 16, 32 or 64), NQ = queries served per pass over the history (1 or 2), NSL = slice columns
// per lane (2, 4 or 8), kWaves = wavefronts per work item (4, or 2 where short items outnumber the resident wavefronts)
// kHot: the first a.hot_rows rows of the item's pools (the most used ones once ckv_remap_hot_rows has renumbered them; the
// appendix on router activations shows how much the activated entries of similar users overlap) are copied into LDS when the
// item starts, and a position whose index is below that count takes its pool row from there instead of from memory.
template <typename T, int G, int NQ, int MODE, int NSL, int kWaves, bool kHot>
__global__ __launch_bounds__(kLanes * kWaves) __attribute__((amdgpu_waves_per_eu(NQ == 1 && NSL <= NSL_MID ? 3 : 2, 8))) void ckv_streamw_kernel(ckv_args a) {
    using S = Store<T>;
    constexpr int EPL = S::EPL;
    constexpr int R = kLanes / G;  // rows per load instruction = row groups
    constexpr int NB = 8 * R;      // positions per batch
    constexpr int LP = G / 8;      // lanes that share a position's slice
    constexpr int WMAX = G * EPL + NSL * LP;  // most columns of a final row
    __shared__ float sm_acc[kWaves][NQ][WMAX];
    __shared__ float sm_ml[kWaves][NQ][2];
    extern __shared__ __attribute__((aligned(16))) unsigned char hot_lds[];  // kHot: a.hot_rows K rows, then as many V rows

    const ckv_item it = a.items[blockIdx.x];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane / G, lg = lane % G;  // row group, lane within the row
    const int x = lane & 7, o = lg >> 3;    // batch position (x, g) whose score this lane ends up with; octet within the row
    const int d_a = a.d_a;
    // per side: wide part (pool row of d_g columns, or the whole d_a-wide row of a side without pool) and slice
    const bool ksh = a.d_gk > 0, vsh = a.d_gv > 0;
    const int wk = ksh ? a.d_gk : d_a, sk = ksh ? a.d_uk : 0;  // wide and slice columns of a K row; the wide part starts at column sk
    const int wv = vsh ? a.d_gv : d_a, sv = vsh ? a.d_uv : 0;
    const int64_t hT = (int64_t)it.h * a.T + it.t0;
    const int32_t* ik = a.idx_k + hT;
    const int32_t* iv = a.idx_v + hT;
    const unsigned char* kwide = ksh ? (const unsigned char*)a.pool_k + (int64_t)it.h * a.P * a.pool_ld * sizeof(T)
                                     : (const unsigned char*)a.user_k + hT * d_a * (int64_t)sizeof(T);
    const unsigned char* vwide = vsh ? (const unsigned char*)a.pool_v + (int64_t)it.h * a.P * a.pool_ld * sizeof(T)
                                     : (const unsigned char*)a.user_v + hT * d_a * (int64_t)sizeof(T);
    const int64_t kstride = (ksh ? a.pool_ld : (int64_t)d_a) * sizeof(T), vstride = (vsh ? a.pool_ld : (int64_t)d_a) * sizeof(T);
    const T* kslice = (const T*)a.user_k + hT * sk;
    const T* vslice = (const T*)a.user_v + hT * sv;
    const int n = it.n;
    // byte offset of this lane's 16 bytes in a row (lanes past the row's last 16 bytes fetch those again: every lane loads,
    // without a branch; what they get is masked off)
    const int koff = min(lg, (wk * (int)sizeof(T) + 15) / 16 - 1) * 16, voff = min(lg, (wv * (int)sizeof(T) + 15) / 16 - 1) * 16;
    // (only K is masked: a V column past the row's width only reaches an accumulator that is never stored)
    uint32_t kmask[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) kmask[i] = S::mask(lg * EPL, i, wk);
    const int nslk = (sk + LP - 1) / LP, nslv = (sv + LP - 1) / LP;  // slice columns per lane in use (wavefront-uniform)
    // hot rows: whole 16-byte lanes of the rows 0 .. hot - 1 of each pool of the item's head; no more of them than a quarter
    // of the item's positions, so that fetching them stays a small part of the item
    const int rbk = (wk * (int)sizeof(T) + 15) / 16 * 16, rbv = (wv * (int)sizeof(T) + 15) / 16 * 16;
    const int hotk = kHot && ksh ? min(min(a.hot_rows, a.P), n >> 2) : 0, hotv = kHot && vsh ? min(min(a.hot_rows, a.P), n >> 2) : 0;
    const uint32_t hotv_base = kHot ? (uint32_t)a.hot_rows * rbk : 0;
    if (kHot) {
        for (int c = threadIdx.x; c < hotk * (rbk / 16); c += kLanes * kWaves) {
            const int r = c / (rbk / 16), ch = c % (rbk / 16);
            *reinterpret_cast<u32x4*>(hot_lds + r * rbk + ch * 16) = *reinterpret_cast<const u32x4*>(kwide + r * kstride + ch * 16);
        }
        for (int c = threadIdx.x; c < hotv * (rbv / 16); c += kLanes * kWaves) {
            const int r = c / (rbv / 16), ch = c % (rbv / 16);
            *reinterpret_cast<u32x4*>(hot_lds + hotv_base + r * rbv + ch * 16) = *reinterpret_cast<const u32x4*>(vwide + r * vstride + ch * 16);
        }
        __syncthreads();
    }

    for (int j0 = 0; j0 < a.QB; j0 += NQ) {
        if (it.q0 + j0 >= a.Nq) break;
        // queries: this lane's columns of the wide part and of the slice (zero past the row's width)
        float qw[NQ][EPL], qs[NQ][NSL];
        int64_t qo[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int qj = min(it.q0 + j0 + q, a.Nq - 1);  // (a second query past the last one repeats it; its result is not written)
            qo[q] = (((int64_t)it.b * a.H + it.h) * a.Nq + qj) * d_a;
            const T* qp = (const T*)a.q + qo[q];
#pragma unroll
            for (int e = 0; e < EPL; ++e) qw[q][e] = lg * EPL + e < wk ? S::up(qp[sk + lg * EPL + e]) : 0.f;
#pragma unroll
            for (int k = 0; k < NSL; ++k) qs[q][k] = o + LP * k < sk ? S::up(qp[o + LP * k]) : 0.f;
        }
        float acc[NQ][EPL], accu[NQ][NSL], m_run[NQ], l_run[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            m_run[q] = -INFINITY;
            l_run[q] = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[q][e] = 0.f;
#pragma unroll
            for (int k = 0; k < NSL; ++k) accu[q][k] = 0.f;
        }

        // ---- the wavefront's batches: tiles wave, wave + kWaves, ... of 64 positions, batches of NB positions inside a tile;
        // the indices run one tile ahead.  With two queries per pass (two wavefronts per SIMD by the registers) the loads
        // run one batch ahead into the same registers: the K rows (and K slices) of the next batch are requested as soon as
        // this batch's partial dot products are taken, the V rows (and V slices) as soon as this batch's are added up.  With
        // one query the kernel fits three wavefronts per SIMD without that, which measured faster than two with it
        // (256 bf16 columns, 1024 users of 1000 positions: 128 against 137 us; two queries: 296 -> 159 us with it).
        constexpr bool kAhead = NQ == 2 && NSL <= NSL_SMALL;  // (with wide slices as well it would not fit the registers)
        u32x4 kraw[8], vraw[8];
        T ks[NSL], vs[NSL];
#pragma unroll
        for (int i = 0; i < 8; ++i) kraw[i] = vraw[i] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int k = 0; k < NSL; ++k) ks[k] = vs[k] = T(0);
        // (rows past the end of the tile fetch its last one; their weight is zero.  Slice columns past d_u repeat the last one; q is zero there.)
        auto issue_k = [&](int t0, int nt, int b0, int idx) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int tp = min(b0 + i * R + g, nt - 1);
                const int row = ksh ? __shfl(idx, tp, kLanes) : tp + t0;
                // (hot rows: one load through the flat address space, whose address is the row's copy in LDS or the row in memory,
                // lane by lane; a branch around two kinds of load measured twice as slow as no hot rows at all)
                const unsigned char* src = kwide + row * kstride + koff;
                if (kHot) src = row < hotk ? (const unsigned char*)hot_lds + row * rbk + koff : src;
                kraw[i] = *reinterpret_cast<const u32x4*>(src);
            }
            const int64_t ps = t0 + min(b0 + x * R + g, nt - 1);
#pragma unroll
            for (int k = 0; k < NSL; ++k)
                if (k < nslk) ks[k] = kslice[ps * sk + min(o + LP * k, sk - 1)];
        };
        auto issue_v = [&](int t0, int nt, int b0, int idx) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int tp = min(b0 + i * R + g, nt - 1);
                const int row = vsh ? __shfl(idx, tp, kLanes) : tp + t0;
                const unsigned char* src = vwide + row * vstride + voff;
                if (kHot) src = row < hotv ? (const unsigned char*)hot_lds + hotv_base + row * rbv + voff : src;
                vraw[i] = *reinterpret_cast<const u32x4*>(src);
            }
            const int64_t ps = t0 + min(b0 + x * R + g, nt - 1);
#pragma unroll
            for (int k = 0; k < NSL; ++k)
                if (k < nslv) vs[k] = vslice[ps * sv + min(o + LP * k, sv - 1)];
        };
        auto load_idx = [&](int t0, int& jk, int& jv) {
            const int p = min(t0 + lane, n - 1);
            if (ksh) jk = ik[p];
            if (vsh) jv = iv[p];
        };
        int t0 = wave * kLanes;
        if (t0 < n) {
            int nt = min(n - t0, kLanes), b0 = 0;
            int cur_ik = 0, cur_iv = 0, nxt_ik = 0, nxt_iv = 0;
            load_idx(t0, cur_ik, cur_iv);
            if (t0 + kLanes * kWaves < n) load_idx(t0 + kLanes * kWaves, nxt_ik, nxt_iv);
            if (kAhead) {
                issue_k(t0, nt, b0, cur_ik);
                issue_v(t0, nt, b0, cur_iv);
            }
            while (true) {
                if (!kAhead) {
                    issue_k(t0, nt, b0, cur_ik);
                    issue_v(t0, nt, b0, cur_iv);
                }
                // the batch after this one
                int t0n = t0, ntn = nt, b0n = b0 + NB;
                const bool same = b0n < nt;
                if (!same) {
                    t0n = t0 + kLanes * kWaves;
                    ntn = min(n - t0n, kLanes);
                    b0n = 0;
                }
                const bool more = t0n < n;
                if (!more) {  // (past the last batch the loads below fetch this batch again, so that no load sits under a branch)
                    t0n = t0;
                    ntn = nt;
                    b0n = b0;
                }
                const bool from_cur = same || !more;
                const bool valid = b0 + x * R + g < nt;  // (x, g): the batch position whose score this lane ends up with
                // ---- scores: eight partial dot products per lane and query, and this lane's share of its position's slice
                float part[NQ][8], spart[NQ];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    float kf[EPL];
                    u32x4 w = kraw[i];
#pragma unroll
                    for (int c = 0; c < 4; ++c) w[c] &= kmask[c];
                    S::unpack(w, kf);
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        float p = 0.f;
#pragma unroll
                        for (int e = 0; e < EPL; ++e) p = fmaf(kf[e], qw[q][e], p);
                        part[q][i] = p;
                    }
                }
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    spart[q] = 0.f;
#pragma unroll
                    for (int k = 0; k < NSL; ++k)
                        if (k < nslk) spart[q] = fmaf(S::up(ks[k]), qs[q][k], spart[q]);
                }
                if (kAhead) {
                    // (the loads below overwrite the operands of the arithmetic above: its results are pinned here, so that the
                    // compiler neither moves the loads up nor the arithmetic down, which would take a second set of registers)
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(part[q][i])::"memory");
                        asm volatile("" : "+v"(spart[q])::"memory");
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    issue_k(t0n, ntn, b0n, from_cur ? cur_ik : nxt_ik);
                    __builtin_amdgcn_sched_barrier(0);
                }
                float wgt[NQ];
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    // butterfly over the lanes of an octet: after the three steps lane x holds instruction x's sum
                    float r4[4], r2[2], s;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float keep = (x & 4) ? part[q][i + 4] : part[q][i], send = (x & 4) ? part[q][i] : part[q][i + 4];
                        r4[i] = keep + __shfl_xor(send, 4, kLanes);
                    }
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        const float keep = (x & 2) ? r4[i + 2] : r4[i], send = (x & 2) ? r4[i] : r4[i + 2];
                        r2[i] = keep + __shfl_xor(send, 2, kLanes);
                    }
                    {
                        const float keep = (x & 1) ? r2[1] : r2[0], send = (x & 1) ? r2[0] : r2[1];
                        s = keep + __shfl_xor(send, 1, kLanes);
                    }
                    // the slice's share, then the octets of the row
                    s += spart[q];
#pragma unroll
                    for (int m = 8; m < G; m <<= 1) s += __shfl_xor(s, m, kLanes);
                    // ---- weight of this lane's position
                    if (MODE == CKV_SOFTMAX) {
                        const float sc = valid ? s * a.scale : -INFINITY;
                        float bm = sc;  // maximum over the eight positions of the row group in this batch
                        bm = fmaxf(bm, __shfl_xor(bm, 1, kLanes));
                        bm = fmaxf(bm, __shfl_xor(bm, 2, kLanes));
                        bm = fmaxf(bm, __shfl_xor(bm, 4, kLanes));
                        if (__any(bm > m_run[q])) {
                            const float m_new = fmaxf(m_run[q], bm);
                            const float alpha = m_new == m_run[q] ? 1.f : __expf(m_run[q] - m_new);  // (first batch: exp(-inf) = 0)
                            l_run[q] *= alpha;
#pragma unroll
                            for (int e = 0; e < EPL; ++e) acc[q][e] *= alpha;
#pragma unroll
                            for (int k = 0; k < NSL; ++k) accu[q][k] *= alpha;
                            m_run[q] = m_new;
                        }
                        wgt[q] = valid ? __expf(sc - m_run[q]) : 0.f;
                        l_run[q] += o == 0 ? wgt[q] : 0.f;  // (every octet of the row holds the same weight: counted once)
                    } else {
                        const float sc = s * a.scale;
                        wgt[q] = valid ? sc / (1.f + __expf(-sc)) : 0.f;
                    }
#pragma unroll
                    for (int k = 0; k < NSL; ++k)
                        if (k < nslv) accu[q][k] = fmaf(wgt[q], S::up(vs[k]), accu[q][k]);
                }
                // ---- weighted sum of the wide V rows: instruction i's row has its weight in lane i of this lane's octet
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    float vf[EPL];
                    S::unpack(vraw[i], vf);
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        const float wr = __shfl(wgt[q], (lane & ~7) | i, kLanes);
#pragma unroll
                        for (int e = 0; e < EPL; ++e) acc[q][e] = fmaf(wr, vf[e], acc[q][e]);
                    }
                }
                if (kAhead) {
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
#pragma unroll
                        for (int e = 0; e < EPL; ++e) asm volatile("" : "+v"(acc[q][e])::"memory");
#pragma unroll
                        for (int k = 0; k < NSL; ++k) asm volatile("" : "+v"(accu[q][k])::"memory");
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    issue_v(t0n, ntn, b0n, from_cur ? cur_iv : nxt_iv);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (!more) break;
                if (!same) {
                    cur_ik = nxt_ik;
                    cur_iv = nxt_iv;
                    if (t0n + kLanes * kWaves < n) load_idx(t0n + kLanes * kWaves, nxt_ik, nxt_iv);
                }
                t0 = t0n;
                nt = ntn;
                b0 = b0n;
            }
        }
        // ---- merge the row groups of the wavefront (common maximum first), then the wavefronts through LDS
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            float M = m_run[q];
            if (MODE == CKV_SOFTMAX) {
#pragma unroll
                for (int m = G; m < kLanes; m <<= 1) M = fmaxf(M, __shfl_xor(M, m, kLanes));
                const float f = m_run[q] == -INFINITY ? 0.f : __expf(m_run[q] - M);
                l_run[q] *= f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[q][e] *= f;
#pragma unroll
                for (int k = 0; k < NSL; ++k) accu[q][k] *= f;
            }
#pragma unroll
            for (int e = 0; e < EPL; ++e)
#pragma unroll
                for (int m = G; m < kLanes; m <<= 1) acc[q][e] += __shfl_xor(acc[q][e], m, kLanes);
#pragma unroll
            for (int k = 0; k < NSL; ++k) {
                if (k < nslv) {
                    float v = accu[q][k];
#pragma unroll
                    for (int m = 1; m < 8; m <<= 1) v += __shfl_xor(v, m, kLanes);
#pragma unroll
                    for (int m = G; m < kLanes; m <<= 1) v += __shfl_xor(v, m, kLanes);
                    accu[q][k] = v;
                }
            }
            float L = l_run[q];
#pragma unroll
            for (int m = 1; m < kLanes; m <<= 1) L += __shfl_xor(L, m, kLanes);
            if (g == 0) {
#pragma unroll
                for (int e = 0; e < EPL; ++e)
                    if (lg * EPL + e < wv) sm_acc[wave][q][sv + lg * EPL + e] = acc[q][e];
                if (x == 0) {
#pragma unroll
                    for (int k = 0; k < NSL; ++k)
                        if (o + LP * k < sv) sm_acc[wave][q][o + LP * k] = accu[q][k];
                }
            }
            if (lane == 0) {
                sm_ml[wave][q][0] = M;
                sm_ml[wave][q][1] = L;
            }
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const int j = j0 + q;
                if (it.q0 + j >= a.Nq) break;
                float M = -INFINITY, L = 0.f, wg[kWaves];
                if (MODE == CKV_SOFTMAX) {
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sm_ml[w][q][0]);
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) {
                        wg[w] = sm_ml[w][q][0] == -INFINITY ? 0.f : __expf(sm_ml[w][q][0] - M);
                        L += wg[w] * sm_ml[w][q][1];
                    }
                } else {
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) wg[w] = 1.f;
                }
                float norm;
                if (MODE == CKV_SOFTMAX) norm = L > 0.f ? 1.f / L : 0.f;
                else norm = it.n_total > 0 ? 1.f / (float)it.n_total : 0.f;
                float* ws = it.part < 0 ? nullptr : a.partial + (int64_t)it.part * a.QB * (d_a + 2);
                for (int c = lane; c < d_a; c += kLanes) {
                    float v = 0.f;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) v += wg[w] * sm_acc[w][q][c];
                    if (!ws) ((T*)a.out)[qo[q] + c] = S::down(v * norm);
                    else ws[(int64_t)j * d_a + c] = v;
                }
                if (ws && lane == 0) {
                    ws[(int64_t)a.QB * d_a + j] = M;
                    ws[(int64_t)a.QB * d_a + a.QB + j] = L;
                }
            }
        }
        __syncthreads();  // the next queries reuse the LDS buffers
    }
}

template <typename T, int G, int NQ, int NSL, int NWV>
hipError_t launch_mode(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    dim3 grid(c->n_items), block(kLanes * NWV);
    if constexpr (G >= 16 && NQ == 1 && NSL <= NSL_MID) {  // the instantiations that exist with hot rows in LDS
        if (a.hot_rows > 0) {
            const size_t lds = (size_t)a.hot_rows * ckv_streamw_hot_row_bytes(c->shape);
            if (c->shape.mode == CKV_SOFTMAX)
                hipLaunchKernelGGL((ckv_streamw_kernel<T, G, NQ, CKV_SOFTMAX, NSL, NWV, true>), grid, block, lds, s, a);
            else
                hipLaunchKernelGGL((ckv_streamw_kernel<T, G, NQ, CKV_SILU_OVER_N, NSL, NWV, true>), grid, block, lds, s, a);
            return hipGetLastError();
        }
    }
    if (a.hot_rows > 0) return hipErrorInvalidValue;  // (the host asks for hot rows only where ckv_streamw_hot_rows allows them)
    if (c->shape.mode == CKV_SOFTMAX) hipLaunchKernelGGL((ckv_streamw_kernel<T, G, NQ, CKV_SOFTMAX, NSL, NWV, false>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((ckv_streamw_kernel<T, G, NQ, CKV_SILU_OVER_N, NSL, NWV, false>), grid, block, 0, s, a);
    return hipGetLastError();
}

template <typename T, int G, int NQ, int NSL>
hipError_t launch_waves(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    return c->nw == 2 ? launch_mode<T, G, NQ, NSL, 2>(c, a, s) : launch_mode<T, G, NQ, NSL, 4>(c, a, s);
}

// (slices of at most two and of at most four columns per lane have instantiations of their own, 24 and 16 registers
// smaller: with one query they fit three wavefronts per SIMD, the second with a dozen registers spilled)
template <typename T, int G, int NQ>
hipError_t launch_nsl(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    const int slice = a.d_gk > 0 && a.d_gv > 0 ? (a.d_uk > a.d_uv ? a.d_uk : a.d_uv) : (a.d_gk > 0 ? a.d_uk : (a.d_gv > 0 ? a.d_uv : 0));
    if (slice <= NSL_SMALL * (G / 8)) return launch_waves<T, G, NQ, NSL_SMALL>(c, a, s);
    if (slice <= NSL_MID * (G / 8)) return launch_waves<T, G, NQ, NSL_MID>(c, a, s);
    return launch_waves<T, G, NQ, NSL_MAX>(c, a, s);
}

template <typename T, int G>
hipError_t launch_nq(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    return c->sw_nq == 2 ? launch_nsl<T, G, 2>(c, a, s) : launch_nsl<T, G, 1>(c, a, s);
}

template <typename T>
hipError_t launch_g(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    switch (c->sw_g) {
        case 8: return launch_nq<T, 8>(c, a, s);
        case 16: return launch_nq<T, 16>(c, a, s);
        case 32: return launch_nq<T, 32>(c, a, s);
        case 64: return launch_nq<T, 64>(c, a, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

// Bytes of LDS one hot row takes (its K row and its V row in whole 16-byte lanes; a side without pool takes none).
size_t ckv_streamw_hot_row_bytes(const ckv_shape& s) {
    const int e = s.dtype == CKV_F32 ? 4 : 2;
    size_t bytes = 0;
    for (int side = 0; side < 2; ++side) {
        int du, dg;
        ckv_side_dims(s, side, &du, &dg);
        // (the kernel places the V rows behind hot_rows K rows of the K side's row size, whatever the K side is)
        const int wide = dg > 0 ? dg : s.d_g + s.d_u;
        bytes += (size_t)((wide * e + 15) / 16 * 16);
    }
    return bytes;
}

// Most pool rows the kernel that serves the shape (G lanes per row, nq queries per pass) can keep in LDS: a multiple of
// eight, at most 32, within 40 KB; 0 where the instantiation does not exist (fewer than 16 lanes per row, two queries per
// pass, slices of more than four columns per lane) or the shape has no pool.
int ckv_streamw_hot_rows(const ckv_shape& s, int G, int nq) {
    if (G < 16 || nq != 1 || s.d_g == 0) return 0;
    int slice = 0;
    for (int side = 0; side < 2; ++side) {
        int du, dg;
        ckv_side_dims(s, side, &du, &dg);
        if (dg > 0) slice = slice > du ? slice : du;
    }
    if (slice > NSL_MID * (G / 8)) return 0;
    const int fit = (int)(40960 / ckv_streamw_hot_row_bytes(s)) / 8 * 8;
    return fit > 32 ? 32 : fit;
}

// Lanes per row with which this kernel serves the shape (8, 16, 32 or 64), or 0 if it does not: the wide
// part of each side must be addressable in whole 16-byte lanes (row strides that are multiples of 16 bytes),
// fit 64 lanes, and the slice must fit eight columns per lane of the G / 8 lanes that share it.
int ckv_streamw_lanes(const ckv_shape& s) {
    const int e = s.dtype == CKV_F32 ? 4 : 2;
    const int d_a = s.d_g + s.d_u;
    int need = 1, slice = 0;
    for (int side = 0; side < 2; ++side) {
        int du, dg;
        ckv_side_dims(s, side, &du, &dg);
        const int64_t stride = dg > 0 ? s.pool_ld : d_a;
        if ((stride * e) % 16) return 0;
        const int wide = dg > 0 ? dg : d_a;
        need = need > (wide * e + 15) / 16 ? need : (wide * e + 15) / 16;
        if (dg > 0) slice = slice > du ? slice : du;
    }
    if (need > 64) return 0;
    int G = 8;
    while (G < need) G <<= 1;
    while (G <= 64 && slice > NSL_MAX * (G / 8)) G <<= 1;  // more lanes per row also means more lanes per slice
    return G <= 64 ? G : 0;
}

// Wavefronts per SIMD the kernel that serves the shape is built for (its register budget).
int ckv_streamw_waves_per_simd(const ckv_shape& s, int G, int nq) {
    int slice = 0;
    for (int side = 0; side < 2; ++side) {
        int du, dg;
        ckv_side_dims(s, side, &du, &dg);
        if (dg > 0) slice = slice > du ? slice : du;
    }
    return nq == 1 && slice <= NSL_MID * (G / 8) ? 3 : 2;
}

hipError_t ckv_launch_streamw(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    if (c->n_items == 0) return hipSuccess;
    return c->shape.dtype == CKV_F32 ? launch_g<float>(c, a, s) : launch_g<uint16_t>(c, a, s);
}
