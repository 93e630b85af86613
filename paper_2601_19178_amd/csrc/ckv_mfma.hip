// Matrix-core gather-concat-attend kernel for many candidate queries per user (bf16 storage,
// fp32 accumulation, built for rows of DA = 64, 128 or 256 columns; a narrower d_a runs in the next
// wider kernel with its missing columns as zeros of K, V and q; the 256-column kernel keeps one
// workgroup of four wavefronts per compute unit, its accumulators need the whole register file).
//
// A workgroup of NW wavefronts serves one work item: a run of positions of one user and head
// and a block of 32*NW queries; wavefront w owns queries 32w .. 32w+31 and every wavefront
// sees every position.  Positions are processed in tiles of TP.  For a tile the workgroup
// gathers the final K and V rows into LDS, 16 bytes per lane: lane (row p, chunk c) reads
// pool[idx[p]][8c .. 8c+8) and patches in the user slice where the chunk reaches past d_g.
// Inside the kernel a final row is laid out [pool columns | user columns]; the dot product
// and the output do not care about column order as long as q and out are permuted the same
// way, and this order keeps the 16-byte pool chunks aligned.  The concat of the paper
// (eq. "eq: K", user columns first) is restored when q is read and out is written.
//
// Per 32-position sub-tile each wavefront computes with v_mfma_f32_32x32x16_bf16
//   S^T (32 pos x 32 q)  = K (32 x d_a, A operand from LDS) * Q^T (B operand, registers)
//   O^T (d_a x 32 q)    += V^T (A operand, LDS transpose reads) * P^T (B operand = weights)
// Both products put one query per lane (query = lane % 32), so the running maximum, the
// running sum and the weights never cross lanes except for one exchange between lane l and
// l ^ 32, which hold the two halves of a query's 32 positions.  The accumulator layout of
// S^T (lane holds positions 8*(r/4) + 4*(lane/32) + r%4, r = 0..15) is used directly as the
// k-slot order of the second product; V^T is read with ds_read_b64_tr_b16 in that same order.
#include "ckv_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLazy = 8.f;  // rescale only when the maximum grows by more than 2^8

__device__ __forceinline__ float other_half(float x) {
    // value of the same register in lane ^ 32, combined by the caller
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return threadIdx.x & 32 ? __uint_as_float(r[0]) : __uint_as_float(r[1]);
}

__device__ __forceinline__ uint16_t f2bf(float f) {
    return __builtin_bit_cast(uint16_t, (__bf16)f);
}

// One 16-byte chunk of a final row in kernel order [pool | user]: elements 8c .. 8c+7.
__device__ __forceinline__ uint4 gather_chunk(const uint16_t* __restrict__ pool_h, int row, int64_t pool_ld,
                                              const uint16_t* __restrict__ user_pos, int c, int d_g, int d_u) {
    uint4 v = make_uint4(0, 0, 0, 0);
    const int c0 = 8 * c;
    if (c0 < d_g) v = *reinterpret_cast<const uint4*>(pool_h + (int64_t)row * pool_ld + c0);
    if (c0 + 8 > d_g) {
        const int first = d_g > c0 ? d_g - c0 : 0;  // first element of the chunk that is a user column
        const uint16_t* u = user_pos + (c0 + first - d_g);
        if (first == 0 && c0 + 8 <= d_g + d_u && ((d_g | d_u) & 7) == 0) {
            v = *reinterpret_cast<const uint4*>(u);
        } else if (first == 4 && d_u == 4) {
            const uint2 x = *reinterpret_cast<const uint2*>(u);
            v.z = x.x;
            v.w = x.y;
        } else if (first == 6 && d_u == 2) {
            v.w = *reinterpret_cast<const uint32_t*>(u);
        } else {
            uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (e >= first) {  // a user column, or past the end of a row narrower than the kernel's: zero
                    const uint32_t x = c0 + e < d_g + d_u ? u[e - first] : 0u;
                    w[e >> 1] = (e & 1) ? ((w[e >> 1] & 0x0000FFFFu) | (x << 16)) : ((w[e >> 1] & 0xFFFF0000u) | x);
                }
            }
            v = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
    return v;
}

template <int DA, int NW, int TP, int MODE>
__global__ __launch_bounds__(NW * 64, (DA == 256 ? 1 : 2)) void ckv_mfma_kernel(ckv_args a) {
    constexpr int NT = NW * 64;        // threads
    constexpr int CH = DA / 8;         // 16-byte chunks per row
    constexpr int RPP = NT / CH;       // rows gathered per pass
    constexpr int NL = TP / RPP;       // passes per tile (chunks per lane per tile, K and V each)
    constexpr int KS = DA * 2 + 16;    // LDS row stride of K in bytes (conflict-free 16-byte row reads)
    constexpr int VS = DA * 2 + 64;    // LDS row stride of V in bytes (conflict-free transpose reads: four rows x 64 bytes per clock)
    constexpr int BUF = TP * (KS + VS);
    constexpr int NKK = DA / 16;       // k-steps of S^T = K Q^T
    constexpr int NDT = DA / 32;       // 32-row tiles of O^T
    static_assert(TP % RPP == 0 && TP % 32 == 0, "tile shape");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const ckv_item it = a.items[blockIdx.x];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int qn = lane & 31, hh = lane >> 5;
    // pool and user columns of each side (a side that is not shared: all user, no pool)
    const int d_gk = a.d_gk, d_uk = a.d_uk, d_gv = a.d_gv, d_uv = a.d_uv;
    const int d_a = a.d_a;  // <= DA: columns d_a .. DA-1 of the kernel's rows are zeros
    const int n = it.n;

    const int64_t hT = (int64_t)it.h * a.T + it.t0;
    const int32_t* __restrict__ ik = a.idx_k + hT;
    const int32_t* __restrict__ iv = a.idx_v + hT;
    const uint16_t* __restrict__ uk = (const uint16_t*)a.user_k + hT * d_uk;
    const uint16_t* __restrict__ uv = (const uint16_t*)a.user_v + hT * d_uv;
    const uint16_t* __restrict__ pk = (const uint16_t*)a.pool_k + (int64_t)it.h * a.P * a.pool_ld;
    const uint16_t* __restrict__ pv = (const uint16_t*)a.pool_v + (int64_t)it.h * a.P * a.pool_ld;

    // ---- queries of this lane, kernel column order, as B operands
    const int qj = it.q0 + wave * 32 + qn;
    const bool qok = qj < a.Nq;
    const int64_t qo = (((int64_t)it.b * a.H + it.h) * a.Nq + (qok ? qj : 0)) * d_a;
    bf16x8 qreg[NKK];
    {
        const uint16_t* qp = (const uint16_t*)a.q + qo;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int ci = 16 * kk + 8 * hh + e;
                const int pc = ci < d_gk ? ci + d_uk : ci - d_gk;  // kernel column of K -> column of q
                const uint16_t x = qok && ci < d_a ? qp[pc] : (uint16_t)0;
                qreg[kk][e] = __builtin_bit_cast(__bf16, x);
            }
        }
        // the queries have to have arrived before the tile loop: a wait for them that the compiler placed inside
        // the loop would also wait for the row gathers of the next tile, which are meant to stay in flight
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) asm volatile("" : "+v"(qreg[kk]));
    }

    f32x16 oacc[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
    float m_ref = -INFINITY, lsum = 0.f;
    const float sc = MODE == CKV_SOFTMAX ? a.scale * kLog2e : a.scale;

    // ---- gather bookkeeping: this lane owns chunk c of rows p0 + i*RPP
    const int c = tid % CH, p0 = tid / CH;
    int rk[NL], rv[NL];
    uint4 kreg[NL], vreg[NL];
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
    // When pool and user widths are multiples of eight columns on both sides (workgroup-uniform), this lane's chunk
    // lies for every row in one and the same place: in the pool row, in the user row, or past d_a.  Where it comes
    // from is then settled once (source, column), and a row costs one address and one 16-byte load without a
    // branch.  A chunk past d_a fetches chunk 0 instead: for K it meets query columns that are zero, for V it
    // lands in rows of O^T that nobody stores (inputs are finite).
    const bool chunked = ((d_gk | d_uk | d_gv | d_uv) & 7) == 0 && (a.pool_ld & 7) == 0 && a.pool_ld <= 0x7fffffff;
    const int ck = 8 * c < d_a ? 8 * c : 0, cv = ck;
    const bool k_pool = ck < d_gk, v_pool = cv < d_gv;
    // (source of this lane's chunk: first element of its column in row 0, and the distance between rows)
    const uint16_t* const k_src = k_pool ? pk + ck : uk + (ck - d_gk);
    const uint16_t* const v_src = v_pool ? pv + cv : uv + (cv - d_gv);
    const uint32_t k_ld = k_pool ? (uint32_t)a.pool_ld : (uint32_t)d_uk, v_ld = v_pool ? (uint32_t)a.pool_ld : (uint32_t)d_uv;
    // The same with widths that are multiples of four columns (d_u = 4, the paper's usual slice): the two 8-byte halves
    // of the chunk are settled separately and fetched with one 8-byte load each.
    const bool halved = !chunked && ((d_gk | d_uk | d_gv | d_uv) & 3) == 0 && (a.pool_ld & 7) == 0 && a.pool_ld <= 0x7fffffff;
    const uint16_t* kh_src[2];
    const uint16_t* vh_src[2];
    uint32_t kh_ld[2], vh_ld[2];
    bool kh_pool[2], vh_pool[2];
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
        const int col = 8 * c + 4 * hb < d_a ? 8 * c + 4 * hb : 0;
        kh_pool[hb] = col < d_gk;
        vh_pool[hb] = col < d_gv;
        kh_src[hb] = kh_pool[hb] ? pk + col : uk + (col - d_gk);
        vh_src[hb] = vh_pool[hb] ? pv + col : uv + (col - d_gv);
        kh_ld[hb] = kh_pool[hb] ? (uint32_t)a.pool_ld : (uint32_t)d_uk;
        vh_ld[hb] = vh_pool[hb] ? (uint32_t)a.pool_ld : (uint32_t)d_uv;
    }
    auto load_rows = [&](int tile) {
        if (halved) {
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int pos = min(tile * TP + p0 + i * RPP, n - 1);
                uint2 kh[2], vh[2];
#pragma unroll
                for (int hb = 0; hb < 2; ++hb) {
                    const uint32_t krow = (uint32_t)(kh_pool[hb] ? rk[i] : pos), vrow = (uint32_t)(vh_pool[hb] ? rv[i] : pos);
                    kh[hb] = *reinterpret_cast<const uint2*>(kh_src[hb] + (uint64_t)krow * kh_ld[hb]);
                    vh[hb] = *reinterpret_cast<const uint2*>(vh_src[hb] + (uint64_t)vrow * vh_ld[hb]);
                }
                kreg[i] = make_uint4(kh[0].x, kh[0].y, kh[1].x, kh[1].y);
                vreg[i] = make_uint4(vh[0].x, vh[0].y, vh[1].x, vh[1].y);
            }
        } else if (chunked) {
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int pos = min(tile * TP + p0 + i * RPP, n - 1);
                const uint32_t krow = (uint32_t)(k_pool ? rk[i] : pos), vrow = (uint32_t)(v_pool ? rv[i] : pos);
                kreg[i] = *reinterpret_cast<const uint4*>(k_src + (uint64_t)krow * k_ld);
                vreg[i] = *reinterpret_cast<const uint4*>(v_src + (uint64_t)vrow * v_ld);
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
            *reinterpret_cast<uint4*>(kb + p * KS + c * 16) = kreg[i];
            *reinterpret_cast<uint4*>(vb + p * VS + c * 16) = vreg[i];
        }
    };

    if (ntiles > 0) {
        load_idx(0);
        load_rows(0);
        if (ntiles > 1) load_idx(1);
        store_rows(0);
        __syncthreads();
    }

    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) load_rows(t + 1);
        if (t + 2 < ntiles) load_idx(t + 2);

        const unsigned char* kb = smem + buf * BUF;
        const unsigned char* vb = kb + TP * KS;
        const int nt = min(n - t * TP, TP);
#pragma unroll
        for (int s = 0; s < TP / 32; ++s) {
            if (32 * s < nt) {
                // S^T = K Q^T
                f32x16 sacc;
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
                const unsigned char* krow = kb + (32 * s + qn) * KS + hh * 16;
#pragma unroll
                for (int kk = 0; kk < NKK; ++kk) {
                    const bf16x8 ka = *reinterpret_cast<const bf16x8*>(krow + kk * 32);
                    sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[kk], sacc, 0, 0, 0);
                }
                // weights
                const bool ragged = 32 * s + 32 > nt;
                bf16x8 pb[2];
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
                        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[r], sc, -m_ref));
                        psum += p;
                        pb[r >> 3][r & 7] = (__bf16)p;
                    }
                    lsum += psum;
                } else {
                    // (sixteen independent chains, one kind of instruction at a time: the transcendental unit's
                    // latency is then covered by the other fifteen instead of being waited for sixteen times)
                    float x[16], e[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r) x[r] = sacc[r] * sc;
#pragma unroll
                    for (int r = 0; r < 16; ++r) e[r] = __builtin_amdgcn_exp2f(-kLog2e * x[r]);
#pragma unroll
                    for (int r = 0; r < 16; ++r) e[r] = __builtin_amdgcn_rcpf(1.f + e[r]);
#pragma unroll
                    for (int r = 0; r < 16; ++r) x[r] *= e[r];
                    if (ragged) {
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (32 * s + 8 * (r >> 2) + 4 * hh + (r & 3) >= nt) x[r] = 0.f;
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) pb[r >> 3][r & 7] = (__bf16)x[r];
                }
                // O^T += V^T P^T
                const int g16 = lane >> 4, s16 = lane & 15;
                const unsigned char* vrow = vb + (32 * s + 4 * hh + (s16 >> 2)) * VS + (16 * (g16 & 1) + 4 * (s16 & 3)) * 2;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
                    for (int dt = 0; dt < NDT; ++dt) {
                        const unsigned char* p0v = vrow + (16 * ks) * VS + dt * 64;
                        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0v));
                        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0v + 8 * VS));
                        const bf16x8 va = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[ks], oacc[dt], 0, 0, 0);
                    }
                }
            }
        }

        if (t + 1 < ntiles) store_rows((t + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue
    float l_tot = 0.f;
    if (MODE == CKV_SOFTMAX) l_tot = lsum + other_half(lsum);
    if (it.part < 0) {
        float inv;
        if (MODE == CKV_SOFTMAX) inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        else inv = it.n_total > 0 ? 1.f / (float)it.n_total : 0.f;
        if (qok) {
            uint16_t* op = (uint16_t*)a.out + qo;
#pragma unroll
            for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ci = 32 * dt + 8 * (r >> 2) + 4 * hh + (r & 3);
                    const int pc = ci < d_gv ? ci + d_uv : ci - d_gv;  // kernel column of V -> column of out
                    if (ci < d_a) op[pc] = f2bf(oacc[dt][r] * inv);
                }
        }
    } else {
        float* ws = a.partial + (int64_t)it.part * a.QB * (d_a + 2);
        const int j = wave * 32 + qn;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ci = 32 * dt + 8 * (r >> 2) + 4 * hh + (r & 3);
                const int pc = ci < d_gv ? ci + d_uv : ci - d_gv;
                if (ci < d_a) ws[(int64_t)j * d_a + pc] = oacc[dt][r];
            }
        if (hh == 0) {
            ws[(int64_t)a.QB * d_a + j] = m_ref * kLn2;  // natural-log units, as the merge expects
            ws[(int64_t)a.QB * d_a + a.QB + j] = l_tot;
        }
    }
}

template <int DA, int NW, int TP>
constexpr int lds_bytes() {
    return 2 * TP * ((DA * 2 + 16) + (DA * 2 + 64));
}

template <int DA, int NW, int TP, int MODE>
hipError_t prepare() {
    constexpr int lds = lds_bytes<DA, NW, TP>();
    static hipError_t done =
        hipFuncSetAttribute((const void*)ckv_mfma_kernel<DA, NW, TP, MODE>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    return done;
}

template <int DA, int NW, int TP, int MODE>
hipError_t launch(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    hipError_t e = prepare<DA, NW, TP, MODE>();
    if (e != hipSuccess) return e;
    constexpr int lds = lds_bytes<DA, NW, TP>();
    hipLaunchKernelGGL((ckv_mfma_kernel<DA, NW, TP, MODE>), dim3(c->n_items), dim3(NW * 64), lds, s, a);
    return hipGetLastError();
}

template <int DA, int NW, int TP, int MODE>
int occupancy() {
    if (prepare<DA, NW, TP, MODE>() != hipSuccess) return 0;
    int nb = 0;
    constexpr int lds = lds_bytes<DA, NW, TP>();
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, (const void*)ckv_mfma_kernel<DA, NW, TP, MODE>, NW * 64, lds) !=
        hipSuccess)
        return 0;
    return nb;
}

#define CKV_MFMA_SHAPES(X) X(64, 1, 64) X(64, 2, 64) X(64, 4, 64) X(128, 1, 32) X(128, 2, 64) X(128, 4, 64) X(256, 4, 32)

}  // namespace

bool ckv_mfma_supported(int d_a, int nw, int tp) {
#define X(DA, NW, TP) \
    if (d_a == DA && nw == NW && tp == TP) return true;
    CKV_MFMA_SHAPES(X)
#undef X
    return false;
}

int ckv_mfma_occupancy(int d_a, int nw, int tp, int mode) {
#define X(DA, NW, TP)                                                                             \
    if (d_a == DA && nw == NW && tp == TP)                                                        \
        return mode == CKV_SOFTMAX ? occupancy<DA, NW, TP, CKV_SOFTMAX>() : occupancy<DA, NW, TP, CKV_SILU_OVER_N>();
    CKV_MFMA_SHAPES(X)
#undef X
    return 0;
}

hipError_t ckv_launch_mfma(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    if (c->n_items == 0) return hipSuccess;
    const int d_a = a.d_a <= 64 ? 64 : (a.d_a <= 128 ? 128 : 256), nw = c->nw, tp = c->tp;  // the kernel's row width
#define X(DA, NW, TP)                                                                         \
    if (d_a == DA && nw == NW && tp == TP)                                                    \
        return c->shape.mode == CKV_SOFTMAX ? launch<DA, NW, TP, CKV_SOFTMAX>(c, a, s)         \
                                            : launch<DA, NW, TP, CKV_SILU_OVER_N>(c, a, s);
    CKV_MFMA_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}
