// Streaming (vector-ALU) gather-concat-attend kernel: the path for few queries per user
// (target attention, Q in R^{1 x d}, section 2.1) and the general fallback for any shape.
//
// A workgroup of four (or two) 64-lane wavefronts serves one work item (a run of positions of one
// user and head) for every query of the block, one query after the other.  A tile is 64 positions;
// wavefront w takes tiles w, w+4, ... and the partial results (maximum, sum, weighted sum) are
// merged through LDS.  Sixteen
// lanes share one final K (or V) row: lane c of the group owns the columns
// (cb*16 + c)*VEC .. +VEC of every column block cb, taken from the user slice when the
// column is < d_u and from the gathered pool row otherwise (eq. "eq: Kc", "eq: K": the
// concat exists only as this column test; a side that is not shared has d_u = d_a and never
// reaches the pool).  Four rows are processed per step.  The score of
// position 4*t + r ends up in lane 16*r + t, so softmax maxima and sums are wavefront
// shuffles, and the weight is shuffled back to the row's sixteen lanes for the V pass.
#include "ckv_internal.h"

namespace {

constexpr int kLanes = 64;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kLanes));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kLanes);
    return v;
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float up(float x) { return x; }
    static __device__ __forceinline__ float down(float x) { return x; }
};
template <> struct Elem<uint16_t> {  // bfloat16 bit pattern
    static __device__ __forceinline__ float up(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }
    static __device__ __forceinline__ uint16_t down(float f) {  // round to nearest even
        uint32_t u = __float_as_uint(f);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
};

template <typename T, int VEC> struct alignas(sizeof(T) * VEC) Pack { T v[VEC]; };

template <typename T, int VEC>
__device__ __forceinline__ void load_vec(float (&dst)[VEC], const T* src) {
    Pack<T, VEC> p = *reinterpret_cast<const Pack<T, VEC>*>(src);
#pragma unroll
    for (int i = 0; i < VEC; ++i) dst[i] = Elem<T>::up(p.v[i]);
}

// Wavefronts per SIMD the register budget is sized for: a whole tile of K and V rows is held in registers
// (one column block), which costs 64 registers at 8 bytes per lane and row and 128 at 16 bytes.
template <typename T, int VEC, int NCB, int kGroup>
constexpr int stream_waves() { return NCB == 1 ? (kGroup * sizeof(T) * VEC <= 128 ? 4 : 2) : 1; }

// kWaves = wavefronts per work item (2 or 4): four shorten the chain of one item, two let twice as many
// items be resident at once; the host takes two when four would need more than one round of workgroups.
// kGroup = lanes that share one row (16, or 8 when eight lanes of VEC elements cover d_a: half as many
// load instructions per tile); a step covers 64 / kGroup rows and a tile has kGroup steps.
template <typename T, int VEC, int NCB, int MODE, int kWaves, int kGroup>
__global__ __launch_bounds__(kLanes * kWaves)
__attribute__((amdgpu_waves_per_eu(stream_waves<T, VEC, NCB, kGroup>(), 8))) void ckv_stream_kernel(ckv_args a) {
    constexpr int RS = kLanes / kGroup;  // rows per step
    __shared__ float sm_acc[kWaves][NCB * kGroup * VEC];
    __shared__ float sm_ml[kWaves][2];
    const ckv_item it = a.items[blockIdx.x];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane / kGroup, c = lane % kGroup;
    // user columns of each side: d_u of the shape, or all d_a columns for a side that is not shared
    const int d_uk = a.d_uk, d_uv = a.d_uv, d_a = a.d_a;
    const int64_t hT = (int64_t)it.h * a.T + it.t0;
    const int32_t* ik = a.idx_k + hT;
    const int32_t* iv = a.idx_v + hT;
    const T* uk = (const T*)a.user_k + hT * d_uk;
    const T* uv = (const T*)a.user_v + hT * d_uv;
    const T* pk = (const T*)a.pool_k + (int64_t)it.h * a.P * a.pool_ld;
    const T* pv = (const T*)a.pool_v + (int64_t)it.h * a.P * a.pool_ld;
    const int n = it.n;
    const int slot_of_lane = RS * c + r;  // position (within a tile) whose score this lane keeps

    // column ownership: col[cb] = first final-K column of this lane in block cb (or -1)
    int col[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
        int c0 = (cb * kGroup + c) * VEC;
        col[cb] = c0 < d_a ? c0 : -1;
    }

    for (int j = 0; j < a.QB; ++j) {
        const int qj = it.q0 + j;
        if (qj >= a.Nq) break;
        const int64_t qo = (((int64_t)it.b * a.H + it.h) * a.Nq + qj) * d_a;
        const T* qp = (const T*)a.q + qo;
        float qreg[NCB][VEC];
        float acc[NCB][VEC];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) { qreg[cb][v] = 0.f; acc[cb][v] = 0.f; }
            if (col[cb] >= 0) load_vec<T, VEC>(qreg[cb], qp + col[cb]);
        }
        float m_run = -INFINITY, l_run = 0.f;

        for (int t0 = wave * kLanes; t0 < n; t0 += kLanes * kWaves) {
            const int nt = min(n - t0, kLanes);
            const int nsteps = (nt + RS - 1) / RS;
            const int myslot = min(slot_of_lane, nt - 1);
            const int my_ik = a.d_gk > 0 ? ik[t0 + myslot] : 0;
            const int my_iv = a.d_gv > 0 ? iv[t0 + myslot] : 0;
            float s_mine = 0.f;
            float w;
            if constexpr (NCB == 1 && sizeof(T) * VEC >= 4) {
                // One column block: the whole tile's K and V rows (kGroup steps of RS rows) are requested
                // before anything is computed, so that a tile costs one memory round trip after its
                // indices instead of one per group of steps.  Steps past the end of the tile read a
                // clamped position and are masked by their zero weight.
                // rows are kept as raw 32-bit words (two bf16 per word) so that they cost no more registers
                // than their bytes
                constexpr int NWORD = (int)(sizeof(T) * VEC / 4);  // >= 1 here
                typedef uint32_t Raw __attribute__((ext_vector_type(NWORD)));
                auto elem = [](const Raw& w, int v) -> float {
                    if (sizeof(T) == 4) return __uint_as_float(w[v]);
                    return __uint_as_float((v & 1) ? (w[v >> 1] & 0xFFFF0000u) : (w[v >> 1] << 16));
                };
                Raw kraw[kGroup], vraw[kGroup];
                const bool own = col[0] >= 0;
                const int c0 = own ? col[0] : 0;
#pragma unroll
                for (int t = 0; t < kGroup; ++t) {
                    const int pos = min(RS * t + r, nt - 1);
                    const int src_lane = (lane & ~(kGroup - 1)) | t;
                    const int rowk = __shfl(my_ik, src_lane, kLanes);
                    const int rowv = __shfl(my_iv, src_lane, kLanes);
                    const T* ksrc = c0 < d_uk ? uk + (int64_t)(t0 + pos) * d_uk + c0 : pk + (int64_t)rowk * a.pool_ld + (c0 - d_uk);
                    const T* vsrc = c0 < d_uv ? uv + (int64_t)(t0 + pos) * d_uv + c0 : pv + (int64_t)rowv * a.pool_ld + (c0 - d_uv);
                    if (own) {
                        kraw[t] = *reinterpret_cast<const Raw*>(ksrc);
                        vraw[t] = *reinterpret_cast<const Raw*>(vsrc);
                    } else {
#pragma unroll
                        for (int v = 0; v < NWORD; ++v) kraw[t][v] = vraw[t][v] = 0u;
                    }
                }
#pragma unroll
                for (int t = 0; t < kGroup; ++t) {
                    float part = 0.f;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) part = fmaf(elem(kraw[t], v), qreg[0][v], part);
#pragma unroll
                    for (int o = kGroup / 2; o > 0; o >>= 1) part += __shfl_xor(part, o, kLanes);
                    if (c == t) s_mine = part;
                }
                const bool valid = slot_of_lane < nt;
                if (MODE == CKV_SOFTMAX) {
                    const float sv = valid ? s_mine * a.scale : -INFINITY;
                    const float m_new = fmaxf(m_run, wave_max(sv));
                    const float alpha = __expf(m_run - m_new);  // first tile: exp(-inf) = 0
                    w = valid ? __expf(sv - m_new) : 0.f;
                    l_run = l_run * alpha + wave_sum(w);
                    m_run = m_new;
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[0][v] *= alpha;
                } else {
                    const float sv = s_mine * a.scale;
                    w = valid ? sv / (1.f + __expf(-sv)) : 0.f;
                }
#pragma unroll
                for (int t = 0; t < kGroup; ++t) {
                    const float wr = __shfl(w, (lane & ~(kGroup - 1)) | t, kLanes);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[0][v] = fmaf(wr, elem(vraw[t], v), acc[0][v]);
                }
                continue;
            }
            // ---- scores
            for (int tb = 0; tb < nsteps; tb += 4)
#pragma unroll
            for (int t = tb; t < tb + 4; ++t) {  // steps past nsteps touch clamped, masked positions
                const int pos = min(RS * t + r, nt - 1);
                const int row = __shfl(my_ik, (lane & ~(kGroup - 1)) | t, kLanes);
                float part = 0.f;
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) {
                    if (col[cb] >= 0) {
                        float kv[VEC];
                        const T* src = col[cb] < d_uk ? uk + (int64_t)(t0 + pos) * d_uk + col[cb]
                                                      : pk + (int64_t)row * a.pool_ld + (col[cb] - d_uk);
                        load_vec<T, VEC>(kv, src);
#pragma unroll
                        for (int v = 0; v < VEC; ++v) part = fmaf(kv[v], qreg[cb][v], part);
                    }
                }
#pragma unroll
                for (int o = kGroup / 2; o > 0; o >>= 1) part += __shfl_xor(part, o, kLanes);
                if (c == t) s_mine = part;
            }
            // ---- weights
            const bool valid = slot_of_lane < nt;
            if (MODE == CKV_SOFTMAX) {
                const float s = valid ? s_mine * a.scale : -INFINITY;
                const float m_new = fmaxf(m_run, wave_max(s));
                const float alpha = __expf(m_run - m_new);  // first tile: exp(-inf) = 0
                w = valid ? __expf(s - m_new) : 0.f;
                l_run = l_run * alpha + wave_sum(w);
                m_run = m_new;
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[cb][v] *= alpha;
            } else {
                const float s = s_mine * a.scale;
                w = valid ? s / (1.f + __expf(-s)) : 0.f;
            }
            // ---- weighted sum of final V rows
            for (int tb = 0; tb < nsteps; tb += 4)
#pragma unroll
            for (int t = tb; t < tb + 4; ++t) {
                const int pos = min(RS * t + r, nt - 1);
                const int src_lane = (lane & ~(kGroup - 1)) | t;
                const int row = __shfl(my_iv, src_lane, kLanes);
                const float wr = __shfl(w, src_lane, kLanes);
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb) {
                    if (col[cb] >= 0) {
                        float vv[VEC];
                        const T* src = col[cb] < d_uv ? uv + (int64_t)(t0 + pos) * d_uv + col[cb]
                                                      : pv + (int64_t)row * a.pool_ld + (col[cb] - d_uv);
                        load_vec<T, VEC>(vv, src);
#pragma unroll
                        for (int v = 0; v < VEC; ++v) acc[cb][v] = fmaf(wr, vv[v], acc[cb][v]);
                    }
                }
            }
        }
        // ---- fold the four row groups, then write
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                float x = acc[cb][v];
#pragma unroll
                for (int o = kGroup; o < kLanes; o <<= 1) x += __shfl_xor(x, o, kLanes);
                acc[cb][v] = x;
            }
        // ---- merge the four wavefronts through LDS (exact: rescale to the common maximum)
        if (r == 0) {
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                for (int v = 0; v < VEC; ++v) sm_acc[wave][(cb * kGroup + c) * VEC + v] = acc[cb][v];
            if (c == 0) {
                sm_ml[wave][0] = m_run;
                sm_ml[wave][1] = l_run;
            }
        }
        __syncthreads();
        if (wave == 0 && r == 0) {
            float M = -INFINITY, L = 0.f, wgt[kWaves];
            if (MODE == CKV_SOFTMAX) {
#pragma unroll
                for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sm_ml[w][0]);
#pragma unroll
                for (int w = 0; w < kWaves; ++w) {
                    wgt[w] = sm_ml[w][0] == -INFINITY ? 0.f : __expf(sm_ml[w][0] - M);
                    L += wgt[w] * sm_ml[w][1];
                }
            } else {
#pragma unroll
                for (int w = 0; w < kWaves; ++w) wgt[w] = 1.f;
            }
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    float x = 0.f;
#pragma unroll
                    for (int w = 0; w < kWaves; ++w) x += wgt[w] * sm_acc[w][(cb * kGroup + c) * VEC + v];
                    acc[cb][v] = x;
                }
            if (it.part < 0) {
                float norm;
                if (MODE == CKV_SOFTMAX) norm = L > 0.f ? 1.f / L : 0.f;
                else norm = it.n_total > 0 ? 1.f / (float)it.n_total : 0.f;
                T* op = (T*)a.out + qo;
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
                    if (col[cb] >= 0) {
                        Pack<T, VEC> p;
#pragma unroll
                        for (int v = 0; v < VEC; ++v) p.v[v] = Elem<T>::down(acc[cb][v] * norm);
                        *reinterpret_cast<Pack<T, VEC>*>(op + col[cb]) = p;
                    }
            } else {
                float* ws = a.partial + (int64_t)it.part * a.QB * (d_a + 2);
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
                    if (col[cb] >= 0)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) ws[(int64_t)j * d_a + col[cb] + v] = acc[cb][v];
                if (c == 0) {
                    ws[(int64_t)a.QB * d_a + j] = M;
                    ws[(int64_t)a.QB * d_a + a.QB + j] = L;
                }
            }
        }
        __syncthreads();  // the next query reuses the LDS buffers
    }
}

template <typename T, int VEC, int NCB, int NWV, int GRP>
hipError_t launch_group(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    dim3 grid(c->n_items), block(kLanes * NWV);
    if (c->shape.mode == CKV_SOFTMAX)
        hipLaunchKernelGGL((ckv_stream_kernel<T, VEC, NCB, CKV_SOFTMAX, NWV, GRP>), grid, block, 0, s, a);
    else
        hipLaunchKernelGGL((ckv_stream_kernel<T, VEC, NCB, CKV_SILU_OVER_N, NWV, GRP>), grid, block, 0, s, a);
    return hipGetLastError();
}

template <typename T, int VEC, int NCB, int NWV>
hipError_t launch_waves(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    // eight lanes per row only exist for the widest vectors (the host asks for them only there)
    if (c->grp == 8 && sizeof(T) * VEC == 16) return launch_group<T, VEC, NCB, NWV, 8>(c, a, s);
    return launch_group<T, VEC, NCB, NWV, 16>(c, a, s);
}

template <typename T, int VEC, int NCB>
hipError_t launch_mode(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    return c->nw == 2 ? launch_waves<T, VEC, NCB, 2>(c, a, s) : launch_waves<T, VEC, NCB, 4>(c, a, s);
}

template <typename T, int VEC>
hipError_t launch_ncb(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    switch (c->ncb) {
        case 1: return launch_mode<T, VEC, 1>(c, a, s);
        case 2: return launch_mode<T, VEC, 2>(c, a, s);
        case 4: return launch_mode<T, VEC, 4>(c, a, s);
        case 8: return launch_mode<T, VEC, 8>(c, a, s);
        default: break;
    }
    // wide rows that allow no vector loads (odd widths or strides): one element per lane, up to 256 columns
    if constexpr (VEC == 1) {
        if (c->ncb == 16) return launch_mode<T, VEC, 16>(c, a, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t ckv_launch_stream(const ckv_cache* c, const ckv_args& a, hipStream_t s) {
    if (c->n_items == 0) return hipSuccess;
    if (c->shape.dtype == CKV_F32) {
        switch (c->vec) {
            case 1: return launch_ncb<float, 1>(c, a, s);
            case 4: return launch_ncb<float, 4>(c, a, s);
            default: return hipErrorInvalidValue;
        }
    }
    switch (c->vec) {
        case 1: return launch_ncb<uint16_t, 1>(c, a, s);
        case 4: return launch_ncb<uint16_t, 4>(c, a, s);
        case 8: return launch_ncb<uint16_t, 8>(c, a, s);
        default: return hipErrorInvalidValue;
    }
}
