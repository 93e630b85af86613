// Prefill stage of CollectiveKV (paper section 4.2 "In the prefill stage", section 4.3 router):
//   K_u = S W_k + b_k, V_u = S W_v + b_v            (projection to the d_u user-specific columns)
//   M = S W_r + b_r,  I[i] = argmax_j M[i][j]        (router; one for keys, one for values)
// written straight into the packed cache layout the attention kernels stream (indices
// [2][H][T], user slices [H][T][d_u]).  The routing map M (T x P per head and side) is never
// written anywhere: every workgroup keeps a block of positions in registers, streams the
// router weights through LDS in tiles of 32 pool entries and keeps a running (maximum, index)
// per position.
//
// Matrix-core kernel (bf16 storage, d_e = 64, 128 or 256): M^T = W_r S^T with
// v_mfma_f32_32x32x16_bf16, router rows as the A operand (read from LDS), positions as the B
// operand (registers), so that a lane owns one position and sixteen pool entries of the tile;
// the bias enters as the initial value of the accumulator (fp32, exact).  The maximum over the
// lane's sixteen entries costs eight v_max3; only when it beats the lane's running maximum
// (rare after the first tiles) is the entry that attains it located.  Equal scores keep the
// lowest pool entry: tiles are visited in increasing order and replaced only on a strict
// improvement, and inside a tile the lowest matching register wins.
// The projection is one more tile whose 32 "pool entries" are the d_u rows of W_k (or W_v).
//
// Scalar kernel: any d_e and either storage type, one thread per (position, head, side).
#include "ckv_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((address_space(3))) unsigned char lds_u8;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
typedef __attribute__((address_space(3))) f32x4 lds_f32x4;

constexpr int TR = 32;  // pool entries per tile
constexpr int NS = 4;   // stages in the LDS ring

__device__ __forceinline__ void dma16(const void* g, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_base) : "memory");
}
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
__device__ __forceinline__ uint32_t swap_halves(uint32_t x) {
    auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return threadIdx.x & 32 ? r[0] : r[1];
}
__device__ __forceinline__ uint16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

template <int DE, int NW>
struct PGeo {
    static constexpr int CH = DE / 8;            // 16-byte chunks per weight row
    static constexpr int ROWB = DE * 2;          // bytes per weight row
    static constexpr int RPI = 64 / CH;          // rows filled by one wavefront load instruction
    static constexpr int NI = TR / RPI / NW;     // load instructions per wavefront and tile
    static constexpr int WT = TR * ROWB;         // bytes of the weight rows of a stage
    static constexpr int STAGE = WT + NW * 256;  // plus one private copy of the 32 biases per wavefront
    static constexpr int LDS = NS * STAGE;
    static_assert(NI >= 1, "tile too small for this many wavefronts");
};

// One workgroup: NW wavefronts x QG groups x 32 positions, one (head, side).
template <int DE, int NW, int QG>
__global__ __launch_bounds__(NW * 64) void ckv_prefill_mfma_kernel(ckv_prefill_args a) {
    using G = PGeo<DE, NW>;
    constexpr int NKK = DE / 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_u8*)smem;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int qn = lane & 31, hh = lane >> 5;
    const int ncls = 2 * a.H;
    const int cls = blockIdx.x % ncls;
    const int64_t pblock = blockIdx.x / ncls;
    const int h = cls >> 1, side = cls & 1;
    const int P = a.P, d_u = a.d_u;

    const unsigned char* __restrict__ wr = (const unsigned char*)a.w_r[side] + (int64_t)h * P * G::ROWB;
    const float* __restrict__ br = a.b_r[side] + (int64_t)h * P;
    const unsigned char* __restrict__ wu = (const unsigned char*)a.w_u[side] + (int64_t)h * d_u * G::ROWB;
    const float* __restrict__ bu = a.b_u[side] + (int64_t)h * d_u;
    const int nrt = (P + TR - 1) / TR;         // router tiles
    const int ntt = nrt + (d_u > 0 ? 1 : 0);   // plus the projection tile
    if (ntt == 0) return;

    // ---- positions of this wavefront: B operands, 16 bytes per lane and k-step, straight from S
    const int64_t pos0 = pblock * (32 * QG * NW) + (int64_t)wave * QG * 32;
    bf16x8 sreg[QG][NKK];
#pragma unroll
    for (int g = 0; g < QG; ++g) {
        const int64_t pos = pos0 + g * 32 + qn;
        const unsigned char* src = (const unsigned char*)a.S + pos * G::ROWB + hh * 16;
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (pos < a.T) v = *reinterpret_cast<const u32x4*>(src + kk * 32);
            sreg[g][kk] = __builtin_bit_cast(bf16x8, v);
        }
    }
    // these loads have to be complete before the asynchronous loads below start: a wait the
    // compiler placed inside the tile loop would also drain the loads it cannot see
#pragma unroll
    for (int g = 0; g < QG; ++g)
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) asm volatile("" : "+v"(sreg[g][kk]));

    // ---- per-lane constants of the weight loads: instruction i of this wavefront fills rows
    //      (i*NW + wave)*RPI .. +RPI of the stage; chunk c of row p is stored at slot c ^ (p & 7)
    int lrow[G::NI];
    uint32_t lchunk[G::NI];
#pragma unroll
    for (int i = 0; i < G::NI; ++i) {
        lrow[i] = (i * NW + wave) * G::RPI + lane / G::CH;
        lchunk[i] = (uint32_t)(((lane % G::CH) ^ (lrow[i] & 7)) * 16);
    }
    auto issue = [&](int tile) {
        const uint32_t st = lds0 + (tile & (NS - 1)) * G::STAGE;
        tile = min(tile, ntt - 1);  // loads past the last tile repeat it, into a retired stage (never read)
        const bool proj = tile >= nrt;
        const unsigned char* wbase = proj ? wu : wr;
        const float* bbase = proj ? bu : br;
        const int row0 = proj ? 0 : tile * TR;
        const int rmax = (proj ? d_u : P) - 1;
#pragma unroll
        for (int i = 0; i < G::NI; ++i) {
            const int row = min(row0 + lrow[i], rmax);
            dma16(wbase + (int64_t)row * G::ROWB + lchunk[i], st + (i * NW + wave) * G::RPI * G::ROWB);
        }
        dma4(bbase + min(row0 + qn, rmax), st + G::WT + wave * 256);
    };

    float bv[QG];
    int bj[QG];
#pragma unroll
    for (int g = 0; g < QG; ++g) {
        bv[g] = -INFINITY;
        bj[g] = 0;
    }
    const uint32_t arow = qn * G::ROWB;
    const int ax = qn & 7;

    issue(0);
    issue(1);
    issue(2);
    wait_vm<2 * (G::NI + 1)>();
    lds_barrier();
    for (int t = 0; t < ntt; ++t) {
        issue(t + NS - 1);
        const uint32_t st = lds0 + (t & (NS - 1)) * G::STAGE;
        bf16x8 wa[NKK];
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) wa[kk] = *(const lds_bf16x8*)(uintptr_t)(st + arow + (((2 * kk + hh) ^ ax) << 4));
        f32x16 cinit;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const f32x4 b4 = *(const lds_f32x4*)(uintptr_t)(st + G::WT + wave * 256 + (8 * g4 + 4 * hh) * 4);
#pragma unroll
            for (int j = 0; j < 4; ++j) cinit[4 * g4 + j] = b4[j];
        }
        const bool proj = t >= nrt;
#pragma unroll
        for (int g = 0; g < QG; ++g) {
            f32x16 acc = cinit;
#pragma unroll
            for (int kk = 0; kk < NKK; ++kk) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa[kk], sreg[g][kk], acc, 0, 0, 0);
            if (!proj) {
                if (t == nrt - 1 && (P & (TR - 1))) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (t * TR + 8 * (r >> 2) + 4 * hh + (r & 3) >= P) acc[r] = -INFINITY;
                }
                float tmax = acc[0];
#pragma unroll
                for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, acc[r]);
                if (__any(tmax > bv[g])) {
                    int rr = 15;
#pragma unroll
                    for (int r = 14; r >= 0; --r) rr = acc[r] == tmax ? r : rr;
                    if (tmax > bv[g]) {
                        bv[g] = tmax;
                        bj[g] = t * TR + 8 * (rr >> 2) + 4 * hh + (rr & 3);
                    }
                }
            } else {
                // projection tile: row c of the tile is column c of the user slice
                const int64_t pos = pos0 + g * 32 + qn;
                if (pos < a.T) {
                    uint16_t* dst = (uint16_t*)a.user[side] + ((int64_t)h * a.T + pos) * d_u;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int c = 8 * (r >> 2) + 4 * hh + (r & 3);
                        if (c < d_u) dst[c] = f2bf(acc[r]);
                    }
                }
            }
        }
        wait_vm<2 * (G::NI + 1)>();
        lds_barrier();
    }
    wait_vm<0>();  // the repeated loads past the last tile must land before the workgroup gives its LDS back

    if (nrt > 0) {
#pragma unroll
        for (int g = 0; g < QG; ++g) {
            const float ov = __uint_as_float(swap_halves(__float_as_uint(bv[g])));
            const int oj = (int)swap_halves((uint32_t)bj[g]);
            const int best = (ov > bv[g] || (ov == bv[g] && oj < bj[g])) ? oj : bj[g];
            const int64_t pos = pos0 + g * 32 + qn;
            if (hh == 0 && pos < a.T) a.idx[((int64_t)side * a.H + h) * a.T + pos] = best;
        }
    }
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
        if (a.P > 0) {
            const U* __restrict__ w = (const U*)a.w_r[side] + (int64_t)h * a.P * d_e;
            const float* __restrict__ b = a.b_r[side] + (int64_t)h * a.P;
            float best = -INFINITY;
            int bj = 0;
            for (int j = 0; j < a.P; ++j) {
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
        if (a.d_u > 0) {
            const U* __restrict__ w = (const U*)a.w_u[side] + (int64_t)h * a.d_u * d_e;
            const float* __restrict__ b = a.b_u[side] + (int64_t)h * a.d_u;
            U* dst = (U*)a.user[side] + ((int64_t)h * a.T + pos) * a.d_u;
            for (int c0 = 0; c0 < a.d_u; ++c0) {
                float m = 0.f;
                for (int c = 0; c < d_e; ++c) m = fmaf(widen<U>(s[c]), widen<U>(w[(int64_t)c0 * d_e + c]), m);
                narrow(dst + c0, m + b[c0]);
            }
        }
    }
}

template <int DE, int NW, int QG>
hipError_t launch_mfma(const ckv_prefill_args& a, hipStream_t s) {
    constexpr int lds = PGeo<DE, NW>::LDS;
    static hipError_t prepared = hipFuncSetAttribute((const void*)ckv_prefill_mfma_kernel<DE, NW, QG>,
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (prepared != hipSuccess) return prepared;
    const int64_t per_wg = 32 * QG * NW;
    const int64_t blocks = (a.T + per_wg - 1) / per_wg * 2 * a.H;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL((ckv_prefill_mfma_kernel<DE, NW, QG>), dim3((unsigned)blocks), dim3(NW * 64), lds, s, a);
    return hipGetLastError();
}

}  // namespace

bool ckv_prefill_mfma_supported(int dtype, int d_e, int d_u) {
    return dtype == CKV_BF16 && (d_e == 64 || d_e == 128 || d_e == 256) && d_u <= 32;
}

const char* ckv_prefill_variant(int dtype, int d_e, int d_u) {
    if (ckv_prefill_mfma_supported(dtype, d_e, d_u)) return d_e == 64 ? "prefill_mfma_bf16_e64" : (d_e == 128 ? "prefill_mfma_bf16_e128" : "prefill_mfma_bf16_e256");
    return dtype == CKV_F32 ? "prefill_scalar_f32" : "prefill_scalar_bf16";
}

hipError_t ckv_launch_prefill(const ckv_prefill_args& a, int dtype, hipStream_t s) {
    if (a.T == 0 || (a.P == 0 && a.d_u == 0)) return hipSuccess;
    if (ckv_prefill_mfma_supported(dtype, a.d_e, a.d_u)) {
        if (a.d_e == 64) return launch_mfma<64, 4, 2>(a, s);
        if (a.d_e == 128) return launch_mfma<128, 4, 2>(a, s);
        return launch_mfma<256, 4, 1>(a, s);
    }
    const int64_t total = a.T * a.H * 2;
    const int blocks = (int)((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
    if (dtype == CKV_F32) hipLaunchKernelGGL(ckv_prefill_scalar_kernel<float>, dim3(blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL(ckv_prefill_scalar_kernel<uint16_t>, dim3(blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}
