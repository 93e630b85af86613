// C ABI of libckv.so: cache packing, work-list construction, dispatch, verification helpers.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <numeric>
#include <vector>

#include "ckv_internal.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

#define CKV_HIP(call)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            rc = fail(CKV_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_));            \
            goto done;                                                                        \
        }                                                                                     \
    } while (0)

size_t esize(int dtype) { return dtype == CKV_F32 ? 4 : 2; }

// Tuning options of the calling thread (ckv_set_option), read when a handle or a plan is built.
struct Options {
    bool staged = false;       // "mfma_impl" = "staged": register-staged matrix-core kernel where the direct-to-LDS one would run
    int sched = 0;             // "dma_sched": 0 default (static), 1 static, 2 dynamic
    int nw = 0, qg = 0;        // "dma_shape" = "nw,qg": wavefronts per workgroup, query groups per wavefront (0: from Nq)
    double slow_speed = -1.0;  // "dma_slow_speed": weight of a workgroup that shares its SIMDs with an older one (< 0: default)
    int q16 = -1;              // "dma_q16" = "0" | "1": sixteen-query organisation of the direct-to-LDS kernel where it applies (< 0: default, on)
    int scores_ahead = -1;     // "dma_scores_ahead" = "0" | "1": tile loop of the direct-to-LDS kernel with the scores one tile ahead (< 0: default)
    int hot_rows = 0;          // "stream_hot_rows" = n: pool rows the wide-row streaming kernel keeps in LDS per work item (default none)
    int stream_waves = 0;      // "stream_waves" = "2" | "4": wavefronts per work item of the streaming kernels (0: by the number of items)
    bool stream_narrow = false;  // "stream_impl" = "narrow": the column-block streaming kernel also where the wide-row one would run
    bool debug = false;        // "debug" = "1": print the chosen split and list statistics to stderr
};
thread_local Options g_opt;

// Scratch of the entry point that allocates nothing (ckv_attend_static_scratch): the split workspace of the matrix-core
// and streaming kernels, in a fixed array that every GPU the library runs on holds until the process ends.
constexpr size_t kStaticScratchBytes = CKV_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

// ---------------------------------------------------------------------------------------
// Packing: user-major [T][H] records -> head-major planes, with the range check of every
// index done in the same pass.  `bad` receives the smallest offending t*H + h.
template <typename U>
__global__ void ckv_pack_kernel(const int32_t* __restrict__ in_k, const int32_t* __restrict__ in_v,
                                const U* __restrict__ in_uk, const U* __restrict__ in_uv,
                                int32_t* __restrict__ idx, U* __restrict__ uk, U* __restrict__ uv,
                                int64_t T, int H, int d_uk, int d_uv, int P, int pool_k, int pool_v,
                                unsigned long long* __restrict__ bad) {
    const int64_t total = T * H;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t t = i / H;
        const int h = (int)(i - t * H);
        const int64_t o = (int64_t)h * T + t;
        if (idx) {  // a plane whose side has no pool is filled with zeros and never read
            const int32_t a = pool_k ? in_k[i] : 0, b = pool_v ? in_v[i] : 0;
            if (a < 0 || a >= P || b < 0 || b >= P) atomicMin(bad, (unsigned long long)i);
            idx[o] = a;
            idx[(int64_t)H * T + o] = b;
        }
        for (int c = 0; c < d_uk; ++c) uk[o * d_uk + c] = in_uk[i * d_uk + c];
        for (int c = 0; c < d_uv; ++c) uv[o * d_uv + c] = in_uv[i * d_uv + c];
    }
}

// Final K and V rows [H][T][d_a]: user slice then pool row.  Pure copy.
template <typename U>
__global__ void ckv_reconstruct_kernel(const int32_t* __restrict__ idx, const U* __restrict__ user,
                                       const U* __restrict__ pool, U* __restrict__ full,
                                       int64_t T, int H, int d_u, int d_g, int P, int64_t pool_ld) {
    const int d_a = d_u + d_g;
    const int64_t total = (int64_t)H * T * d_a;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t ht = i / d_a;
        const int c = (int)(i - ht * d_a);
        if (c < d_u) {
            full[i] = user[ht * d_u + c];
        } else {
            const int h = (int)(ht / T);
            full[i] = pool[((int64_t)h * P + idx[ht]) * pool_ld + (c - d_u)];
        }
    }
}

// Merge of the pieces of a split history.  Softmax pieces carry (acc, m, l) with acc and l
// relative to the piece maximum m; SiLU pieces carry only acc.  Block (x, y) handles merge
// entry x and queries 16y .. 16y+15, sixteen threads per query, eight columns per thread and pass.
// The kernel is a chain of memory round trips, so it is written to have few: the (m, l) of up to 64
// pieces and the rows of the first four are requested together; the weights exp(m_p - M) are computed
// once per query into LDS; the rows of the next four pieces are requested before the current four are
// accumulated.
template <typename U, int MODE>
__global__ __launch_bounds__(256) void ckv_merge_kernel(const ckv_merge* __restrict__ list, const float* __restrict__ partial,
                                                        U* __restrict__ out, int H, int Nq, int d_a, int QB) {
    constexpr int PCH = 64, CB = 8, SP = 4;
    __shared__ float sw[16][PCH];
    const ckv_merge mg = list[blockIdx.x];
    const int64_t stride = (int64_t)QB * (d_a + 2);
    const int jq = threadIdx.x >> 4;
    const int j = blockIdx.y * 16 + jq;
    const int c0 = threadIdx.x & 15;
    const bool valid = j < QB && mg.q0 + j < Nq;  // (no early exit: the block meets at barriers)
    const int jj = valid ? j : 0;
    const float* base = partial + (int64_t)mg.part0 * stride;
    const float* mrow = base + (int64_t)QB * d_a + jj;  // m of piece p at mrow[p * stride], l at mrow[p * stride + QB]
    const int nparts = mg.nparts;
    float M = -INFINITY, denom = 0.f;
    if (MODE == CKV_SOFTMAX) {
        if (nparts > PCH) {  // more pieces than one chunk: the maximum needs a pass of its own
            for (int p = c0; p < nparts; p += 16) M = fmaxf(M, mrow[p * stride]);
#pragma unroll
            for (int d = 1; d < 16; d <<= 1) M = fmaxf(M, __shfl_xor(M, d));
        }
    } else {
        denom = (float)mg.n_total;
    }
    const int64_t o = (((int64_t)mg.b * H + mg.h) * Nq + mg.q0 + jj) * d_a;
    for (int cbase = 0; cbase < d_a; cbase += 16 * CB) {
        float acc[CB];
#pragma unroll
        for (int k = 0; k < CB; ++k) acc[k] = 0.f;
        auto load_rows = [&](int p, float (&v)[SP][CB]) {  // rows of pieces p .. p+SP-1 (zeros past the last)
#pragma unroll
            for (int i = 0; i < SP; ++i) {
                const float* row = base + (int64_t)(p + i) * stride + (int64_t)jj * d_a + cbase + c0;
#pragma unroll
                for (int k = 0; k < CB; ++k) v[i][k] = (p + i < nparts && cbase + c0 + 16 * k < d_a) ? row[16 * k] : 0.f;
            }
        };
        for (int p0 = 0; p0 < nparts; p0 += PCH) {
            const int np = min(PCH, nparts - p0);
            float v[SP][CB];
            load_rows(p0, v);
            if (MODE == CKV_SOFTMAX) {
                float mp[PCH / 16], lp[PCH / 16];
#pragma unroll
                for (int i = 0; i < PCH / 16; ++i) {
                    const int pp = c0 + 16 * i;
                    mp[i] = pp < np ? mrow[(p0 + pp) * stride] : -INFINITY;
                    lp[i] = pp < np ? mrow[(p0 + pp) * stride + QB] : 0.f;
                }
                if (nparts <= PCH) {
#pragma unroll
                    for (int i = 0; i < PCH / 16; ++i) M = fmaxf(M, mp[i]);
#pragma unroll
                    for (int d = 1; d < 16; d <<= 1) M = fmaxf(M, __shfl_xor(M, d));
                }
                __syncthreads();  // the previous chunk's weights are no longer read
#pragma unroll
                for (int i = 0; i < PCH / 16; ++i) {
                    const float w = mp[i] == -INFINITY ? 0.f : __expf(mp[i] - M);
                    sw[jq][c0 + 16 * i] = w;
                    if (cbase == 0) denom += w * lp[i];
                }
                __syncthreads();
            }
            for (int q0 = 0; q0 < np; q0 += SP) {
                float vn[SP][CB];
                const bool more = q0 + SP < np;
                if (more) load_rows(p0 + q0 + SP, vn);
#pragma unroll
                for (int i = 0; i < SP; ++i) {
                    const float w = MODE == CKV_SOFTMAX ? sw[jq][min(q0 + i, PCH - 1)] : 1.f;
#pragma unroll
                    for (int k = 0; k < CB; ++k) acc[k] += w * v[i][k];  // pieces past the last were loaded as zeros
                }
                if (more) {
#pragma unroll
                    for (int i = 0; i < SP; ++i)
#pragma unroll
                        for (int k = 0; k < CB; ++k) v[i][k] = vn[i][k];
                }
            }
        }
        if (MODE == CKV_SOFTMAX && cbase == 0) {
#pragma unroll
            for (int d = 1; d < 16; d <<= 1) denom += __shfl_xor(denom, d);
        }
        const float inv = denom > 0.f ? 1.f / denom : 0.f;
#pragma unroll
        for (int k = 0; k < CB; ++k) {
            const int c = cbase + c0 + 16 * k;
            if (!valid || c >= d_a) continue;
            const float r = acc[k] * inv;
            if (sizeof(U) == 4) {
                ((float*)out)[o + c] = r;
            } else {
                uint32_t u = __float_as_uint(r);
                if ((u & 0x7FFFFFFFu) > 0x7F800000u) u |= 0x400000u;
                else u += 0x7FFFu + ((u >> 16) & 1u);
                ((uint16_t*)out)[o + c] = (uint16_t)(u >> 16);
            }
        }
    }
}

// Frequency renumbering of pool rows: count how often every row of a head is referred to ...
__global__ void ckv_histogram_kernel(const int32_t* __restrict__ idx, uint32_t* __restrict__ counts, int64_t T, int H, int P) {
    const int64_t total = (int64_t)H * T;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int h = (int)(i / T);
        atomicAdd(&counts[(int64_t)h * P + idx[i]], 1u);
    }
}
// ... rewrite the stored indices with the new row numbers ...
__global__ void ckv_renumber_kernel(int32_t* __restrict__ idx, const int32_t* __restrict__ new_id, int64_t T, int H, int P) {
    const int64_t total = (int64_t)H * T;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int h = (int)(i / T);
        idx[i] = new_id[(int64_t)h * P + idx[i]];
    }
}
// ... and move every pool row to its new place (16 threads per row, whole elements of `e` bytes).
__global__ void ckv_permute_rows_kernel(const unsigned char* __restrict__ src, unsigned char* __restrict__ dst,
                                        const int32_t* __restrict__ new_id, int64_t rows, int P, int64_t row_bytes) {
    const int64_t r = (int64_t)blockIdx.x * (blockDim.x / 16) + threadIdx.x / 16;
    if (r >= rows) return;
    const int64_t h = r / P;
    const unsigned char* s = src + r * row_bytes;
    unsigned char* d = dst + (h * P + new_id[r]) * row_bytes;
    for (int64_t b = (threadIdx.x & 15) * 2; b < row_bytes; b += 32) *(uint16_t*)(d + b) = *(const uint16_t*)(s + b);
}

__global__ void ckv_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16, int tail) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
    if (blockIdx.x == 0 && (int)threadIdx.x < tail)
        ((unsigned char*)(dst + n16))[threadIdx.x] = ((const unsigned char*)(src + n16))[threadIdx.x];
}

// XCC (accelerator complex die) that runs each workgroup of a small launch: the work lists assume workgroup i of a launch
// runs on XCD i mod 8.
__global__ void ckv_xcc_probe_kernel(uint32_t* __restrict__ xcc) {
    if (threadIdx.x == 0) xcc[blockIdx.x] = (uint32_t)__builtin_amdgcn_s_getreg((20 << 0) | (0 << 6) | (3 << 11)) & 15u;  // XCC_ID[3:0]
}

// ---------------------------------------------------------------------------------------
// Work list.  Units are (user, head, query block); long histories are cut into pieces when
// there are too few units to fill and balance the chip.  Pieces are ordered longest first
// (the hardware dispatcher hands out workgroups in grid order, which makes this longest-
// processing-time-first scheduling), interleaved so that workgroup i, which lands on XCD
// i mod 8, keeps to one head class: each XCD's L2 then caches one head's pool rows.
struct Unit {
    int32_t b, h, q0, n;
    int64_t t0;
};

// Vector width (elements per lane) and lanes per row of the streaming kernel: among the widths the
// alignment allows and 16 or 8 lanes per row, the pair with the fewest row-load instructions per tile
// (steps per tile x column blocks); ties go to 16 lanes and to the narrower vector.
void pick_stream_vec(const ckv_shape& s, int* vec, int* grp) {
    const int d_a = s.d_g + s.d_u;
    int best_v = 1, best_g = 16, best_cost = 16 * ((d_a + 15) / 16);
    for (int v : {4, 8}) {
        if (v == 8 && s.dtype == CKV_F32) continue;
        if (s.d_u % v || s.d_g % v || (s.d_g > 0 && s.pool_ld % v)) continue;  // (d_a = d_u + d_g is then a multiple too)
        for (int g : {16, 8}) {
            if (g == 8 && (size_t)v * esize(s.dtype) != 16) continue;  // eight lanes per row only with 16-byte lanes
            const int cost = g * ((d_a + g * v - 1) / (g * v));
            if (cost < best_cost) {
                best_cost = cost;
                best_v = v;
                best_g = g;
            }
        }
    }
    *vec = best_v;
    *grp = best_g;
}

// Number of head classes the work lists keep apart, one (or more) XCD per class: 8 or H when the heads divide over the
// eight XCDs and consecutive workgroups of a launch do land on consecutive XCDs (probed once per device when a handle
// is built; a host-only plan assumes it), else 1: no class, any workgroup takes any head.
int head_classes(const ckv_cache* c) {
    const ckv_shape& s = c->shape;
    if (c->xcd_order_unknown) return 1;
    if (s.H >= 8 && s.H % 8 == 0) return 8;
    if (s.H < 8 && 8 % s.H == 0) return s.H;
    return 1;
}

// Cut units into pieces of at most `piece` positions and order them (see above).
void make_items(const ckv_cache* c, const std::vector<Unit>& units, int64_t piece, std::vector<ckv_item>& items,
                std::vector<ckv_merge>& merges, int* n_parts_out) {
    items.clear();
    merges.clear();
    int n_parts = 0;
    for (const Unit& u : units) {
        const int np = u.n > piece ? (int)((u.n + piece - 1) / piece) : 1;
        if (np == 1) {
            items.push_back({u.b, u.h, u.q0, u.n, u.t0, -1, u.n});
            continue;
        }
        int64_t len = (u.n + np - 1) / np;
        len = (len + 63) / 64 * 64;
        const int real_np = (int)((u.n + len - 1) / len);
        merges.push_back({u.b, u.h, u.q0, n_parts, real_np, u.n});
        for (int p = 0; p < real_np; ++p) {
            const int64_t lo = (int64_t)p * len;
            const int nn = (int)std::min<int64_t>(len, u.n - lo);
            items.push_back({u.b, u.h, u.q0, nn, u.t0 + lo, n_parts++, u.n});
        }
    }
    *n_parts_out = n_parts;

    // head classes for the XCD-aware order
    const int ncls = head_classes(c);
    std::vector<std::vector<ckv_item>> cls((size_t)ncls);
    for (const ckv_item& it : items) cls[(size_t)(it.h % ncls)].push_back(it);
    for (auto& v : cls)
        std::stable_sort(v.begin(), v.end(), [](const ckv_item& x, const ckv_item& y) { return x.n > y.n; });
    std::vector<ckv_item> ordered;
    ordered.reserve(items.size());
    std::vector<size_t> cur((size_t)ncls, 0);
    size_t remaining = items.size();
    for (size_t i = 0; remaining > 0; ++i) {
        size_t k = i % (size_t)ncls;
        if (cur[k] >= cls[k].size()) {  // this class ran dry: take from the fullest one
            size_t best = 0, left = 0;
            for (size_t j = 0; j < (size_t)ncls; ++j)
                if (cls[j].size() - cur[j] > left) { left = cls[j].size() - cur[j]; best = j; }
            k = best;
        }
        ordered.push_back(cls[k][cur[k]++]);
        --remaining;
    }
    items.swap(ordered);
}

// Finish time (in positions) of the last workgroup when the items are handed out in order:
// workgroup i runs on XCD i mod 8, on whichever of that XCD's slots frees up first.
int64_t simulate_dispatch(const std::vector<ckv_item>& items, int64_t slots, int64_t overhead) {
    const int nx = 8;
    const size_t per = (size_t)std::max<int64_t>(1, slots / nx);
    std::vector<std::vector<int64_t>> heap((size_t)nx);  // min-heaps of slot finish times
    for (auto& h : heap) h.assign(per, 0);
    auto cmp = [](int64_t x, int64_t y) { return x > y; };
    int64_t makespan = 0;
    for (size_t i = 0; i < items.size(); ++i) {
        auto& h = heap[i % nx];
        std::pop_heap(h.begin(), h.end(), cmp);
        h.back() += items[i].n + overhead;
        makespan = std::max(makespan, h.back());
        std::push_heap(h.begin(), h.end(), cmp);
    }
    return makespan;
}

// Resident workgroups per CU of the handle's kernel, asked of the runtime (needs a device).
int resident_workgroups(const ckv_cache* c) {
    const ckv_shape& s = c->shape;
    const int d_a = s.d_g + s.d_u;
    if (c->family == CKV_K_MFMA) return std::max(1, ckv_mfma_occupancy(d_a <= 64 ? 64 : (d_a <= 128 ? 128 : 256), c->nw, c->tp, s.mode));
    if (c->family == CKV_K_DMA && c->q16) return std::max(1, ckv_dma_q16_occupancy(s.mode));
    if (c->family == CKV_K_DMA) return std::max(1, ckv_dma_occupancy(d_a, c->nw, c->qg, s.mode, s.d_g == 0 ? 0 : s.d_u));
    if (c->family == CKV_K_MFMA32) return std::max(1, ckv_mfma32_occupancy(d_a <= 64 ? 64 : (d_a <= 128 ? 128 : 256), s.mode, c->QB == 64));
    // (wide-row streaming kernel: workgroups of four wavefronts, two or three wavefronts per SIMD by its registers)
    if (c->sw_g) return ckv_streamw_waves_per_simd(s, c->sw_g, c->sw_nq);
    return 8;
}

void build_work(ckv_cache* c, const int32_t* lengths, const std::vector<int64_t>& offs, int cus, int wg_per_cu,
                std::vector<ckv_item>& items, std::vector<ckv_merge>& merges) {
    const ckv_shape& s = c->shape;
    const int d_a = s.d_g + s.d_u;
    const int nqb = (s.Nq + c->QB - 1) / c->QB;
    const int64_t slots = (int64_t)cus * wg_per_cu;
    std::vector<Unit> units;
    units.reserve((size_t)s.B * s.H * nqb);
    int64_t longest = 0;
    for (int b = 0; b < s.B; ++b)
        for (int h = 0; h < s.H; ++h)
            for (int qb = 0; qb < nqb; ++qb) {
                units.push_back({b, h, qb * c->QB, lengths[b], offs[b]});
                longest = std::max<int64_t>(longest, lengths[b]);
            }
    // Candidate piece lengths: no split, then halvings of the longest history down to 128.
    // Cost of a candidate, in positions per slot: simulated finish time plus the traffic of the
    // split workspace (written and read once) expressed in positions of gather traffic.
    const int64_t overhead = c->family == CKV_K_STREAM ? 16 : 128;  // per-item fill/drain, in positions
    const double e = (double)esize(s.dtype);
    const double part_positions = (double)c->QB * (d_a + 2) * 8.0 / (2.0 * d_a * e + 8.0);
    std::vector<ckv_item> best_items;
    std::vector<ckv_merge> best_merges;
    double best_cost = -1.0;
    int best_parts = 0;
    int64_t best_piece = 0;
    // The merge kernel is a chain of memory round trips, about one per four pieces of a history: in positions
    // of work of one workgroup, a microsecond is ~150 (streaming kernel) or ~25 (matrix-core kernel).
    const int64_t min_piece = 128;
    const double round_trip = c->family == CKV_K_STREAM ? 150.0 : 25.0;
    for (int64_t piece = INT64_MAX; piece >= min_piece; piece = (piece == INT64_MAX ? (longest + 1) / 2 : piece / 2)) {
        if (piece != INT64_MAX) piece = (piece + 63) / 64 * 64;
        std::vector<ckv_item> it2;
        std::vector<ckv_merge> mg2;
        int parts = 0;
        make_items(c, units, piece, it2, mg2, &parts);
        double cost = (double)simulate_dispatch(it2, slots, overhead) + parts * part_positions / (double)slots;
        if (parts > 0) {  // the merge is a second launch
            int most = 0;
            for (const ckv_merge& m : mg2) most = std::max(most, (int)m.nparts);
            cost = cost * 1.02 + round_trip * (2 + (most + 3) / 4);
        }
        if (best_cost < 0 || cost < best_cost) {
            best_cost = cost;
            best_items.swap(it2);
            best_merges.swap(mg2);
            best_parts = parts;
            best_piece = piece;
        }
        if (piece != INT64_MAX && piece <= min_piece) break;
        if (units.size() > (size_t)(64 * slots)) break;  // plenty of units: splitting cannot pay
    }
    items.swap(best_items);
    merges.swap(best_merges);
    c->n_parts = best_parts;
    if (g_opt.debug)
        fprintf(stderr, "ckv: %s: %zu units, %lld slots, piece %lld -> %zu items, %d parts, cost %.0f positions/slot\n", c->variant,
                units.size(), (long long)slots, (long long)(best_piece == INT64_MAX ? -1 : best_piece), items.size(), best_parts,
                best_cost);
}

// Static work lists for the persistent direct-to-LDS kernel: exactly `slots` workgroups are
// launched (all resident at once), workgroup i runs on XCD i mod 8 and serves one head class,
// and every workgroup gets its own list of pieces.  Pieces are assigned longest first to the
// least loaded workgroup of their class; then load is moved from the fullest to the emptiest
// workgroup by cutting the tail off a piece (the two halves become a split history that the
// merge kernel joins), until every workgroup is within a few percent of the mean.  With two
// long histories per workgroup (the long ragged workload) the greedy assignment alone leaves
// the last workgroups running ~10 % longer than the median.
struct Piece {
    int unit;        // index into units
    int64_t lo;      // first position of the piece inside the unit
    int64_t n;       // positions
};

double assign_static(const ckv_cache* c, const std::vector<Unit>& units, int64_t piece_len, int64_t slots, int cus, double slow_speed,
                     int64_t overhead, double part_positions, std::vector<std::vector<Piece>>& lists, int* n_parts_out) {
    const int ncls = head_classes(c);
    lists.assign((size_t)slots, {});
    std::vector<int64_t> load((size_t)slots, 0);
    // Relative speed of a workgroup.  When a SIMD holds more than one wavefront of this kernel the hardware
    // favours the wavefront slot that was filled first: the workgroups of the first dispatch wave (indices
    // below slots / workgroups-per-CU) were measured to advance 1.2 to 1.3 times faster than those that
    // share their SIMDs (traced on both matrix-core workloads), finish early and leave the CU half empty.
    // Giving them proportionally more positions makes all workgroups of a CU finish together.
    const int wg_per_cu = std::max<int>(1, (int)(slots / std::max(1, cus)));
    std::vector<double> speed((size_t)slots, 1.0);
    // (the first 4 / nw workgroups of a CU each find an empty SIMD per wavefront)
    if (wg_per_cu * c->nw > 4)
        for (int64_t i = (slots / wg_per_cu) * std::max(1, 4 / c->nw); i < slots; ++i) speed[(size_t)i] = slow_speed;
    auto time_of = [&](int w) { return (double)load[(size_t)w] / speed[(size_t)w]; };
    std::vector<int> pieces_of_unit(units.size(), 0);
    double worst = 0;
    for (int cls = 0; cls < ncls; ++cls) {
        std::vector<int> wgs;
        for (int i = 0; i < (int)slots; ++i)
            if ((i % 8) % ncls == cls) wgs.push_back(i);
        if (wgs.empty()) continue;
        std::vector<Piece> ps;
        for (int u = 0; u < (int)units.size(); ++u) {
            if (units[u].h % ncls != cls) continue;
            const int64_t n = units[u].n;
            const int np = n > piece_len ? (int)((n + piece_len - 1) / piece_len) : 1;
            int64_t len = np > 1 ? ((n + np - 1) / np + 63) / 64 * 64 : n;
            if (np == 1) {
                ps.push_back({u, 0, n});
                pieces_of_unit[(size_t)u] = 1;
            } else {
                int k = 0;
                for (int64_t lo = 0; lo < n; lo += len, ++k) ps.push_back({u, lo, std::min<int64_t>(len, n - lo)});
                pieces_of_unit[(size_t)u] = k;
            }
        }
        std::stable_sort(ps.begin(), ps.end(), [](const Piece& x, const Piece& y) { return x.n > y.n; });
        // longest first onto the workgroup that would finish it earliest
        for (const Piece& p : ps) {
            int best = wgs[0];
            double best_t = 1e300;
            for (int w : wgs) {
                const double t = (double)(load[(size_t)w] + p.n + overhead) / speed[(size_t)w];
                if (t < best_t) {
                    best_t = t;
                    best = w;
                }
            }
            lists[(size_t)best].push_back(p);
            load[(size_t)best] += p.n + overhead;
        }
        // move load from the workgroup that finishes last to the one that finishes first
        double total = 0, total_speed = 0;
        for (int w : wgs) {
            total += (double)load[(size_t)w];
            total_speed += speed[(size_t)w];
        }
        const double target = total / total_speed;  // common finish time, in positions of a speed-1 workgroup
        const double tol = std::max(target / 50.0, 256.0);
        for (size_t iter = 0; iter < 4 * wgs.size(); ++iter) {
            int d = wgs[0], r = wgs[0];
            for (int w : wgs) {
                if (time_of(w) > time_of(d)) d = w;
                if (time_of(w) < time_of(r)) r = w;
            }
            const double excess = (time_of(d) - target) * speed[(size_t)d];
            const double deficit = (target - time_of(r)) * speed[(size_t)r] - (double)overhead;
            if (time_of(d) - target < tol || deficit < 256) break;
            int64_t move = (int64_t)std::min(excess, deficit) / 32 * 32;
            if (move < 256) break;
            // cut the tail off the longest piece of the donor
            std::vector<Piece>& dl = lists[(size_t)d];
            size_t best = 0;
            for (size_t k = 1; k < dl.size(); ++k)
                if (dl[k].n > dl[best].n) best = k;
            if (dl.empty() || dl[best].n - move < 256) break;
            const int64_t keep = (dl[best].n - move + 31) / 32 * 32;  // keep the cut on a tile boundary
            move = dl[best].n - keep;
            if (move < 256) break;
            lists[(size_t)r].push_back({dl[best].unit, dl[best].lo + keep, move});
            dl[best].n = keep;
            pieces_of_unit[(size_t)dl[best].unit]++;
            load[(size_t)d] -= move;
            load[(size_t)r] += move + overhead;
        }
        for (int w : wgs) worst = std::max(worst, time_of(w));
    }
    int parts = 0;
    for (int k : pieces_of_unit)
        if (k > 1) parts += k;
    *n_parts_out = parts;
    double cost = worst + parts * part_positions / (double)slots;
    if (parts > 0) cost *= 1.01;
    return cost;
}

void build_work_static(ckv_cache* c, const int32_t* lengths, const std::vector<int64_t>& offs, int cus, int wg_per_cu,
                       std::vector<ckv_item>& items, std::vector<ckv_merge>& merges, std::vector<int32_t>& wg_begin) {
    const ckv_shape& s = c->shape;
    const int d_a = s.d_g + s.d_u;
    const int nqb = (s.Nq + c->QB - 1) / c->QB;
    const int64_t slots = (int64_t)cus * wg_per_cu;
    std::vector<Unit> units;
    int64_t longest = 0;
    for (int b = 0; b < s.B; ++b)
        for (int h = 0; h < s.H; ++h)
            for (int qb = 0; qb < nqb; ++qb) {
                units.push_back({b, h, qb * c->QB, lengths[b], offs[b]});
                longest = std::max<int64_t>(longest, lengths[b]);
            }
    const int64_t overhead = 192;  // per-item fill, drain and epilogue, in positions
    const double part_positions = (double)c->QB * (d_a + 2) * 8.0 / (2.0 * d_a * 2.0 + 8.0);
    // speed of a workgroup that shares its SIMDs with an older one (see assign_static); measured best: 0.75 with four
    // wavefronts per workgroup (config 4: 0.465 ms against 0.482 ms at 1.0), no difference with two (config 3), 1.0 with one
    // (config 5: 0.834 ms against 0.867 ms at 0.75)
    double slow_speed = c->nw == 1 ? 1.0 : 0.75;
    if (g_opt.slow_speed >= 0.0) slow_speed = g_opt.slow_speed;  // tuning option
    std::vector<std::vector<Piece>> best;
    double best_cost = -1;
    int64_t best_piece = 0;
    // shortest piece tried: with few users a history is cut until the pieces fill the workgroups (one user of
    // config 4: 64 items of ~590 positions take 37 us, 200 of ~190 take 32; config 3: 24 -> 14 us)
    const int64_t min_piece = 128;
    for (int64_t piece = INT64_MAX; piece >= min_piece; piece = (piece == INT64_MAX ? (longest + 1) / 2 : piece / 2)) {
        if (piece != INT64_MAX) piece = (piece + 63) / 64 * 64;
        std::vector<std::vector<Piece>> lists;
        int parts = 0;
        const double cost = assign_static(c, units, piece, slots, cus, slow_speed, overhead, part_positions, lists, &parts);
        if (best_cost < 0 || cost < best_cost) {
            best_cost = cost;
            best.swap(lists);
            best_piece = piece;
        }
        if (piece != INT64_MAX && piece <= min_piece) break;
        if (units.size() > (size_t)(8 * slots)) break;  // plenty of units per workgroup: uniform cuts cannot pay
    }
    // part slots: the pieces of a split unit get consecutive workspace slots, in position order
    std::vector<std::vector<std::pair<int64_t, std::pair<int, int>>>> by_unit(units.size());  // lo -> (wg, index in list)
    for (int w = 0; w < (int)best.size(); ++w)
        for (int k = 0; k < (int)best[(size_t)w].size(); ++k)
            by_unit[(size_t)best[(size_t)w][(size_t)k].unit].push_back({best[(size_t)w][(size_t)k].lo, {w, k}});
    std::vector<std::vector<int>> part_of(best.size());
    for (size_t w = 0; w < best.size(); ++w) part_of[w].assign(best[w].size(), -1);
    int next_part = 0;
    for (size_t u = 0; u < units.size(); ++u) {
        auto& v = by_unit[u];
        if (v.size() <= 1) continue;
        std::sort(v.begin(), v.end());
        merges.push_back({units[u].b, units[u].h, units[u].q0, next_part, (int)v.size(), units[u].n});
        for (auto& e : v) part_of[(size_t)e.second.first][(size_t)e.second.second] = next_part++;
    }
    c->n_parts = next_part;
    wg_begin.assign(best.size() + 1, 0);
    for (size_t w = 0; w < best.size(); ++w) {
        wg_begin[w] = (int32_t)items.size();
        for (size_t k = 0; k < best[w].size(); ++k) {
            const Piece& p = best[w][k];
            const Unit& u = units[(size_t)p.unit];
            items.push_back({u.b, u.h, u.q0, (int32_t)p.n, u.t0 + p.lo, part_of[w][k], u.n});
        }
    }
    wg_begin[best.size()] = (int32_t)items.size();
    if (g_opt.debug)
        fprintf(stderr, "ckv: %s: %zu units on %lld persistent workgroups, piece %lld -> %zu items, %d parts, cost %.0f positions\n",
                c->variant, units.size(), (long long)slots, (long long)(best_piece == INT64_MAX ? -1 : best_piece), items.size(),
                next_part, best_cost);
}

void choose_variant(ckv_cache* c) {
    const ckv_shape& s = c->shape;
    const int d_a = s.d_g + s.d_u;
    c->family = CKV_K_STREAM;
    // Fewest queries for which a matrix-core kernel beats the streaming kernel (whose time grows with the
    // number of queries while theirs does not, up to 32 per wavefront): measured crossovers on configs 2, 3
    // and 4 are 2-3 queries for the direct-to-LDS kernel, ~5 for the fp32 kernel, ~8 for the register-staged one.
    constexpr int kMinNqDma = 3, kMinNqF32 = 6, kMinNqStaged = 8;
    // the matrix-core kernels take the running maximum before scaling, which needs scale > 0
    if (s.dtype == CKV_BF16 && d_a <= 256 && s.Nq >= kMinNqDma && (s.d_g == 0 || s.pool_ld % 8 == 0) &&
        (s.mode == CKV_SILU_OVER_N || s.scale > 0.f)) {
        const int dak = d_a <= 64 ? 64 : (d_a <= 128 ? 128 : 256);  // row width the register-staged kernel is built for
        const bool staged = g_opt.staged;  // tuning option: forces the register-staged kernel
        {
            // direct-to-LDS kernel: 32 queries per wavefront, up to 4 wavefronts per workgroup (two
            // wavefronts per SIMD overlap better than one wavefront with two query groups)
            // (256 columns: always four wavefronts, those without queries only gather)
            int nw = dak == 256 ? 4 : (s.Nq <= 32 ? 1 : (s.Nq <= 64 ? 2 : 4)), qg = 1;
            // (64 columns, 33 to 64 queries: one wavefront with two query groups and the two-stage ring, eight workgroups
            // per CU, measured faster than two wavefronts with four stages: config 3 77.8 -> 75.4 us, a config-5-like batch
            // with 64 queries 349 -> 309 us; at 128 columns it is the other way round, 380 against 575 us, and so it is
            // for an ordinary cache, d_g = 0, whose rows all stream from HBM: 113 against 128 us)
            if (dak == 64 && s.Nq > 32 && s.Nq <= 64 && s.d_g > 0 && !(s.d_u & 1) && s.d_u <= 8) nw = 1, qg = 2;
            if (g_opt.nw > 0 && g_opt.qg > 0) nw = g_opt.nw, qg = g_opt.qg;  // tuning option "dma_shape"
            // (d_g = 0, ordinary attention over the user arrays: rows are fetched by position, nothing is appended)
            const int nui = d_a == dak && ckv_dma_supported(d_a, nw, qg) && (s.d_g == 0 || qg == 1 || (!(s.d_u & 1) && (s.d_u <= 8 || dak == 256)))
                                ? (s.d_g == 0 ? 0 : ckv_dma_nui(d_a, nw, s.d_u)) : -1;
            if (nui >= 0 && !staged) {
                c->family = CKV_K_DMA;
                c->nw = nw;
                c->qg = qg;
                c->tp = 32;
                c->nui = nui;
                // (the loop with the scores one tile ahead exists for four wavefronts of one query group at 128 columns; measured
                // on the long ragged configuration: 449 -> 444 us where both sides gather from pools, 518 -> 531 us on an
                // ordinary cache, whose rows all stream from HBM and want the deeper prefetch of the other loop; at 256 columns,
                // one wavefront per SIMD, it is the faster loop throughout: 432 -> 391 us, one side shared 490 -> 445 us, an
                // ordinary cache 517 -> 491 us)
                c->scores_ahead = g_opt.scores_ahead < 0 ? (dak == 256 || (s.share == CKV_SHARE_KV && s.d_g > 0)) : g_opt.scores_ahead;
                c->QB = 32 * nw * qg;
                // (sixteen queries or fewer at 64 columns: the organisation on the 16x16x32 instruction, which they fill)
                c->q16 = g_opt.q16 != 0 && nw == 1 && qg == 1 && s.Nq <= 16 && ckv_dma_q16_supported(d_a, s.d_u, s.d_g);
                if (c->q16) {
                    c->QB = 16;
                    snprintf(c->variant, sizeof c->variant, "mfma_dma_bf16_d%d_w1_q16_%s", d_a, s.mode == CKV_SOFTMAX ? "softmax" : "silu");
                    return;
                }
                snprintf(c->variant, sizeof c->variant, "mfma_dma_bf16_d%d_w%d_g%d_%s", d_a, nw, qg,
                         s.mode == CKV_SOFTMAX ? "softmax" : "silu");
                return;
            }
        }
        const int nw = dak == 256 ? 4 : (s.Nq <= 32 ? 1 : (s.Nq <= 64 ? 2 : 4));
        const int tp = (dak == 256 || (dak == 128 && nw == 1)) ? 32 : 64;
        if (s.Nq >= kMinNqStaged && ckv_mfma_supported(dak, nw, tp)) {
            c->family = CKV_K_MFMA;
            c->nw = nw;
            c->tp = tp;
            c->QB = 32 * nw;
            snprintf(c->variant, sizeof c->variant, "mfma_bf16_d%d_w%d_t%d_%s", dak, nw, tp,
                     s.mode == CKV_SOFTMAX ? "softmax" : "silu");
            return;
        }
    }
    // fp32 storage, many queries: the same organisation on the fp32 matrix instruction
    if (s.dtype == CKV_F32 && d_a <= 256 && s.Nq >= kMinNqF32 && (s.d_g == 0 || s.pool_ld % 4 == 0) &&
        (s.mode == CKV_SILU_OVER_N || s.scale > 0.f)) {
        const int dak = d_a <= 64 ? 64 : (d_a <= 128 ? 128 : 256);
        c->family = CKV_K_MFMA32;
        c->nw = 4;
        const bool split = ckv_mfma32_split(dak, s.Nq);
        c->tp = ckv_mfma32_tile(dak, split);
        c->QB = ckv_mfma32_queries(split);
        snprintf(c->variant, sizeof c->variant, "mfma_f32_d%d_w4_t%d%s_%s", dak, c->tp, split ? "_c2" : "", s.mode == CKV_SOFTMAX ? "softmax" : "silu");
        return;
    }
    pick_stream_vec(s, &c->vec, &c->grp);
    int ncb = (d_a + c->grp * c->vec - 1) / (c->grp * c->vec);
    c->ncb = ncb <= 1 ? 1 : (ncb <= 2 ? 2 : (ncb <= 4 ? 4 : (ncb <= 8 ? 8 : 16)));
    c->QB = s.Nq;
    c->nw = 4;  // wavefronts per item; plan_work drops to 2 when the items outnumber the resident workgroups
    // Rows that the kernel above would fetch in several column blocks, or in lanes of less than 16 bytes because the
    // user slice breaks the alignment (d_u = 1, 2, 3, 6, 10 of Table 1's 256 columns), go to the wide-row kernel, which
    // fetches pool row and slice separately.
    // (A row that the kernel above holds in one block of vector lanes stays there, also with 8-byte lanes: 64 bf16 columns with
    // d_u = 4 or 12 measured 22 us there against 24 and 47 us; so do fp32 rows of several blocks with one query: 238 against 265 us.)
    const bool one_block = c->ncb == 1 && c->vec > 1;
    const bool f32_blocks = s.dtype == CKV_F32 && c->vec == 4 && s.Nq == 1;
    c->sw_g = one_block || f32_blocks || g_opt.stream_narrow ? 0 : ckv_streamw_lanes(s);
    if (c->sw_g) {
        c->sw_nq = s.Nq >= 2 ? 2 : 1;
        // (hot rows in LDS, the second half of the frequency renumbering: only where the option asks for them; with them the
        // kernel measured twice as slow on Zipf indices as with the same rows left to the L2s)
        c->hot_rows = g_opt.hot_rows > 0 ? std::min(g_opt.hot_rows, ckv_streamw_hot_rows(s, c->sw_g, c->sw_nq)) : 0;
        snprintf(c->variant, sizeof c->variant, "streamw_%s_g%d_q%d_%s", s.dtype == CKV_F32 ? "f32" : "bf16", c->sw_g, c->sw_nq,
                 s.mode == CKV_SOFTMAX ? "softmax" : "silu");
        return;
    }
    snprintf(c->variant, sizeof c->variant, "stream_%s_v%d_c%d%s_%s", s.dtype == CKV_F32 ? "f32" : "bf16", c->vec,
             c->ncb, c->grp == 8 ? "_g8" : "", s.mode == CKV_SOFTMAX ? "softmax" : "silu");
}

// The packed cache lives in device memory, or (offloaded handle) in pinned host memory that the
// GPU reads in place.
// *host receives the host address of an offloaded buffer (what hipHostFree takes back), nullptr otherwise.
hipError_t cache_alloc(const ckv_cache* c, void** p, void** host, size_t bytes) {
    *host = nullptr;
    if (!c->offloaded) return hipMalloc(p, bytes);
    void* h = nullptr;
    hipError_t e = hipHostMalloc(&h, bytes, hipHostMallocMapped | hipHostMallocPortable);
    if (e != hipSuccess) return e;
    e = hipHostGetDevicePointer(p, h, 0);
    if (e != hipSuccess) {
        (void)hipHostFree(h);
        *p = nullptr;
        return e;
    }
    *host = h;
    return e;
}
void cache_free(const ckv_cache* c, void* p, void* host) {
    if (c->offloaded) {
        if (host) (void)hipHostFree(host);
    } else if (p) {
        (void)hipFree(p);
    }
}

void destroy(ckv_cache* c) {
    if (!c) return;
    cache_free(c, c->d_idx, c->h_idx);
    cache_free(c, c->d_user_k, c->h_user_k);
    cache_free(c, c->d_user_v, c->h_user_v);
    (void)hipFree(c->d_lengths);
    (void)hipFree(c->d_items);
    (void)hipFree(c->d_wg_begin);
    (void)hipFree(c->d_merge);
    (void)hipFree(c->d_partial);
    (void)hipFree(c->d_trace);
    (void)hipFree(c->d_pf_ws);
    for (int i = 0; i < 3 * c->timing; ++i) (void)hipEventDestroy(c->ev[i]);
    delete[] c->ev;
    delete c;
}

}  // namespace

// Scratch of ckv_attend_static_scratch.  In host code the array's name is only a stand-in: its device address is
// asked of the runtime once per device (each GPU holds its own copy at its own address) and kept.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};
bool g_scratch_known[kMaxDevices] = {};

// Device address of `scratch` on device `dev`, which must be the current device.
hipError_t static_scratch_address(int dev, float** out) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_known[dev]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = (float*)ptr;
        g_scratch_known[dev] = true;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

extern "C" {

const char* ckv_last_error(void) { return g_err; }

// Validate the shape and the lengths, choose the kernel, allocate the handle and the buffers of
// the packed cache (device memory, or pinned host memory for an offloaded handle) and upload the
// lengths.  offs receives the B+1 prefix sums of the lengths.
static int cache_new(const char* who, const ckv_shape* shape, const int32_t* lengths, bool offloaded, hipStream_t st,
                     ckv_cache** out, std::vector<int64_t>& offs, hipDeviceProp_t* prop) {
    const ckv_shape s = *shape;
    const int64_t d_a = (int64_t)s.d_g + s.d_u;
    if (s.B < 1 || s.H < 1 || s.d_g < 0 || s.d_u < 0 || d_a < 1 || s.Nq < 1)
        return fail(CKV_ERR_SHAPE, "%s: need B,H,Nq >= 1, d_g,d_u >= 0, d_g+d_u >= 1 (B=%d H=%d d_g=%d d_u=%d Nq=%d)", who,
                    s.B, s.H, s.d_g, s.d_u, s.Nq);
    if (s.share != CKV_SHARE_KV && s.share != CKV_SHARE_K && s.share != CKV_SHARE_V)
        return fail(CKV_ERR_SHAPE, "%s: unknown sharing mode %d", who, s.share);
    if (s.d_g > 0 && (s.P < 1 || s.pool_ld < s.d_g))
        return fail(CKV_ERR_SHAPE, "%s: need P >= 1 and pool_ld >= d_g (P=%d pool_ld=%lld d_g=%d)", who, s.P,
                    (long long)s.pool_ld, s.d_g);
    if ((s.dtype != CKV_F32 && s.dtype != CKV_BF16) || (s.mode != CKV_SOFTMAX && s.mode != CKV_SILU_OVER_N))
        return fail(CKV_ERR_SHAPE, "%s: unknown dtype %d or mode %d", who, s.dtype, s.mode);
    if (!(s.scale == s.scale) || s.scale - s.scale != 0.f) return fail(CKV_ERR_SHAPE, "%s: scale must be finite", who);
    offs.assign((size_t)s.B + 1, 0);
    for (int b = 0; b < s.B; ++b) {
        if (lengths[b] < 0) return fail(CKV_ERR_LENGTH, "%s: lengths[%d] = %d is negative", who, b, lengths[b]);
        offs[(size_t)b + 1] = offs[(size_t)b] + lengths[b];
    }
    const int64_t T = offs[(size_t)s.B];
    if (T * s.H > ((int64_t)1 << 40)) return fail(CKV_ERR_LENGTH, "%s: T*H = %lld is too large", who, (long long)(T * s.H));

    ckv_cache* c = new (std::nothrow) ckv_cache();
    if (!c) return fail(CKV_ERR_HIP, "%s: out of host memory", who);
    memset(c, 0, sizeof *c);
    c->shape = s;
    c->T = T;
    c->offloaded = offloaded ? 1 : 0;
    choose_variant(c);
    // column blocks the streaming kernel is built for: 8 (16 when it moves single elements)
    if (c->family == CKV_K_STREAM && !c->sw_g && (d_a + c->grp * c->vec - 1) / (c->grp * c->vec) > (c->vec == 1 ? 16 : 8)) {
        const int limit = c->grp * c->vec * (c->vec == 1 ? 16 : 8);
        delete c;
        return fail(CKV_ERR_UNSUPPORTED, "%s: d_a = %lld exceeds the streaming kernel's limit of %d columns at this alignment", who,
                    (long long)d_a, limit);
    }
    int rc = CKV_OK;
    const size_t n_ph = (size_t)T * s.H;
    CKV_HIP(hipGetDevice(&c->device));
    CKV_HIP(hipGetDeviceProperties(prop, c->device));
    if (strncmp(prop->gcnArchName, "gfx950", 6) != 0) {
        rc = fail(CKV_ERR_UNSUPPORTED, "%s: device is %s, this library is built for gfx950 only", who, prop->gcnArchName);
        goto done;
    }
    CKV_HIP(hipMalloc((void**)&c->d_lengths, sizeof(int32_t) * (size_t)s.B));
    CKV_HIP(hipMemcpyAsync(c->d_lengths, lengths, sizeof(int32_t) * (size_t)s.B, hipMemcpyHostToDevice, st));
    {
        int d_uk, d_gk, d_uv, d_gv;
        ckv_side_dims(s, 0, &d_uk, &d_gk);
        ckv_side_dims(s, 1, &d_uv, &d_gv);
        if (n_ph > 0 && s.d_g > 0) CKV_HIP(cache_alloc(c, (void**)&c->d_idx, &c->h_idx, sizeof(int32_t) * 2 * n_ph));
        // (rounded up to whole 16-byte chunks: an odd number of bf16 elements is read in aligned dwords)
        if (n_ph > 0 && d_uk > 0) CKV_HIP(cache_alloc(c, &c->d_user_k, &c->h_user_k, (n_ph * (size_t)d_uk * esize(s.dtype) + 15) / 16 * 16));
        if (n_ph > 0 && d_uv > 0) CKV_HIP(cache_alloc(c, &c->d_user_v, &c->h_user_v, (n_ph * (size_t)d_uv * esize(s.dtype) + 15) / 16 * 16));
    }
done:
    if (rc != CKV_OK) {
        destroy(c);
        return rc;
    }
    *out = c;
    return CKV_OK;
}

// The work lists of a handle: items (in workgroup order for the persistent kernel), merge entries of split
// histories, and for the persistent kernel the first item of every workgroup.  Host arithmetic only.
struct ckv_plan_lists {
    std::vector<ckv_item> items;
    std::vector<ckv_merge> merges;
    std::vector<int32_t> wg_begin;  // persistent kernel only
};

static void plan_work(ckv_cache* c, const int32_t* lengths, const std::vector<int64_t>& offs, int cus, int wg_per_cu,
                      ckv_plan_lists& p) {
    if (c->family == CKV_K_DMA) {
        // Two ways to hand out work.  Static (default): one resident workgroup per slot with its
        // own item list, no relaunch gaps.  Dynamic: one workgroup per item in longest-first order,
        // scheduled by the hardware dispatcher as slots free up.  Static measured faster on every
        // workload (uniform lengths: by 20 %; two long ragged histories per slot: by 2 %).
        const bool use_static = g_opt.sched != 2;  // tuning option "dma_sched"
        if (use_static) {
            build_work_static(c, lengths, offs, cus, wg_per_cu, p.items, p.merges, p.wg_begin);
        } else {
            build_work(c, lengths, offs, cus, wg_per_cu, p.items, p.merges);
            p.wg_begin.resize(p.items.size() + 1);
            for (size_t i = 0; i <= p.items.size(); ++i) p.wg_begin[i] = (int32_t)i;
        }
        c->n_wg = (int)p.wg_begin.size() - 1;
    } else {
        build_work(c, lengths, offs, cus, wg_per_cu, p.items, p.merges);
    }
    c->n_items = (int)p.items.size();
    c->n_merge = (int)p.merges.size();
    if (c->family == CKV_K_STREAM && (c->ncb == 1 || c->sw_g)) {
        // The column-block kernel holds a tile in registers, which leaves room for four wavefronts per SIMD at 8 bytes
        // per lane and row and two at 16; the wide-row kernel has two or three.  Four wavefronts per item give the
        // shortest chain for one item; when that needs more than one round of workgroups, two per item are faster
        // (the column-block kernel: where two per item fit in a single round; the wide-row kernel: where an item is at most
        // one tile per wavefront, 256 positions: 1024 users of 200 positions at 256 bf16 columns 44 -> 33 us, pieces of 500
        // positions 127 -> 132 us).
        const int per_simd = c->sw_g ? ckv_streamw_waves_per_simd(c->shape, c->sw_g, c->sw_nq)
                                     : ((size_t)c->grp * esize(c->shape.dtype) * (size_t)c->vec <= 128 ? 4 : 2);
        const int64_t resident = (int64_t)cus * 4 * per_simd;
        int64_t positions = 0;
        for (const ckv_item& it : p.items) positions += it.n;
        const bool fits = c->sw_g ? positions <= (int64_t)256 * c->n_items : (int64_t)c->n_items * 2 <= resident;
        if (g_opt.stream_waves ? g_opt.stream_waves == 2 : ((int64_t)c->n_items * 4 > resident && fits)) {
            c->nw = 2;
            const size_t len = strlen(c->variant);
            if (len + 4 < sizeof c->variant) memcpy(c->variant + len, "_w2", 4);
        }
    }
}

// Whether consecutive workgroups of a launch land on consecutive XCDs of this device (round robin over eight), asked of
// the hardware once per device with a launch of 64 one-wavefront workgroups.  A failure to ask counts as "no".
static bool xcd_round_robin(int device, hipStream_t st) {
    static std::mutex m;
    static int known[64] = {};  // 0 unknown, 1 yes, 2 no
    std::lock_guard<std::mutex> lock(m);
    if (device < 0 || device >= 64) return false;
    if (known[device]) return known[device] == 1;
    constexpr int kBlocks = 64;
    uint32_t* d = nullptr;
    uint32_t h[kBlocks];
    bool ok = hipMalloc((void**)&d, sizeof h) == hipSuccess;
    if (ok) {
        hipLaunchKernelGGL(ckv_xcc_probe_kernel, dim3(kBlocks), dim3(64), 0, st, d);
        ok = hipGetLastError() == hipSuccess && hipMemcpyAsync(h, d, sizeof h, hipMemcpyDeviceToHost, st) == hipSuccess &&
             hipStreamSynchronize(st) == hipSuccess;
    }
    (void)hipFree(d);
    if (ok)
        for (int i = 0; i < kBlocks; ++i) ok = ok && h[i] == (h[0] + (uint32_t)i) % 8u;
    known[device] = ok ? 1 : 2;
    return ok;
}

// Build and upload the work lists (and the split workspace) of a handle whose packed cache is in place.
static int cache_finish(ckv_cache* c, const int32_t* lengths, const std::vector<int64_t>& offs, const hipDeviceProp_t& prop,
                        hipStream_t st) {
    int rc = CKV_OK;
    const int64_t d_a = (int64_t)c->shape.d_g + c->shape.d_u;
    ckv_plan_lists plan;
    c->xcd_order_unknown = xcd_round_robin(c->device, st) ? 0 : 1;
    if (g_opt.debug && c->xcd_order_unknown) fprintf(stderr, "ckv: workgroups do not land on XCD i mod 8 here: heads are not kept apart\n");
    plan_work(c, lengths, offs, prop.multiProcessorCount, resident_workgroups(c), plan);
    std::vector<ckv_item>& items = plan.items;
    std::vector<ckv_merge>& merges = plan.merges;
    if (c->family == CKV_K_DMA) {
        CKV_HIP(hipMalloc((void**)&c->d_wg_begin, sizeof(int32_t) * plan.wg_begin.size()));
        CKV_HIP(hipMemcpy(c->d_wg_begin, plan.wg_begin.data(), sizeof(int32_t) * plan.wg_begin.size(), hipMemcpyHostToDevice));
    }
    if (c->n_items > 0) {
        CKV_HIP(hipMalloc((void**)&c->d_items, sizeof(ckv_item) * items.size()));
        CKV_HIP(hipMemcpyAsync(c->d_items, items.data(), sizeof(ckv_item) * items.size(), hipMemcpyHostToDevice, st));
    }
    if (c->n_merge > 0) {
        CKV_HIP(hipMalloc((void**)&c->d_merge, sizeof(ckv_merge) * merges.size()));
        CKV_HIP(hipMemcpyAsync(c->d_merge, merges.data(), sizeof(ckv_merge) * merges.size(), hipMemcpyHostToDevice, st));
        CKV_HIP(hipMalloc((void**)&c->d_partial, sizeof(float) * (size_t)c->n_parts * c->QB * (size_t)(d_a + 2)));
    }
    CKV_HIP(hipStreamSynchronize(st));  // the host vectors above go out of scope
done:
    return rc;
}

static int build_cache_impl(const ckv_shape* shape, const int32_t* lengths, const int32_t* idx_k, const int32_t* idx_v,
                            const void* user_k, const void* user_v, ckv_cache** out, void* stream, bool offloaded) {
    if (out) *out = nullptr;
    if (!shape || !lengths || !out) return fail(CKV_ERR_NULL, "ckv_build_cache: shape, lengths and out must not be NULL");
    hipStream_t st = (hipStream_t)stream;
    ckv_cache* c = nullptr;
    std::vector<int64_t> offs;
    hipDeviceProp_t prop;
    {
        int64_t T = 0;
        for (int b = 0; b < shape->B; ++b) T += lengths[b] > 0 ? lengths[b] : 0;
        int d_uk = 0, d_gk = 0, d_uv = 0, d_gv = 0;
        if (shape->share >= CKV_SHARE_KV && shape->share <= CKV_SHARE_V) {
            ckv_side_dims(*shape, 0, &d_uk, &d_gk);
            ckv_side_dims(*shape, 1, &d_uv, &d_gv);
        }
        if (T > 0 && ((d_gk > 0 && !idx_k) || (d_gv > 0 && !idx_v)))
            return fail(CKV_ERR_NULL, "ckv_build_cache: an index array is NULL but its side gathers from a pool");
        if (T > 0 && ((d_uk > 0 && !user_k) || (d_uv > 0 && !user_v)))
            return fail(CKV_ERR_NULL, "ckv_build_cache: a user array is NULL but its side has user columns");
    }
    int rc = cache_new("ckv_build_cache", shape, lengths, offloaded, st, &c, offs, &prop);
    if (rc != CKV_OK) return rc;
    const ckv_shape& s = c->shape;
    const int64_t T = c->T;
    const size_t e = esize(s.dtype);
    const size_t n_ph = (size_t)T * s.H;
    int32_t *s_ik = nullptr, *s_iv = nullptr;
    void *s_uk = nullptr, *s_uv = nullptr;
    unsigned long long* d_bad = nullptr;
    unsigned long long h_bad = ~0ull;

    int d_uk, d_gk, d_uv, d_gv;
    ckv_side_dims(s, 0, &d_uk, &d_gk);
    ckv_side_dims(s, 1, &d_uv, &d_gv);
    if (n_ph > 0) {
        if (d_gk > 0) {
            CKV_HIP(hipMalloc((void**)&s_ik, sizeof(int32_t) * n_ph));
            CKV_HIP(hipMemcpyAsync(s_ik, idx_k, sizeof(int32_t) * n_ph, hipMemcpyHostToDevice, st));
        }
        if (d_gv > 0) {
            CKV_HIP(hipMalloc((void**)&s_iv, sizeof(int32_t) * n_ph));
            CKV_HIP(hipMemcpyAsync(s_iv, idx_v, sizeof(int32_t) * n_ph, hipMemcpyHostToDevice, st));
        }
        if (d_uk > 0) {
            CKV_HIP(hipMalloc(&s_uk, n_ph * (size_t)d_uk * e));
            CKV_HIP(hipMemcpyAsync(s_uk, user_k, n_ph * (size_t)d_uk * e, hipMemcpyHostToDevice, st));
        }
        if (d_uv > 0) {
            CKV_HIP(hipMalloc(&s_uv, n_ph * (size_t)d_uv * e));
            CKV_HIP(hipMemcpyAsync(s_uv, user_v, n_ph * (size_t)d_uv * e, hipMemcpyHostToDevice, st));
        }
        CKV_HIP(hipMalloc((void**)&d_bad, sizeof h_bad));
        CKV_HIP(hipMemcpyAsync(d_bad, &h_bad, sizeof h_bad, hipMemcpyHostToDevice, st));
        {
            const int threads = 256;
            const int blocks = (int)std::min<size_t>((n_ph + threads - 1) / threads, 65536);
            if (e == 4)
                hipLaunchKernelGGL(ckv_pack_kernel<uint32_t>, dim3(blocks), dim3(threads), 0, st, s_ik, s_iv,
                                   (const uint32_t*)s_uk, (const uint32_t*)s_uv, c->d_idx, (uint32_t*)c->d_user_k,
                                   (uint32_t*)c->d_user_v, T, s.H, d_uk, d_uv, s.P, d_gk > 0 ? 1 : 0, d_gv > 0 ? 1 : 0, d_bad);
            else
                hipLaunchKernelGGL(ckv_pack_kernel<uint16_t>, dim3(blocks), dim3(threads), 0, st, s_ik, s_iv,
                                   (const uint16_t*)s_uk, (const uint16_t*)s_uv, c->d_idx, (uint16_t*)c->d_user_k,
                                   (uint16_t*)c->d_user_v, T, s.H, d_uk, d_uv, s.P, d_gk > 0 ? 1 : 0, d_gv > 0 ? 1 : 0, d_bad);
            CKV_HIP(hipGetLastError());
        }
        CKV_HIP(hipMemcpyAsync(&h_bad, d_bad, sizeof h_bad, hipMemcpyDeviceToHost, st));
    }
    CKV_HIP(hipStreamSynchronize(st));
    if (h_bad != ~0ull) {
        const long long t = (long long)(h_bad / (unsigned long long)s.H);
        const int h = (int)(h_bad % (unsigned long long)s.H);
        rc = fail(CKV_ERR_INDEX, "ckv_build_cache: pool index out of range [0,%d) at position %lld head %d (idx_k=%d idx_v=%d)", s.P,
                  t, h, d_gk > 0 ? idx_k[h_bad] : 0, d_gv > 0 ? idx_v[h_bad] : 0);
        goto done;
    }
    rc = cache_finish(c, lengths, offs, prop, st);

done:
    (void)hipFree(s_ik);
    (void)hipFree(s_iv);
    (void)hipFree(s_uk);
    (void)hipFree(s_uv);
    (void)hipFree(d_bad);
    if (rc != CKV_OK) {
        destroy(c);
        return rc;
    }
    *out = c;
    return CKV_OK;
}

// Check a router against a shape and fill the kernel arguments that do not depend on the handle.
static int router_args(const char* who, const ckv_shape& s, const ckv_router* r, const void* S, int64_t T, ckv_prefill_args* a) {
    if (!r) return fail(CKV_ERR_NULL, "%s: router is NULL", who);
    if (r->d_e < 1) return fail(CKV_ERR_SHAPE, "%s: d_e = %d must be >= 1", who, r->d_e);
    if (T > 0 && !S) return fail(CKV_ERR_NULL, "%s: S is NULL", who);
    int d_uk, d_gk, d_uv, d_gv;
    ckv_side_dims(s, 0, &d_uk, &d_gk);
    ckv_side_dims(s, 1, &d_uv, &d_gv);
    if (T > 0 && ((d_gk > 0 && (!r->w_rk || !r->b_rk)) || (d_gv > 0 && (!r->w_rv || !r->b_rv))))
        return fail(CKV_ERR_NULL, "%s: router weights or biases are NULL for a side that gathers from a pool", who);
    if (T > 0 && ((d_uk > 0 && (!r->w_k || !r->b_k)) || (d_uv > 0 && (!r->w_v || !r->b_v))))
        return fail(CKV_ERR_NULL, "%s: projection weights or biases are NULL for a side that has user columns", who);
    const uintptr_t align = (uintptr_t)S | (uintptr_t)r->w_rk | (uintptr_t)r->w_rv | (uintptr_t)r->w_k | (uintptr_t)r->w_v |
                            (uintptr_t)r->b_rk | (uintptr_t)r->b_rv | (uintptr_t)r->b_k | (uintptr_t)r->b_v;
    if (align & 15) return fail(CKV_ERR_UNSUPPORTED, "%s: every device pointer must be 16-byte aligned", who);
    a->S = S;
    a->w_r[0] = r->w_rk;
    a->w_r[1] = r->w_rv;
    a->b_r[0] = r->b_rk;
    a->b_r[1] = r->b_rv;
    a->w_u[0] = r->w_k;
    a->w_u[1] = r->w_v;
    a->b_u[0] = r->b_k;
    a->b_u[1] = r->b_v;
    a->T = T;
    a->H = s.H;
    a->P[0] = d_gk > 0 ? s.P : 0;
    a->P[1] = d_gv > 0 ? s.P : 0;
    a->d_u[0] = d_uk;
    a->d_u[1] = d_uv;
    a->d_e = r->d_e;
    a->ws = nullptr;
    a->ws_entries = 0;
    a->split_first = 0;
    a->split_s = 1;
    return CKV_OK;
}

int ckv_build_cache(const ckv_shape* shape, const int32_t* lengths, const int32_t* idx_k, const int32_t* idx_v,
                    const void* user_k, const void* user_v, ckv_cache** out, void* stream) {
    return build_cache_impl(shape, lengths, idx_k, idx_v, user_k, user_v, out, stream, false);
}

int ckv_build_cache_offloaded(const ckv_shape* shape, const int32_t* lengths, const int32_t* idx_k, const int32_t* idx_v,
                              const void* user_k, const void* user_v, ckv_cache** out, void* stream) {
    return build_cache_impl(shape, lengths, idx_k, idx_v, user_k, user_v, out, stream, true);
}

int ckv_prefill_into(ckv_cache* c, const ckv_router* router, const void* S, void* stream) {
    if (!c) return fail(CKV_ERR_NULL, "ckv_prefill_into: cache is NULL");
    ckv_prefill_args a;
    int rc = router_args("ckv_prefill_into", c->shape, router, S, c->T, &a);
    if (rc != CKV_OK) return rc;
    a.idx = c->d_idx;
    a.user[0] = c->d_user_k;
    a.user[1] = c->d_user_v;
    a.ws = c->d_pf_ws;
    a.ws_entries = c->pf_ws_entries;
    hipError_t e = ckv_launch_prefill(a, c->shape.dtype, (hipStream_t)stream);
    if (e != hipSuccess) return fail(CKV_ERR_HIP, "ckv_prefill_into: kernel launch (%s): %s",
                                     ckv_prefill_variant(c->shape.dtype, router->d_e), hipGetErrorString(e));
    return CKV_OK;
}

int ckv_prefill(const ckv_shape* shape, const ckv_router* router, const int32_t* lengths, const void* S, ckv_cache** out,
                void* stream) {
    if (out) *out = nullptr;
    if (!shape || !lengths || !out || !router) return fail(CKV_ERR_NULL, "ckv_prefill: shape, router, lengths and out must not be NULL");
    hipStream_t st = (hipStream_t)stream;
    ckv_cache* c = nullptr;
    std::vector<int64_t> offs;
    hipDeviceProp_t prop;
    int rc = cache_new("ckv_prefill", shape, lengths, false, st, &c, offs, &prop);
    if (rc != CKV_OK) return rc;
    {
        // workspace that lets the matrix-core kernel fill the chip when its last round of workgroups is short
        ckv_prefill_args a;
        rc = router_args("ckv_prefill", c->shape, router, S, c->T, &a);
        const int64_t entries = rc == CKV_OK ? ckv_prefill_workspace_entries(a, c->shape.dtype) : 0;
        if (entries > 0) {
            hipError_t e = hipMalloc((void**)&c->d_pf_ws, sizeof(unsigned long long) * (size_t)entries);
            if (e == hipSuccess) e = hipMemsetAsync(c->d_pf_ws, 0, sizeof(unsigned long long) * (size_t)entries, st);
            if (e != hipSuccess) {
                destroy(c);
                return fail(CKV_ERR_HIP, "ckv_prefill: workspace of %lld entries: %s", (long long)entries, hipGetErrorString(e));
            }
            c->pf_ws_entries = entries;
        }
    }
    if (rc == CKV_OK) rc = ckv_prefill_into(c, router, S, stream);
    if (rc == CKV_OK) rc = cache_finish(c, lengths, offs, prop, st);
    if (rc != CKV_OK) {
        destroy(c);
        return rc;
    }
    *out = c;
    return CKV_OK;
}

int64_t ckv_cache_prefill_workspace(const ckv_cache* c) { return c ? c->pf_ws_entries : 0; }

const char* ckv_prefill_kernel_name(const ckv_shape* shape, const ckv_router* router) {
    if (!shape || !router) return "";
    return ckv_prefill_variant(shape->dtype, router->d_e);
}

int64_t ckv_plan(const ckv_shape* shape, const int32_t* lengths, int cus, int wg_per_cu, int64_t* records, int64_t max_records,
                 int32_t* n_workgroups, char* variant, size_t variant_size) {
    if (!shape || !lengths) return fail(CKV_ERR_NULL, "ckv_plan: shape and lengths must not be NULL");
    if (cus < 1 || wg_per_cu < 1) return fail(CKV_ERR_SHAPE, "ckv_plan: cus and wg_per_cu must be >= 1");
    const ckv_shape s = *shape;
    if (s.B < 1 || s.H < 1 || s.d_g < 0 || s.d_u < 0 || s.d_g + s.d_u < 1 || s.Nq < 1 || s.share < CKV_SHARE_KV || s.share > CKV_SHARE_V)
        return fail(CKV_ERR_SHAPE, "ckv_plan: bad shape");
    std::vector<int64_t> offs((size_t)s.B + 1, 0);
    for (int b = 0; b < s.B; ++b) {
        if (lengths[b] < 0) return fail(CKV_ERR_LENGTH, "ckv_plan: lengths[%d] = %d is negative", b, lengths[b]);
        offs[(size_t)b + 1] = offs[(size_t)b] + lengths[b];
    }
    ckv_cache c;
    memset(&c, 0, sizeof c);
    c.shape = s;
    c.T = offs[(size_t)s.B];
    choose_variant(&c);
    ckv_plan_lists plan;
    plan_work(&c, lengths, offs, cus, wg_per_cu, plan);
    if (n_workgroups) *n_workgroups = c.family == CKV_K_DMA ? c.n_wg : c.n_items;
    if (variant && variant_size > 0) snprintf(variant, variant_size, "%s", c.variant);
    const int64_t n = (int64_t)plan.items.size();
    if (records) {
        size_t wg = 0;
        for (int64_t i = 0; i < n && i < max_records; ++i) {
            const ckv_item& it = plan.items[(size_t)i];
            if (c.family == CKV_K_DMA)
                while (wg + 1 < plan.wg_begin.size() && plan.wg_begin[wg + 1] <= i) ++wg;
            int64_t* r = records + 8 * i;
            r[0] = it.b;
            r[1] = it.h;
            r[2] = it.q0;
            r[3] = it.n;
            r[4] = it.t0;
            r[5] = it.part;
            r[6] = it.n_total;
            r[7] = c.family == CKV_K_DMA ? (int64_t)wg : i;
        }
    }
    return n;
}

int ckv_cache_is_offloaded(const ckv_cache* c) { return c ? c->offloaded : 0; }

const int32_t* ckv_cache_idx(const ckv_cache* c) { return c ? c->d_idx : nullptr; }
const void* ckv_cache_user_k(const ckv_cache* c) { return c ? c->d_user_k : nullptr; }
const void* ckv_cache_user_v(const ckv_cache* c) { return c ? c->d_user_v : nullptr; }
const int32_t* ckv_cache_lengths(const ckv_cache* c) { return c ? c->d_lengths : nullptr; }
int64_t ckv_cache_positions(const ckv_cache* c) { return c ? c->T : -1; }
int64_t ckv_cache_stored_bytes(const ckv_cache* c) {
    if (!c) return -1;
    const int64_t ph = c->T * c->shape.H;
    int64_t per = 0;
    for (int side = 0; side < 2; ++side) {
        int d_u, d_g;
        ckv_side_dims(c->shape, side, &d_u, &d_g);
        per += (d_g > 0 ? (int64_t)sizeof(int32_t) : 0) + (int64_t)d_u * (int64_t)esize(c->shape.dtype);
    }
    return ph * per;
}
const char* ckv_variant(const ckv_cache* c) { return c ? c->variant : ""; }

// The body of both attention entry points: `partial` is the split workspace the kernels use (the handle's own, or the
// static scratch), `who` the name for error messages.
static int attend_common(const char* who, const ckv_cache* c, const void* pool_k, const void* pool_v, const int32_t* idx,
                         const void* user_k, const void* user_v, const void* q, const int32_t* lengths, void* out,
                         float* partial, hipStream_t st) {
    if (!c || !q || !out || !lengths) return fail(CKV_ERR_NULL, "%s: cache, q, lengths and out must not be NULL", who);
    // The work lists (pieces, offsets, merge entries) were built from the lengths given when the handle was made and
    // are not rebuilt here: other lengths would be ignored silently, so only the handle's own array is taken.
    if (lengths != c->d_lengths)
        return fail(CKV_ERR_UNSUPPORTED, "%s: lengths must be ckv_cache_lengths(cache): the work lists follow the lengths the handle was built with", who);
    const ckv_shape& s = c->shape;
    int d_uk, d_gk, d_uv, d_gv;
    ckv_side_dims(s, 0, &d_uk, &d_gk);
    ckv_side_dims(s, 1, &d_uv, &d_gv);
    if (c->T > 0 && ((d_gk > 0 && (!pool_k || !idx)) || (d_gv > 0 && (!pool_v || !idx))))
        return fail(CKV_ERR_NULL, "%s: pool_k, pool_v or idx is NULL for a side that gathers from a pool", who);
    if (c->T > 0 && ((d_uk > 0 && !user_k) || (d_uv > 0 && !user_v))) return fail(CKV_ERR_NULL, "%s: user_k or user_v is NULL", who);
    const uintptr_t align = (uintptr_t)pool_k | (uintptr_t)pool_v | (uintptr_t)idx | (uintptr_t)user_k | (uintptr_t)user_v |
                            (uintptr_t)q | (uintptr_t)out;
    if (align & 15) return fail(CKV_ERR_UNSUPPORTED, "%s: every device pointer must be 16-byte aligned", who);
    ckv_args a;
    a.pool_k = pool_k;
    a.pool_v = pool_v;
    a.idx_k = idx;
    a.idx_v = idx ? idx + (int64_t)s.H * c->T : nullptr;
    a.user_k = user_k;
    a.user_v = user_v;
    a.q = q;
    a.out = out;
    a.items = c->d_items;
    a.wg_begin = c->d_wg_begin;
    a.partial = partial;
    a.trace = c->d_trace;
    a.T = c->T;
    a.pool_ld = s.pool_ld;
    a.H = s.H;
    a.P = s.P;
    a.d_g = s.d_g;
    a.d_u = s.d_u;
    a.d_a = s.d_g + s.d_u;
    a.d_uk = d_uk;
    a.d_gk = d_gk;
    a.d_uv = d_uv;
    a.d_gv = d_gv;
    a.Nq = s.Nq;
    a.QB = c->QB;
    a.scale = s.scale;
    a.scores_ahead = c->scores_ahead;
    a.hot_rows = c->family == CKV_K_STREAM && c->sw_g ? c->hot_rows : 0;
    ckv_cache* mc = const_cast<ckv_cache*>(c);
    hipError_t e;
    // timing: three events per launch (start, main kernel done, merge done)
    const int slot = c->timing ? (int)(c->ev_count % c->timing) : 0;
    if (c->timing) {
        e = hipEventRecord(c->ev[3 * slot], st);
        if (e != hipSuccess) return fail(CKV_ERR_HIP, "%s: hipEventRecord: %s", who, hipGetErrorString(e));
    }
    e = c->family == CKV_K_DMA      ? ckv_launch_dma(c, a, st)
        : c->family == CKV_K_MFMA   ? ckv_launch_mfma(c, a, st)
        : c->family == CKV_K_MFMA32 ? ckv_launch_mfma32(c, a, st)
        : c->sw_g                   ? ckv_launch_streamw(c, a, st)
                                    : ckv_launch_stream(c, a, st);
    if (e != hipSuccess) return fail(CKV_ERR_HIP, "%s: kernel launch (%s): %s", who, c->variant, hipGetErrorString(e));
    if (c->timing) {
        e = hipEventRecord(c->ev[3 * slot + 1], st);
        if (e != hipSuccess) return fail(CKV_ERR_HIP, "%s: hipEventRecord: %s", who, hipGetErrorString(e));
    }
    if (c->n_merge > 0) {
        const int d_a = a.d_a;
        const dim3 mgrid(c->n_merge, (c->QB + 15) / 16), threads(256);
        if (s.dtype == CKV_F32) {
            if (s.mode == CKV_SOFTMAX)
                hipLaunchKernelGGL((ckv_merge_kernel<float, CKV_SOFTMAX>), mgrid, threads, 0, st, c->d_merge,
                                   partial, (float*)out, s.H, s.Nq, d_a, c->QB);
            else
                hipLaunchKernelGGL((ckv_merge_kernel<float, CKV_SILU_OVER_N>), mgrid, threads, 0, st, c->d_merge,
                                   partial, (float*)out, s.H, s.Nq, d_a, c->QB);
        } else {
            if (s.mode == CKV_SOFTMAX)
                hipLaunchKernelGGL((ckv_merge_kernel<uint16_t, CKV_SOFTMAX>), mgrid, threads, 0, st, c->d_merge,
                                   partial, (uint16_t*)out, s.H, s.Nq, d_a, c->QB);
            else
                hipLaunchKernelGGL((ckv_merge_kernel<uint16_t, CKV_SILU_OVER_N>), mgrid, threads, 0, st,
                                   c->d_merge, partial, (uint16_t*)out, s.H, s.Nq, d_a, c->QB);
        }
        e = hipGetLastError();
        if (e != hipSuccess) return fail(CKV_ERR_HIP, "%s: merge launch: %s", who, hipGetErrorString(e));
    }
    if (c->timing) {
        e = hipEventRecord(c->ev[3 * slot + 2], st);
        if (e != hipSuccess) return fail(CKV_ERR_HIP, "%s: hipEventRecord: %s", who, hipGetErrorString(e));
        mc->ev_count++;
    }
    return CKV_OK;
}

int ckv_attend(const ckv_cache* c, const void* pool_k, const void* pool_v, const int32_t* idx, const void* user_k,
               const void* user_v, const void* q, const int32_t* lengths, void* out, void* stream) {
    return attend_common("ckv_attend", c, pool_k, pool_v, idx, user_k, user_v, q, lengths, out, c ? c->d_partial : nullptr,
                         (hipStream_t)stream);
}

// Bytes of split workspace the handle's kernels use per call (0: no history is split).
static size_t split_workspace_bytes(const ckv_cache* c) {
    if (!c || c->n_merge == 0) return 0;
    return sizeof(float) * (size_t)c->n_parts * (size_t)c->QB * (size_t)(c->shape.d_g + c->shape.d_u + 2);
}

int ckv_attend_static_scratch(const ckv_cache* c, const void* pool_k, const void* pool_v, const int32_t* idx,
                              const void* user_k, const void* user_v, const void* q, const int32_t* lengths, void* out,
                              void* stream) {
    static const char* who = "ckv_attend_static_scratch";
    if (!c) return fail(CKV_ERR_NULL, "%s: cache is NULL", who);
    const size_t need = split_workspace_bytes(c);
    if (need > kStaticScratchBytes)
        return fail(CKV_ERR_UNSUPPORTED, "%s: the handle's split workspace is %zu bytes, the static scratch holds %zu; use ckv_attend",
                    who, need, kStaticScratchBytes);
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(CKV_ERR_HIP, "%s: hipGetDevice: %s", who, hipGetErrorString(e));
    if (dev != c->device) return fail(CKV_ERR_UNSUPPORTED, "%s: the handle was built on device %d, the current device is %d", who, c->device, dev);
    if (dev < 0 || dev >= kMaxDevices) return fail(CKV_ERR_UNSUPPORTED, "%s: device %d is beyond the %d devices this entry point keeps scratch for", who, dev, kMaxDevices);
    float* scratch_ptr = nullptr;
    e = static_scratch_address(dev, &scratch_ptr);
    if (e != hipSuccess) return fail(CKV_ERR_HIP, "%s: hipGetSymbolAddress(scratch): %s", who, hipGetErrorString(e));
    // (nothing in the workspace has to start at zero: every slot a merge entry reads is written by its piece in the same call)
    return attend_common(who, c, pool_k, pool_v, idx, user_k, user_v, q, lengths, out, scratch_ptr, (hipStream_t)stream);
}

int ckv_set_option(const char* key, const char* value) {
    if (!key) {
        g_opt = Options();
        return CKV_OK;
    }
    const bool unset = !value || !*value;
    if (strcmp(key, "mfma_impl") == 0) {
        if (!unset && strcmp(value, "staged") != 0 && strcmp(value, "auto") != 0)
            return fail(CKV_ERR_UNSUPPORTED, "ckv_set_option: mfma_impl takes \"staged\" or \"auto\", not \"%s\"", value);
        g_opt.staged = !unset && strcmp(value, "staged") == 0;
    } else if (strcmp(key, "dma_sched") == 0) {
        if (!unset && strcmp(value, "static") != 0 && strcmp(value, "dynamic") != 0)
            return fail(CKV_ERR_UNSUPPORTED, "ckv_set_option: dma_sched takes \"static\" or \"dynamic\", not \"%s\"", value);
        g_opt.sched = unset ? 0 : (strcmp(value, "static") == 0 ? 1 : 2);
    } else if (strcmp(key, "dma_shape") == 0) {
        int nw = 0, qg = 0;
        if (!unset && (sscanf(value, "%d,%d", &nw, &qg) != 2 || nw < 1 || qg < 1))
            return fail(CKV_ERR_UNSUPPORTED, "ckv_set_option: dma_shape takes \"nw,qg\" with both >= 1, not \"%s\"", value);
        g_opt.nw = nw;
        g_opt.qg = qg;
    } else if (strcmp(key, "dma_slow_speed") == 0) {
        char* end = nullptr;
        const double v = unset ? -1.0 : strtod(value, &end);
        if (!unset && (end == value || !(v > 0.0) || v > 4.0))
            return fail(CKV_ERR_UNSUPPORTED, "ckv_set_option: dma_slow_speed takes a number in (0, 4], not \"%s\"", value);
        g_opt.slow_speed = v;
    } else if (strcmp(key, "dma_q16") == 0) {
        if (!unset && strcmp(value, "0") != 0 && strcmp(value, "1") != 0)
            return fail(CKV_ERR_UNSUPPORTED, "ckv_set_option: dma_q16 takes \"0\" or \"1\", not \"%s\"", value);
        g_opt.q16 = unset ? -1 : atoi(value);
    } else if (strcmp(key, "dma_scores_ahead") == 0) {
        if (!unset && strcmp(value, "0") != 0 && strcmp(value, "1") != 0)
            return fail(CKV_ERR_UNSUPPORTED, "ckv_set_option: dma_scores_ahead takes \"0\" or \"1\", not \"%s\"", value);
        g_opt.scores_ahead = unset ? -1 : atoi(value);
    } else if (strcmp(key, "stream_hot_rows") == 0) {
        char* end = nullptr;
        const long v = unset ? 0 : strtol(value, &end, 10);
        if (!unset && (end == value || *end || v < 0 || v > 32))
            return fail(CKV_ERR_UNSUPPORTED, "ckv_set_option: stream_hot_rows takes a number from 0 to 32, not \"%s\"", value);
        g_opt.hot_rows = (int)v;
    } else if (strcmp(key, "stream_waves") == 0) {
        if (!unset && strcmp(value, "2") != 0 && strcmp(value, "4") != 0)
            return fail(CKV_ERR_UNSUPPORTED, "ckv_set_option: stream_waves takes \"2\" or \"4\", not \"%s\"", value);
        g_opt.stream_waves = unset ? 0 : atoi(value);
    } else if (strcmp(key, "stream_impl") == 0) {
        if (!unset && strcmp(value, "narrow") != 0 && strcmp(value, "auto") != 0)
            return fail(CKV_ERR_UNSUPPORTED, "ckv_set_option: stream_impl takes \"narrow\" or \"auto\", not \"%s\"", value);
        g_opt.stream_narrow = !unset && strcmp(value, "narrow") == 0;
    } else if (strcmp(key, "debug") == 0) {
        g_opt.debug = !unset && strcmp(value, "0") != 0;
    } else {
        return fail(CKV_ERR_UNSUPPORTED, "ckv_set_option: unknown option \"%s\"", key);
    }
    return CKV_OK;
}

int ckv_reconstruct(const ckv_cache* c, const void* pool_k, const void* pool_v, void* k_full, void* v_full, void* stream) {
    if (!c) return fail(CKV_ERR_NULL, "ckv_reconstruct: cache is NULL");
    const ckv_shape& s = c->shape;
    int side_du[2], side_dg[2];
    ckv_side_dims(s, 0, &side_du[0], &side_dg[0]);
    ckv_side_dims(s, 1, &side_du[1], &side_dg[1]);
    if (c->T > 0 && ((k_full && side_dg[0] > 0 && !pool_k) || (v_full && side_dg[1] > 0 && !pool_v)))
        return fail(CKV_ERR_NULL, "ckv_reconstruct: pool pointer is NULL");
    const int64_t total = (int64_t)s.H * c->T * (s.d_g + s.d_u);
    if (total == 0) return CKV_OK;
    const int threads = 256;
    const int blocks = (int)std::min<int64_t>((total + threads - 1) / threads, 1 << 20);
    hipStream_t st = (hipStream_t)stream;
    for (int side = 0; side < 2; ++side) {
        void* full = side == 0 ? k_full : v_full;
        if (!full) continue;
        const void* pool = side == 0 ? pool_k : pool_v;
        const void* user = side == 0 ? c->d_user_k : c->d_user_v;
        const int32_t* idx = c->d_idx ? c->d_idx + (int64_t)side * s.H * c->T : nullptr;
        if (s.dtype == CKV_F32)
            hipLaunchKernelGGL(ckv_reconstruct_kernel<uint32_t>, dim3(blocks), dim3(threads), 0, st, idx, (const uint32_t*)user,
                               (const uint32_t*)pool, (uint32_t*)full, c->T, s.H, side_du[side], side_dg[side], s.P, s.pool_ld);
        else
            hipLaunchKernelGGL(ckv_reconstruct_kernel<uint16_t>, dim3(blocks), dim3(threads), 0, st, idx, (const uint16_t*)user,
                               (const uint16_t*)pool, (uint16_t*)full, c->T, s.H, side_du[side], side_dg[side], s.P, s.pool_ld);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(CKV_ERR_HIP, "ckv_reconstruct: launch: %s", hipGetErrorString(e));
    }
    return CKV_OK;
}

void ckv_free(ckv_cache* c) { destroy(c); }

int ckv_set_timing(ckv_cache* c, int pairs) {
    if (!c) return fail(CKV_ERR_NULL, "ckv_set_timing: cache is NULL");
    if (pairs < 0 || pairs > 4096) return fail(CKV_ERR_SHAPE, "ckv_set_timing: pairs must be in [0, 4096]");
    for (int i = 0; i < 3 * c->timing; ++i) (void)hipEventDestroy(c->ev[i]);
    delete[] c->ev;
    c->ev = nullptr;
    c->timing = 0;
    c->ev_count = 0;
    if (pairs == 0) return CKV_OK;
    c->ev = new (std::nothrow) hipEvent_t[3 * (size_t)pairs];
    if (!c->ev) return fail(CKV_ERR_HIP, "ckv_set_timing: out of host memory");
    for (int i = 0; i < 3 * pairs; ++i) {
        hipError_t e = hipEventCreate(&c->ev[i]);
        if (e != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(c->ev[j]);
            delete[] c->ev;
            c->ev = nullptr;
            return fail(CKV_ERR_HIP, "ckv_set_timing: hipEventCreate: %s", hipGetErrorString(e));
        }
    }
    c->timing = pairs;
    return CKV_OK;
}

int ckv_kernel_times(ckv_cache* c, float* kernel_ms, float* merge_ms, int max_launches) {
    if (!c) return fail(CKV_ERR_NULL, "ckv_kernel_times: cache is NULL");
    if (!c->timing || c->ev_count == 0) return 0;
    const int n = (int)std::min<long long>(std::min<long long>(c->ev_count, c->timing), std::max(0, max_launches));
    // oldest recorded launch first: the ring holds the last `timing` launches
    const long long first = c->ev_count > c->timing ? c->ev_count - c->timing : 0;
    for (int i = 0; i < n; ++i) {
        const int slot = (int)((first + i) % c->timing);
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(c->ev[3 * slot + 2]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, c->ev[3 * slot], c->ev[3 * slot + 1]);
        if (e == hipSuccess && kernel_ms) kernel_ms[i] = ms;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, c->ev[3 * slot + 1], c->ev[3 * slot + 2]);
        if (e != hipSuccess) return fail(CKV_ERR_HIP, "ckv_kernel_times: %s", hipGetErrorString(e));
        if (merge_ms) merge_ms[i] = c->n_merge > 0 ? ms : 0.f;
    }
    return n;
}

float ckv_kernel_ms(ckv_cache* c) {
    if (!c || !c->timing || c->ev_count == 0) return -1.f;
    const int n = (int)std::min<long long>(c->ev_count, c->timing);
    double sum = 0;
    for (int i = 0; i < n; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(c->ev[3 * i + 2]) != hipSuccess) return -1.f;
        if (hipEventElapsedTime(&ms, c->ev[3 * i], c->ev[3 * i + 1]) != hipSuccess) return -1.f;
        sum += ms;
    }
    return (float)(sum / n);
}

int ckv_trace_enable(ckv_cache* c, int enable) {
    if (!c) return fail(CKV_ERR_NULL, "ckv_trace_enable: cache is NULL");
    (void)hipFree(c->d_trace);
    c->d_trace = nullptr;
    if (!enable || c->n_items == 0) return CKV_OK;
    const size_t bytes = sizeof(unsigned long long) * 8 * (size_t)c->n_items;
    hipError_t e = hipMalloc((void**)&c->d_trace, bytes);
    if (e == hipSuccess) e = hipMemset(c->d_trace, 0, bytes);
    if (e != hipSuccess) {
        c->d_trace = nullptr;
        return fail(CKV_ERR_HIP, "ckv_trace_enable: %s", hipGetErrorString(e));
    }
    return CKV_OK;
}

int64_t ckv_trace_read(ckv_cache* c, unsigned long long* host, int64_t max_items) {
    if (!c || !host) return fail(CKV_ERR_NULL, "ckv_trace_read: NULL argument");
    if (!c->d_trace) return 0;
    const int64_t n = std::min<int64_t>(max_items, c->n_items);
    if (n <= 0) return 0;
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(host, c->d_trace, sizeof(unsigned long long) * 8 * (size_t)n, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(CKV_ERR_HIP, "ckv_trace_read: %s", hipGetErrorString(e));
    return n;
}

int ckv_remap_hot_rows(ckv_cache* c, const void* pool_k, const void* pool_v, void* pool_k_out, void* pool_v_out,
                       int32_t* new_id, void* stream) {
    if (!c) return fail(CKV_ERR_NULL, "ckv_remap_hot_rows: cache is NULL");
    const ckv_shape& s = c->shape;
    if (c->offloaded) return fail(CKV_ERR_UNSUPPORTED, "ckv_remap_hot_rows: the handle's cache lives in host memory");
    int side_du[2], side_dg[2];
    ckv_side_dims(s, 0, &side_du[0], &side_dg[0]);
    ckv_side_dims(s, 1, &side_du[1], &side_dg[1]);
    const void* pin[2] = {pool_k, pool_v};
    void* pout[2] = {pool_k_out, pool_v_out};
    for (int side = 0; side < 2; ++side)
        if (side_dg[side] > 0 && (!pin[side] || !pout[side] || pin[side] == pout[side]))
            return fail(CKV_ERR_NULL, "ckv_remap_hot_rows: a shared side needs distinct input and output pools");
    if (s.d_g == 0) return CKV_OK;
    hipStream_t st = (hipStream_t)stream;
    int rc = CKV_OK;
    const size_t hp = (size_t)s.H * (size_t)s.P;
    uint32_t* d_counts = nullptr;
    int32_t* d_new = nullptr;
    std::vector<uint32_t> counts(2 * hp, 0);
    std::vector<int32_t> ids(2 * hp, 0);
    std::vector<int32_t> order((size_t)s.P);
    const int64_t n_ph = (int64_t)s.H * c->T;
    const int blocks = (int)std::max<int64_t>(1, std::min<int64_t>((n_ph + 255) / 256, 65536));
    CKV_HIP(hipMalloc((void**)&d_counts, sizeof(uint32_t) * 2 * hp));
    CKV_HIP(hipMalloc((void**)&d_new, sizeof(int32_t) * 2 * hp));
    CKV_HIP(hipMemsetAsync(d_counts, 0, sizeof(uint32_t) * 2 * hp, st));
    for (int side = 0; side < 2; ++side)
        if (side_dg[side] > 0 && n_ph > 0)
            hipLaunchKernelGGL(ckv_histogram_kernel, dim3(blocks), dim3(256), 0, st, c->d_idx + (int64_t)side * n_ph,
                               d_counts + (size_t)side * hp, c->T, s.H, s.P);
    CKV_HIP(hipGetLastError());
    CKV_HIP(hipMemcpyAsync(counts.data(), d_counts, sizeof(uint32_t) * 2 * hp, hipMemcpyDeviceToHost, st));
    CKV_HIP(hipStreamSynchronize(st));
    // most used first, equal counts by row number (a stable sort of the row numbers)
    for (int side = 0; side < 2; ++side) {
        if (side_dg[side] == 0) continue;
        for (int h = 0; h < s.H; ++h) {
            const uint32_t* cnt = counts.data() + (size_t)side * hp + (size_t)h * s.P;
            std::iota(order.begin(), order.end(), 0);
            std::stable_sort(order.begin(), order.end(), [cnt](int32_t x, int32_t y) { return cnt[x] > cnt[y]; });
            int32_t* id = ids.data() + (size_t)side * hp + (size_t)h * s.P;
            for (int32_t k = 0; k < s.P; ++k) id[order[(size_t)k]] = k;
        }
    }
    CKV_HIP(hipMemcpyAsync(d_new, ids.data(), sizeof(int32_t) * 2 * hp, hipMemcpyHostToDevice, st));
    for (int side = 0; side < 2; ++side) {
        if (side_dg[side] == 0) continue;
        const int64_t rows = (int64_t)hp;
        const int64_t row_bytes = s.pool_ld * (int64_t)esize(s.dtype);
        hipLaunchKernelGGL(ckv_permute_rows_kernel, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, (const unsigned char*)pin[side],
                           (unsigned char*)pout[side], d_new + (size_t)side * hp, rows, s.P, row_bytes);
        if (n_ph > 0)
            hipLaunchKernelGGL(ckv_renumber_kernel, dim3(blocks), dim3(256), 0, st, c->d_idx + (int64_t)side * n_ph,
                               d_new + (size_t)side * hp, c->T, s.H, s.P);
    }
    CKV_HIP(hipGetLastError());
    if (new_id) CKV_HIP(hipMemcpyAsync(new_id, d_new, sizeof(int32_t) * 2 * hp, hipMemcpyDeviceToDevice, st));
    CKV_HIP(hipStreamSynchronize(st));
done:
    (void)hipFree(d_counts);
    (void)hipFree(d_new);
    return rc;
}

int ckv_copy(void* dst, const void* src, size_t nbytes, void* stream) {
    if (!dst || !src) return fail(CKV_ERR_NULL, "ckv_copy: NULL pointer");
    if (((uintptr_t)dst | (uintptr_t)src) & 15) return fail(CKV_ERR_UNSUPPORTED, "ckv_copy: pointers must be 16-byte aligned");
    if (nbytes == 0) return CKV_OK;
    const size_t n16 = nbytes / 16;
    const int blocks = (int)std::max<size_t>(1, std::min<size_t>((n16 + 255) / 256, 256 * 32));
    hipLaunchKernelGGL(ckv_copy_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (uint4*)dst, (const uint4*)src, n16,
                       (int)(nbytes & 15));
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(CKV_ERR_HIP, "ckv_copy: launch: %s", hipGetErrorString(e));
    return CKV_OK;
}

}  // extern "C"
