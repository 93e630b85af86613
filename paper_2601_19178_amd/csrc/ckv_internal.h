// Internal declarations shared by the translation units of libckv.so (not part of the ABI).
#ifndef CKV_INTERNAL_H
#define CKV_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ckv.h"

// One piece of work for one workgroup: a contiguous run of positions of one user and head,
// attended by one block of queries.
struct ckv_item {
    int32_t b, h;      // user, head
    int32_t q0;        // first query of the block this item serves
    int32_t n;         // positions in this piece (0 for an empty history)
    int64_t t0;        // first flattened position of the piece, in [0, T]
    int32_t part;      // slot in the split workspace, or -1 if the piece is the whole history
    int32_t n_total;   // n_b, the user's full history length
};

// A (user, head, query block) whose history was split into pieces; merged by a second kernel.
struct ckv_merge {
    int32_t b, h, q0;
    int32_t part0, nparts;  // consecutive workspace slots
    int32_t n_total;
};

// Kernel arguments common to both attention kernels.
struct ckv_args {
    const void* pool_k;
    const void* pool_v;
    const int32_t* idx_k;  // plane 0 of idx, [H][T]
    const int32_t* idx_v;  // plane 1
    const void* user_k;    // [H][T][d_u]
    const void* user_v;
    const void* q;         // [B][H][Nq][d_a]
    void* out;             // [B][H][Nq][d_a]
    const ckv_item* items;
    const int32_t* wg_begin;  // persistent kernel: items [wg_begin[i], wg_begin[i+1]) belong to workgroup i
    float* partial;        // split workspace: per slot [QB][d_a] acc, [QB] m, [QB] l
    unsigned long long* trace;  // optional: 8 words per item (timestamps, hardware id), or nullptr
    int64_t T;
    int64_t pool_ld;
    int32_t H, P, d_g, d_u, d_a, Nq;
    int32_t d_uk, d_gk, d_uv, d_gv;  // per side: d_u, d_g of the shape for a shared side, (d_a, 0) otherwise
    int32_t QB;            // queries per block (rows of a workspace slot)
    float scale;
    int32_t hot_rows;      // wide-row streaming kernel: pool rows 0 .. hot_rows - 1 of the item's head are kept in LDS (0: none)
    int32_t scores_ahead;  // direct-to-LDS kernel, four wavefronts at 128 columns: tile loop with the scores one tile ahead
};

// Columns of one side (0 = K, 1 = V) that come from the user array and from the pool.
inline void ckv_side_dims(const ckv_shape& s, int side, int* d_u, int* d_g) {
    const bool shared = s.share == CKV_SHARE_KV || (s.share == CKV_SHARE_K && side == 0) || (s.share == CKV_SHARE_V && side == 1);
    *d_u = shared ? s.d_u : s.d_u + s.d_g;
    *d_g = shared ? s.d_g : 0;
}

// Kernel arguments of the prefill kernels.  Index 0 of every pair is the key side, 1 the value side.
struct ckv_prefill_args {
    const void* S;            // [T][d_e]
    const void* w_r[2];       // [H][P[side]][d_e]
    const float* b_r[2];      // [H][P[side]]
    const void* w_u[2];       // [H][d_u[side]][d_e]
    const float* b_u[2];      // [H][d_u[side]]
    int32_t* idx;             // out [2][H][T]
    void* user[2];            // out [H][T][d_u[side]]
    int64_t T;
    int32_t P[2];             // pool entries routed to (0: that side has no router)
    int32_t d_u[2];           // projected columns
    int32_t H, d_e;
    // blocks of a partly filled last round, cut into split_s workgroups each (matrix-core kernel; set by its launcher)
    unsigned long long* ws;   // one 64-bit maximum per position of a split block, zero between calls; may be NULL
    int64_t ws_entries;
    int64_t split_first;      // first split block
    int32_t split_s;
};

enum ckv_kernel_family { CKV_K_STREAM = 0, CKV_K_MFMA = 1, CKV_K_DMA = 2, CKV_K_MFMA32 = 3 };

struct ckv_cache {
    ckv_shape shape;
    int64_t T;
    int device;
    int offloaded;       // packed cache in pinned host memory, read by the kernels in place
    // packed cache (device, owned)
    int32_t* d_idx;      // [2][H][T]
    void* d_user_k;      // [H][T][d_u]
    void* d_user_v;
    // offloaded handle: host addresses of the three buffers above (what hipHostFree takes back), else nullptr
    void* h_idx;
    void* h_user_k;
    void* h_user_v;
    int32_t* d_lengths;  // [B]
    // launch metadata
    int family;          // ckv_kernel_family
    int vec, ncb;        // stream kernel: elements per lane per column block, column blocks
    int grp;             // stream kernel: lanes that share a row (16 or 8)
    int hot_rows;        // wide-row stream kernel: pool rows kept in LDS per work item (0: none; tuning option stream_hot_rows)
    int sw_g, sw_nq;     // wide-row stream kernel: lanes per row (0: the shape runs in the other stream kernel), queries per pass
    int nw, tp;          // mfma kernels: waves per workgroup, positions per tile
    int nui;             // dma kernel: user-slice load instructions per wavefront and tile
    int qg;              // dma kernel: groups of 32 queries per wavefront
    int q16;             // dma kernel: sixteen queries per work item on the 16x16x32 matrix instruction
    int scores_ahead;    // dma kernel: tile loop with the scores one tile ahead (four wavefronts, one query group, 128 columns)
    int QB;              // queries per block
    int n_items, n_merge, n_parts;
    ckv_item* d_items;
    int32_t* d_wg_begin;  // persistent kernel only
    int n_wg;             // persistent kernel only: workgroups launched
    int xcd_order_unknown;  // 1: consecutive workgroups were not seen to land on consecutive XCDs; heads are then not kept apart
    ckv_merge* d_merge;
    float* d_partial;
    unsigned long long* d_trace;  // 8 words per item while tracing is on
    unsigned long long* d_pf_ws;  // handles made by ckv_prefill: workspace of the split last round, zero between calls
    int64_t pf_ws_entries;
    // timing: ring of event triples (start, main kernel done, merge done), filled while timing > 0
    int timing;            // number of triples in the ring (0 = off)
    long long ev_count;    // launches recorded since timing was switched on
    hipEvent_t* ev;        // 3 * timing events
    char variant[96];
};

// Launchers (each returns hipGetLastError() of its launch).
hipError_t ckv_launch_stream(const ckv_cache* c, const ckv_args& a, hipStream_t s);
// Streaming kernel for wide rows and user slices of any width; lanes per row it would use for a shape (0: not served).
hipError_t ckv_launch_streamw(const ckv_cache* c, const ckv_args& a, hipStream_t s);
int ckv_streamw_lanes(const ckv_shape& s);
int ckv_streamw_waves_per_simd(const ckv_shape& s, int G, int nq);
size_t ckv_streamw_hot_row_bytes(const ckv_shape& s);
int ckv_streamw_hot_rows(const ckv_shape& s, int G, int nq);  // most hot rows the kernel can keep in LDS (0: none)
hipError_t ckv_launch_mfma(const ckv_cache* c, const ckv_args& a, hipStream_t s);
// Resident workgroups per CU of the chosen mfma kernel (0 if the shape has no mfma kernel).
int ckv_mfma_occupancy(int d_a, int nw, int tp, int mode);
// Whether (d_a, nw, tp) has an instantiated mfma kernel.
bool ckv_mfma_supported(int d_a, int nw, int tp);
// Direct-to-LDS variant of the mfma kernel.
hipError_t ckv_launch_dma(const ckv_cache* c, const ckv_args& a, hipStream_t s);
int ckv_dma_nui(int d_a, int nw, int d_u);  // -1: shape not served
int ckv_dma_occupancy(int d_a, int nw, int qg, int mode, int d_u);
bool ckv_dma_supported(int d_a, int nw, int qg);
// sixteen queries per work item on the 16x16x32 matrix instruction (64 columns, one wavefront)
bool ckv_dma_q16_supported(int d_a, int d_u, int d_g);
int ckv_dma_q16_occupancy(int mode);

// fp32-storage variant of the register-staged mfma kernel (four wavefronts, 128 queries per block).
hipError_t ckv_launch_mfma32(const ckv_cache* c, const ckv_args& a, hipStream_t s);
// dak: row width the kernel is built for (64, 128 or 256); split: wavefront pairs split the columns instead of the queries
// (always at 256 columns, otherwise for 64 queries or fewer), which makes a work item 64 queries instead of 128
bool ckv_mfma32_split(int dak, int Nq);
int ckv_mfma32_occupancy(int dak, int mode, bool split);
int ckv_mfma32_tile(int dak, bool split);     // positions per tile
int ckv_mfma32_queries(bool split);           // queries per work item

// Prefill (projection + router argmax into the packed cache layout).
hipError_t ckv_launch_prefill(const ckv_prefill_args& a, int dtype, hipStream_t s);
// 64-bit workspace entries the matrix-core prefill kernel would use to split its partly filled last round (0: none).
int64_t ckv_prefill_workspace_entries(const ckv_prefill_args& a, int dtype);
const char* ckv_prefill_variant(int dtype, int d_e);
bool ckv_prefill_mfma_supported(int dtype, int d_e);

#endif
