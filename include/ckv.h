/*
 * ckv.h - C ABI of the CollectiveKV decode hot path on AMD MI355X (gfx950).
 *
 * CollectiveKV (paper section 4.2) stores, for every position of a user's history and
 * every head, two pool indices I_k, I_v and two low-dimensional user-specific slices
 * K_u, V_u (d_u columns).  At decode time the collective part is gathered from the global
 * pools, K_c[i] = P_k[I_k[i]], V_c[i] = P_v[I_v[i]] (eq. "eq: Kc"), concatenated behind the
 * user slice, K = concat(K_u, K_c), V = concat(V_u, V_c) with d_a = d_u + d_g (eq. "eq: K";
 * the first d_u columns are the user-specific ones, appendix "Discussion of the sharing
 * mechanism"), and the user's queries attend over the final K, V.
 *
 * This library does gather + concat + attention in one fused pass that never writes a
 * full-width K or V to memory.  Notation: B users, n_b = lengths[b] positions of user b,
 * T = sum n_b, H heads, P pool rows per head, Nq queries per user and head.
 *
 * Conventions
 *  - Every entry point returns 0 (CKV_OK) or a negative CKV_ERR_* code; the text of the
 *    last error of the calling thread is available from ckv_last_error().  No C++
 *    exception crosses this boundary.
 *  - "device" pointers are HIP device memory on the current device, allocated and owned by
 *    the caller and only borrowed for the duration of the enqueued work; "host" pointers
 *    are ordinary host memory.  `stream` is a hipStream_t passed as void* (NULL = the
 *    default stream).
 *  - dtype selects the storage type of pools, user slices, q and out: CKV_F32 (float) or
 *    CKV_BF16 (bfloat16, upper half of a binary32).  Accumulation is always fp32.
 *  - The library needs a gfx950 device; there is no CPU fallback.
 */
#ifndef CKV_H
#define CKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { CKV_F32 = 0, CKV_BF16 = 1 };
enum { CKV_SOFTMAX = 0, CKV_SILU_OVER_N = 1 };
/* Which sides gather from a pool (ablation "sharing keys or values"): both (CollectiveKV), only the
 * keys (CollectiveK) or only the values (CollectiveV).  A side that is not shared is the ordinary
 * cache: its user array holds all d_a columns of every position (d_u' = d_a, d_g' = 0), and its
 * index plane, pool and router are never read. */
enum { CKV_SHARE_KV = 0, CKV_SHARE_K = 1, CKV_SHARE_V = 2 };

enum {
    CKV_OK = 0,
    CKV_ERR_NULL = -1,        /* a required pointer is NULL                              */
    CKV_ERR_SHAPE = -2,       /* a field of ckv_shape is out of range                    */
    CKV_ERR_INDEX = -3,       /* a pool index lies outside [0, P)                        */
    CKV_ERR_LENGTH = -4,      /* a history length is negative or T*H overflows           */
    CKV_ERR_UNSUPPORTED = -5, /* valid but not implemented (alignment, size)             */
    CKV_ERR_HIP = -6          /* a HIP runtime call failed                               */
};

/*
 * Problem shape (section 4.2 notation: n -> lengths, m -> P, d_u, d_g, d_a = d_u + d_g).
 * mode:  CKV_SOFTMAX      out_j = sum_i softmax_i(scale * q_j . K_i) V_i
 *        CKV_SILU_OVER_N  out_j = sum_i SiLU(scale * q_j . K_i) V_i / n_b   (HSTU-style pointwise)
 * Attention is non-causal over the user's n_b positions.  A user with n_b = 0 gets out = 0.
 * pool_ld is the row stride of both pools in elements, pool_ld >= d_g; columns
 * [d_g, pool_ld) of a pool row are padding and are never interpreted.
 * Limits (checked by ckv_build_cache / ckv_prefill, which fail with the code named):
 *   B, H, Nq >= 1; d_g, d_u >= 0 with d_a >= 1; P >= 1 when d_g > 0 (CKV_ERR_SHAPE);
 *   lengths >= 0 and T * H <= 2^40 (CKV_ERR_LENGTH); pools may exceed 4 GiB (row offsets are 64-bit);
 *   d_a <= 256 for any widths and stride; d_a <= 512 when d_u, d_g and pool_ld are multiples of 4,
 *   <= 1024 for bf16 when they are multiples of 8; also rows of up to 1024 bytes (512 bf16 or 256 fp32 columns) with any
 *   d_u <= 64 when the row strides (pool_ld, and d_a for a side that is not shared) are whole multiples of 16 bytes
 *   (CKV_ERR_UNSUPPORTED beyond);
 *   every device pointer 16-byte aligned (CKV_ERR_UNSUPPORTED); device gfx950 (CKV_ERR_UNSUPPORTED).
 * The matrix-core kernels take Nq >= 8 (>= 3 for the fastest bf16 shapes, >= 6 in fp32; scale > 0 for
 * softmax): bf16 with d_a <= 256 and pool_ld a multiple
 * of 8 (fastest at d_a of exactly 64, 128 or 256 with d_u odd up to 7 or even up to 16, up to 32 at 256 columns), fp32 with d_a <= 256 and pool_ld a
 * multiple of 4 (on the fp32 matrix instruction, a sixteenth of the bf16 rate).  Every other shape runs one of the two streaming
 * kernels, which are made for one or two queries (target attention): column blocks, or, for wide rows and user widths that
 * break the alignment of the final row, pool rows in 16-byte lanes and user slices apart.  ckv_variant names the choice.
 */
typedef struct ckv_shape {
    int32_t B, H, d_g, d_u, P, Nq;
    int32_t dtype;   /* CKV_F32 | CKV_BF16 */
    int32_t mode;    /* CKV_SOFTMAX | CKV_SILU_OVER_N */
    float scale;
    int32_t share;   /* CKV_SHARE_KV (0) | CKV_SHARE_K | CKV_SHARE_V */
    int64_t pool_ld;
} ckv_shape;

/* Opaque handle: the packed compressed cache of B users plus launch metadata. Owned by the
 * library from ckv_build_cache until ckv_free. */
typedef struct ckv_cache ckv_cache;

/*
 * Pack the compressed cache of B users ("both the global K/V indices and the user-specific
 * K/V will be cached", section 4.2, prefill stage) into the device layout the attention
 * kernels stream, and precompute launch metadata (per-user offsets, the work list).
 *
 *   shape     host.  Copied.
 *   lengths   host int32 [B], each >= 0.
 *   idx_k,
 *   idx_v     host int32 [T][H]: pool row of flattened position t (users back to back) and
 *             head h, 0-based, each in [0, P).  Ignored (may be NULL) when d_g == 0.
 *   user_k,
 *   user_v    host [T][H][d_u] in shape->dtype.  Ignored (may be NULL) when d_u == 0.
 *             With share = CKV_SHARE_K, user_v is [T][H][d_a] and idx_v is ignored (may be NULL);
 *             with CKV_SHARE_V the same holds for user_k and idx_k.
 *   out       receives the handle.
 *   stream    uploads and the packing kernel run on this stream; the call synchronises it
 *             before returning (it has to read back the index check).
 *
 * Device layout produced (see the accessors): indices as two planes [2][H][T] (plane 0 =
 * I_k, plane 1 = I_v), user slices [H][T][d_u], so that one head's positions are one
 * contiguous, coalesced stream.  Packing and the range check of every index run on the GPU.
 * Errors: CKV_ERR_NULL, _SHAPE, _LENGTH, _INDEX (message names the first offending
 * position and head; nothing is clamped), _HIP.  On error *out is NULL and nothing leaks.
 */
int ckv_build_cache(const ckv_shape* shape, const int32_t* lengths,
                    const int32_t* idx_k, const int32_t* idx_v,
                    const void* user_k, const void* user_v,
                    ckv_cache** out, void* stream);

/*
 * Offloaded cache (latency analysis, section 4.4: the cache of a large user base does not fit
 * GPU memory and is kept in CPU memory; the load term shrinks from s*d_a to s*d_u + s).  Same
 * arguments and packing as ckv_build_cache, but the packed indices and user slices are placed
 * in pinned, GPU-mapped host memory.  The views below then return device-visible addresses of
 * that host memory, and ckv_attend streams the compressed cache over PCIe while it gathers
 * from the GPU-resident pools and attends: load, gather, concat and attention are one pass,
 * with no staging copy.  Everything else about the handle is unchanged.
 */
int ckv_build_cache_offloaded(const ckv_shape* shape, const int32_t* lengths,
                              const int32_t* idx_k, const int32_t* idx_v,
                              const void* user_k, const void* user_v,
                              ckv_cache** out, void* stream);
int ckv_cache_is_offloaded(const ckv_cache* c);

/*
 * Prefill stage (section 4.2 "In the prefill stage" and section 4.3 "CollectiveKV Router"): from the
 * history embedding S (T x d_e, users back to back, shared by the heads) compute, per head,
 *   K_u = S W_k + b_k,  V_u = S W_v + b_v                 the d_u user-specific columns, and
 *   M = S W_r + b_r,  I[i] = argmax_j M[i][j]             one router for keys, one for values,
 * and write them straight into the packed cache of a new handle; the T x P routing map is never
 * stored.  Inference form only (the sigmoid weighting and the router losses exist in training).
 *
 * ckv_router: device pointers, borrowed for the duration of the enqueued work.  Weights are in
 * shape->dtype, one row per output: row j of w_rk[h] is column j of that head's W_r, row c of
 * w_k[h] is column c of W_k.  Biases are always float.
 *   w_rk, w_rv  [H][P][d_e]    b_rk, b_rv  [H][P]       (ignored when d_g == 0)
 *   w_k,  w_v   [H][d_u][d_e]  b_k,  b_v   [H][d_u]     (ignored when d_u == 0)
 * For a side that is not shared (shape->share) the router is ignored and the projection has d_a
 * rows: w_v [H][d_a][d_e], b_v [H][d_a] with CKV_SHARE_K, likewise w_k, b_k with CKV_SHARE_V.
 * Arithmetic: products of the stored values accumulated in fp32, bias added in fp32; user slices
 * are rounded to shape->dtype (nearest even).  Of equal routing scores the lowest pool entry
 * wins.  Scores that differ by less than the fp32 rounding of their sums may resolve either way;
 * inputs must be finite.  Every index written lies in [0, P).
 *
 *   lengths   host int32 [B]; T = sum.       S   device [T][d_e] in shape->dtype.
 * ckv_prefill allocates the handle (device-resident), enqueues the kernels on `stream`, builds the
 * launch metadata and synchronises the stream before returning.  ckv_prefill_into recomputes the
 * packed cache of an existing, device-resident handle (same shape and lengths) from new S or
 * weights: no allocation, no synchronisation.
 * The matrix-core kernel runs equal workgroups of 256 positions x one (head, side) in rounds; when
 * the last round (for a short batch: the only one) would leave most compute units idle, its
 * workgroups are cut along the pool entries and meet in a 64-bit atomic maximum per position, which
 * needs a small workspace.  ckv_prefill sizes and owns it (ckv_cache_prefill_workspace returns its
 * number of 8-byte entries, 0 if none is needed); a handle made by ckv_build_cache has none, and
 * ckv_prefill_into on it simply runs the uncut rounds.  Results do not depend on the cut: ties
 * still go to the lowest pool entry.  Calls on one handle must not overlap (they share it).  ckv_prefill_kernel_name names the kernel the pair
 * (shape, router) dispatches to: a matrix-core kernel when a row of d_e elements is a whole number of
 * 16-byte chunks and d_e <= 256 (bf16 storage on the bf16 matrix instruction, fp32 storage on the fp32
 * one; built for 64, 128 and 256 columns, a narrower row runs in the next wider kernel), a scalar
 * kernel, slower by orders of magnitude, for any other d_e.
 * Errors: CKV_ERR_NULL, _SHAPE, _LENGTH, _UNSUPPORTED (pointer not 16-byte aligned), _HIP.
 */
typedef struct ckv_router {
    int32_t d_e;
    int32_t reserved; /* must be 0 */
    const void* w_rk;
    const float* b_rk;
    const void* w_rv;
    const float* b_rv;
    const void* w_k;
    const float* b_k;
    const void* w_v;
    const float* b_v;
} ckv_router;
int ckv_prefill(const ckv_shape* shape, const ckv_router* router, const int32_t* lengths, const void* S,
                ckv_cache** out, void* stream);
int ckv_prefill_into(ckv_cache* cache, const ckv_router* router, const void* S, void* stream);
int64_t ckv_cache_prefill_workspace(const ckv_cache* cache);
const char* ckv_prefill_kernel_name(const ckv_shape* shape, const ckv_router* router);

/* Borrowed device views of the packed cache; valid until ckv_free. */
const int32_t* ckv_cache_idx(const ckv_cache* c);     /* device int32 [2][H][T]        */
const void* ckv_cache_user_k(const ckv_cache* c);     /* device [H][T][d_u] ([H][T][d_a] if K is not shared) */
const void* ckv_cache_user_v(const ckv_cache* c);     /* device [H][T][d_u] ([H][T][d_a] if V is not shared) */
const int32_t* ckv_cache_lengths(const ckv_cache* c); /* device int32 [B]              */
int64_t ckv_cache_positions(const ckv_cache* c);      /* T                             */
/* Bytes of the stored cache (indices + user slices; the quantity whose ratio to the full
 * K/V size 2*T*H*d_a*e is the compression rate of section 5.1). */
int64_t ckv_cache_stored_bytes(const ckv_cache* c);

/*
 * Fused gather + concat + attend (section 4.2, decode stage), enqueued on `stream`.
 *
 *   cache     handle from ckv_build_cache: shape, offsets, work list, split workspace.
 *   pool_k,
 *   pool_v    device [H][P][pool_ld]: the global K/V pools P_k, P_v.
 *   idx       device int32 [2][H][T]            } normally the handle's own views; other buffers of
 *   user_k,                                     } the same layout (same lengths, indices in [0, P))
 *   user_v    device [H][T][d_u]                } are accepted.
 *   lengths   must be ckv_cache_lengths(cache).  The argument is there for the call's signature; it is not read:
 *             pieces, offsets and merge entries were computed from the lengths given when the handle was built,
 *             and a history that has grown needs a new handle.  Any other pointer is refused
 *             (CKV_ERR_UNSUPPORTED) rather than silently ignored.
 *   q         device [B][H][Nq][d_a]: queries, columns in final-K order (user columns first).
 *   out       device [B][H][Nq][d_a]: written completely (zeros for users with n_b = 0).
 *
 * With bf16 and an odd d_u the user arrays are read in aligned 4-byte words: they must be readable up to
 * a multiple of 4 bytes (the handle's own views are).
 * No allocation, no synchronisation, no validation pass over the data: indices were checked
 * when the cache was built; passing other index buffers with out-of-range entries is
 * undefined.  Calls on the same handle share its split workspace, so two calls on one handle
 * must not overlap in time (serialise them on one stream).  The call enqueues kernel launches
 * only (no memset, no copy, no event unless ckv_set_timing switched timing on), so it may be
 * recorded into a HIP graph by stream capture and replayed; a replay reads the buffers whose
 * addresses were captured.
 * Errors: CKV_ERR_NULL, CKV_ERR_UNSUPPORTED (a pointer not 16-byte aligned, foreign lengths), CKV_ERR_HIP (launch failure).
 */
int ckv_attend(const ckv_cache* cache, const void* pool_k, const void* pool_v,
               const int32_t* idx, const void* user_k, const void* user_v,
               const void* q, const int32_t* lengths, void* out, void* stream);

/*
 * ckv_attend for callers that must not touch the allocator at all (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, same kernels, same results bit for bit, but the split
 * workspace (the unnormalised partial outputs of histories that were cut into pieces, joined by the merge
 * kernel) is a fixed array of CKV_STATIC_SCRATCH_BYTES inside the library instead of the buffer the handle
 * owns.  Every GPU the library runs on holds that array until the process ends.  A handle whose pieces need more
 * (partial slots x queries per block x (d_a + 2) floats) is refused with CKV_ERR_UNSUPPORTED: use ckv_attend.
 * The handle's device must be the current device (CKV_ERR_UNSUPPORTED otherwise).  The call allocates and frees
 * nothing and calls no allocating routine.  All calls on one GPU share the one array, which keeps the last
 * call's contents (nothing in it has to start at zero: every slot that is read was written earlier in the same
 * call): calls that overlap in time on one GPU race, on any handle; serialise them on one stream.
 */
#define CKV_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int ckv_attend_static_scratch(const ckv_cache* cache, const void* pool_k, const void* pool_v,
                              const int32_t* idx, const void* user_k, const void* user_v,
                              const void* q, const int32_t* lengths, void* out, void* stream);

/*
 * Materialise the final K and V rows, k_full, v_full device [H][T][d_a], each row the
 * user slice followed by the gathered pool row (eq. "eq: Kc", "eq: K").  A pure copy,
 * bit-exact.  Exists for verification of the gather and the layouts; the attention path
 * never calls it.  Either output may be NULL to skip it.
 */
int ckv_reconstruct(const ckv_cache* cache, const void* pool_k, const void* pool_v,
                    void* k_full, void* v_full, void* stream);

/*
 * Host only (no device is touched): the work lists ckv_build_cache would attach to a handle of this shape
 * and these lengths on a GPU with `cus` compute units that keeps `wg_per_cu` workgroups of the chosen
 * kernel resident per unit.  One record of 8 int64 per work item, in launch order:
 *   [0] user b  [1] head h  [2] first query q0 of the block  [3] positions n of the piece
 *   [4] first flattened position t0  [5] slot in the split workspace, or -1 for a whole history
 *   [6] the user's full length n_b  [7] workgroup that runs the item
 * Every (user, head, query block) is covered by pieces that tile [0, n_b) exactly once; pieces of a split
 * history carry consecutive workspace slots in position order.  Up to max_records records are written
 * (records may be NULL); the return value is the total number of items, or a negative CKV_ERR_* code.
 * n_workgroups receives the number of workgroups launched, variant (if not NULL) the kernel name.
 * Exists so that the scheduling arithmetic can be checked without a GPU.
 */
int64_t ckv_plan(const ckv_shape* shape, const int32_t* lengths, int cus, int wg_per_cu,
                 int64_t* records, int64_t max_records, int32_t* n_workgroups,
                 char* variant, size_t variant_size);

/*
 * Frequency renumbering of the pool rows.  The router sends many positions of many users to the same pool
 * entries (appendix "Analysis of Router Activations for Highly Similar Users"); this call counts, per head
 * and side, how often the handle's cache refers to every row, renumbers the rows most used first (equal
 * counts keep their order), writes the permuted pools and rewrites the handle's stored indices, so that
 * the hot rows of a head are one contiguous block at the start of its pool.  A pure relabeling: ckv_attend
 * with the new pools gives bit-identical results.
 *
 *   pool_k, pool_v          device [H][P][pool_ld], the current pools (a side that is not shared is ignored)
 *   pool_k_out, pool_v_out  device [H][P][pool_ld], receive the permuted pools; must not alias the inputs
 *   new_id                  device int32 [2][H][P] or NULL: new number of every old row (plane 0 keys,
 *                           plane 1 values), e.g. to permute the rows of a router the same way
 * The handle must be device-resident.  Allocates temporaries, sorts on the host and synchronises `stream`:
 * a maintenance call (after a pool refresh), not part of the request path.  After it the handle is only
 * valid together with the new pools.  Errors: CKV_ERR_NULL, _UNSUPPORTED (offloaded handle), _HIP.
 */
int ckv_remap_hot_rows(ckv_cache* cache, const void* pool_k, const void* pool_v, void* pool_k_out, void* pool_v_out,
                       int32_t* new_id, void* stream);

/*
 * Tuning options of the calling thread, read by the calls that build a handle or a plan afterwards
 * (ckv_build_cache, ckv_build_cache_offloaded, ckv_prefill, ckv_plan); handles that exist are not affected.
 * None changes a result beyond the order of summation; they exist for measurement and so that tests reach
 * every kernel.  value NULL or "" restores the option's default, key NULL restores all defaults.
 *   "mfma_impl"       "staged": the register-staged matrix-core kernel where the direct-to-LDS one would run; "auto"
 *   "stream_impl"     "narrow": the column-block streaming kernel where the wide-row one would run; "auto"
 *   "stream_hot_rows" 0 .. 32: pool rows 0 .. n-1 of a work item's head that the wide-row streaming kernel copies into LDS and serves
 *                     from there (the most used rows after ckv_remap_hot_rows; default 0: measured slower than leaving them to the L2s)
 *   "stream_waves"    "2" | "4": wavefronts per work item of the streaming kernels (default: by the number and length of the items)
 *   "dma_sched"       "static" (default: persistent workgroups with their own item lists) | "dynamic"
 *   "dma_shape"       "nw,qg": wavefronts per workgroup and query groups per wavefront of the direct-to-LDS kernel
 *   "dma_q16"         "0" | "1": up to sixteen queries at 64 columns run sixteen to a work item on the 16x16x32 matrix instruction
 *                     (default "1") or 32 to a work item like larger query counts
 *   "dma_scores_ahead" "0" | "1": tile loop of the direct-to-LDS kernel that takes the scores of a tile one iteration early (exists
 *                     for four wavefronts at 128 columns and for 256 columns; default: on at 256 columns, at 128 where both sides gather from pools)
 *   "dma_slow_speed"  weight in (0, 4] of a workgroup that shares its SIMDs with an older one (default 0.75 / 1.0)
 *   "debug"           "1": print the chosen split and list statistics to stderr
 * Errors: CKV_ERR_UNSUPPORTED (unknown key, malformed value).
 */
int ckv_set_option(const char* key, const char* value);

/* Release the handle and the device memory it owns.  NULL is allowed. */
void ckv_free(ckv_cache* cache);

/* Message of the last error on this thread ("" if none). Never NULL. */
const char* ckv_last_error(void);

/*
 * Measurement helpers.
 * ckv_set_timing(cache, n) with n > 0 makes every following ckv_attend on this handle record three
 * HIP events on the launch stream (before the main attention kernel, after it, after the merge
 * kernel of split histories), kept in a ring of n launches; n = 0 switches it off.  ckv_kernel_ms
 * synchronises them and returns the mean milliseconds of the main kernel over the last
 * min(calls, n) launches (negative if none).  ckv_kernel_times writes the per-launch times, oldest
 * launch first, of the main kernel (kernel_ms) and of the merge kernel (merge_ms, zeros for a handle
 * without split histories) for up to max_launches launches (either array may be NULL) and returns
 * how many it wrote, or a negative error.  ckv_variant names the kernel family the handle dispatches to.
 * ckv_copy enqueues a plain device-to-device copy kernel of nbytes (16-byte aligned device
 * pointers), used to calibrate hardware byte counters against a transfer of known size and
 * to read the packed cache back in tests.
 */
int ckv_set_timing(ckv_cache* cache, int pairs);
float ckv_kernel_ms(ckv_cache* cache);
int ckv_kernel_times(ckv_cache* cache, float* kernel_ms, float* merge_ms, int max_launches);
const char* ckv_variant(const ckv_cache* cache);
int ckv_copy(void* dst, const void* src, size_t nbytes, void* stream);
/*
 * Per-workgroup timeline of the matrix-core kernel, for load-balance studies.  After
 * ckv_trace_enable(cache, 1) every ckv_attend on the handle records, per work item in launch
 * order, 8 words: [0] start, [1] tile loop entered, [2] tile loop left, [3] end (all in ticks of
 * the 100 MHz wall clock), [4] hardware id (XCC id << 32 | HW_ID), [5] positions, [6..7] unused.
 * ckv_trace_read synchronises the device and copies up to max_items records to `host`
 * (8 * max_items words); it returns the number of records or a negative error.  Costs one
 * allocation; switch it off (enable = 0) for timed runs.
 */
int ckv_trace_enable(ckv_cache* cache, int enable);
int64_t ckv_trace_read(ckv_cache* cache, unsigned long long* host, int64_t max_items);

#ifdef __cplusplus
}
#endif
#endif /* CKV_H */
