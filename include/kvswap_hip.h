/*
 * kvswap_hip -- the decode-step hot path of KVSwap (arXiv 2511.11907) as
 * hand-written HIP kernels for gfx950 (MI355X), behind a plain C ABI.
 *
 * One decode step of one layer, per (sequence b, KV head k) problem:
 *   predict : s[n] = sum_{h: g(h)=k} (q[h] . A[k]) . K_lr[n]       (Sec. 3.3, Eq. 1)
 *   group   : gs[j] = max (or mean) of s over the G tokens of group j
 *   select  : idx = the M groups with the largest gs               (ReduceMax + TopK)
 *   attend  : out[h] = softmax(scale * q[h] . K[sel]^T) . V[sel]    over the selected
 *             groups' tokens only                                   (Sec. 3.4, KV cache manager)
 * with the compact metadata K_lr = K . A built once per token (Sec. 3.2).
 * Sec. 3.2 considers two designs of the adapter and both are implemented
 * (kvs_params.head_mode):
 *   KVS_HEADS_SEPARATE  design (a): one adapter A[k] (d x r), one K_lr and one
 *                       selection per KV head, as written above;
 *   KVS_HEADS_JOINT     design (b), the one the paper adopts: the keys of all KV
 *                       heads of a token are flattened into one row of H_kv*d values
 *                       (head-major) and projected by a single adapter
 *                       A [(H_kv*d) x r]; one K_lr row per token; the token score
 *                       is summed over ALL query heads, head h using the block
 *                       A_{g(h)} = rows g(h)*d .. g(h)*d+d-1 of the adapter (Eq. 1);
 *                       one selection per sequence, shared by all its KV heads.
 * The full K/V cache lives in device memory (it stands in for the paper's disk
 * tier plus preload buffer).
 *
 * Metadata precision (Sec. 3.2: the compressed K cache only ranks tokens, so its
 * precision may be traded for memory): meta_dtype may be fp32, bf16 or the 8-bit float
 * OCP E4M3 (finite-only, largest value 448; one byte per element, which halves the
 * stream of the prediction again).  K_lr is stored as round(K.A / meta_scale), nearest
 * even, saturating for E4M3; scores use meta_scale * stored.  meta_scale is one number for
 * the whole call, or (meta_scales) one per selection set.
 *
 * Memory: every pointer below is a DEVICE pointer unless it says "host".  All
 * tensors are contiguous and row-major, 16-byte aligned:
 *   K, V          [B, H_kv, N, d]   kv_dtype      (a group = G consecutive rows,
 *                                                  i.e. one contiguous G*d run)
 *   q, out        [B, H_q, d]       kv_dtype
 *   A             [H_kv, d, r]      fp32
 *   K_lr          [B, H_kv, N, r]   meta_dtype
 *   idx           [B, H_kv, M]      int32 group indices in [0, N/G), unique,
 *                                   ascending as written by kvs_predict_select
 *   group_scores  [B, H_kv, N/G]    fp32
 * g(h) = h / (H_q / H_kv).
 * With ctx_capacity = C > 0 the N axis of K, V and K_lr has C >= N rows allocated
 * (K, V [B, H_kv, C, d], K_lr [B, H_kv, C, r]); only the first N are the cache.
 * Rolling buffer (Sec. 3.4.1): the newest tokens, which do not yet form a group,
 * live in rb_K, rb_V [B, H_kv, rb_capacity, d] (kv_dtype), first rb_len rows valid;
 * they are never scored and always attended (the *_rb calls).
 * In joint mode the per-selection tensors have no H_kv axis: K_lr [B, N, r],
 * idx [B, M], group_scores [B, N/G]; A has the same memory layout as above
 * ([H_kv*d, r] row-major == [H_kv, d, r]).
 *
 * Ownership: the caller owns every buffer.  The library allocates nothing,
 * frees nothing, keeps no state between calls and never synchronises; all work
 * is enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 * stream).  Inputs are read-only.  `workspace` is caller-provided scratch of at
 * least kvs_workspace_bytes() bytes.  It starts with a small area of counters
 * (per-problem score histograms, and the arrival counters with which the
 * attention kernel hands the final merge to the workgroup that finishes last)
 * that must be zero when a call starts: call kvs_workspace_init once after
 * allocating (or zero-fill the buffer yourself); every call then leaves the
 * counters zero for the next one, PROVIDED all of its launches ran: after any call
 * that returned KVS_ERR_DEVICE (a launch failed part-way through a call) the counters
 * may be left non-zero, and the workspace must be prepared with kvs_workspace_init
 * again before it is reused.  This counter area is the only thing the library keeps
 * from one call to the next, and it keeps it in the caller's buffer.
 * The rest of the workspace is undefined on entry and on return.  Calls that
 * share a workspace must be ordered on one stream (they would race otherwise).
 * The layout of the counter area depends only on batch, n_kv_heads and head_mode:
 * a buffer that is large enough stays valid while those are unchanged (e.g. through
 * a decode loop whose ctx_len grows: size it for the largest ctx_len); when they
 * change, call kvs_workspace_init again with the new params first.
 *
 * Values: inputs are expected to be finite.  Infinities or NaNs in q, K, V, A or K_lr
 * are not detected; they give unspecified selections and outputs (never an access
 * outside the buffers).
 *
 * Errors: every function validates its arguments on the host before anything is
 * launched and returns a kvs_status; nothing is thrown or aborted across the
 * ABI.  Contents of idx are NOT validated on the device: out-of-range indices
 * passed to kvs_sparse_decode_attn are a caller error.
 *
 * Supported shapes: d in {64, 128}; r in {16, 32, 64, 128} with r <= d
 * (r <= H_kv*d in joint mode); 1 <= G <= 16, any integer (the parameter solver of
 * App. A.4 searches G upwards from 1, and the appendix's rolling-buffer table uses
 * G = 12); H_q / H_kv from 1 to 8 (the models of Sec. 4.1 have 3, 4, 5, 7 or 8 query
 * heads per KV head);
 * N % G == 0; 1 <= M <= N/G; N/G <= 32768; B * H_kv <= 65535; N * d < 2^31;
 * joint mode: H_kv * d <= 4096; ctx_capacity * d < 2^31; rb_len <= 256.
 */
#ifndef KVSWAP_HIP_H
#define KVSWAP_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  KVS_OK = 0,
  KVS_ERR_NULL = 1,        /* a required pointer is NULL                      */
  KVS_ERR_SHAPE = 2,       /* inconsistent or non-positive sizes              */
  KVS_ERR_DTYPE = 3,       /* unknown dtype / reduce / head-mode code         */
  KVS_ERR_UNSUPPORTED = 4, /* consistent but outside the supported set        */
  KVS_ERR_WORKSPACE = 5,   /* workspace NULL, misaligned or too small         */
  KVS_ERR_DEVICE = 6,      /* a HIP launch reported an error                  */
  KVS_ERR_ALIGN = 7,       /* a tensor pointer is not 16-byte aligned         */
  KVS_ERR_SCRATCH = 8      /* kvs_decode_step_static: the problem needs more scratch than
                              KVS_STATIC_SCRATCH_BYTES                        */
} kvs_status;

typedef enum { KVS_F32 = 0, KVS_BF16 = 1, KVS_FP8_E4M3 = 2 /* meta_dtype only */ } kvs_dtype;
typedef enum { KVS_REDUCE_MAX = 0, KVS_REDUCE_MEAN = 1 } kvs_reduce;
typedef enum { KVS_HEADS_SEPARATE = 0, KVS_HEADS_JOINT = 1 } kvs_head_mode;

typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim, rank; /* B, H_q, H_kv, d, r          */
  int32_t ctx_len, group_size, n_select;                /* N, G, M                     */
  int32_t kv_dtype;      /* kvs_dtype of K, V, q, out                                  */
  int32_t meta_dtype;    /* kvs_dtype of K_lr                                          */
  int32_t reduce;        /* kvs_reduce; MAX is the paper's ReduceMax                   */
  float softmax_scale;   /* 0 => 1/sqrt(d)                                             */
  int32_t head_mode;     /* kvs_head_mode; SEPARATE (0) = one adapter per KV head      */
  float meta_scale;      /* K_lr is stored divided by this and multiplied back when it is
                            scored (0 => 1): fits the metadata to a narrow meta_dtype     */
  int32_t ctx_capacity;  /* rows allocated per (b, kv head) in K and V, and per selection
                            set in K_lr; 0 => ctx_len.  Rows ctx_len .. capacity-1 are room
                            for the groups a decode loop appends and are never read.       */
  const float* meta_scales; /* NULL, or a DEVICE array with one metadata scale per selection
                            set - [B, H_kv], or [B] in joint mode - used instead of
                            meta_scale: heads (or sequences) whose keys differ by orders of
                            magnitude then each fit a narrow meta_dtype.  Values must be
                            positive and finite (not checked: the array is device memory);
                            16-byte alignment is not required.  A per-head calibration
                            constant is simply repeated for every sequence.               */
} kvs_params;

/* Bytes of workspace that any of the calls below may need for these params
 * (0 if the params are invalid). */
size_t kvs_workspace_bytes(const kvs_params* p);

/* Zero the arrival counters at the start of `workspace` (one small fill kernel
 * on `stream`).  Needed once per workspace buffer, before its first use. */
kvs_status kvs_workspace_init(const kvs_params* p, void* workspace, size_t workspace_bytes,
                              void* stream);

/* Diagnostic: has a wait between workgroups of kvs_decode_step_single_launch ever run out on this
 * workspace since it was prepared?  Copies one word to the host and SYNCHRONISES `stream`.
 * KVS_OK if not; KVS_ERR_DEVICE if so (text in kvs_last_device_error): results of that step
 * are incomplete and the workspace needs kvs_workspace_init before it is used again. */
kvs_status kvs_workspace_check(const kvs_params* p, const void* workspace, size_t workspace_bytes,
                               void* stream);

/* Bound of the waits between workgroups inside kvs_decode_step_single_launch, in polls of a counter (a
 * poll takes one to two microseconds); process-wide, takes effect with the next call;
 * polls <= 0 restores the default (about a second).  Meant for tests and diagnostics. */
void kvs_set_wait_limit(int32_t polls);

/* Validate params without touching a device: KVS_OK or the error the other
 * calls would return for them. */
kvs_status kvs_check_params(const kvs_params* p);

/* Sec. 3.2: K_lr[b,k,n,:] = K[b,k,n,:] . A[k] (joint mode: K_lr[b,n,:] =
 * Flatten(K)[b,n,:] . A), fp32 accumulation, one rounding (nearest-even) to meta_dtype.  Run at prefill and whenever new groups are
 * appended; not part of the per-step latency.  n_select is ignored. */
kvs_status kvs_build_metadata(const kvs_params* p, const void* K, const float* A,
                              void* K_lr, void* stream);

/* The same for token rows first_row .. first_row + n_rows - 1 only (they may lie
 * beyond ctx_len, inside the capacity): the incremental update of the compressed K
 * cache when new groups are completed (Sec. 3.4.1).  KVS_ERR_SHAPE if the range
 * leaves the allocated rows. */
kvs_status kvs_build_metadata_rows(const kvs_params* p, const void* K, const float* A,
                                   void* K_lr, int32_t first_row, int32_t n_rows, void* stream);

/* Sec. 3.4.1: a completed group leaves the rolling buffer.  Copies the first G rows
 * of every (b, kv head) of rb_K / rb_V into cache rows ctx_len .. ctx_len+G-1 of K / V
 * (written here) and builds the K_lr rows of the new group; two small launches.
 * Needs ctx_len + G <= ctx_capacity and rb_capacity >= G (KVS_ERR_SHAPE otherwise).
 * Afterwards the caller uses ctx_len + G and restarts (or shifts) its buffer. */
kvs_status kvs_append_group(const kvs_params* p, const void* rb_K, const void* rb_V,
                            int32_t rb_capacity, void* K, void* V, const float* A, void* K_lr,
                            void* stream);

/* Sec. 3.3 (Eq. 1, "Scoring and selection"): low-rank token scores summed over
 * the query heads of each KV head, group representative (max or mean), and the
 * indices of the M best groups per (b, kv head): ties go to the lower index,
 * output ascending.  Two launches: the streaming kernel also histograms the
 * scores, the selection kernel starts from that histogram.  group_scores may be
 * NULL; if given it receives gs.  Joint mode: one more small launch first, which
 * projects the head-summed queries of each sequence into the rank-r space (kept
 * in the workspace); scores are summed over all query heads and idx is [B, M]. */
kvs_status kvs_predict_select(const kvs_params* p, const void* q, const void* K_lr,
                              const float* A, int32_t* idx, float* group_scores,
                              void* workspace, size_t workspace_bytes, void* stream);

/* The two launches of kvs_predict_select as separate calls (same kernels).
 * kvs_predict_scores writes group_scores [B,H_kv,N/G] (required here);
 * kvs_select_topk reads them and writes idx.  workspace may be NULL in both: the
 * selection then builds its own score histogram (joint mode: kvs_predict_scores
 * needs the workspace, KVS_ERR_WORKSPACE without).
 * Contract of a non-NULL workspace: if kvs_predict_scores is given a workspace it also
 * leaves the per-problem score histograms there (for up to 32 selection sets; beyond that
 * the selection is faster building its own), and the NEXT call on that workspace
 * must be kvs_select_topk with the same workspace, params and group_scores (it consumes
 * the histograms and zeroes them again).  Conversely, a workspace passed to
 * kvs_select_topk is expected to hold the histograms of exactly these group_scores.
 * The selection checks that a histogram counts N/G scores in all; one that does not
 * (scores that came from elsewhere, or from kvs_predict_scores without a workspace)
 * is ignored, the selection builds its own and is still exact, and the counters are
 * zeroed all the same.  A histogram of the right total that belongs to other scores
 * cannot be told apart and gives an unspecified (in-range, M-element) selection. */
kvs_status kvs_predict_scores(const kvs_params* p, const void* q, const void* K_lr,
                              const float* A, float* group_scores, void* workspace,
                              size_t workspace_bytes, void* stream);
kvs_status kvs_select_topk(const kvs_params* p, const float* group_scores, int32_t* idx,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Sec. 3.4 (attention consumes only the selected KV groups): softmax attention
 * of every query head over the G*M tokens named by idx of its KV head (joint
 * mode: by the idx of its sequence), gathered
 * from the full K/V, fp32 online softmax, result rounded to kv_dtype.  One
 * launch (split over the selected groups, merged by the last workgroup). */
kvs_status kvs_sparse_decode_attn(const kvs_params* p, const void* q, const void* K,
                                  const void* V, const int32_t* idx, void* out,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* The same with a rolling buffer: every head also attends the first rb_len tokens of
 * its KV head's rows of rb_K / rb_V, in one softmax with the selected tokens.
 * rb_len = 0 (pointers may then be NULL) is kvs_sparse_decode_attn.  The buffer's
 * tokens are handled by the last split of each problem; rb_len <= 256. */
kvs_status kvs_sparse_decode_attn_rb(const kvs_params* p, const void* q, const void* K,
                                     const void* V, const int32_t* idx, const void* rb_K,
                                     const void* rb_V, int32_t rb_len, int32_t rb_capacity,
                                     void* out, void* workspace, size_t workspace_bytes,
                                     void* stream);

/* Sec. 3.4.4 (KV cache manager): the same attention with the KV groups addressed
 * through a mapping table, as an operating system addresses pages.  K_pool, V_pool
 * [n_slots, G, d] (kv_dtype) are pools of group-sized slots shared by all problems;
 * slot_table [B, H_kv, N/G] int32 gives the slot that holds logical group j of
 * (b, kv head); group idx[m] of a head is read from slot_table[b, g(h), idx[m]].  Slots may
 * be in any order, need not all be used, and only the selected ones are read.  Slot
 * numbers are not validated on the device (0 <= slot < n_slots is the caller's duty,
 * like the contents of idx).  ctx_capacity plays no role here.  The rolling-buffer
 * arguments are as above (rb_len = 0: none). */
kvs_status kvs_sparse_decode_attn_paged(const kvs_params* p, const void* q, const void* K_pool,
                                        const void* V_pool, const int32_t* slot_table,
                                        int32_t n_slots, const int32_t* idx, const void* rb_K,
                                        const void* rb_V, int32_t rb_len, int32_t rb_capacity,
                                        void* out, void* workspace, size_t workspace_bytes,
                                        void* stream);

/* Sec. 3.4.2 (reuse of groups across steps): common[s] = number of group indices that
 * occur in both idx_prev[s,:] and idx_cur[s,:], per selection set ([B, H_kv], or [B] in
 * joint mode; int32, device).  Divided by M it is the overlap ratio of two consecutive
 * steps.  Indices of a row must be unique (any order); out-of-range ones are ignored. */
kvs_status kvs_selection_overlap(const kvs_params* p, const int32_t* idx_prev,
                                 const int32_t* idx_cur, int32_t* common, void* stream);

/* One whole decode step of a layer: kvs_predict_select followed by
 * kvs_sparse_decode_attn on the same stream (three launches in all).  idx
 * receives the selection (it is an output here); group_scores may be NULL. */
kvs_status kvs_decode_step(const kvs_params* p, const void* q, const void* K_lr,
                           const float* A, const void* K, const void* V, int32_t* idx,
                           float* group_scores, void* out, void* workspace,
                           size_t workspace_bytes, void* stream);

/* The same step as ONE launch: a persistent grid whose workgroups draw prediction, selection
 * and attention work items of all (sequence, KV head) problems from one counter, ordered so
 * that the selection of a problem runs while other problems stream and no phase waits for a
 * launch boundary.  Items wait for the items they depend on through counters in the
 * workspace; such a wait is bounded (kvs_set_wait_limit) and cannot block the grid (an item
 * only waits for items drawn before it, which running workgroups hold).  Should a wait run
 * out all the same, the step's results are incomplete, the error word of the workspace is
 * set (kvs_workspace_check) and the workspace must be prepared again.
 * Covers the layouts of the evaluated models' layers only - bf16 K/V and metadata, d = 128,
 * four query heads per KV head, r = 32 with G = 4 or r = 64 with G = 8, per-head adapters,
 * at most 16384 groups and 4096 selected groups per problem - and returns
 * KVS_ERR_UNSUPPORTED for every other.  Scores and selection are bit for bit those of
 * kvs_decode_step; `out` may differ from it in the last bits (the selected tokens are cut
 * into another number of splits, i.e. summed in another order) and is the same from call to
 * call.  On MI355X it is SLOWER than the three launches at every evaluated size (inside a
 * grid that saturates the memory system every dependent step of the selection takes several
 * times longer, and the attention of a problem still has to wait for it): kvs_decode_step
 * does not use it.  It is kept for callers to whom the number of launches matters more. */
kvs_status kvs_decode_step_single_launch(const kvs_params* p, const void* q, const void* K_lr,
                                         const float* A, const void* K, const void* V, int32_t* idx,
                                         float* group_scores, void* out, void* workspace,
                                         size_t workspace_bytes, void* stream);

/* Sec. 3.3 / 3.4 (the pipeline over layers: the groups of the next layer are predicted
 * while this layer computes): the attention of one layer and the top-M selection for the
 * NEXT layer in one launch.  The selection is latency-bound and the attention is the one
 * kernel of a pipelined step it does not depend on, so the selection's workgroups ride along
 * in the attention's grid.  Equivalent, bit for bit, to
 *     kvs_sparse_decode_attn(p, q, K, V, idx, out, workspace, ...);
 *     kvs_select_topk(p, next_group_scores, next_idx, workspace, ...);
 * with the workspace contract of kvs_select_topk (the histograms that kvs_predict_scores left
 * in this workspace for next_group_scores are consumed and zeroed).  A pipelined step of
 * layer i is then two launches: kvs_predict_scores for layer i+1, then this call (attention
 * of layer i with the idx this call produced one step earlier, selection of layer i+1).
 * idx and next_idx must not overlap.  Both layers have the shape `p`.  Hidden behind the
 * attention, the selection gains nothing from the histogram hand-over, which costs the
 * prediction kernel about a microsecond: in this form kvs_predict_scores is best called
 * without a workspace (per-head mode), and the selection builds its own histogram.
 * Covers bf16 K/V with d = 128, 3 to 8 query heads per KV head and at most 16384 groups per
 * selection set (either head mode); KVS_ERR_UNSUPPORTED otherwise. */
kvs_status kvs_attend_select_next(const kvs_params* p, const void* q, const void* K, const void* V,
                                  const int32_t* idx, void* out, const float* next_group_scores,
                                  int32_t* next_idx, void* workspace, size_t workspace_bytes,
                                  void* stream);

/* The same with the rolling buffer in the attention (Sec. 3.4.1; arguments and limits as in
 * kvs_sparse_decode_attn_rb): equivalent, bit for bit, to kvs_sparse_decode_attn_rb followed
 * by kvs_select_topk.  rb_len = 0 is kvs_attend_select_next. */
kvs_status kvs_attend_select_next_rb(const kvs_params* p, const void* q, const void* K, const void* V,
                                     const int32_t* idx, const void* rb_K, const void* rb_V,
                                     int32_t rb_len, int32_t rb_capacity, void* out,
                                     const float* next_group_scores, int32_t* next_idx, void* workspace,
                                     size_t workspace_bytes, void* stream);

/* kvs_decode_step with the rolling buffer in the attention (kvs_predict_select, then
 * kvs_sparse_decode_attn_rb). */
kvs_status kvs_decode_step_rb(const kvs_params* p, const void* q, const void* K_lr,
                              const float* A, const void* K, const void* V, const void* rb_K,
                              const void* rb_V, int32_t rb_len, int32_t rb_capacity,
                              int32_t* idx, float* group_scores, void* out, void* workspace,
                              size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid it): kvs_decode_step without a workspace argument.
 * The scratch memory of the step's kernels lives in a static device array inside the
 * library, KVS_STATIC_SCRATCH_BYTES per GPU, held by every GPU the library runs on until
 * the process ends.  The call allocates and frees nothing (no hipMalloc, no hipFree, no
 * allocating library routine) and does not synchronise; it enqueues one small fill kernel
 * that zeroes the counter area, then the launches of kvs_decode_step, on `stream`.  Params
 * whose kvs_workspace_bytes() exceeds KVS_STATIC_SCRATCH_BYTES are refused with
 * KVS_ERR_SCRATCH before anything is launched (every workload of the evaluation fits: the
 * largest, 128 problems of 4096 groups, needs 5.1 MiB).  The device that `stream` belongs to
 * must be the current device.  On the first call per device the library looks up that
 * device's address of the array; make that first call outside a graph capture.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 * (different streams, or graphs replayed concurrently) race and give undefined results;
 * calls ordered on one stream are safe, whatever their shapes.  Results are bit-identical
 * to kvs_decode_step's. */
#define KVS_STATIC_SCRATCH_BYTES (8u << 20)
kvs_status kvs_decode_step_static(const kvs_params* p, const void* q, const void* K_lr,
                                  const float* A, const void* K, const void* V, int32_t* idx,
                                  float* group_scores, void* out, void* stream);

/* Static, NUL-terminated description of a status code (host pointer). */
const char* kvs_status_str(kvs_status s);

/* Text of the HIP error behind the calling thread's most recent KVS_ERR_DEVICE
 * ("" if none yet); diagnostics only (host pointer, static storage). */
const char* kvs_last_device_error(void);

/* Library version string, e.g. "kvswap_hip 0.1 gfx950" (host pointer). */
const char* kvs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVSWAP_HIP_H */
