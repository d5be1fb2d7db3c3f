/*
 * CPU oracle of the KVSwap decode-step hot path -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 implementation of what the path computes, written out
 * step by step in the order the paper states the method.  It shares no code
 * with the GPU library and may be used only by the tests, by the smoke check
 * and by the bench's CPU-baseline leg; no product path may call it.
 *
 * Conventions (all arrays contiguous, row-major, host memory):
 *   K, V    [B, H_kv, N, d]   storage dtype kv_dtype
 *   q       [B, H_q, d]       storage dtype kv_dtype
 *   A       [H_kv, d, r]      fp32 (per-KV-head adapter, Sec. 3.2 design (a))
 *   K_lr    [B, H_kv, N, r]   storage dtype meta_dtype
 *   idx     [B, H_kv, M]      int32 group indices, ascending
 *   g(h) = h / (H_q / H_kv)   query head -> shared KV head (Eq. 1)
 * Joint-head mode (head_mode = ORC_HEADS_JOINT; Sec. 3.2 design (b), the one the
 * paper adopts): the keys of all KV heads of a token are flattened into one row
 * of H_kv*d values (head-major) and projected by a single adapter; there is one
 * K_lr row per token and one selection per sequence:
 *   A       [H_kv * d, r]     fp32; rows k*d .. k*d+d-1 form A_k of Eq. (1)
 *   K_lr    [B, N, r]
 *   idx     [B, M]            shared by all KV heads of the sequence
 *   gs, s, boundary           [B, NG], [B, N], [B, 2]
 * Capacity: if ctx_capacity > 0 the arrays K, V and K_lr hold ctx_capacity rows per
 * (b, kv head) [per b for the joint K_lr] of which the first ctx_len are the cache
 * (room for the groups a decode loop appends); 0 means exactly ctx_len rows.
 * Rolling buffer (Sec. 3.4.1 "New KV entries management"): the newest tokens, not yet
 * a complete group, live outside the cache in rb_K, rb_V [B, H_kv, rb_capacity, d]
 * (first rb_len rows valid); they are never scored and always attended.
 * Metadata precision (Sec. 3.2: the compressed K cache only ranks tokens, so its precision
 * may be traded for memory): meta_dtype may also be 8-bit floating point (OCP E4M3,
 * uint8 codes), and K_lr is stored as round(K.A / meta_scale) and read back as
 * meta_scale * stored (meta_scale 0 => 1; it applies to every meta_dtype).  With
 * meta_scales every selection set (b, kv head; b in joint mode) has a scale of its own.
 * Storage dtypes: 0 = fp32 (float), 1 = bf16 (uint16 bit patterns), 2 = fp8 E4M3 (uint8).  Stored
 * values are widened to fp64 exactly; every sum is an fp64 sum in natural
 * index order.
 *
 * Pins (tests/test_oracle_*.py): numpy brute force on tiny shapes; r = d with
 * A = I gives exact q.K scores; exactly rank-r keys give exact scores; both
 * sides of Eq. (1) agree; G = 1 is plain token top-k; selecting every group
 * equals dense softmax attention; planted ties resolve to the lower index;
 * closed-form softmax cases; bf16 rounding at known midpoints.  Joint mode: numpy
 * brute force; one KV head makes both modes coincide; a block-diagonal adapter
 * makes the joint scores the sum of the per-head ones; identity adapter gives the
 * sum of the exact logits of all heads; shared idx equals replicated idx.
 * Rolling buffer / capacity: numpy brute force over the concatenated token list; an
 * empty buffer changes nothing; a cache group moved into the buffer gives the same
 * output; all groups + buffer equals dense attention over the concatenated cache;
 * padded (capacity > ctx_len) arrays with poisoned padding give the compact results;
 * metadata of a row range equals the same rows of the full build.
 * Mapping table: the identity table over the cache viewed as slots equals the unpaged
 * call; a random permutation of the slots gives the same output; brute force over the
 * gathered rows.  Overlap: numpy's intersect1d and hand cases.
 * fp8: every code's value and the rounding of many values against the float8 type of a
 * tensor library and against a nearest-neighbour search over all codes; hand-derived
 * ties and saturation; the whole path against brute force on the decoded values.
 * The paper prints no worked numeric example of this path, so numeric parity
 * with the authors' own implementation is unpinned (parity unpinned on that
 * point only; every function below has the pins listed above).
 */
#ifndef KVSWAP_ORACLE_H
#define KVSWAP_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_FP8_E4M3 = 2 /* meta_dtype only */ };
enum { ORC_REDUCE_MAX = 0, ORC_REDUCE_MEAN = 1 };
enum { ORC_HEADS_SEPARATE = 0, ORC_HEADS_JOINT = 1 };

typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim, rank; /* B, H_q, H_kv, d, r */
  int32_t ctx_len, group_size, n_select;                /* N, G, M            */
  int32_t kv_dtype, meta_dtype;                         /* ORC_F32 / ORC_BF16 */
  int32_t reduce;                                       /* ORC_REDUCE_*       */
  int32_t head_mode;                                    /* ORC_HEADS_*        */
  int32_t ctx_capacity; /* rows allocated per problem in K, V, K_lr; 0 => ctx_len      */
  int32_t n_threads;   /* OpenMP threads over the (b, kv head) problems; <=1: serial */
  double meta_scale;   /* K_lr is stored divided by this; 0 => 1 */
  double softmax_scale; /* 0 => 1/sqrt(d) */
  const double* meta_scales; /* nullable: one scale per selection set ([B*H_kv], or [B] in
                                joint mode), positive and finite; overrides meta_scale */
} orc_params;

/* K_lr = K . A per KV head, or Flatten(K) . A in joint mode (Sec. 3.2), fp64
 * accumulation, then one rounding to meta_dtype (round-to-nearest-even).
 * K_lr_exact (nullable, doubles, shape of K_lr) receives the unrounded products.
 * Returns 0, or -1 on bad params. */
int oracle_build_metadata(const orc_params* p, const void* K, const float* A,
                          void* K_lr, double* K_lr_exact);

/* The same for token rows first_row .. first_row + n_rows - 1 only (the metadata of
 * newly completed groups, Sec. 3.4.1); other rows of K_lr / K_lr_exact are untouched.
 * Rows may lie beyond ctx_len but must lie inside the capacity. */
int oracle_build_metadata_rows(const orc_params* p, const void* K, const float* A,
                               void* K_lr, double* K_lr_exact, int32_t first_row,
                               int32_t n_rows);

/* Prediction and selection (Sec. 3.3, Eq. 1 and "Scoring and selection"):
 *   q_lr[h]  = q[h] . A[g(h)]                          (low-rank query vector)
 *   s[n]     = sum_{h: g(h)=k} q_lr[h] . K_lr[n]       (raw logits summed over heads)
 *   gs[j]    = max (or mean) of s over the G tokens of group j
 *   idx      = the M groups with the largest gs, ties to the lower index,
 *              written in ascending index order.
 * Optional outputs (nullable): gs [B,H_kv,NG], s [B,H_kv,N],
 * boundary [B,H_kv,2] = {M-th largest gs, (M+1)-th largest gs (or -inf if M = NG)}.
 * Joint mode: the sum runs over all H_q heads, each with the A_{g(h)} block of the
 * adapter, against the single K_lr of the sequence; outputs lose the H_kv axis. */
int oracle_predict_select(const orc_params* p, const void* q, const void* K_lr,
                          const float* A, int32_t* idx, double* gs, double* s,
                          double* boundary);

/* Softmax attention of each query head over the tokens of the selected groups
 * of its KV head only: out[b,h,:] in fp64.  idx is [B,H_kv,n_sel] with
 * n_sel = p->n_select ([B,n_sel] in joint mode: every head of the sequence attends
 * the same groups); order of idx is irrelevant, duplicates are not allowed. */
int oracle_sparse_attn(const orc_params* p, const void* q, const void* K,
                       const void* V, const int32_t* idx, double* out);

/* The same with a rolling buffer: every head also attends the first rb_len tokens of
 * its KV head's rows of rb_K / rb_V [B, H_kv, rb_capacity, d] (one softmax over the
 * selected tokens and the buffer together).  rb_len = 0 is oracle_sparse_attn. */
int oracle_sparse_attn_rb(const orc_params* p, const void* q, const void* K,
                          const void* V, const int32_t* idx, const void* rb_K,
                          const void* rb_V, int32_t rb_len, int32_t rb_capacity,
                          double* out);

/* The same through a mapping table (Sec. 3.4.4 "KV cache manager": attention addresses
 * its KV groups logically, a table maps them to where they physically are).  K_pool and
 * V_pool are [n_slots, G, d]: slots of one group each, in any order and shared by all
 * problems; slot_table [B, H_kv, NG] gives the slot of logical group j of (b, kv head).
 * Group idx[m] of head h is read from slot slot_table[b, g(h), idx[m]].  The rolling
 * buffer arguments are as in oracle_sparse_attn_rb.  Returns -1 for a slot outside
 * [0, n_slots). */
int oracle_sparse_attn_paged(const orc_params* p, const void* q, const void* K_pool,
                             const void* V_pool, const int32_t* slot_table, int32_t n_slots,
                             const int32_t* idx, const void* rb_K, const void* rb_V,
                             int32_t rb_len, int32_t rb_capacity, double* out);

/* Overlap of two selections (Sec. 3.4.2: the overlap ratio between consecutive steps
 * that motivates reusing loaded groups): common[s] = number of group indices that occur
 * in both idx_prev[s, :] and idx_cur[s, :], per selection set.  Each row must hold
 * unique indices (any order). */
int oracle_selection_overlap(const orc_params* p, const int32_t* idx_prev,
                             const int32_t* idx_cur, int32_t* common);

/* Ordinary softmax attention over all N tokens. */
int oracle_dense_attn(const orc_params* p, const void* q, const void* K,
                      const void* V, double* out);

/* fp64 -> storage dtype rounding used by oracle_build_metadata (exposed so the
 * tests can pin it against hand-derived values). */
uint16_t oracle_round_to_bf16(double x);
/* the same for the 8-bit E4M3 format: nearest-even, saturating at +-448 */
uint8_t oracle_round_to_fp8_e4m3(double x);
double oracle_fp8_e4m3_value(uint8_t code);

#ifdef __cplusplus
}
#endif
#endif
