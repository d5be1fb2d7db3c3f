// C ABI of kvswap_hip: argument validation, launch planning and the entry points
// declared in include/kvswap_hip.h.  Everything here runs on the host; all checks
// are done before the first launch.
#include <math.h>

#include <mutex>
#ifdef KVS_TUNING
#include <stdlib.h>
#endif

#include "kernels.h"

namespace kvs {

namespace {

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline int round_up(int a, int b) { return ceil_div(a, b) * b; }
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Launch-shape targets.  A tuning build (-DKVS_TUNING) lets the environment override
// them for sweeps; the shipped library uses the constants.
inline int target(const char* env_name, int dflt) {
#ifdef KVS_TUNING
  if (const char* v = getenv(env_name)) {
    const int x = atoi(v);
    if (x > 0) return x;
  }
#else
  (void)env_name;
#endif
  return dflt;
}

}  // namespace

Plan make_plan(const kvs_params& p) {
  Plan pl{};
  pl.problems = p.batch * p.n_kv_heads;
  const bool joint = p.head_mode == KVS_HEADS_JOINT;
  pl.sets = joint ? p.batch : pl.problems;
  pl.kv_heads_per_set = joint ? p.n_kv_heads : 1;
  pl.ctx_rows = p.ctx_capacity > 0 ? p.ctx_capacity : p.ctx_len;
  pl.n_groups = p.ctx_len / p.group_size;
  pl.q_per_kv = p.n_q_heads / p.n_kv_heads;

  // predict: two workgroups per compute unit over the whole chip, each streaming at
  // least one full step of its waves
  const int meta_epl = p.meta_dtype == KVS_FP8_E4M3 ? 16 : (p.meta_dtype == KVS_BF16 ? 8 : 4);
  pl.meta_lanes_per_row = p.rank / meta_epl;
  pl.meta_rows_per_unit = 64 / pl.meta_lanes_per_row;
  pl.group_slots = 1;  // row slots per group in the prediction pass: G or the next power of two
  while (pl.group_slots < p.group_size) pl.group_slots *= 2;
  pl.predict_units = ceil_div(pl.n_groups * pl.group_slots, pl.meta_rows_per_unit);
  {
    const int want = ceil_div(target("KVS_PREDICT_WGS", kPredictTargetWgs), pl.sets);
    const int most = ceil_div(pl.predict_units, kPredictUnitsPerWgStep);
    const int chunks = want < 1 ? 1 : (want > most ? most : want);
    pl.predict_units_per_wg = round_up(ceil_div(pl.predict_units, chunks), kPredictUnitsPerWgStep);
    pl.predict_chunks = ceil_div(pl.predict_units, pl.predict_units_per_wg);
    // single-launch step: two prediction items per workgroup slot
    const int want_s = ceil_div(target("KVS_STEP_PREDICT_ITEMS", 2 * kStepTargetWgs), pl.sets);
    const int most_s = ceil_div(pl.predict_units, kStepPredictUnitsPerWgStep);
    const int chunks_s = want_s < 1 ? 1 : (want_s > most_s ? most_s : want_s);
    pl.step_predict_units_per_wg = round_up(ceil_div(pl.predict_units, chunks_s), kStepPredictUnitsPerWgStep);
    pl.step_predict_chunks = ceil_div(pl.predict_units, pl.step_predict_units_per_wg);
  }

  // attention: split the selected tokens of a problem over workgroups
  const int kv_epl = p.kv_dtype == KVS_BF16 ? 8 : 4;
  pl.kv_lanes_per_tok = p.head_dim / kv_epl;
  pl.kv_toks_per_unit = 64 / pl.kv_lanes_per_tok;
  pl.attn_units = ceil_div(p.n_select * p.group_size, pl.kv_toks_per_unit);
  {
    const int wgs = attn_mfma_applies(p, pl) ? kAttnMfmaTargetWgs : kAttnTargetWgs;
    const int want = ceil_div(target("KVS_ATTN_WGS", wgs), pl.problems);
    const int most = ceil_div(pl.attn_units, kAttnUnitsPerWgStep);
    int splits = want < 1 ? 1 : (want > most ? most : want);
    if (splits > kAttnMaxSplitsPerProblem) splits = kAttnMaxSplitsPerProblem;
    // (rounded to one wave's batch only: rounding to a whole workgroup step would make e.g.
    // 7 splits of 128 units out of 820 where 8 of 104 fill the chip evenly)
    pl.attn_units_per_split = round_up(ceil_div(pl.attn_units, splits), kAttnUnitsPerWave);
    pl.attn_splits = ceil_div(pl.attn_units, pl.attn_units_per_split);
    int step = ceil_div(target("KVS_STEP_ATTN_WGS", kStepTargetWgs), pl.problems);
    step = step < 1 ? 1 : (step > most ? most : step);
    if (step > kAttnMaxSplitsPerProblem) step = kAttnMaxSplitsPerProblem;
    pl.step_attn_units_per_split = round_up(ceil_div(pl.attn_units, step), kAttnUnitsPerWave);
    pl.step_attn_splits = ceil_div(pl.attn_units, pl.step_attn_units_per_split);
  }

  size_t off = 0;
  // zero-on-entry area: three counters per problem and the launch-wide words of the
  // single-launch step, then one histogram of kSelectHistBins counters per selection set
  pl.off_sync = off;
  pl.sync_arrivals = 0;
  pl.sync_pred_done = pl.problems;
  pl.sync_sel_done = 2 * pl.problems;
  pl.sync_ticket = 3 * pl.problems;
  pl.off_hist = align256((size_t)(3 * pl.problems + 4) * sizeof(int));
  pl.sync_bytes = pl.off_hist + align256((size_t)pl.sets * kSelectHistBins * sizeof(int));
  off += pl.sync_bytes;
  pl.off_gs = off;
  off += align256(((size_t)pl.sets * pl.n_groups + kSelectScorePad) * sizeof(float));
  pl.off_part_ml = off;
  const int most_splits = pl.attn_splits > pl.step_attn_splits ? pl.attn_splits : pl.step_attn_splits;
  off += align256((size_t)pl.problems * most_splits * pl.q_per_kv * 2 * sizeof(float));
  pl.off_part_o = off;
  off += align256((size_t)pl.problems * most_splits * pl.q_per_kv * p.head_dim * sizeof(float));
  pl.off_qlr = off;  // low-rank queries of the joint-head mode
  off += align256((size_t)pl.sets * p.rank * sizeof(float));
  pl.total_bytes = off;
  return pl;
}

namespace {

kvs_status check_params(const kvs_params* p, bool need_select) {
  if (!p) return KVS_ERR_NULL;
  if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1 || p->head_dim < 1 || p->rank < 1 ||
      p->ctx_len < 1 || p->group_size < 1)
    return KVS_ERR_SHAPE;
  if ((p->kv_dtype != KVS_F32 && p->kv_dtype != KVS_BF16) ||
      (p->meta_dtype != KVS_F32 && p->meta_dtype != KVS_BF16 && p->meta_dtype != KVS_FP8_E4M3) ||
      (p->reduce != KVS_REDUCE_MAX && p->reduce != KVS_REDUCE_MEAN) ||
      (p->head_mode != KVS_HEADS_SEPARATE && p->head_mode != KVS_HEADS_JOINT))
    return KVS_ERR_DTYPE;
  if (p->n_q_heads % p->n_kv_heads) return KVS_ERR_SHAPE;
  if (p->ctx_len % p->group_size) return KVS_ERR_SHAPE;
  if (p->ctx_capacity != 0 && p->ctx_capacity < p->ctx_len) return KVS_ERR_SHAPE;
  const bool joint = p->head_mode == KVS_HEADS_JOINT;
  if (p->rank > (joint ? p->n_kv_heads : 1) * p->head_dim) return KVS_ERR_SHAPE;
  if (!(p->softmax_scale >= 0.f) || isinf(p->softmax_scale)) return KVS_ERR_SHAPE;
  if (!(p->meta_scale >= 0.f) || isinf(p->meta_scale)) return KVS_ERR_SHAPE;
  const int ng = p->ctx_len / p->group_size;
  if (need_select && (p->n_select < 1 || p->n_select > ng)) return KVS_ERR_SHAPE;
  // supported set
  if (p->head_dim != 64 && p->head_dim != 128) return KVS_ERR_UNSUPPORTED;
  if (p->rank != 16 && p->rank != 32 && p->rank != 64 && p->rank != 128) return KVS_ERR_UNSUPPORTED;
  if (p->group_size > 16) return KVS_ERR_UNSUPPORTED;
  const int qpk = p->n_q_heads / p->n_kv_heads;
  if (qpk > 8) return KVS_ERR_UNSUPPORTED;
  if (ng > 32768) return KVS_ERR_UNSUPPORTED;
  // index arithmetic inside the kernels is 32-bit per problem and 64-bit across problems
  const long long rows = p->ctx_capacity > 0 ? p->ctx_capacity : p->ctx_len;
  if (rows * p->head_dim >= (1ll << 31)) return KVS_ERR_UNSUPPORTED;
  if ((long long)p->batch * p->n_kv_heads > 65535) return KVS_ERR_UNSUPPORTED;  // gridDim.y
  if (joint && (long long)p->n_kv_heads * p->head_dim > kJointMaxFlatDim) return KVS_ERR_UNSUPPORTED;
  return KVS_OK;
}

inline bool misaligned(const void* ptr) { return ((uintptr_t)ptr & 15u) != 0; }

// rolling-buffer arguments of the *_rb calls -> RollingBuffer (len 0: no buffer at all)
kvs_status check_rb(const void* rb_K, const void* rb_V, int32_t rb_len, int32_t rb_capacity,
                    RollingBuffer* rb) {
  if (rb_len < 0 || rb_capacity < 0 || rb_len > rb_capacity) return KVS_ERR_SHAPE;
  if (rb_len > kRollingBufferMaxLen) return KVS_ERR_UNSUPPORTED;
  if (rb_len == 0) return KVS_OK;
  if (!rb_K || !rb_V) return KVS_ERR_NULL;
  if (misaligned(rb_K) || misaligned(rb_V)) return KVS_ERR_ALIGN;
  rb->K = rb_K, rb->V = rb_V, rb->len = rb_len, rb->capacity = rb_capacity;
  return KVS_OK;
}

// The score histograms in the workspace, if prediction and selection hand them over for
// this many selection sets (both sides decide by this one rule), else nullptr.
int* hist_handed_over(const Plan& pl, void* workspace) {
  if (pl.sets > kHistHandOverMaxSets) return nullptr;
  return (int*)((char*)workspace + pl.off_hist);
}

kvs_status check_workspace(const Plan& pl, const void* ws, size_t bytes) {
  if (!ws || misaligned(ws) || bytes < pl.total_bytes) return KVS_ERR_WORKSPACE;
  return KVS_OK;
}

// Text of the most recent HIP error seen by this thread (diagnostics only).
thread_local const char* g_last_device_error = "";

inline kvs_status dev(hipError_t e) {
  if (e == hipSuccess) return KVS_OK;
  g_last_device_error = hipGetErrorString(e);
  return KVS_ERR_DEVICE;
}

}  // namespace
}  // namespace kvs

using namespace kvs;

extern "C" {

kvs_status kvs_check_params(const kvs_params* p) { return check_params(p, true); }

size_t kvs_workspace_bytes(const kvs_params* p) {
  if (check_params(p, true) != KVS_OK) return 0;
  return make_plan(*p).total_bytes;
}

kvs_status kvs_workspace_init(const kvs_params* p, void* workspace, size_t workspace_bytes,
                              void* stream) {
  if (!p) return KVS_ERR_NULL;
  kvs_status s = check_params(p, true);
  if (s != KVS_OK) return s;
  const Plan pl = make_plan(*p);
  if ((s = check_workspace(pl, workspace, workspace_bytes)) != KVS_OK) return s;
  return dev(launch_fill_zero((char*)workspace + pl.off_sync, pl.sync_bytes, (hipStream_t)stream));
}

kvs_status kvs_workspace_check(const kvs_params* p, const void* workspace, size_t workspace_bytes,
                               void* stream) {
  if (!p) return KVS_ERR_NULL;
  kvs_status s = check_params(p, true);
  if (s != KVS_OK) return s;
  const Plan pl = make_plan(*p);
  if ((s = check_workspace(pl, workspace, workspace_bytes)) != KVS_OK) return s;
  const int* word = (const int*)((const char*)workspace + pl.off_sync) + pl.sync_ticket + 2;
  int flag = 0;
  if ((s = dev(hipMemcpyAsync(&flag, word, sizeof(int), hipMemcpyDeviceToHost, (hipStream_t)stream))) != KVS_OK)
    return s;
  if ((s = dev(hipStreamSynchronize((hipStream_t)stream))) != KVS_OK) return s;
  if (flag != 0) {
    g_last_device_error = "a wait between workgroups of kvs_decode_step_single_launch ran out; results of that call are incomplete";
    return KVS_ERR_DEVICE;
  }
  return KVS_OK;
}

void kvs_set_wait_limit(int32_t polls) { set_fused_wait_limit(polls); }

kvs_status kvs_build_metadata_rows(const kvs_params* p, const void* K, const float* A, void* K_lr,
                                   int32_t first_row, int32_t n_rows, void* stream) {
  if (!p || !K || !A || !K_lr) return KVS_ERR_NULL;
  kvs_params q = *p;
  q.n_select = 1;  // not used by this call
  const kvs_status s = check_params(&q, false);
  if (s != KVS_OK) return s;
  if (misaligned(K) || misaligned(A) || misaligned(K_lr)) return KVS_ERR_ALIGN;
  const Plan pl = make_plan(q);
  if (first_row < 0 || n_rows < 0 || (long long)first_row + n_rows > pl.ctx_rows) return KVS_ERR_SHAPE;
  return dev(launch_build_metadata(q, pl, K, A, K_lr, first_row, n_rows, (hipStream_t)stream));
}

kvs_status kvs_build_metadata(const kvs_params* p, const void* K, const float* A, void* K_lr,
                              void* stream) {
  if (!p) return KVS_ERR_NULL;
  return kvs_build_metadata_rows(p, K, A, K_lr, 0, p->ctx_len, stream);
}

kvs_status kvs_append_group(const kvs_params* p, const void* rb_K, const void* rb_V,
                            int32_t rb_capacity, void* K, void* V, const float* A, void* K_lr,
                            void* stream) {
  if (!p || !rb_K || !rb_V || !K || !V || !A || !K_lr) return KVS_ERR_NULL;
  kvs_params q = *p;
  q.n_select = 1;  // not used by this call
  kvs_status s = check_params(&q, false);
  if (s != KVS_OK) return s;
  if (misaligned(rb_K) || misaligned(rb_V) || misaligned(K) || misaligned(V) || misaligned(A) ||
      misaligned(K_lr))
    return KVS_ERR_ALIGN;
  const Plan pl = make_plan(q);
  if (rb_capacity < q.group_size) return KVS_ERR_SHAPE;               // no complete group to move
  if ((long long)q.ctx_len + q.group_size > pl.ctx_rows) return KVS_ERR_SHAPE;  // cache is full
  RollingBuffer rb;
  rb.K = rb_K, rb.V = rb_V, rb.len = q.group_size, rb.capacity = rb_capacity;
  hipStream_t st = (hipStream_t)stream;
  if ((s = dev(launch_append_rows(q, pl, rb, K, V, st))) != KVS_OK) return s;
  return dev(launch_build_metadata(q, pl, K, A, K_lr, q.ctx_len, q.group_size, st));
}

kvs_status kvs_predict_select(const kvs_params* p, const void* q, const void* K_lr, const float* A,
                              int32_t* idx, float* group_scores, void* workspace,
                              size_t workspace_bytes, void* stream) {
  if (!p || !q || !K_lr || !A || !idx) return KVS_ERR_NULL;
  kvs_status s = check_params(p, true);
  if (s != KVS_OK) return s;
  if (misaligned(q) || misaligned(K_lr) || misaligned(A) || misaligned(idx) ||
      (group_scores && misaligned(group_scores)))
    return KVS_ERR_ALIGN;
  const Plan pl = make_plan(*p);
  if ((s = check_workspace(pl, workspace, workspace_bytes)) != KVS_OK) return s;
  float* gs = group_scores ? group_scores : (float*)((char*)workspace + pl.off_gs);
  hipStream_t st = (hipStream_t)stream;
  int* hist = hist_handed_over(pl, workspace);
  float* qlr = pl.kv_heads_per_set > 1 ? (float*)((char*)workspace + pl.off_qlr) : nullptr;
  if ((s = dev(launch_predict(*p, pl, q, K_lr, A, gs, hist, qlr, st))) != KVS_OK) return s;
  return dev(launch_topk(*p, pl, gs, idx, hist, st));
}

kvs_status kvs_predict_scores(const kvs_params* p, const void* q, const void* K_lr, const float* A,
                              float* group_scores, void* workspace, size_t workspace_bytes,
                              void* stream) {
  if (!p || !q || !K_lr || !A || !group_scores) return KVS_ERR_NULL;
  kvs_status s = check_params(p, true);
  if (s != KVS_OK) return s;
  if (misaligned(q) || misaligned(K_lr) || misaligned(A) || misaligned(group_scores))
    return KVS_ERR_ALIGN;
  const Plan pl = make_plan(*p);
  int* hist = nullptr;
  float* qlr = nullptr;
  if (!workspace && pl.kv_heads_per_set > 1) return KVS_ERR_WORKSPACE;  // holds the low-rank queries
  if (workspace) {
    if ((s = check_workspace(pl, workspace, workspace_bytes)) != KVS_OK) return s;
    hist = hist_handed_over(pl, workspace);
    if (pl.kv_heads_per_set > 1) qlr = (float*)((char*)workspace + pl.off_qlr);
  }
  return dev(launch_predict(*p, pl, q, K_lr, A, group_scores, hist, qlr, (hipStream_t)stream));
}

kvs_status kvs_select_topk(const kvs_params* p, const float* group_scores, int32_t* idx,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (!p || !group_scores || !idx) return KVS_ERR_NULL;
  kvs_status s = check_params(p, true);
  if (s != KVS_OK) return s;
  if (misaligned(group_scores) || misaligned(idx)) return KVS_ERR_ALIGN;
  const Plan pl = make_plan(*p);
  int* hist = nullptr;
  if (workspace) {
    if ((s = check_workspace(pl, workspace, workspace_bytes)) != KVS_OK) return s;
    hist = hist_handed_over(pl, workspace);
  }
  return dev(launch_topk(*p, pl, group_scores, idx, hist, (hipStream_t)stream));
}

namespace {
// shared body of the attention entry points; slot_table == nullptr: K, V are the caches
kvs_status attend(const kvs_params* p, const void* q, const void* K, const void* V,
                  const int32_t* slot_table, const int32_t* idx, const void* rb_K,
                  const void* rb_V, int32_t rb_len, int32_t rb_capacity, void* out,
                  void* workspace, size_t workspace_bytes, void* stream) {
  if (!p || !q || !K || !V || !idx || !out) return KVS_ERR_NULL;
  kvs_status s = check_params(p, true);
  if (s != KVS_OK) return s;
  RollingBuffer rb;
  if ((s = check_rb(rb_K, rb_V, rb_len, rb_capacity, &rb)) != KVS_OK) return s;
  if (misaligned(q) || misaligned(K) || misaligned(V) || misaligned(idx) || misaligned(out) ||
      (slot_table && misaligned(slot_table)))
    return KVS_ERR_ALIGN;
  const Plan pl = make_plan(*p);
  if ((s = check_workspace(pl, workspace, workspace_bytes)) != KVS_OK) return s;
  float* part_ml = (float*)((char*)workspace + pl.off_part_ml);
  float* part_o = (float*)((char*)workspace + pl.off_part_o);
  int* arrivals = (int*)((char*)workspace + pl.off_sync) + pl.sync_arrivals;
  return dev(launch_attn(*p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table,
                         (hipStream_t)stream));
}
}  // namespace

kvs_status kvs_attend_select_next_rb(const kvs_params* p, const void* q, const void* K, const void* V,
                                     const int32_t* idx, const void* rb_K, const void* rb_V,
                                     int32_t rb_len, int32_t rb_capacity, void* out,
                                     const float* next_group_scores, int32_t* next_idx, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  if (!p || !q || !K || !V || !idx || !out || !next_group_scores || !next_idx) return KVS_ERR_NULL;
  kvs_status s = check_params(p, true);
  if (s != KVS_OK) return s;
  RollingBuffer rb;
  if ((s = check_rb(rb_K, rb_V, rb_len, rb_capacity, &rb)) != KVS_OK) return s;
  if (misaligned(q) || misaligned(K) || misaligned(V) || misaligned(idx) || misaligned(out) ||
      misaligned(next_group_scores) || misaligned(next_idx))
    return KVS_ERR_ALIGN;
  const Plan pl = make_plan(*p);
  if (!attn_select_applies(*p, pl)) return KVS_ERR_UNSUPPORTED;
  if ((s = check_workspace(pl, workspace, workspace_bytes)) != KVS_OK) return s;
  float* part_ml = (float*)((char*)workspace + pl.off_part_ml);
  float* part_o = (float*)((char*)workspace + pl.off_part_o);
  int* arrivals = (int*)((char*)workspace + pl.off_sync) + pl.sync_arrivals;
  return dev(launch_attn_select(*p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, next_group_scores,
                                next_idx, hist_handed_over(pl, workspace), (hipStream_t)stream));
}

kvs_status kvs_attend_select_next(const kvs_params* p, const void* q, const void* K, const void* V,
                                  const int32_t* idx, void* out, const float* next_group_scores,
                                  int32_t* next_idx, void* workspace, size_t workspace_bytes,
                                  void* stream) {
  return kvs_attend_select_next_rb(p, q, K, V, idx, nullptr, nullptr, 0, 0, out, next_group_scores, next_idx,
                                   workspace, workspace_bytes, stream);
}

kvs_status kvs_sparse_decode_attn_rb(const kvs_params* p, const void* q, const void* K,
                                     const void* V, const int32_t* idx, const void* rb_K,
                                     const void* rb_V, int32_t rb_len, int32_t rb_capacity,
                                     void* out, void* workspace, size_t workspace_bytes,
                                     void* stream) {
  return attend(p, q, K, V, nullptr, idx, rb_K, rb_V, rb_len, rb_capacity, out, workspace,
                workspace_bytes, stream);
}

kvs_status kvs_sparse_decode_attn_paged(const kvs_params* p, const void* q, const void* K_pool,
                                        const void* V_pool, const int32_t* slot_table,
                                        int32_t n_slots, const int32_t* idx, const void* rb_K,
                                        const void* rb_V, int32_t rb_len, int32_t rb_capacity,
                                        void* out, void* workspace, size_t workspace_bytes,
                                        void* stream) {
  if (!slot_table) return KVS_ERR_NULL;
  if (n_slots < 1) return KVS_ERR_SHAPE;
  return attend(p, q, K_pool, V_pool, slot_table, idx, rb_K, rb_V, rb_len, rb_capacity, out,
                workspace, workspace_bytes, stream);
}

kvs_status kvs_selection_overlap(const kvs_params* p, const int32_t* idx_prev,
                                 const int32_t* idx_cur, int32_t* common, void* stream) {
  if (!p || !idx_prev || !idx_cur || !common) return KVS_ERR_NULL;
  const kvs_status s = check_params(p, true);
  if (s != KVS_OK) return s;
  if (misaligned(idx_prev) || misaligned(idx_cur) || misaligned(common)) return KVS_ERR_ALIGN;
  const Plan pl = make_plan(*p);
  return dev(launch_overlap(*p, pl, idx_prev, idx_cur, common, (hipStream_t)stream));
}

kvs_status kvs_sparse_decode_attn(const kvs_params* p, const void* q, const void* K, const void* V,
                                  const int32_t* idx, void* out, void* workspace,
                                  size_t workspace_bytes, void* stream) {
  return kvs_sparse_decode_attn_rb(p, q, K, V, idx, nullptr, nullptr, 0, 0, out, workspace,
                                   workspace_bytes, stream);
}

kvs_status kvs_decode_step_rb(const kvs_params* p, const void* q, const void* K_lr, const float* A,
                              const void* K, const void* V, const void* rb_K, const void* rb_V,
                              int32_t rb_len, int32_t rb_capacity, int32_t* idx,
                              float* group_scores, void* out, void* workspace,
                              size_t workspace_bytes, void* stream) {
  if (!p || !q || !K_lr || !A || !K || !V || !idx || !out) return KVS_ERR_NULL;
  RollingBuffer rb;  // validated before anything is launched
  kvs_status s = check_rb(rb_K, rb_V, rb_len, rb_capacity, &rb);
  if (s != KVS_OK) return s;
  if (misaligned(K) || misaligned(V) || misaligned(out)) return KVS_ERR_ALIGN;
  s = kvs_predict_select(p, q, K_lr, A, idx, group_scores, workspace, workspace_bytes, stream);
  if (s != KVS_OK) return s;
  return kvs_sparse_decode_attn_rb(p, q, K, V, idx, rb_K, rb_V, rb_len, rb_capacity, out,
                                   workspace, workspace_bytes, stream);
}

kvs_status kvs_decode_step_single_launch(const kvs_params* p, const void* q, const void* K_lr,
                                         const float* A, const void* K, const void* V, int32_t* idx,
                                         float* group_scores, void* out, void* workspace,
                                         size_t workspace_bytes, void* stream) {
  if (!p || !q || !K_lr || !A || !K || !V || !idx || !out) return KVS_ERR_NULL;
  kvs_status s = check_params(p, true);
  if (s != KVS_OK) return s;
  if (misaligned(q) || misaligned(K_lr) || misaligned(A) || misaligned(K) || misaligned(V) ||
      misaligned(idx) || misaligned(out) || (group_scores && misaligned(group_scores)))
    return KVS_ERR_ALIGN;
  const Plan pl = make_plan(*p);
  if (!fused_step_applies(*p, pl)) return KVS_ERR_UNSUPPORTED;
  if ((s = check_workspace(pl, workspace, workspace_bytes)) != KVS_OK) return s;
  char* ws = (char*)workspace;
  return dev(launch_fused_step(*p, pl, q, K_lr, A, K, V, (float*)(ws + pl.off_gs), group_scores, idx,
                               (float*)(ws + pl.off_part_ml), (float*)(ws + pl.off_part_o), out,
                               (int*)(ws + pl.off_sync), (hipStream_t)stream));
}

kvs_status kvs_decode_step(const kvs_params* p, const void* q, const void* K_lr, const float* A,
                           const void* K, const void* V, int32_t* idx, float* group_scores,
                           void* out, void* workspace, size_t workspace_bytes, void* stream) {
  return kvs_decode_step_rb(p, q, K_lr, A, K, V, nullptr, nullptr, 0, 0, idx, group_scores, out,
                            workspace, workspace_bytes, stream);
}

}  // extern "C"

// ---- a whole decode step for callers that cannot allocate ------------------------------------
// The scratch memory of the step's kernels (arrival counters, score histograms, group scores,
// split partial results) lives in a device array of the library itself instead of a caller's
// workspace.  Every GPU the library runs on holds its own copy of the array, at its own
// address; in host code the array's name is only a handle for hipGetSymbolAddress, never a
// device address.
static __device__ __align__(256) unsigned char scratch[KVS_STATIC_SCRATCH_BYTES];

namespace kvs {
namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device, looked up once

// Address of the current device's copy of the array (set-up on the first call per device).
kvs_status static_scratch(void** ptr_out) {
  int device = -1;
  kvs_status s = dev(hipGetDevice(&device));
  if (s != KVS_OK) return s;
  if (device < 0 || device >= kMaxDevices) return KVS_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    if ((s = dev(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)))) != KVS_OK) return s;
    if (!ptr) return KVS_ERR_DEVICE;
    g_scratch_ptr[device] = ptr;
  }
  *ptr_out = g_scratch_ptr[device];
  return KVS_OK;
}

}  // namespace
}  // namespace kvs

extern "C" {

kvs_status kvs_decode_step_static(const kvs_params* p, const void* q, const void* K_lr,
                                  const float* A, const void* K, const void* V, int32_t* idx,
                                  float* group_scores, void* out, void* stream) {
  if (!p || !q || !K_lr || !A || !K || !V || !idx || !out) return KVS_ERR_NULL;
  kvs_status s = check_params(p, true);
  if (s != KVS_OK) return s;
  const Plan pl = make_plan(*p);
  if (pl.total_bytes > (size_t)KVS_STATIC_SCRATCH_BYTES) return KVS_ERR_SCRATCH;
  void* ptr = nullptr;
  if ((s = static_scratch(&ptr)) != KVS_OK) return s;
  // The array keeps whatever the last call on this device left (possibly of another shape,
  // whose counter area was laid out differently): the counters of this call start at zero.
  if ((s = dev(launch_fill_zero((char*)ptr + pl.off_sync, pl.sync_bytes, (hipStream_t)stream))) != KVS_OK)
    return s;
  return kvs_decode_step(p, q, K_lr, A, K, V, idx, group_scores, out, ptr,
                         (size_t)KVS_STATIC_SCRATCH_BYTES, stream);
}

const char* kvs_status_str(kvs_status s) {
  switch (s) {
    case KVS_OK: return "ok";
    case KVS_ERR_NULL: return "a required pointer is NULL";
    case KVS_ERR_SHAPE: return "inconsistent sizes";
    case KVS_ERR_DTYPE: return "unknown dtype, reduce or head-mode code";
    case KVS_ERR_UNSUPPORTED: return "shape outside the supported set";
    case KVS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case KVS_ERR_DEVICE: return "HIP launch failed";
    case KVS_ERR_ALIGN: return "a tensor pointer is not 16-byte aligned";
    case KVS_ERR_SCRATCH: return "the problem needs more scratch memory than the library's static buffer holds";
  }
  return "unknown status";
}

const char* kvs_last_device_error(void) { return g_last_device_error; }

const char* kvs_version(void) { return "kvswap_hip 0.1 gfx950"; }

}  // extern "C"
