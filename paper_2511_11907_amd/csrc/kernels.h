// Internal launch interface between the C-ABI layer (api.hip) and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/kvswap_hip.h"

namespace kvs {

// Work granules of the streaming kernels (units = wave-wide 1 KiB loads).
// (prediction: 1024-lane workgroups whose 16 waves share the workgroup's rows dynamically,
// two per compute unit, four loads in flight per wave: at the 128K workload 79.9 us against
// 85.4 us for four 512-lane workgroups per compute unit with a fixed split over the waves)
constexpr int kPredictWgThreads = 1024;
constexpr int kPredictUnitsPerWgStep = (kPredictWgThreads / 64) * 4;  // 16 waves x 4 loads in flight (54-64 registers: two workgroups per CU)
constexpr int kPredictTargetWgs = 512;         // two 1024-lane workgroups per CU, all resident (256: the same; 1024 x 512 lanes: slower)
// (512-lane attention workgroups: in one run, same 512-workgroup grid, 256 -> 512 lanes took
// c4 from 64.8 to 58.6 us and c2 from 16.1 to 13.5 us, c3 unchanged)
#ifndef KVS_ATTN_THREADS
#define KVS_ATTN_THREADS 512
#endif
constexpr int kAttnWgThreads = KVS_ATTN_THREADS;
constexpr int kAttnUnitsPerWave = 4;  // (K,V) load pairs a wave keeps in flight (5: no gain, 6: spills)
constexpr int kAttnUnitsPerWgStep = (kAttnWgThreads / 64) * kAttnUnitsPerWave;
constexpr int kSelectScorePad = 2304;           // floats of padding behind the workspace's group scores
// Up to this many selection sets the prediction kernel also accumulates the sets' score
// histograms for the selection kernel (measured: with 8 sets the selection is 0.2 us shorter for it,
// with 32 it makes no difference, with 64 or 128 the prediction kernel's extra atomics cost
// 1 us more than the selection saves).
constexpr int kHistHandOverMaxSets = 32;
constexpr int kSelectHistBins = 4096;          // per-problem histogram of the top 12 key bits
// The matrix-core attention kernel (bf16, d = 128) takes over from this many query heads
// per KV head on (measured: level with the vector-ALU kernel at 1 and 2, 5 % faster at 3,
// 12 % at 4, 20 % at 5, 45 % at 7 and 8), with one workgroup per compute unit as its target
// (swept 128 ... 1024: 256 is best at 32K and 128K contexts).
#ifndef KVS_ATTN_MFMA_MIN_QPK
#define KVS_ATTN_MFMA_MIN_QPK 3
#endif
constexpr int kAttnMfmaMinHeadsPerKv = KVS_ATTN_MFMA_MIN_QPK;
constexpr int kAttnMfmaTargetWgs = 256;
constexpr int kAttnInterleaveFromSteps = 12;   // workgroup steps per split from which the splits are interleaved
#ifndef KVS_STEP_PREDICT_UNROLL
#define KVS_STEP_PREDICT_UNROLL 8
#endif
constexpr int kStepPredictUnroll = KVS_STEP_PREDICT_UNROLL;  // wave-loads in flight per wave in the single-launch step (16 waves per compute unit)
constexpr int kStepPredictUnitsPerWgStep = 8 * kStepPredictUnroll;
constexpr int kStepTargetWgs = 512;            // workgroup slots of the single-launch step on 256 compute units
constexpr int kAttnTargetWgs = 512;            // measured best: fewer, longer splits (less merge traffic)
constexpr int kAttnMaxSplitsPerProblem = 256;   // the merge keeps one weight per split in LDS
constexpr int kMetaMfmaTargetWgs = 512;          // workgroups of the matrix-core metadata kernel: two per compute unit (measured best)
constexpr int kJointMaxFlatDim = 4096;          // H_kv * d the query projection kernel stages in LDS

// Launch geometry derived from the params alone (the host computes it once per
// call; kvs_workspace_bytes uses the same numbers).
// The newest tokens of every (b, kv head), kept outside the cache until they form a
// group (Sec. 3.4.1): K, V [B, H_kv, capacity, d], the first `len` rows valid.
struct RollingBuffer {
  const void* K = nullptr;
  const void* V = nullptr;
  int len = 0;
  int capacity = 0;
};
constexpr int kRollingBufferMaxLen = 256;

struct Plan {
  int problems;          // P = B * H_kv: attention problems
  int sets;              // selection sets: P, or B in joint-head mode (one K_lr, one idx each)
  int kv_heads_per_set;  // 1, or H_kv in joint-head mode
  int ctx_rows;          // rows held per problem by K, V and K_lr (>= N)
  int n_groups;          // NG = N / G
  int q_per_kv;          // H_q / H_kv
  // predict
  int meta_lanes_per_row;   // lanes of 16 B that cover one K_lr row
  int meta_rows_per_unit;   // rows covered by one wave-wide 1 KiB load
  int group_slots;          // row slots per group in the prediction pass (G, or the next power of two)
  int predict_units;        // wave-loads per problem
  int predict_units_per_wg;
  int predict_chunks;       // workgroups per problem
  // the same for the single-launch step (its workgroups keep more loads in flight per wave,
  // so its workgroup step is longer)
  int step_predict_units_per_wg;
  int step_predict_chunks;
  // attention
  int kv_lanes_per_tok;     // lanes of 16 B that cover one K (or V) row
  int kv_toks_per_unit;     // tokens covered by one wave-wide load
  int attn_units;           // wave-loads (of K, and as many of V) per problem
  int attn_units_per_split;
  int attn_splits;          // workgroups per problem
  // the same for the single-launch step, whose attention items share the grid's workgroup
  // slots with everything else: one item per slot (two per compute unit) where the problems
  // are long enough, so that the slots stay evenly loaded
  int step_attn_units_per_split;
  int step_attn_splits;
  // workspace layout (byte offsets, 256-byte aligned).  The counter area at off_sync
  // (sync_bytes long: the counters below, then the score histograms at off_hist) must be zero
  // when a call starts; every call leaves it zero.
  size_t off_sync, sync_bytes, off_hist, off_gs, off_part_ml, off_part_o, off_qlr, total_bytes;
  // counters at the start of that area, as int offsets from off_sync: per problem the arrival
  // counter of the attention splits, the count of finished prediction chunks and the
  // selection-done flag; then three launch-wide words of the single-launch step (next work
  // item, workgroups that have left, error)
  int sync_arrivals, sync_pred_done, sync_sel_done, sync_ticket;
};

Plan make_plan(const kvs_params& p);

// rows [first_row, first_row + n_rows) of every selection set
hipError_t launch_build_metadata(const kvs_params& p, const Plan& pl, const void* K,
                                 const float* A, void* K_lr, int first_row, int n_rows,
                                 hipStream_t st);
// cache rows [N, N + G) of every (b, kv head) <- the first G rows of its rolling buffer
hipError_t launch_append_rows(const kvs_params& p, const Plan& pl, const RollingBuffer& rb,
                              void* K, void* V, hipStream_t st);
// hist == nullptr: scores only.  Otherwise the kernel also adds the histogram of the top
// 12 key bits of every score to `hist` (kSelectHistBins ints per problem, zero on entry).
// qlr: joint-head mode only (nullptr otherwise): pl.sets * r floats of scratch that receive
// the low-rank queries from a small projection kernel launched first.
hipError_t launch_predict(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                          const float* A, float* gs, int* hist, float* qlr, hipStream_t st);
// hist == nullptr: the selection builds its own histogram.  Otherwise it starts from the
// finished per-problem histograms and leaves them zeroed.
hipError_t launch_topk(const kvs_params& p, const Plan& pl, const float* gs, int32_t* idx,
                       int* hist, hipStream_t st);
hipError_t launch_attn(const kvs_params& p, const Plan& pl, const void* q, const void* K,
                       const void* V, const int32_t* idx, float* part_ml, float* part_o,
                       void* out, int* arrivals, const RollingBuffer& rb, const int32_t* slot_table,
                       hipStream_t st);
// Matrix-core variant of the attention kernel (bf16 keys/values, d = 128): whether it is
// the one to run for these parameters, and its launch (same arguments as launch_attn).
bool attn_mfma_applies(const kvs_params& p, const Plan& pl);
hipError_t launch_attn_mfma(const kvs_params& p, const Plan& pl, const void* q, const void* K,
                       const void* V, const int32_t* idx, float* part_ml, float* part_o,
                       void* out, int* arrivals, const RollingBuffer& rb, const int32_t* slot_table,
                       hipStream_t st);
// slot_table != nullptr: K and V are pools [n_slots, G, d] and slot_table [P, NG] maps the
// logical groups of each problem to slots (Sec. 3.4.4).
// common[s] = |idx_prev[s,:] ∩ idx_cur[s,:]| per selection set
hipError_t launch_overlap(const kvs_params& p, const Plan& pl, const int32_t* idx_prev,
                          const int32_t* idx_cur, int32_t* common, hipStream_t st);
hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t st);

// The attention of one layer and the selection for the next in one launch (matrix-core
// attention layouts, at most 16384 groups per set): whether it covers these parameters, and
// its launch.  hist as in launch_topk.
bool attn_select_applies(const kvs_params& p, const Plan& pl);
hipError_t launch_attn_select(const kvs_params& p, const Plan& pl, const void* q, const void* K, const void* V,
                              const int32_t* idx, float* part_ml, float* part_o, void* out, int* arrivals,
                              const RollingBuffer& rb, const float* next_gs, int32_t* next_idx, int* hist,
                              hipStream_t st);

// The whole step (prediction, selection, attention) as one launch of a persistent grid:
// whether it covers these parameters, and its launch.  gs: the workspace's score area (the
// selection items read a little beyond its end, into the padding make_plan leaves there);
// gs_copy: nullable, the caller's array that receives the scores as well; sync: the counter
// area of the workspace (zero on entry, left zero).  Same results, bit for bit, as launch_predict + launch_topk + launch_attn.
bool fused_step_applies(const kvs_params& p, const Plan& pl);
hipError_t launch_fused_step(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                             const float* A, const void* K, const void* V, float* gs, float* gs_copy,
                             int32_t* idx, float* part_ml, float* part_o, void* out, int* sync,
                             hipStream_t st);
// Bound of the in-kernel waits of that launch, in polls (<= 0: the default).
void set_fused_wait_limit(int polls);

}  // namespace kvs
