// One launch for a whole decode step (Sec. 3.3 prediction and selection, Sec. 3.4 attention over
// the selected groups): prediction, top-M selection and gathered attention of all (sequence,
// KV head) problems run as work items of one persistent grid instead of three dependent
// launches.
//
// The idea: the three phases of one problem depend on each other, but the problems do not.  As
// three launches every phase waits for the slowest workgroup of the previous one, the
// latency-bound selection (5 us of dependent steps on a few KiB) sits between the two
// streaming kernels with the memory system idle, and each launch pays its own ramp-up and
// drain.  Here a workgroup draws work items from one counter, in an order that puts the
// selection of a problem behind the prediction of later problems and all attention items at
// the end, so that selections run while other workgroups stream, and the attention of the
// first problems starts while the last predictions drain.
//
// Work items, in draw order (P problems, C prediction chunks and S attention splits each, D
// = the number of problems whose prediction items the grid holds at once):
//   predict(0..D-1, all chunks); then for s = D..P-1: predict(s, all chunks), select(s - D);
//   select(P-D..P-1); attend(0..P-1, all splits).
// Dependencies: select(p) needs the C chunks of predict(p) (counter pred_done[p]); attend(p, *)
// needs select(p) (flag sel_done[p]).  An item only ever waits for items drawn before it, which
// are held by workgroups that are already running: whatever the number of resident
// workgroups, the item with the lowest unfinished ticket never waits for an unfinished one,
// so the grid always drains.  Waits are bounded all the same: a wait that runs out sets the
// error word of the workspace, the item and its dependants are skipped, every workgroup still
// leaves.
//
// Which workgroup runs which item depends on timing; what an item computes does not: scores
// and indices are functions of the inputs alone and equal those of the three separate
// launches bit for bit; every attention split sums a fixed set of tokens in a fixed order
// and the splits are merged in index order, so the outputs are reproducible bit for bit.
// They differ from the three launches' outputs in the last fp32 roundings only, because this
// launch cuts a problem's selected tokens into its own number of splits.
//
// Measured on an MI355X this form is slower than the three launches at every benchmark
// shape (a memory round trip takes several times longer inside a grid that saturates the
// memory system, and the selection is a chain of such round trips), so the library's default
// step keeps the three launches and this launch is an entry point of its own.
//
// Values that cross workgroups inside the launch (group scores, selected indices, split
// partial results, counters) move with device-scope stores and loads (see device_utils.h);
// K_lr, K, V, q and the adapter are read-only and are read normally.
#include <hip/hip_runtime.h>
#include <stddef.h>

// Work-item timestamps for the debugging harness (compiled only with -DKVS_FUSED_TRACE_BUILD):
// one row of 8 words per work item: kind, problem, part, workgroup, start, dependencies
// met, done, compute unit.
#ifdef KVS_FUSED_TRACE_BUILD
static __device__ long long g_fused_select_trace[512 * 8];
#define KVS_TOPK_TRACE(i)                                                                    \
  do {                                                                                       \
    if (threadIdx.x == 0) g_fused_select_trace[(blockIdx.x & 511) * 8 + (i)] = wall_clock64(); \
  } while (0)
extern "C" int kvs_debug_fused_select_trace(long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_fused_select_trace), sizeof(long long) * (size_t)n);
}
static __device__ long long g_fused_predict_trace[512 * 8];
#define KVS_PREDICT_TRACE(i)                                                                  \
  do {                                                                                        \
    if (threadIdx.x == 0) g_fused_predict_trace[(blockIdx.x & 511) * 8 + (i)] = wall_clock64(); \
  } while (0)
extern "C" int kvs_debug_fused_predict_trace(long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_fused_predict_trace), sizeof(long long) * (size_t)n);
}
static __device__ long long g_fused_trace[8 << 14];
extern "C" int kvs_debug_fused_trace(long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_fused_trace), sizeof(long long) * (size_t)n);
}
#define KVS_FUSED_TRACE(item, slot, value)                                                  \
  do {                                                                                      \
    if (threadIdx.x == 0 && (item) < (1 << 14)) g_fused_trace[(item) * 8 + (slot)] = (value); \
  } while (0)
#else
#define KVS_FUSED_TRACE(item, slot, value)
#endif

#include "attn_mfma_item.h"
#include "predict_item.h"

namespace kvs {

constexpr int kFusedThreads = 512;
static_assert(kFusedThreads == kStepPredictThreads && kFusedThreads == kAttnThreads, "one workgroup size for all items");
constexpr int kFusedSelCap = 4096;        // selected groups per problem the attention items hold in LDS
constexpr int kFusedMaxGroups = kFusedThreads * kTopkMaxPerLane;  // 16384 scores per problem
constexpr int kFusedWgsPerCu = 2;         // 128 registers per lane, < 80 KiB of LDS

struct FusedArgs {
  int* ticket;     // next work item to draw (beyond the first gridDim.x, which are dealt by blockIdx)
  int* pred_done;  // [P] prediction chunks of the problem that have published their scores
  int* sel_done;   // [P] 1: the selection of the problem is published, 2: it was given up
  int* error;      // sticky: set when a wait ran out
  float* gs;       // [P, NG]
  int32_t* idx;    // [P, M]
  int P, C, S, D, n_items, NG, M, spin_limit;
};

// Thread 0 polls *flag (device scope) until it is at least `need`, at most `limit` times; every
// lane gets the last value read.  One barrier.
__device__ __forceinline__ int wait_until(const int* flag, int need, int limit, int* s_slot) {
  if (threadIdx.x == 0) {
    int v = load_published(flag);
    for (int n = 1; v < need && n < limit; ++n) {
      __builtin_amdgcn_s_sleep(16);
      v = load_published(flag);
    }
    *s_slot = v;
  }
  lds_barrier();
  const int v = __builtin_amdgcn_readfirstlane(*s_slot);  // (uniform, and known to be)
  consume_fence();
  return v;
}

// All arguments of the launch as one structure: the single kernel argument.  The work-item
// functions below read the member they need from the kernel-argument segment themselves.
struct StepArgs {
  PredictArgs predict;
  AttnMfmaArgs attn;
  FusedArgs fused;
};

// The address of the kernel-argument segment.  Only a kernel can ask for it (inside a
// function that is not inlined the compiler's intrinsic yields a null pointer), so the kernel
// hands it to the work-item functions as two 32-bit halves.
struct ArgSegment {
  uint32_t lo, hi;
};
__device__ __forceinline__ ArgSegment kernel_arg_segment() {
  const uint64_t a = (uint64_t)(uintptr_t)__builtin_amdgcn_kernarg_segment_ptr();
  return ArgSegment{(uint32_t)a, (uint32_t)(a >> 32)};
}

// One member of the argument structure, read from the kernel-argument segment (constant
// address space, scalar loads).
template <class T>
__device__ __forceinline__ T read_step_args(ArgSegment seg, size_t offset) {
  typedef const uint32_t __attribute__((address_space(4))) const_word;
  static_assert(sizeof(T) % 4 == 0, "copied word by word");
  const uint64_t address = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)seg.hi) << 32) |
                           (uint32_t)__builtin_amdgcn_readfirstlane((int)seg.lo);
  const_word* base = (const_word*)(uintptr_t)address;
  T out;
  uint32_t* words = reinterpret_cast<uint32_t*>(&out);
#pragma unroll
  for (size_t i = 0; i < sizeof(T) / 4; ++i) words[i] = base[offset / 4 + i];
  return out;
}
#define KVS_STEP_ARGS(seg, member) read_step_args<decltype(StepArgs::member)>(seg, offsetof(StepArgs, member))

// The three kinds of work item are functions of their own (not inlined into the kernel's
// loop): each then gets the register allocation it has as a kernel of its own - the
// attention item needs all 128 registers, the selection up to 32 keys per lane and many
// uniform values - instead of one allocation over the union of the three, which spills
// inside the streaming loops.  A function's arguments arrive in vector registers; they are
// uniform, and are told to be.  The LDS block travels as an LDS pointer so that the
// routines' accesses to it stay LDS instructions.
__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }
template <class T>
__device__ __forceinline__ T& lds_block(uint32_t lds_address) {
  typedef T __attribute__((address_space(3))) * lds_ptr;
  return *(T*)(lds_ptr)(uintptr_t)uniform((int)lds_address);
}
template <class T>
__device__ __forceinline__ uint32_t lds_address_of(T& block) {
  typedef T __attribute__((address_space(3))) * lds_ptr;
  return (uint32_t)(uintptr_t)(lds_ptr)&block;
}

template <typename E, int R, int G, bool PAD>
__device__ __noinline__ void predict_work(ArgSegment seg, int p_in, int chunk_in, uint32_t lds) {
  const int p = uniform(p_in), chunk = uniform(chunk_in);
  KVS_PREDICT_TRACE(0);
  const PredictArgs pa = KVS_STEP_ARGS(seg, predict);
  predict_item<E, R, G, false, PAD, true, kStepPredictUnroll, kFusedThreads>(
      lds_block<PredictShared<E, R, G, false, kStepPredictUnroll, kFusedThreads>>(lds), pa, p, chunk);
  publish_complete_and_barrier();  // the scores are out before the chunk is counted
  KVS_PREDICT_TRACE(4);
  if (threadIdx.x == 0) atomicAdd(as_global(KVS_STEP_ARGS(seg, fused).pred_done) + p, 1);
  KVS_PREDICT_TRACE(5);
}

// (the caller has waited for the problem's prediction chunks: ready = whether they all came)
__device__ __noinline__ void select_work(ArgSegment seg, int p_in, uint32_t lds, int ready_in) {
  const int p = uniform(p_in), ready = uniform(ready_in);
  const FusedArgs fa = KVS_STEP_ARGS(seg, fused);
  int* pred_done = as_global(fa.pred_done) + p;
  int* sel_done = as_global(fa.sel_done) + p;
  if (ready) {  // uniform
    if (threadIdx.x == 0) publish_store(pred_done, 0);  // (its only reader; ready for the next call)
    const float* g = as_global(fa.gs) + (size_t)p * fa.NG;
    int32_t* out = as_global(fa.idx) + (size_t)p * fa.M;
    TopkShared& sh = lds_block<TopkShared>(lds);
    if (fa.NG <= kFusedThreads * 16) topk_block<16, kFusedThreads, true>(g, out, fa.NG, fa.M, nullptr, sh);
    else topk_block<kTopkMaxPerLane, kFusedThreads, true>(g, out, fa.NG, fa.M, nullptr, sh);
    publish_complete_and_barrier();  // the indices are out before the flag goes up
    if (threadIdx.x == 0) publish_store(sel_done, 1);
  } else if (threadIdx.x == 0) {
    publish_store(as_global(fa.error), 1);
    publish_store(sel_done, 2);
  }
}

// (the caller has waited for the problem's selection)
template <int QPK, bool INTERLEAVE>
__device__ __noinline__ void attend_work(ArgSegment seg, int p_in, int split_in, uint32_t lds) {
  const int p = uniform(p_in), split = uniform(split_in);
  const AttnMfmaArgs aa = KVS_STEP_ARGS(seg, attn);
  const bool wrote = attn_mfma_item<QPK, kAttnPlain, INTERLEAVE, kFusedSelCap>(
      lds_block<AttnMfmaShared<QPK, kFusedSelCap>>(lds), aa, p, split);
  // every split has read the flag; ready for the next call
  if (wrote && threadIdx.x == 0) publish_store(as_global(KVS_STEP_ARGS(seg, fused).sel_done) + p, 0);
}

template <typename E, int R, int G, bool PAD, int QPK, bool INTERLEAVE>
__global__ __launch_bounds__(kFusedThreads, 4) void decode_step_kernel(StepArgs all_args) {
  union Shared {
    PredictShared<E, R, G, false, kStepPredictUnroll, kFusedThreads> predict;
    TopkShared topk;
    AttnMfmaShared<QPK, kFusedSelCap> attn;
  };
  __shared__ Shared sh;
  __shared__ int s_next;
  __shared__ int s_seen;
  (void)all_args;  // (read from the argument segment, here and in the work-item functions)
  const int tid = threadIdx.x;
  const ArgSegment seg = kernel_arg_segment();
  const FusedArgs fa = KVS_STEP_ARGS(seg, fused);
  const int first_mixed = fa.D * fa.C;                               // items before the first selection
  const int first_tail = first_mixed + (fa.P - fa.D) * (fa.C + 1);   // the last D selections
  const int first_attn = first_tail + fa.D;
  for (int item = blockIdx.x; item < fa.n_items;) {
    int kind, p, part;  // 0 predict(p, chunk), 1 select(p), 2 attend(p, split)
    if (item < first_mixed) {
      kind = 0, p = item / fa.C, part = item % fa.C;
    } else if (item < first_tail) {
      const int t = item - first_mixed, s = t / (fa.C + 1), r = t % (fa.C + 1);
      if (r < fa.C) kind = 0, p = fa.D + s, part = r;
      else kind = 1, p = s, part = 0;
    } else if (item < first_attn) {
      kind = 1, p = fa.P - fa.D + (item - first_tail), part = 0;
    } else {
      const int t = item - first_attn;
      kind = 2, p = t / fa.S, part = t % fa.S;
    }
    KVS_FUSED_TRACE(item, 0, kind);
    KVS_FUSED_TRACE(item, 1, p);
    KVS_FUSED_TRACE(item, 2, part);
    KVS_FUSED_TRACE(item, 3, blockIdx.x);
    KVS_FUSED_TRACE(item, 4, wall_clock64());
    KVS_FUSED_TRACE(item, 7, ((long long)__builtin_amdgcn_s_getreg((31 << 11) | 20) << 32) | (unsigned)__builtin_amdgcn_s_getreg((31 << 11) | 4));
    if (kind == 0) predict_work<E, R, G, PAD>(seg, p, part, lds_address_of(sh.predict));
    else if (kind == 1) {
      const int seen = wait_until(as_global(fa.pred_done) + p, fa.C, fa.spin_limit, &s_seen);
      KVS_FUSED_TRACE(item, 5, wall_clock64());
      select_work(seg, p, lds_address_of(sh.topk), seen >= fa.C);
    } else {
      const int seen = wait_until(as_global(fa.sel_done) + p, 1, fa.spin_limit, &s_seen);
      KVS_FUSED_TRACE(item, 5, wall_clock64());
      if (seen == 1) attend_work<QPK, INTERLEAVE>(seg, p, part, lds_address_of(sh.attn));  // uniform
      else if (tid == 0) publish_store(as_global(fa.error), 1);
    }
    KVS_FUSED_TRACE(item, 6, wall_clock64());
    // the next work item
    if (tid == 0) s_next = atomicAdd(as_global(fa.ticket), 1);
    lds_barrier();  // (also: the item's LDS is free for the next one)
    const int drawn = uniform(s_next);
    lds_barrier();  // (s_next is read before the next round rewrites it)
    // Every workgroup draws once per item it takes and once more to learn that nothing is
    // left: n_items draws in all.  Whoever makes the last of them knows that every other
    // workgroup has made its last draw, i.e. has finished: it puts the counter back to zero.
    if (drawn == fa.n_items - 1 && tid == 0) publish_store(as_global(fa.ticket), 0);
    item = (int)gridDim.x + drawn;
  }
}

namespace {

constexpr int kDefaultWaitLimit = 1 << 19;  // about a second: a poll is a memory round trip plus a short sleep
int g_wait_limit = kDefaultWaitLimit;      // polls of one in-kernel wait

int compute_units(hipError_t* err) {
  static int cached[64];
  int dev = 0;
  if ((*err = hipGetDevice(&dev)) != hipSuccess) return 0;
  if (dev < 0 || dev >= 64) return 256;
  if (!cached[dev]) {
    int n = 0;
    if ((*err = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return 0;
    cached[dev] = n > 0 ? n : 256;
  }
  return cached[dev];
}

template <typename E, int R, int G, int QPK>
hipError_t launch_fused_one(const kvs_params& p, const Plan& pl, const PredictArgs& pa, const AttnMfmaArgs& aa,
                            FusedArgs fa, hipStream_t st) {
  static_assert(offsetof(StepArgs, predict) == 0, "the kernel reads its argument segment as a StepArgs");
  hipError_t err = hipSuccess;
  const int cus = compute_units(&err);
  if (err != hipSuccess) return err;
  // prediction items of as many problems as the grid holds at once come before the first selection
  const int grid = fa.n_items < kFusedWgsPerCu * cus ? fa.n_items : kFusedWgsPerCu * cus;
  int D = (grid + fa.C - 1) / fa.C;
  fa.D = D < 1 ? 1 : (D > fa.P ? fa.P : D);
  const bool interleave = aa.units_per_split >= kAttnInterleaveFromSteps * kAttnUnitsPerWgStep;
  const StepArgs all{pa, aa, fa};
  if (interleave)
    hipLaunchKernelGGL((decode_step_kernel<E, R, G, false, QPK, true>), dim3(grid), dim3(kFusedThreads), 0, st, all);
  else
    hipLaunchKernelGGL((decode_step_kernel<E, R, G, false, QPK, false>), dim3(grid), dim3(kFusedThreads), 0, st, all);
  return hipGetLastError();
}

}  // namespace

void set_fused_wait_limit(int polls) { g_wait_limit = polls > 0 ? polls : kDefaultWaitLimit; }

bool fused_step_applies(const kvs_params& p, const Plan& pl) {
  if (p.head_mode != KVS_HEADS_SEPARATE || p.meta_dtype != KVS_BF16) return false;
  if (!attn_mfma_applies(p, pl) || pl.q_per_kv != 4) return false;
  if (!((p.rank == 32 && p.group_size == 4) || (p.rank == 64 && p.group_size == 8))) return false;
  if (pl.n_groups > kFusedMaxGroups || p.n_select > kFusedSelCap) return false;
  return true;
}

hipError_t launch_fused_step(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                             const float* A, const void* K, const void* V, float* gs, float* gs_copy,
                             int32_t* idx, float* part_ml, float* part_o, void* out, int* sync, hipStream_t st) {
  using S = uint16_t;
  const float mscale = p.meta_scale != 0.f ? p.meta_scale : 1.0f;
  const PredictArgs pa{q, (int)(p.kv_dtype == KVS_BF16), K_lr, A, gs, gs_copy, p.n_kv_heads, pl.q_per_kv, p.head_dim,
                       pl.n_groups, p.group_size, pl.ctx_rows, pl.predict_units, pl.step_predict_units_per_wg,
                       (int)(p.reduce == KVS_REDUCE_MEAN), nullptr, nullptr, mscale, p.meta_scales};
  const int G = p.group_size;
  int log2G = 0;
  while ((1 << log2G) < G) ++log2G;
  const float scale = p.softmax_scale != 0.f ? p.softmax_scale : 1.0f / sqrtf((float)p.head_dim);
  const AttnMfmaArgs aa{(const S*)q, (const S*)K, (const S*)V, idx, part_ml, part_o, (S*)out,
                        sync + pl.sync_arrivals, p.n_kv_heads, 1, pl.ctx_rows, p.n_select, G, log2G, 0u,
                        pl.attn_units, pl.step_attn_units_per_split, pl.step_attn_splits, scale * kLog2e,
                        nullptr, nullptr, 0, 0, nullptr, pl.n_groups};
  FusedArgs fa{};
  fa.ticket = sync + pl.sync_ticket;
  fa.error = sync + pl.sync_ticket + 2;
  fa.pred_done = sync + pl.sync_pred_done;
  fa.sel_done = sync + pl.sync_sel_done;
  fa.gs = gs, fa.idx = idx;
  fa.P = pl.problems, fa.C = pl.step_predict_chunks, fa.S = pl.step_attn_splits;
  fa.n_items = pl.problems * (pl.step_predict_chunks + 1 + pl.step_attn_splits);
  fa.NG = pl.n_groups, fa.M = p.n_select, fa.spin_limit = g_wait_limit;
  if (p.rank == 32) return launch_fused_one<BF16Elem, 32, 4, 4>(p, pl, pa, aa, fa, st);
  return launch_fused_one<BF16Elem, 64, 8, 4>(p, pl, pa, aa, fa, st);
}

}  // namespace kvs
