// Prediction pass over the compact key metadata (Sec. 3.3, Eq. 1 and "Scoring and
// selection"): for every (sequence, KV head) problem, project the query heads
// that share the KV head into the rank-r space, stream all N rows of K_lr once,
// and write one representative score per group of G consecutive tokens.
//
//   q_lr  = (sum_{h: g(h)=k} q[h]) . A[k]           (the head sum commutes with the
//                                                    projection and with the dot product)
//   s[n]  = q_lr . K_lr[n]
//   gs[j] = max_t s[jG+t]   (or the mean)
//
// HBM-bound: the kernel's job is to keep wide, fully coalesced 16-byte-per-lane
// loads of K_lr in flight.  One wave-wide load ("unit") is 1 KiB = 64/LPR
// consecutive rows, LPR lanes per row; the dot product is finished with an
// in-register all-reduce over those LPR lanes and the group max with a second
// all-reduce over the lanes (or consecutive units) that hold the group's rows.
//
// Group sizes that are not a power of two run on the PAD instantiation of the next power
// of two G: every group gets G row slots of which the last G - g_real stay empty (no
// load is useful there, the score counts as -inf for the max and 0 for the mean), so
// groups still never straddle a unit or a batch.  The bytes moved are the same; the
// empty slots only cost issue slots.
//
// Joint-head mode (Sec. 3.2 design (b)): there is one K_lr per sequence and the score is
// summed over all query heads, head h projected with the block A_{g(h)} of the single
// adapter.  The sum still commutes:
//   q_lr = sum_k (sum_{h: g(h)=k} q[h]) . A_k = qcat . A,   qcat = the per-KV-head query
//                                                            sums laid side by side
// a contraction over H_kv*d values.  It is done once per sequence by a small kernel of
// its own (project_query_kernel); the streaming kernel then starts from the r finished
// values instead of projecting in its prologue.
//
// With HIST the kernel also prepares the selection: while a group score is still in a
// register its top 12 key bits are counted in a workgroup-local LDS histogram, and at
// the end the non-empty bins are added to the problem's histogram in global memory.
// The selection kernel that follows starts from that finished histogram instead of
// building it with heavily contended atomics.
#include "predict_item.h"

namespace kvs {

// Start and end time of every workgroup for the debugging harness (compiled only with
// -DKVS_WG_TRACE_BUILD): two words per workgroup, in launch order.
#ifdef KVS_WG_TRACE_BUILD
static __device__ long long g_predict_wg_trace[2 * 8192];
extern "C" int kvs_debug_predict_wg_trace(long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_predict_wg_trace), sizeof(long long) * (size_t)n);
}
#define KVS_WG_TRACE(i)                                                                        \
  do {                                                                                         \
    const int wg_ = blockIdx.y * gridDim.x + blockIdx.x;                                       \
    if (threadIdx.x == 0 && wg_ < 8192) g_predict_wg_trace[2 * wg_ + (i)] = wall_clock64();    \
  } while (0)
#else
#define KVS_WG_TRACE(i)
#endif

template <typename E, int R, int G, bool HIST, bool PAD>
__global__ __launch_bounds__(kPredictThreads) void predict_kernel(PredictArgs a) {
  __shared__ PredictShared<E, R, G, HIST> sh;
  KVS_WG_TRACE(0);
  predict_item<E, R, G, HIST, PAD, false, kPredictUnroll, kPredictThreads, true>(sh, a, blockIdx.y, blockIdx.x);
  KVS_WG_TRACE(1);
}


// Joint-head mode: q_lr[b,:] = qcat[b,:] . A for one sequence per workgroup, where
// qcat[k*d + i] = sum_{h: g(h)=k} q[b,h,i] and A is [(H_kv*d), R].  Lane (slice, j)
// sums every NSL-th row of column j (consecutive lanes read consecutive floats of a
// row), the slices are added through LDS.
constexpr int kProjectThreads = 1024;

template <int R>
__global__ __launch_bounds__(kProjectThreads) void project_query_kernel(
    const void* __restrict__ q, int q_is_bf16, const float* __restrict__ A,
    float* __restrict__ qlr, int n_kv_heads, int q_per_kv, int d) {
  constexpr int NSL = kProjectThreads / R;
  __shared__ float s_qcat[kJointMaxFlatDim];
  __shared__ float s_part[kProjectThreads];
  const int tid = threadIdx.x, b = blockIdx.x;
  const int L = n_kv_heads * d;  // flattened length, <= kJointMaxFlatDim
  const int n_q_heads = n_kv_heads * q_per_kv;
  for (int i = tid; i < L; i += kProjectThreads) {
    const int k = i / d, e = i % d;
    StridedSum heads;
    heads.request(q, q_is_bf16, ((size_t)b * n_q_heads + (size_t)k * q_per_kv) * d + e, d, q_per_kv);
    s_qcat[i] = heads.sum(q_is_bf16, q_per_kv);
  }
  lds_barrier();
  const int j = tid % R, sl = tid / R;
  float acc = 0.f;
#pragma unroll 8
  for (int i = sl; i < L; i += NSL) acc = fmaf(s_qcat[i], A[(size_t)i * R + j], acc);
  s_part[tid] = acc;
  lds_barrier();
  if (tid < R) {
    float tot = 0.f;
#pragma unroll 8
    for (int s = 0; s < NSL; ++s) tot += s_part[s * R + tid];
    qlr[(size_t)b * R + tid] = tot;
  }
}

namespace {

template <typename E, int R, int G, bool PAD>
hipError_t launch_one(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                      const float* A, float* gs, int* hist, float* qlr, hipStream_t st) {
  dim3 grid(pl.predict_chunks, pl.sets), block(kPredictThreads);
  const int q_bf16 = (int)(p.kv_dtype == KVS_BF16), mean = (int)(p.reduce == KVS_REDUCE_MEAN);
  const float scale = p.meta_scale != 0.f ? p.meta_scale : 1.0f;
  if (qlr) {
    hipLaunchKernelGGL((project_query_kernel<R>), dim3(pl.sets), dim3(kProjectThreads), 0, st, q,
                       q_bf16, A, qlr, p.n_kv_heads, pl.q_per_kv, p.head_dim);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  PredictArgs a{q, q_bf16, K_lr, A, gs, nullptr, p.n_kv_heads, pl.q_per_kv, p.head_dim, pl.n_groups, p.group_size,
                pl.ctx_rows, pl.predict_units, pl.predict_units_per_wg, mean, hist, (const float*)qlr, scale,
                p.meta_scales};
  if (hist) hipLaunchKernelGGL((predict_kernel<E, R, G, true, PAD>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((predict_kernel<E, R, G, false, PAD>), grid, block, 0, st, a);
  return hipGetLastError();
}

template <typename E, int R>
hipError_t launch_g(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                    const float* A, float* gs, int* hist, float* qlr, hipStream_t st) {
  const bool pad = pl.group_slots != p.group_size;  // G is not a power of two
  switch (pl.group_slots) {  // the group size, or the next power of two
    case 1: return launch_one<E, R, 1, false>(p, pl, q, K_lr, A, gs, hist, qlr, st);
    case 2: return launch_one<E, R, 2, false>(p, pl, q, K_lr, A, gs, hist, qlr, st);
    case 4:
      return pad ? launch_one<E, R, 4, true>(p, pl, q, K_lr, A, gs, hist, qlr, st)
                 : launch_one<E, R, 4, false>(p, pl, q, K_lr, A, gs, hist, qlr, st);
    case 8:
      return pad ? launch_one<E, R, 8, true>(p, pl, q, K_lr, A, gs, hist, qlr, st)
                 : launch_one<E, R, 8, false>(p, pl, q, K_lr, A, gs, hist, qlr, st);
    case 16:
      return pad ? launch_one<E, R, 16, true>(p, pl, q, K_lr, A, gs, hist, qlr, st)
                 : launch_one<E, R, 16, false>(p, pl, q, K_lr, A, gs, hist, qlr, st);
  }
  return hipErrorInvalidValue;
}

template <typename E>
hipError_t launch_r(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                    const float* A, float* gs, int* hist, float* qlr, hipStream_t st) {
  switch (p.rank) {
    case 16: return launch_g<E, 16>(p, pl, q, K_lr, A, gs, hist, qlr, st);
    case 32: return launch_g<E, 32>(p, pl, q, K_lr, A, gs, hist, qlr, st);
    case 64: return launch_g<E, 64>(p, pl, q, K_lr, A, gs, hist, qlr, st);
    case 128: return launch_g<E, 128>(p, pl, q, K_lr, A, gs, hist, qlr, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_predict(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                          const float* A, float* gs, int* hist, float* qlr, hipStream_t st) {
  if (p.meta_dtype == KVS_BF16) return launch_r<BF16Elem>(p, pl, q, K_lr, A, gs, hist, qlr, st);
  if (p.meta_dtype == KVS_FP8_E4M3) return launch_r<FP8Elem>(p, pl, q, K_lr, A, gs, hist, qlr, st);
  return launch_r<F32Elem>(p, pl, q, K_lr, A, gs, hist, qlr, st);
}

}  // namespace kvs
