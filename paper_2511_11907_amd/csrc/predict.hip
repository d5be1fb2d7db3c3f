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
#include "device_utils.h"
#include "kernels.h"
#include "topk_block.h"

namespace kvs {

static_assert(kTopkBins == kSelectHistBins, "workspace layout and selection routine disagree");

constexpr int kPredictThreads = kPredictWgThreads;
constexpr int kPredictWaves = kPredictThreads / kWave;
constexpr int kPredictUnroll = kPredictUnitsPerWgStep / kPredictWaves;  // wave-loads in flight per wave
static_assert(kPredictUnroll * kPredictWaves == kPredictUnitsPerWgStep, "granule mismatch");

template <typename E, int R, int G, bool HIST, bool PAD>
__global__ __launch_bounds__(kPredictThreads) void predict_kernel(
    const void* __restrict__ q, int q_is_bf16, const typename E::storage* __restrict__ K_lr,
    const float* __restrict__ A, float* gs, int n_kv_heads, int q_per_kv, int d,
    int n_groups, int g_real, int ctx_rows, int units, int units_per_wg, int mean,
    int* __restrict__ hist, const float* __restrict__ qlr, float meta_scale) {
  constexpr int EPL = E::kPerLane;
  constexpr int LPR = R / EPL;          // lanes per row
  constexpr int RPU = kWave / LPR;      // rows per unit
  static_assert(LPR >= 1 && LPR <= 32 && (LPR & (LPR - 1)) == 0, "row must span 1..32 lanes");
  constexpr bool kGroupInUnit = (G <= RPU);
  constexpr int UPG = kGroupInUnit ? 1 : G / RPU;  // units per group otherwise
  // wave-loads in flight per wave; a group must not straddle two batches
  constexpr int U = UPG > kPredictUnroll ? UPG : kPredictUnroll;
  static_assert(U % UPG == 0, "a group must not straddle two batches");

  __shared__ float s_qsum[128];
  __shared__ float s_red[kPredictThreads];
  __shared__ float s_qlr[R];
  __shared__ int s_hist[HIST ? kTopkBins : 1];
  constexpr int kGroupsPerBatch = kGroupInUnit ? U * (RPU / G) : U / UPG;  // per wave
  __shared__ float s_stage[kPredictWaves][kGroupsPerBatch];  // group scores of a wave's batch

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int p = blockIdx.y;
  const int b = p / n_kv_heads, k = p % n_kv_heads;
  const int n_q_heads = n_kv_heads * q_per_kv;
  const int c = lane % LPR;   // 16-byte column of the row
  const int rl = lane / LPR;  // row within the unit

  const typename E::storage* Kp = K_lr + (size_t)p * ctx_rows * R;
  float* gsp = gs + (size_t)p * n_groups;
  const int N = n_groups * g_real;   // rows of the compressed cache
  const int n_slots = n_groups * G;  // row slots (== N unless the groups are padded)
  const int u0 = blockIdx.x * units_per_wg;
  const int u1 = min(units, u0 + units_per_wg);

  // A workgroup step covers kPredictWaves * U consecutive units; wave w takes the U
  // consecutive units starting at w * U, i.e. one contiguous run of U KiB, whose group
  // scores are U * RPU / G consecutive floats that leave in one coalesced store.
  constexpr int kStep = kPredictWaves * U;
  auto unit_of = [&](int step_base, int j) { return step_base + wave * U + j; };
  uint4 v[U];
  bool ok[U];
  auto issue = [&](int step_base) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int unit = unit_of(step_base, u);
      const int slot = unit * RPU + rl;
      size_t off;
      if constexpr (PAD) {
        const int row = (slot / G) * g_real + (slot % G);
        ok[u] = (unit < u1) && (slot < n_slots) && ((slot % G) < g_real);
        // (a slot without a row reads a valid row nearby, one its neighbours fetch anyway)
        off = (size_t)(unit < u1 ? min(row, N - 1) : 0) * R + (size_t)c * EPL;
      } else {
        ok[u] = (unit < u1) && (slot < N);
        off = (size_t)(ok[u] ? slot : 0) * R + (size_t)c * EPL;
      }
      v[u] = *reinterpret_cast<const uint4*>(Kp + off);
    }
  };
  // Everything the prologue needs from memory is requested up front - the queries, this
  // lane's entries of the adapter, and the first batch of K_lr - so that the workgroup
  // pays one memory latency before it streams, not three in a row.
  constexpr int NSL = kPredictThreads / R;  // slices of the d axis in the projection
  constexpr int kSpanMax = 128 / NSL;       // adapter rows per lane at d = 128
  const int pj = tid % R, psl = tid / R;
  const int span = d / NSL;
  const bool project = (qlr == nullptr);  // uniform: false when the low-rank query is given
  StridedSum qheads;
  float a_reg[kSpanMax];
  float qr[EPL];
  if (project) {
    // the query heads of this KV head, element tid of each (lanes beyond d repeat the last)
    qheads.request(q, q_is_bf16, ((size_t)b * n_q_heads + (size_t)k * q_per_kv) * d + min(tid, d - 1), d, q_per_kv);
    const float* Ak = A + (size_t)k * d * R;
#pragma unroll
    for (int i = 0; i < kSpanMax; ++i)
      a_reg[i] = Ak[(size_t)min(psl * span + i, d - 1) * R + pj];  // rows past the span are never used
  } else {
#pragma unroll
    for (int e = 0; e < EPL; ++e) qr[e] = qlr[(size_t)p * R + c * EPL + e] * meta_scale;
  }
  int ub = u0;  // base of the current workgroup step
  if (ub < u1) issue(ub);

  if constexpr (HIST) {  // this workgroup's share of the score histogram
    for (int i = tid; i < kTopkBins; i += kPredictThreads) s_hist[i] = 0;
  }

  if (project) {
    // ---- low-rank query vector of this KV head (head-summed) --------------------
    if (tid < d) s_qsum[tid] = qheads.sum(q_is_bf16, q_per_kv);
    lds_barrier();
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < kSpanMax; ++i)
      if (i < span) acc = fmaf(s_qsum[psl * span + i], a_reg[i], acc);
    s_red[tid] = acc;
    lds_barrier();
    if (tid < R) {
      float tot = 0.f;
#pragma unroll 8
      for (int s = 0; s < NSL; ++s) tot += s_red[s * R + tid];
      s_qlr[tid] = tot;
    }
    lds_barrier();
#pragma unroll
    // the stored metadata is K.A / meta_scale: the factor goes into the query once
    for (int e = 0; e < EPL; ++e) qr[e] = s_qlr[c * EPL + e] * meta_scale;
  } else if constexpr (HIST) {
    lds_barrier();  // the histogram is cleared before anyone counts into it
  }

  const float inv_g = 1.0f / (float)g_real;
  const float empty = mean ? 0.f : -__builtin_huge_valf();  // score of an empty row slot

  while (ub < u1) {
    float sc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float f[EPL];
      unpack16<E>(v[u], f);
      float acc = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc = fmaf(qr[e], f[e], acc);
      sc[u] = allreduce_lanes<OpSum, 1, LPR>(acc);  // token score, on all LPR lanes of the row
      if constexpr (PAD) sc[u] = ok[u] ? sc[u] : empty;
    }
    // Group representatives go through a per-wave LDS line so that they leave as one
    // coalesced store per batch (scattered 4-byte stores per unit cost ~8 % of the
    // streaming bandwidth).  Only this wave touches its line, in program order.
    if constexpr (kGroupInUnit) {
      constexpr int GPU_ = RPU / G;  // groups per unit
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float g;
        if (mean) g = allreduce_lanes<OpSum, LPR, LPR * G>(sc[u]) * inv_g;
        else g = allreduce_lanes<OpMax, LPR, LPR * G>(sc[u]);
        if ((lane % (LPR * G)) == 0) s_stage[wave][u * GPU_ + lane / (LPR * G)] = g;
      }
    } else {
#pragma unroll
      for (int u0g = 0; u0g < U; u0g += UPG) {
        float g = sc[u0g];
#pragma unroll
        for (int t = 1; t < UPG; ++t) g = mean ? g + sc[u0g + t] : fmaxf(g, sc[u0g + t]);
        if (mean) g = allreduce_lanes<OpSum, LPR, kWave>(g) * inv_g;
        else g = allreduce_lanes<OpMax, LPR, kWave>(g);
        if (lane == 0) s_stage[wave][u0g / UPG] = g;
      }
    }
    {
      // first group of this wave's batch; groups never straddle units' ends, so a group is
      // valid iff its first row is
      const int row0 = unit_of(ub, 0) * RPU;
      const int grp0 = row0 / G;
      const int row_end = min(n_slots, u1 * RPU);
#pragma unroll
      for (int t = lane; t < kGroupsPerBatch; t += kWave) {
        if ((grp0 + t) * G < row_end) {
          const float g = s_stage[wave][t];
          gsp[grp0 + t] = g;
          if constexpr (HIST) atomicAdd(&s_hist[score_key(g) >> kTopkLowBits], 1);
        }
      }
    }
    ub += kStep;
    if (ub < u1) issue(ub);
  }

  if constexpr (HIST) {
    // add this workgroup's histogram to the problem's (only the bins it touched)
    lds_barrier();
    int* hg = hist + (size_t)p * kTopkBins;
    for (int i = tid; i < kTopkBins; i += kPredictThreads) {
      const int n = s_hist[i];
      if (n) atomicAdd(&hg[i], n);
    }
  }
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
  if (hist)
    hipLaunchKernelGGL((predict_kernel<E, R, G, true, PAD>), grid, block, 0, st, q, q_bf16,
                       (const typename E::storage*)K_lr, A, gs, p.n_kv_heads, pl.q_per_kv,
                       p.head_dim, pl.n_groups, p.group_size, pl.ctx_rows, pl.predict_units,
                       pl.predict_units_per_wg, mean, hist, (const float*)qlr, scale);
  else
    hipLaunchKernelGGL((predict_kernel<E, R, G, false, PAD>), grid, block, 0, st, q, q_bf16,
                       (const typename E::storage*)K_lr, A, gs, p.n_kv_heads, pl.q_per_kv,
                       p.head_dim, pl.n_groups, p.group_size, pl.ctx_rows, pl.predict_units,
                       pl.predict_units_per_wg, mean, (int*)nullptr, (const float*)qlr, scale);
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
