// Prediction pass over the compact key metadata (Sec. 4.3, Eq. 1 and "Scoring and
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

constexpr int kPredictThreads = kTopkThreads;  // the selection tail wants the full 1024 lanes
constexpr int kPredictWaves = kPredictThreads / kWave;
constexpr int kPredictUnroll = kPredictUnitsPerWgStep / kPredictWaves;  // wave-loads in flight per wave
static_assert(kPredictUnroll * kPredictWaves == kPredictUnitsPerWgStep, "granule mismatch");

template <typename E, int R, int G, bool HIST>
__global__ __launch_bounds__(kPredictThreads) void predict_kernel(
    const void* __restrict__ q, int q_is_bf16, const typename E::storage* __restrict__ K_lr,
    const float* __restrict__ A, float* gs, int n_kv_heads, int q_per_kv, int d,
    int N, int units, int units_per_wg, int mean, int* __restrict__ hist) {
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

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int p = blockIdx.y;
  const int b = p / n_kv_heads, k = p % n_kv_heads;
  const int n_q_heads = n_kv_heads * q_per_kv;
  const int c = lane % LPR;   // 16-byte column of the row
  const int rl = lane / LPR;  // row within the unit

  const typename E::storage* Kp = K_lr + (size_t)p * N * R;
  float* gsp = gs + (size_t)p * (N / G);
  const int u0 = blockIdx.x * units_per_wg;
  const int u1 = min(units, u0 + units_per_wg);

  uint4 v[U];
  bool ok[U];
  auto issue = [&](int ub) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = (ub + u) * RPU + rl;
      ok[u] = (ub + u < u1) && (row < N);
      const size_t off = (size_t)(ok[u] ? row : 0) * R + (size_t)c * EPL;
      v[u] = *reinterpret_cast<const uint4*>(Kp + off);
    }
  };
  // The first batch of K_lr is requested before anything else, so that its latency
  // overlaps the query projection below.
  int ub = u0 + wave * U;
  if (ub < u1) issue(ub);

  if constexpr (HIST) {  // this workgroup's share of the score histogram
    for (int i = tid; i < kTopkBins; i += kPredictThreads) s_hist[i] = 0;
  }

  // ---- low-rank query vector of this KV head (head-summed) --------------------
  if (tid < d) {
    float acc = 0.f;
    for (int hh = 0; hh < q_per_kv; ++hh)
      acc += load_as_float(q, q_is_bf16, ((size_t)b * n_q_heads + (size_t)k * q_per_kv + hh) * d + tid);
    s_qsum[tid] = acc;
  }
  lds_barrier();
  {
    constexpr int NSL = kPredictThreads / R;  // slices of the d axis
    const int j = tid % R, sl = tid / R;
    const int span = d / NSL;
    const float* Ak = A + (size_t)k * d * R;
    float acc = 0.f;
    for (int i = sl * span; i < (sl + 1) * span; ++i) acc = fmaf(s_qsum[i], Ak[(size_t)i * R + j], acc);
    s_red[tid] = acc;
    lds_barrier();
    if (tid < R) {
      float tot = 0.f;
#pragma unroll 8
      for (int s = 0; s < NSL; ++s) tot += s_red[s * R + tid];
      s_qlr[tid] = tot;
    }
    lds_barrier();
  }
  float qr[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) qr[e] = s_qlr[c * EPL + e];
  const float inv_g = 1.0f / (float)G;

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
    }
    if constexpr (kGroupInUnit) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float g;
        if (mean) g = allreduce_lanes<OpSum, LPR, LPR * G>(sc[u]) * inv_g;
        else g = allreduce_lanes<OpMax, LPR, LPR * G>(sc[u]);
        if (ok[u] && (lane % (LPR * G)) == 0) {
          gsp[((ub + u) * RPU + rl) / G] = g;
          if constexpr (HIST) atomicAdd(&s_hist[score_key(g) >> kTopkLowBits], 1);
        }
      }
    } else {
#pragma unroll
      for (int u0g = 0; u0g < U; u0g += UPG) {
        float g = sc[u0g];
#pragma unroll
        for (int t = 1; t < UPG; ++t) g = mean ? g + sc[u0g + t] : fmaxf(g, sc[u0g + t]);
        if (mean) g = allreduce_lanes<OpSum, LPR, kWave>(g) * inv_g;
        else g = allreduce_lanes<OpMax, LPR, kWave>(g);
        if (ok[u0g] && lane == 0) {
          gsp[((ub + u0g) * RPU) / G] = g;
          if constexpr (HIST) atomicAdd(&s_hist[score_key(g) >> kTopkLowBits], 1);
        }
      }
    }
    ub += kPredictWaves * U;
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

namespace {

template <typename E, int R, int G>
hipError_t launch_one(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                      const float* A, float* gs, int* hist, hipStream_t st) {
  dim3 grid(pl.predict_chunks, pl.problems), block(kPredictThreads);
  const int q_bf16 = (int)(p.kv_dtype == KVS_BF16), mean = (int)(p.reduce == KVS_REDUCE_MEAN);
  if (hist)
    hipLaunchKernelGGL((predict_kernel<E, R, G, true>), grid, block, 0, st, q, q_bf16,
                       (const typename E::storage*)K_lr, A, gs, p.n_kv_heads, pl.q_per_kv,
                       p.head_dim, p.ctx_len, pl.predict_units, pl.predict_units_per_wg, mean, hist);
  else
    hipLaunchKernelGGL((predict_kernel<E, R, G, false>), grid, block, 0, st, q, q_bf16,
                       (const typename E::storage*)K_lr, A, gs, p.n_kv_heads, pl.q_per_kv,
                       p.head_dim, p.ctx_len, pl.predict_units, pl.predict_units_per_wg, mean,
                       (int*)nullptr);
  return hipGetLastError();
}

template <typename E, int R>
hipError_t launch_g(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                    const float* A, float* gs, int* hist, hipStream_t st) {
  switch (p.group_size) {
    case 1: return launch_one<E, R, 1>(p, pl, q, K_lr, A, gs, hist, st);
    case 2: return launch_one<E, R, 2>(p, pl, q, K_lr, A, gs, hist, st);
    case 4: return launch_one<E, R, 4>(p, pl, q, K_lr, A, gs, hist, st);
    case 8: return launch_one<E, R, 8>(p, pl, q, K_lr, A, gs, hist, st);
    case 16: return launch_one<E, R, 16>(p, pl, q, K_lr, A, gs, hist, st);
  }
  return hipErrorInvalidValue;
}

template <typename E>
hipError_t launch_r(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                    const float* A, float* gs, int* hist, hipStream_t st) {
  switch (p.rank) {
    case 16: return launch_g<E, 16>(p, pl, q, K_lr, A, gs, hist, st);
    case 32: return launch_g<E, 32>(p, pl, q, K_lr, A, gs, hist, st);
    case 64: return launch_g<E, 64>(p, pl, q, K_lr, A, gs, hist, st);
    case 128: return launch_g<E, 128>(p, pl, q, K_lr, A, gs, hist, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_predict(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                          const float* A, float* gs, int* hist, hipStream_t st) {
  if (p.meta_dtype == KVS_BF16) return launch_r<BF16Elem>(p, pl, q, K_lr, A, gs, hist, st);
  return launch_r<F32Elem>(p, pl, q, K_lr, A, gs, hist, st);
}

}  // namespace kvs
