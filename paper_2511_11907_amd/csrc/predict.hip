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
#include "device_utils.h"
#include "kernels.h"

namespace kvs {

constexpr int kPredictThreads = 256;
constexpr int kPredictWaves = kPredictThreads / kWave;
constexpr int kPredictUnroll = 8;  // wave-loads in flight per wave

template <typename E, int R, int G>
__global__ __launch_bounds__(kPredictThreads) void predict_kernel(
    const void* __restrict__ q, int q_is_bf16, const typename E::storage* __restrict__ K_lr,
    const float* __restrict__ A, float* __restrict__ gs, int n_kv_heads, int q_per_kv, int d,
    int N, int units, int units_per_wg, int mean) {
  constexpr int EPL = E::kPerLane;
  constexpr int LPR = R / EPL;          // lanes per row
  constexpr int RPU = kWave / LPR;      // rows per unit
  static_assert(LPR >= 1 && LPR <= 32 && (LPR & (LPR - 1)) == 0, "row must span 1..32 lanes");
  constexpr bool kGroupInUnit = (G <= RPU);
  constexpr int UPG = kGroupInUnit ? 1 : G / RPU;  // units per group otherwise
  static_assert(kPredictUnroll % UPG == 0, "a group must not straddle two batches");

  __shared__ float s_qsum[128];
  __shared__ float s_red[kPredictThreads];
  __shared__ float s_qlr[R];

  const int tid = threadIdx.x;
  const int p = blockIdx.y;
  const int b = p / n_kv_heads, k = p % n_kv_heads;
  const int n_q_heads = n_kv_heads * q_per_kv;

  // ---- low-rank query vector of this KV head (head-summed) --------------------
  if (tid < d) {
    float acc = 0.f;
    for (int hh = 0; hh < q_per_kv; ++hh)
      acc += load_as_float(q, q_is_bf16, ((size_t)b * n_q_heads + (size_t)k * q_per_kv + hh) * d + tid);
    s_qsum[tid] = acc;
  }
  __syncthreads();
  {
    constexpr int NSL = kPredictThreads / R;  // slices of the d axis
    const int j = tid % R, sl = tid / R;
    const int span = d / NSL;
    const float* Ak = A + (size_t)k * d * R;
    float acc = 0.f;
    for (int i = sl * span; i < (sl + 1) * span; ++i) acc = fmaf(s_qsum[i], Ak[(size_t)i * R + j], acc);
    s_red[tid] = acc;
    __syncthreads();
    if (tid < R) {
      float tot = 0.f;
#pragma unroll
      for (int s = 0; s < NSL; ++s) tot += s_red[s * R + tid];
      s_qlr[tid] = tot;
    }
    __syncthreads();
  }

  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int c = lane % LPR;   // 16-byte column of the row
  const int rl = lane / LPR;  // row within the unit
  float qr[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) qr[e] = s_qlr[c * EPL + e];

  const typename E::storage* Kp = K_lr + (size_t)p * N * R;
  float* gsp = gs + (size_t)p * (N / G);
  const int u0 = blockIdx.x * units_per_wg;
  const int u1 = min(units, u0 + units_per_wg);
  const float inv_g = 1.0f / (float)G;

  for (int ub = u0 + wave * kPredictUnroll; ub < u1; ub += kPredictWaves * kPredictUnroll) {
    uint4 v[kPredictUnroll];
    bool ok[kPredictUnroll];
#pragma unroll
    for (int u = 0; u < kPredictUnroll; ++u) {
      const int row = (ub + u) * RPU + rl;
      ok[u] = (ub + u < u1) && (row < N);
      const size_t off = (size_t)(ok[u] ? row : 0) * R + (size_t)c * EPL;
      v[u] = *reinterpret_cast<const uint4*>(Kp + off);
    }
    float sc[kPredictUnroll];
#pragma unroll
    for (int u = 0; u < kPredictUnroll; ++u) {
      float f[EPL];
      unpack16<E>(v[u], f);
      float acc = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc = fmaf(qr[e], f[e], acc);
      sc[u] = allreduce_lanes<OpSum, 1, LPR>(acc);  // token score, on all LPR lanes of the row
    }
    if constexpr (kGroupInUnit) {
#pragma unroll
      for (int u = 0; u < kPredictUnroll; ++u) {
        float g;
        if (mean) g = allreduce_lanes<OpSum, LPR, LPR * G>(sc[u]) * inv_g;
        else g = allreduce_lanes<OpMax, LPR, LPR * G>(sc[u]);
        if (ok[u] && (lane % (LPR * G)) == 0) gsp[((ub + u) * RPU + rl) / G] = g;
      }
    } else {
#pragma unroll
      for (int u0g = 0; u0g < kPredictUnroll; u0g += UPG) {
        float g = sc[u0g];
#pragma unroll
        for (int t = 1; t < UPG; ++t) g = mean ? g + sc[u0g + t] : fmaxf(g, sc[u0g + t]);
        if (mean) g = allreduce_lanes<OpSum, LPR, kWave>(g) * inv_g;
        else g = allreduce_lanes<OpMax, LPR, kWave>(g);
        if (ok[u0g] && lane == 0) gsp[((ub + u0g) * RPU) / G] = g;
      }
    }
  }
}

namespace {

template <typename E, int R, int G>
hipError_t launch_one(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                      const float* A, float* gs, hipStream_t st) {
  dim3 grid(pl.predict_chunks, pl.problems), block(kPredictThreads);
  hipLaunchKernelGGL((predict_kernel<E, R, G>), grid, block, 0, st, q, (int)(p.kv_dtype == KVS_BF16),
                     (const typename E::storage*)K_lr, A, gs, p.n_kv_heads, pl.q_per_kv, p.head_dim,
                     p.ctx_len, pl.predict_units, pl.predict_units_per_wg,
                     (int)(p.reduce == KVS_REDUCE_MEAN));
  return hipGetLastError();
}

template <typename E, int R>
hipError_t launch_g(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                    const float* A, float* gs, hipStream_t st) {
  switch (p.group_size) {
    case 1: return launch_one<E, R, 1>(p, pl, q, K_lr, A, gs, st);
    case 2: return launch_one<E, R, 2>(p, pl, q, K_lr, A, gs, st);
    case 4: return launch_one<E, R, 4>(p, pl, q, K_lr, A, gs, st);
    case 8: return launch_one<E, R, 8>(p, pl, q, K_lr, A, gs, st);
    case 16: return launch_one<E, R, 16>(p, pl, q, K_lr, A, gs, st);
  }
  return hipErrorInvalidValue;
}

template <typename E>
hipError_t launch_r(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                    const float* A, float* gs, hipStream_t st) {
  switch (p.rank) {
    case 16: return launch_g<E, 16>(p, pl, q, K_lr, A, gs, st);
    case 32: return launch_g<E, 32>(p, pl, q, K_lr, A, gs, st);
    case 64: return launch_g<E, 64>(p, pl, q, K_lr, A, gs, st);
    case 128: return launch_g<E, 128>(p, pl, q, K_lr, A, gs, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_predict(const kvs_params& p, const Plan& pl, const void* q, const void* K_lr,
                          const float* A, float* gs, hipStream_t st) {
  if (p.meta_dtype == KVS_BF16) return launch_r<BF16Elem>(p, pl, q, K_lr, A, gs, st);
  return launch_r<F32Elem>(p, pl, q, K_lr, A, gs, st);
}

}  // namespace kvs
