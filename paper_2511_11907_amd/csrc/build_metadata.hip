// Compact key metadata (Sec. 3.2): K_lr[b,k,n,:] = K[b,k,n,:] . A[k], fp32
// accumulation over the head dimension in natural order, one rounding to the
// metadata dtype.  Runs at prefill and when new groups are appended, outside the
// per-step latency.  In joint-head mode the row that is projected is the token's
// keys of all KV heads side by side, K_lr[b,n,:] = sum_k K[b,k,n,:] . A_k with A_k
// the k-th block of d rows of the single adapter: the same tile loop, run over the
// KV heads with the accumulators kept.
//
// A workgroup owns a tile of 64 consecutive token rows of one (sequence, KV head)
// problem (of one sequence in joint-head mode).  The K tile is brought in with coalesced 16-byte loads and parked in
// LDS as fp32 (row stride d+1 words, so the 64 lanes of a wave, one row each, hit
// 64 different banks); wave w produces the w-th quarter of the r output columns
// for all 64 rows, so the adapter entries it needs are the same for every lane of
// the wave (uniform loads).
#include "device_utils.h"
#include "kernels.h"

namespace kvs {

constexpr int kMetaThreads = 256;
constexpr int kMetaRows = 64;

template <typename EK, typename EM, int RC>  // RC = r / 4 output columns per lane
__global__ __launch_bounds__(kMetaThreads) void build_metadata_kernel(
    const typename EK::storage* __restrict__ K, const float* __restrict__ A,
    typename EM::storage* __restrict__ K_lr, int n_kv_heads, int heads_per_set, int ctx_rows,
    int first_row, int row_end, int d, float meta_scale) {
  constexpr int R = RC * 4;
  extern __shared__ float s_k[];  // [kMetaRows][d + 1]
  const int tid = threadIdx.x;
  const int set = blockIdx.y;  // (b, k), or b alone when the heads are projected jointly
  const int row0 = first_row + blockIdx.x * kMetaRows;  // rows [first_row, row_end) are built
  const int ld = d + 1;
  constexpr int EPL = EK::kPerLane;
  const int lanes_per_row = d / EPL;
  const int row = tid & (kMetaRows - 1);
  const int jq = __builtin_amdgcn_readfirstlane(tid / kMetaRows);  // wave-uniform column quarter
  float acc[RC];
#pragma unroll
  for (int j = 0; j < RC; ++j) acc[j] = 0.f;

  for (int kk = 0; kk < heads_per_set; ++kk) {
    const int p = set * heads_per_set + kk;  // (b, k) problem whose keys are staged
    const int k = p % n_kv_heads;
    if (kk > 0) lds_barrier();               // everyone is done with the previous tile
    // stage the tile: 16 bytes per lane, consecutive lanes along the row
    const typename EK::storage* Kp = K + ((size_t)p * ctx_rows + row0) * d;
    for (int i = tid; i < kMetaRows * lanes_per_row; i += kMetaThreads) {
      const int r_ = i / lanes_per_row, cc = i % lanes_per_row;
      float f[EPL];
      if (row0 + r_ < row_end) {
        const uint4 v = *reinterpret_cast<const uint4*>(Kp + (size_t)r_ * d + (size_t)cc * EPL);
        unpack16<EK>(v, f);
      } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) f[e] = 0.f;
      }
#pragma unroll
      for (int e = 0; e < EPL; ++e) s_k[r_ * ld + cc * EPL + e] = f[e];
    }
    lds_barrier();
    const float* Ak = A + (size_t)k * d * R + (size_t)jq * RC;
    for (int i = 0; i < d; ++i) {
      const float kv = s_k[row * ld + i];
#pragma unroll
      for (int j = 0; j < RC; ++j) acc[j] = fmaf(kv, Ak[(size_t)i * R + j], acc[j]);
    }
  }
  if (row0 + row < row_end) {
    typename EM::storage* o = K_lr + ((size_t)set * ctx_rows + row0 + row) * R + (size_t)jq * RC;
#pragma unroll
    for (int j = 0; j < RC; ++j) {
      const float v = acc[j] / meta_scale;  // (exact when the scale is 1)
      if constexpr (EM::kBytes == 2) o[j] = float_to_bf16_bits(v);
      else if constexpr (EM::kBytes == 1) o[j] = float_to_fp8_e4m3(v);
      else o[j] = v;
    }
  }
}

namespace {

template <typename EK, typename EM, int RC>
hipError_t launch_one(const kvs_params& p, const Plan& pl, const void* K, const float* A,
                      void* K_lr, int first_row, int n_rows, hipStream_t st) {
  dim3 grid((n_rows + kMetaRows - 1) / kMetaRows, pl.sets), block(kMetaThreads);
  const size_t lds = (size_t)kMetaRows * (p.head_dim + 1) * sizeof(float);
  hipLaunchKernelGGL((build_metadata_kernel<EK, EM, RC>), grid, block, lds, st,
                     (const typename EK::storage*)K, A, (typename EM::storage*)K_lr, p.n_kv_heads,
                     pl.kv_heads_per_set, pl.ctx_rows, first_row, first_row + n_rows, p.head_dim,
                     p.meta_scale != 0.f ? p.meta_scale : 1.0f);
  return hipGetLastError();
}

template <typename EK, typename EM>
hipError_t launch_r(const kvs_params& p, const Plan& pl, const void* K, const float* A,
                    void* K_lr, int first_row, int n_rows, hipStream_t st) {
  switch (p.rank) {
    case 16: return launch_one<EK, EM, 4>(p, pl, K, A, K_lr, first_row, n_rows, st);
    case 32: return launch_one<EK, EM, 8>(p, pl, K, A, K_lr, first_row, n_rows, st);
    case 64: return launch_one<EK, EM, 16>(p, pl, K, A, K_lr, first_row, n_rows, st);
    case 128: return launch_one<EK, EM, 32>(p, pl, K, A, K_lr, first_row, n_rows, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_build_metadata(const kvs_params& p, const Plan& pl, const void* K,
                                 const float* A, void* K_lr, int first_row, int n_rows,
                                 hipStream_t st) {
  if (n_rows <= 0) return hipSuccess;
  const bool kb = p.kv_dtype == KVS_BF16, mb = p.meta_dtype == KVS_BF16;
  if (p.meta_dtype == KVS_FP8_E4M3) {
    if (kb) return launch_r<BF16Elem, FP8Elem>(p, pl, K, A, K_lr, first_row, n_rows, st);
    return launch_r<F32Elem, FP8Elem>(p, pl, K, A, K_lr, first_row, n_rows, st);
  }
  if (kb && mb) return launch_r<BF16Elem, BF16Elem>(p, pl, K, A, K_lr, first_row, n_rows, st);
  if (kb && !mb) return launch_r<BF16Elem, F32Elem>(p, pl, K, A, K_lr, first_row, n_rows, st);
  if (!kb && mb) return launch_r<F32Elem, BF16Elem>(p, pl, K, A, K_lr, first_row, n_rows, st);
  return launch_r<F32Elem, F32Elem>(p, pl, K, A, K_lr, first_row, n_rows, st);
}

// A completed group leaves the rolling buffer (Sec. 3.4.1): the first G rows of every
// (b, kv head)'s buffer become cache rows N .. N+G-1.  16 bytes per lane, one workgroup
// per problem (G*d elements of K and of V: a few KiB).
__global__ __launch_bounds__(256) void append_rows_kernel(const uint4* __restrict__ rb_K,
                                                          const uint4* __restrict__ rb_V,
                                                          uint4* __restrict__ K, uint4* __restrict__ V,
                                                          size_t rb_stride16, size_t cache_stride16,
                                                          size_t dst_off16, int n16) {
  const size_t p = blockIdx.x;
  for (int i = threadIdx.x; i < n16; i += blockDim.x) {
    K[p * cache_stride16 + dst_off16 + i] = rb_K[p * rb_stride16 + i];
    V[p * cache_stride16 + dst_off16 + i] = rb_V[p * rb_stride16 + i];
  }
}

hipError_t launch_append_rows(const kvs_params& p, const Plan& pl, const RollingBuffer& rb,
                              void* K, void* V, hipStream_t st) {
  const size_t row16 = (size_t)p.head_dim * (p.kv_dtype == KVS_BF16 ? 2 : 4) / 16;  // 16-byte pieces per row
  hipLaunchKernelGGL(append_rows_kernel, dim3(pl.problems), dim3(256), 0, st, (const uint4*)rb.K,
                     (const uint4*)rb.V, (uint4*)K, (uint4*)V, (size_t)rb.capacity * row16,
                     (size_t)pl.ctx_rows * row16, (size_t)p.ctx_len * row16,
                     (int)(p.group_size * row16));
  return hipGetLastError();
}

}  // namespace kvs
