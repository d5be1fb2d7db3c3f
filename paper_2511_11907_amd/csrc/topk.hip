// Top-M selection kernel (Sec. 3.3, "TopK"): one workgroup of 1024 lanes per (sequence,
// KV head) problem runs kvs::topk_block on that problem's group scores, either from
// scratch (kvs_select_topk) or starting from the histogram the prediction kernel left
// in the workspace (kvs_predict_select).  The small fill kernel that prepares a
// workspace lives here too.
#include "kernels.h"
#include "topk_block.h"

namespace kvs {

// SLOTS: register slots per lane, i.e. problems of up to kTopkThreads * SLOTS scores.
template <int SLOTS>
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float* __restrict__ gs,
                                                            int32_t* __restrict__ idx, int NG,
                                                            int M, int* __restrict__ hist) {
  __shared__ TopkShared sh;
  const int p = blockIdx.x;
  topk_block<SLOTS>(gs + (size_t)p * NG, idx + (size_t)p * M, NG, M,
                    hist ? hist + (size_t)p * kTopkBins : nullptr, sh);
}

hipError_t launch_topk(const kvs_params& p, const Plan& pl, const float* gs, int32_t* idx,
                       int* hist, hipStream_t st) {
  dim3 grid(pl.sets), block(kTopkThreads);
  if (pl.n_groups <= kTopkThreads * kTopkSmallPerLane)
    hipLaunchKernelGGL(topk_kernel<kTopkSmallPerLane>, grid, block, 0, st, gs, idx, pl.n_groups, p.n_select, hist);
  else
    hipLaunchKernelGGL(topk_kernel<kTopkMaxPerLane>, grid, block, 0, st, gs, idx, pl.n_groups, p.n_select, hist);
  return hipGetLastError();
}

// Zero-fill of the workspace's arrival counters (a kernel rather than a memset so that
// it can be recorded into a captured graph like every other launch of the library).
__global__ void fill_zero_kernel(uint32_t* ptr, size_t words) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < words) ptr[i] = 0u;
}

hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t st) {
  const size_t words = bytes / 4;
  if (words == 0) return hipSuccess;
  dim3 grid((unsigned)((words + 255) / 256)), block(256);
  hipLaunchKernelGGL(fill_zero_kernel, grid, block, 0, st, (uint32_t*)ptr, words);
  return hipGetLastError();
}

// Overlap of two selections of one set (Sec. 3.4.2: how many of this step's groups were
// already selected in the previous step).  The previous selection is marked in a bitmap
// of N/G bits in LDS, then every current index is looked up; indices of a row are unique,
// in any order.
constexpr int kOverlapThreads = 256;

__global__ __launch_bounds__(kOverlapThreads) void overlap_kernel(const int32_t* __restrict__ idx_prev,
                                                                  const int32_t* __restrict__ idx_cur,
                                                                  int32_t* __restrict__ common, int M,
                                                                  int n_groups) {
  __shared__ uint32_t s_bits[kTopkThreads * kTopkMaxPerLane / 32];  // one bit per group
  __shared__ int s_count;
  const int tid = threadIdx.x, set = blockIdx.x;
  const int words = (n_groups + 31) / 32;
  for (int i = tid; i < words; i += kOverlapThreads) s_bits[i] = 0u;
  if (tid == 0) s_count = 0;
  lds_barrier();
  const int32_t* a = idx_prev + (size_t)set * M;
  const int32_t* b = idx_cur + (size_t)set * M;
  for (int i = tid; i < M; i += kOverlapThreads) {
    const int g = a[i];
    if (g >= 0 && g < n_groups) atomicOr(&s_bits[g >> 5], 1u << (g & 31));
  }
  lds_barrier();
  int mine = 0;
  for (int i = tid; i < M; i += kOverlapThreads) {
    const int g = b[i];
    if (g >= 0 && g < n_groups) mine += (s_bits[g >> 5] >> (g & 31)) & 1u;
  }
  if (mine) atomicAdd(&s_count, mine);
  lds_barrier();
  if (tid == 0) common[set] = s_count;
}

hipError_t launch_overlap(const kvs_params& p, const Plan& pl, const int32_t* idx_prev,
                          const int32_t* idx_cur, int32_t* common, hipStream_t st) {
  hipLaunchKernelGGL(overlap_kernel, dim3(pl.sets), dim3(kOverlapThreads), 0, st, idx_prev, idx_cur,
                     common, p.n_select, pl.n_groups);
  return hipGetLastError();
}

}  // namespace kvs
