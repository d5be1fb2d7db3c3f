// Top-M selection kernel (Sec. 3.3, "TopK"): one workgroup of 1024 lanes per (sequence,
// KV head) problem runs kvs::topk_block on that problem's group scores, either from
// scratch (kvs_select_topk) or starting from the histogram the prediction kernel left
// in the workspace (kvs_predict_select).  The small fill kernel that prepares a
// workspace lives here too.
#include "kernels.h"
#include "topk_block.h"

namespace kvs {

__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float* __restrict__ gs,
                                                            int32_t* __restrict__ idx, int NG,
                                                            int M, int* __restrict__ hist) {
  __shared__ TopkShared sh;
  const int p = blockIdx.x;
  topk_block(gs + (size_t)p * NG, idx + (size_t)p * M, NG, M,
             hist ? hist + (size_t)p * kTopkBins : nullptr, sh);
}

hipError_t launch_topk(const kvs_params& p, const Plan& pl, const float* gs, int32_t* idx,
                       int* hist, hipStream_t st) {
  dim3 grid(pl.sets), block(kTopkThreads);
  hipLaunchKernelGGL(topk_kernel, grid, block, 0, st, gs, idx, pl.n_groups, p.n_select, hist);
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

}  // namespace kvs
