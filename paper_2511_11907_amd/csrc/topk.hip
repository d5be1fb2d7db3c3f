// Top-M group selection (Sec. 4.3, "TopK"): for each (sequence, KV head) problem,
// the indices of the M groups with the largest representative score, ties going
// to the lower group index, written in ascending index order.
//
// One workgroup of 1024 lanes per problem; every lane keeps a blocked slice of
// the scores in registers as order-preserving 32-bit keys.  An exact MSB-first
// radix select (11 + 11 + 10 bits, LDS histograms) finds the key of the M-th
// largest score; one block-wide prefix sum over (greater, equal) flags then
// places every selected index at its final position.  Integer work only, so the
// result is a deterministic function of the fp32 scores.
#include "device_utils.h"
#include "kernels.h"

namespace kvs {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / kWave;
constexpr int kTopkBins = 2048;

// float -> uint32 whose unsigned order equals the float order; -0 is folded into +0
// so that equal scores have equal keys.
__device__ __forceinline__ uint32_t score_key(float x) {
  const uint32_t u = __float_as_uint(x + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inclusive prefix sum across the workgroup (thread order).  s_wave needs
// kTopkWaves entries; contains two barriers, safe to call back to back.
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t v, uint32_t* s_wave) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  uint32_t incl = wave_inclusive_scan(v);
  if (lane == kWave - 1) s_wave[wave] = incl;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += s_wave[w];
  __syncthreads();
  return incl + base;
}

// hist[digit] += 1 for every lane with `active`, with the few most common digits of
// the wave combined into one LDS atomic each (scores of similar magnitude share
// their leading bits, which would otherwise serialise the atomics).
__device__ __forceinline__ void histogram_add(int* hist, bool active, int digit) {
  const int lane = threadIdx.x & (kWave - 1);
  bool todo = active;
#pragma unroll 1
  for (int it = 0; it < 4; ++it) {
    const unsigned long long pending = __ballot(todo);
    if (pending == 0ull) return;  // wave-uniform
    const int leader = __ffsll((long long)pending) - 1;
    const int d0 = __shfl(digit, leader, kWave);
    const bool mine = todo && (digit == d0);
    const unsigned long long same = __ballot(mine);
    if (lane == leader) atomicAdd(&hist[d0], __popcll(same));
    todo = todo && !mine;
  }
  if (todo) atomicAdd(&hist[digit], 1);
}

template <int KPT>
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float* __restrict__ gs,
                                                            int32_t* __restrict__ idx, int NG,
                                                            int M) {
  __shared__ int s_hist[kTopkBins];
  __shared__ uint32_t s_wave[kTopkWaves];
  __shared__ int s_sel[2];  // {digit of the M-th key, number of candidates in higher bins}

  const int tid = threadIdx.x;
  const int p = blockIdx.x;
  const float* g = gs + (size_t)p * NG;
  int32_t* out = idx + (size_t)p * M;

  uint32_t key[KPT];
  const int first = tid * KPT;
#pragma unroll
  for (int j = 0; j < KPT; ++j) key[j] = (first + j < NG) ? score_key(g[first + j]) : 0u;

  uint32_t prefix = 0u, pmask = 0u;
  int need = M;  // rank of the wanted key among the keys that still match the prefix
#pragma unroll 1
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = (pass == 0) ? 21 : (pass == 1) ? 10 : 0;
    const int bits = (pass == 2) ? 10 : 11;
    const int nb = 1 << bits;
    for (int i = tid; i < kTopkBins; i += kTopkThreads) s_hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
      const bool active = (first + j < NG) && ((key[j] & pmask) == prefix);
      histogram_add(s_hist, active, (int)((key[j] >> shift) & (uint32_t)(nb - 1)));
    }
    __syncthreads();
    // scan the bins from the top: thread t owns bins nb-1-t*bpt downwards
    const int bpt = nb / kTopkThreads;  // 2, 2, 1
    uint32_t mine = 0;
    for (int c = 0; c < bpt; ++c) mine += (uint32_t)s_hist[nb - 1 - (tid * bpt + c)];
    const uint32_t incl = block_inclusive_scan(mine, s_wave);
    int above = (int)(incl - mine);  // candidates in bins above my first bin
    for (int c = 0; c < bpt; ++c) {
      const int bin = nb - 1 - (tid * bpt + c);
      const int cnt = s_hist[bin];
      if (above < need && need <= above + cnt) {
        s_sel[0] = bin;
        s_sel[1] = above;
      }
      above += cnt;
    }
    __syncthreads();
    prefix |= (uint32_t)s_sel[0] << shift;
    pmask |= (uint32_t)(nb - 1) << shift;
    need -= s_sel[1];
    __syncthreads();  // s_sel and s_hist are rewritten by the next pass
  }
  // prefix is now the key of the M-th largest score; `need` of the groups that
  // carry exactly this key are selected, lowest indices first.
  const uint32_t T = prefix;
  uint32_t packed = 0;  // low half: keys > T, high half: keys == T, in my slice
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    if (first + j < NG) {
      packed += (key[j] > T) ? 1u : 0u;
      packed += (key[j] == T) ? 0x10000u : 0u;
    }
  }
  const uint32_t excl = block_inclusive_scan(packed, s_wave) - packed;
  int gt_before = (int)(excl & 0xFFFFu);
  int eq_before = (int)(excl >> 16);
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    if (first + j < NG) {
      const bool gt = key[j] > T, eq = key[j] == T;
      if (gt || (eq && eq_before < need)) out[gt_before + min(eq_before, need)] = first + j;
      gt_before += gt ? 1 : 0;
      eq_before += eq ? 1 : 0;
    }
  }
}

hipError_t launch_topk(const kvs_params& p, const Plan& pl, const float* gs, int32_t* idx,
                       hipStream_t st) {
  const int NG = pl.n_groups, M = p.n_select;
  dim3 grid(pl.problems), block(kTopkThreads);
  const int kpt = (NG + kTopkThreads - 1) / kTopkThreads;
#define KVS_TOPK(KPT) hipLaunchKernelGGL((topk_kernel<KPT>), grid, block, 0, st, gs, idx, NG, M)
  if (kpt <= 1) KVS_TOPK(1);
  else if (kpt <= 2) KVS_TOPK(2);
  else if (kpt <= 4) KVS_TOPK(4);
  else if (kpt <= 8) KVS_TOPK(8);
  else if (kpt <= 16) KVS_TOPK(16);
  else if (kpt <= 32) KVS_TOPK(32);
  else return hipErrorInvalidValue;
#undef KVS_TOPK
  return hipGetLastError();
}

}  // namespace kvs
