// Second half of the split-K attention kernels, shared by the vector-ALU and the
// matrix-core variant: merge the per-wave online-softmax states of a workgroup, publish
// the workgroup's partial result, and let the workgroup of a problem that arrives last
// merge the splits and write the output (log-sum-exp rescaling throughout; logits are in
// log2 units).
#pragma once

#include <type_traits>

#include "device_utils.h"
#include "kernels.h"

// Phase timestamps for the debugging harness (compiled only with -DKVS_ATTN_TRACE_BUILD): one
// row of 8 wall-clock stamps per workgroup, in an array of the including source file's own.
#ifdef KVS_ATTN_TRACE_BUILD
static __device__ long long g_attn_trace[1 << 16];
#define KVS_ATTN_TRACE(i)                                                                           \
  do {                                                                                               \
    if (threadIdx.x == 0) g_attn_trace[((blockIdx.y * gridDim.x + blockIdx.x) * 8 + (i)) & 0xFFFF] = wall_clock64(); \
  } while (0)
#define KVS_ATTN_TRACE_ACCESSOR(name)                                                               \
  extern "C" int name(long long* host, int n) {                                                     \
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_attn_trace), sizeof(long long) * (size_t)n); \
  }
#else
#define KVS_ATTN_TRACE(i)
#define KVS_ATTN_TRACE_ACCESSOR(name)
#endif

namespace kvs {

constexpr int kAttnThreads = kAttnWgThreads;
constexpr int kAttnWaves = kAttnThreads / kWave;
constexpr int kAttnMaxSplits = kAttnMaxSplitsPerProblem;
constexpr int kAttnMergeRound = 32;  // splits whose partial results the final merge requests together
constexpr float kNegBig = -1.0e30f;  // "no token seen yet" running max (finite on purpose)
constexpr float kLog2e = 1.4426950408889634f;

// MODE selects what the gather has to support beyond the plain cache; each feature is
// compiled out of the modes below it, so the plain path pays nothing for them:
//   kAttnPlain   selected groups are rows of this problem's contiguous cache
//   kAttnRolling + the attended-token list continues into a rolling buffer (Sec. 3.4.1)
//   kAttnPaged   + groups are addressed through a mapping table (Sec. 3.4.4): K and V are
//                  pools of group-sized slots shared by all problems, slot_table[p][j]
//                  is the slot that holds logical group j of problem p
constexpr int kAttnPlain = 0, kAttnRolling = 1, kAttnPaged = 2;

// Units per split when the attended-token list is longer than the selection the plan was
// made for (the rolling buffer's tokens follow the selected ones): the number of splits -
// and with it the workspace layout - stays, the units are dealt out evenly again, so the
// buffer does not cost the last split an extra batch.
inline int attn_units_per_split_with_buffer(const Plan& pl, int units) {
  const int even = (units + pl.attn_splits - 1) / pl.attn_splits;
  const int rounded = (even + kAttnUnitsPerWave - 1) / kAttnUnitsPerWave * kAttnUnitsPerWave;
  return rounded > pl.attn_units_per_split ? rounded : pl.attn_units_per_split;
}

// Per-wave states as the first half leaves them in LDS: for wave w and head h the running
// max m, the sum l of 2^(z - m) and the accordingly weighted sum o of value rows.
//
// o is stored with the heads innermost - element (h, d) of a wave at d * QPK + h - plus a
// pad after every 32 values of d that moves consecutive blocks 16 banks apart.  The merge
// then reads consecutive words; the matrix-core kernel, whose store instructions have lane
// (h, g) write d = 32 g + const, hits 16 g + h: a different bank for every active lane
// (with the plain [h][d] layout all of them fell on two banks, 1.6 us per workgroup).  The
// partial results in the workspace use the same heads-innermost order (without the pads).
template <int D, int QPK>
struct AttnWaveStates {
  static constexpr int kPad = (QPK % 2 == 0) ? 16 : 48;  // (32 * QPK + kPad) % 64 == 16
  static constexpr int kWords = QPK * D + (D / 32) * kPad;
  static __device__ __forceinline__ int pos(int h, int d) { return d * QPK + h + (d / 32) * kPad; }
  float m[kAttnWaves][QPK];
  float l[kAttnWaves][QPK];
  float o[kAttnWaves][kWords];
};

// LDS of the merge over the splits (used by the last workgroup of a problem only).
template <int QPK>
struct AttnMergeShared {
  int last;
  float cw[kAttnMaxSplits][QPK];  // weight of each split, per head
  float cl[QPK];                  // merged softmax denominators
};

// Every lane of the workgroup calls this after its wave's state is written to `ws` (no
// barrier needed before the call).  p: problem (sequence, KV head); op: the QPK output
// rows of this problem.  Returns true (on all lanes) in the workgroup that wrote the
// problem's output: the only one, or the one that arrived last.
template <typename E, int D, int QPK>
__device__ __forceinline__ bool attn_merge_and_finish(AttnWaveStates<D, QPK>& ws, AttnMergeShared<QPK>& ms,
                                                      float* part_ml, float* part_o,
                                                      typename E::storage* op, int* __restrict__ arrivals,
                                                      int p, int split, int n_splits) {
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  auto& s_m = ws.m;
  auto& s_l = ws.l;
  auto& s_o = ws.o;
  lds_barrier();
  // Every lane merges the waves' states for its own (head, d) elements.  The waves' weights
  // exp2(m_wave - m) are recomputed by every lane (a few instructions) rather than computed
  // once and handed on through LDS, which would cost a barrier.
  float* ml = part_ml + ((size_t)p * n_splits + split) * QPK * 2;
  float* po = part_o + ((size_t)p * n_splits + split) * QPK * D;
  for (int i = tid; i < QPK * D; i += kAttnThreads) {  // i = d * QPK + h
    const int h = i % QPK, dd = i / QPK;
    const int at = AttnWaveStates<D, QPK>::pos(h, dd);
    float m_w[kAttnWaves], l_w[kAttnWaves], o_w[kAttnWaves];
#pragma unroll
    for (int s = 0; s < kAttnWaves; ++s) m_w[s] = s_m[s][h], l_w[s] = s_l[s][h], o_w[s] = s_o[s][at];
    float mt = kNegBig;
#pragma unroll
    for (int s = 0; s < kAttnWaves; ++s) mt = fmaxf(mt, m_w[s]);
    float lt = 0.f, acc = 0.f;
#pragma unroll
    for (int s = 0; s < kAttnWaves; ++s) {
      const float w = __builtin_amdgcn_exp2f(m_w[s] - mt);
      lt += w * l_w[s];
      acc = fmaf(w, o_w[s], acc);
    }
    if (n_splits == 1) {  // uniform: the problem was not split, this is its result
      const float r = acc / lt;
      if constexpr (E::kBytes == 2) op[h * D + dd] = float_to_bf16_bits(r);
      else op[h * D + dd] = r;
    } else {
      publish_store(&po[i], acc);
      if (dd == 0) {
        publish_store(&ml[h * 2 + 0], mt);
        publish_store(&ml[h * 2 + 1], lt);
      }
    }
  }
  if (n_splits == 1) return true;  // uniform

  // ---- the last workgroup of the problem merges the splits ------------------------
  int& s_last = ms.last;
  auto& s_cw = ms.cw;
  auto& s_cl = ms.cl;
  KVS_ATTN_TRACE(3);
  publish_complete_and_barrier();  // the partials are out before the arrival is announced
  KVS_ATTN_TRACE(4);
  if (tid == 0) {
    const int old = atomicAdd(&arrivals[p], 1);
    s_last = (old == n_splits - 1);
    if (s_last) publish_store(&arrivals[p], 0);  // leave the counter ready for the next call
  }
  lds_barrier();
  KVS_ATTN_TRACE(5);
  if (!s_last) return false;
  consume_fence();
  const float* pml = part_ml + (size_t)p * n_splits * QPK * 2;
  for (int h = wave; h < QPK; h += kAttnWaves) {  // one wave per head, lanes over splits
    // (m, l) of this lane's splits, all requested at once: one memory latency
    constexpr int kPerLane = kAttnMaxSplits / kWave;
    float m_s[kPerLane], l_s[kPerLane];
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) {
      const size_t at = ((size_t)min(lane + j * kWave, n_splits - 1) * QPK + h) * 2;
      m_s[j] = load_published(&pml[at]);
      l_s[j] = load_published(&pml[at + 1]);
    }
    float mt = kNegBig;
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) mt = (lane + j * kWave < n_splits) ? fmaxf(mt, m_s[j]) : mt;
    mt = allreduce_lanes<OpMax, 1, kWave>(mt);
    float lt = 0.f;
#pragma unroll
    for (int j = 0; j < kPerLane; ++j) {
      const int s = lane + j * kWave;
      if (s < n_splits) {
        const float w = __builtin_amdgcn_exp2f(m_s[j] - mt);
        s_cw[s][h] = w;
        lt = fmaf(w, l_s[j], lt);
      }
    }
    lt = allreduce_lanes<OpSum, 1, kWave>(lt);
    if (lane == 0) s_cl[h] = lt;
  }
  lds_barrier();
  const float* ppo = part_o + (size_t)p * n_splits * QPK * D;
  for (int i = tid; i < QPK * D; i += kAttnThreads) {  // i = d * QPK + h
    const int h = i % QPK, dd = i / QPK;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    // The partial results of many splits are requested together before the first is used:
    // these loads go past the caches, so every round of requests costs a full memory
    // latency.  Whole rounds of kAttnMergeRound splits, then one round for the rest, sized
    // to the next power of two (indices clamped, surplus weights zero).
    auto take = [&](auto round_size, int s0) __attribute__((always_inline)) {
      constexpr int kRound = decltype(round_size)::value;
      float v[kRound];
#pragma unroll
      for (int j = 0; j < kRound; ++j)
        v[j] = load_published(&ppo[(size_t)min(s0 + j, n_splits - 1) * QPK * D + i]);
#pragma unroll
      for (int j = 0; j < kRound; ++j) {
        const float w = (s0 + j < n_splits) ? s_cw[min(s0 + j, n_splits - 1)][h] : 0.f;
        acc[j & 3] = fmaf(w, v[j], acc[j & 3]);
      }
    };
    int s0 = 0;
    for (; s0 + kAttnMergeRound <= n_splits; s0 += kAttnMergeRound)
      take(std::integral_constant<int, kAttnMergeRound>{}, s0);
    const int rest = n_splits - s0;  // uniform
    if (rest > 16) take(std::integral_constant<int, 32>{}, s0);
    else if (rest > 8) take(std::integral_constant<int, 16>{}, s0);
    else if (rest > 4) take(std::integral_constant<int, 8>{}, s0);
    else if (rest > 0) take(std::integral_constant<int, 4>{}, s0);
    const float r = ((acc[0] + acc[1]) + (acc[2] + acc[3])) / s_cl[h];
    if constexpr (E::kBytes == 2) op[h * D + dd] = float_to_bf16_bits(r);
    else op[h * D + dd] = r;
  }
  return true;
}

}  // namespace kvs
