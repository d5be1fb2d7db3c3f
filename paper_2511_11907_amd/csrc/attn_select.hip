// Attention of one layer and top-M selection for the next layer in one launch.
//
// The method runs as a pipeline over layers (Sec. 3.3, 3.4): the groups of layer i+1 are
// predicted from a query that is known one layer early, while layer i is still computing.
// On the GPU the latency-bound part of that prediction is the selection: a chain of about a
// dozen dependent steps over a few KiB that keeps one compute unit per problem busy for
// 7-12 us while the memory system idles.  Here it shares a launch with the one kernel it
// does not depend on, the gathered attention of the layer before: the first workgroups of
// the grid (one per selection set) run the selection routine on the next layer's group
// scores, all others are the attention kernel's workgroups, unchanged.  Nothing in the
// launch waits for anything else in it: the two parts touch disjoint data.
//
// Results are those of the separate kernels bit for bit: the attention workgroups run the
// same routine on the same split plan, and the selection is a function of the scores alone
// (here by 512 lanes with twice the keys per lane, which does not change what is selected).
#include "attn_mfma_item.h"
#include "topk_block.h"

#include <type_traits>

namespace kvs {

constexpr int kAttnSelectThreads = 512;
static_assert(kAttnSelectThreads == kAttnThreads, "the attention routine's workgroup size");
constexpr int kAttnSelectMaxGroups = kAttnSelectThreads * kTopkMaxPerLane;  // 16384 scores per selection set

struct SelectNextArgs {
  const float* gs;  // [sets, NG] group scores of the next layer
  int32_t* idx;     // [sets, M] receives its selection
  int* hist;        // nullable: finished score histograms (kTopkBins per set), left zeroed
  int sets, NG, M;
};

// MODE: kAttnPlain or kAttnRolling (the attention also covers the rolling buffer's tokens).
template <int QPK, int MODE, bool INTERLEAVE, int SLOTS>
__global__ __launch_bounds__(kAttnSelectThreads, 4) void attn_select_kernel(AttnMfmaArgs a, SelectNextArgs s) {
  union Shared {
    AttnMfmaShared<QPK, 0> attn;
    TopkShared topk;
  };
  __shared__ Shared sh;
  const int wg = blockIdx.x;
  if (wg < s.sets) {  // (uniform) the selection workgroups come first: they are dispatched first
    topk_block<SLOTS, kAttnSelectThreads>(s.gs + (size_t)wg * s.NG, s.idx + (size_t)wg * s.M, s.NG, s.M,
                                          s.hist ? s.hist + (size_t)wg * kTopkBins : nullptr, sh.topk);
    return;
  }
  const int item = wg - s.sets;
  attn_mfma_item<QPK, MODE, INTERLEAVE, 0>(sh.attn, a, item / a.n_splits, item % a.n_splits);
}

namespace {

template <int QPK>
hipError_t launch_qpk(const kvs_params& p, const Plan& pl, const void* q, const void* K, const void* V,
                      const int32_t* idx, float* part_ml, float* part_o, void* out, int* arrivals,
                      const RollingBuffer& rb, const float* next_gs, int32_t* next_idx, int* hist,
                      hipStream_t st) {
  using S = uint16_t;
  const int G = p.group_size;
  int log2G = 0;
  while ((1 << log2G) < G) ++log2G;
  if ((1 << log2G) != G) log2G = -1;
  const uint32_t recipG = (uint32_t)((1ull << 32) / (unsigned)G + 1);  // (only read when log2G < 0)
  const float scale = p.softmax_scale != 0.f ? p.softmax_scale : 1.0f / sqrtf((float)p.head_dim);
  // the split plan of the stand-alone attention kernel
  const int units = (p.n_select * p.group_size + rb.len + pl.kv_toks_per_unit - 1) / pl.kv_toks_per_unit;
  const int units_per_split = attn_units_per_split_with_buffer(pl, units);
  const bool interleave = units_per_split >= kAttnInterleaveFromSteps * kAttnUnitsPerWgStep;
  const AttnMfmaArgs a{(const S*)q, (const S*)K, (const S*)V, idx, part_ml, part_o, (S*)out, arrivals,
                       p.n_kv_heads, pl.kv_heads_per_set, pl.ctx_rows, p.n_select, G, log2G, recipG, units,
                       units_per_split, pl.attn_splits, scale * kLog2e, (const S*)rb.K, (const S*)rb.V, rb.len,
                       rb.capacity, nullptr, pl.n_groups};
  const SelectNextArgs s{next_gs, next_idx, hist, pl.sets, pl.n_groups, p.n_select};
  const dim3 grid(pl.sets + pl.problems * pl.attn_splits), block(kAttnSelectThreads);
  const bool small = pl.n_groups <= kAttnSelectThreads * 16;
  auto launch = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, block, 0, st, a, s); };
  auto pick = [&](auto mode, auto il) {
    constexpr int M_ = decltype(mode)::value;
    constexpr bool I_ = decltype(il)::value;
    if (small) launch(attn_select_kernel<QPK, M_, I_, 16>);
    else launch(attn_select_kernel<QPK, M_, I_, kTopkMaxPerLane>);
  };
  using Plain = std::integral_constant<int, kAttnPlain>;
  using Rolling = std::integral_constant<int, kAttnRolling>;
  if (rb.len > 0) {
    if (interleave) pick(Rolling{}, std::true_type{});
    else pick(Rolling{}, std::false_type{});
  } else {
    if (interleave) pick(Plain{}, std::true_type{});
    else pick(Plain{}, std::false_type{});
  }
  return hipGetLastError();
}

}  // namespace

bool attn_select_applies(const kvs_params& p, const Plan& pl) {
  return attn_mfma_applies(p, pl) && pl.q_per_kv >= 3 && pl.n_groups <= kAttnSelectMaxGroups;
}

hipError_t launch_attn_select(const kvs_params& p, const Plan& pl, const void* q, const void* K, const void* V,
                              const int32_t* idx, float* part_ml, float* part_o, void* out, int* arrivals,
                              const RollingBuffer& rb, const float* next_gs, int32_t* next_idx, int* hist,
                              hipStream_t st) {
#define KVS_CASE(n) \
  case n: return launch_qpk<n>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, next_gs, next_idx, hist, st);
  switch (pl.q_per_kv) {
    KVS_CASE(3) KVS_CASE(4) KVS_CASE(5) KVS_CASE(6) KVS_CASE(7) KVS_CASE(8)
  }
#undef KVS_CASE
  return hipErrorInvalidValue;
}

}  // namespace kvs
