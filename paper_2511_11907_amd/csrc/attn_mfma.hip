// Attention over the selected KV groups on the matrix cores (Sec. 3.4; bf16, d = 128).
//
// Same split-K flash-decode as the vector-ALU kernel (same splits, same per-wave batches of
// 16 tokens, same merge), but the two contractions of a 16-token tile run as MFMA
// instructions with the query heads of the KV head as one matrix dimension, padded to 16:
//
//   S^T (16 tokens x 16 heads) = K_tile (16 x 128) . Q^T (128 x 16)       4 x 16x16x32
//   O^T (128 x 16 heads)      += V_tile^T (128 x 16) . P^T (16 x 16)      8 x 16x16x16
//
// which leaves the vector ALU the softmax of one head per lane (5 exponentials per tile and
// lane instead of 20) and removes its multiply-adds altogether; with more than four query
// heads per KV head the vector-ALU kernel is bound by exactly that arithmetic.
//
// Operand layouts (lane l, c = l % 16, g = l / 16; an instruction takes row/column c and
// the contraction indices of slice g from lane l, and returns column c, rows 4g .. 4g+3):
//   K_tile   row c = token c of the tile; contraction = head dimension, the lane's four
//            16-byte loads are d = 32 j + 8 g .. + 7 (64 contiguous bytes per token and
//            instruction over the four lanes that share the token);
//   Q^T      column c = head c (zero beyond the real heads), same d indices: loaded once;
//   S^T      lane (c, g) receives head c, tokens 4g .. 4g+3: exactly the four contraction
//            indices slice g of the second product needs, so P goes from the accumulator
//            to the operand without crossing lanes (scaled, exponentiated, rounded to bf16);
//   V^T      row c, contraction = tokens 4g .. 4g+3.  The lane loads, for each of these four
//            tokens, the 16 bytes d = 8c .. 8c+7 (each load instruction covers four whole
//            rows); instruction b (0..7) takes element b of the four loads, i.e. its row c
//            stands for d = 8c + b.  The transposition V^T needs is thus only a choice of
//            which output column an accumulator register stands for;
//   O^T      lane (c, g), register i of instruction b: head c, d = 8 (4g + i) + b.
// Every lane therefore owns one head (c) from the logits to the output, so the running
// maximum, the denominator and the rescaling of the accumulators stay in the lane.
#include "attn_mfma_item.h"

KVS_ATTN_TRACE_ACCESSOR(kvs_debug_attn_mfma_trace)

namespace kvs {

// (registers: the plain and rolling-buffer modes fit the 128 that let two workgroups share a
// compute unit; the mapping table's extra look-ahead does not, and a spilled register is
// reloaded in order behind the key loads, i.e. stalls the value loads for a full latency,
// so that mode takes what it needs)
// Start and end time of every workgroup for the debugging harness (compiled only with
// -DKVS_WG_TRACE_BUILD): two words per workgroup, in launch order.
#ifdef KVS_WG_TRACE_BUILD
static __device__ long long g_attn_wg_trace[2 * 8192];
extern "C" int kvs_debug_attn_wg_trace(long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_attn_wg_trace), sizeof(long long) * (size_t)n);
}
extern "C" int kvs_debug_attn_wave_end(long long* host, int n) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_attn_wave_end), sizeof(long long) * (size_t)n);
}
#define KVS_WG_TRACE(i)                                                                     \
  do {                                                                                      \
    const int wg_ = blockIdx.y * gridDim.x + blockIdx.x;                                    \
    if (threadIdx.x == 0 && wg_ < 8192) g_attn_wg_trace[2 * wg_ + (i)] = wall_clock64();    \
  } while (0)
#else
#define KVS_WG_TRACE(i)
#endif

template <int QPK, int MODE, bool INTERLEAVE>
__global__ __launch_bounds__(kAttnThreads, MODE == kAttnPaged ? 2 : 4) void attn_mfma_kernel(AttnMfmaArgs a) {
  __shared__ AttnMfmaShared<QPK, 0> sh;
  KVS_WG_TRACE(0);
  attn_mfma_item<QPK, MODE, INTERLEAVE, 0>(sh, a, blockIdx.y, blockIdx.x);
  KVS_WG_TRACE(1);
}

namespace {

template <int QPK>
hipError_t launch_mfma_qpk(const kvs_params& p, const Plan& pl, const void* q, const void* K,
                           const void* V, const int32_t* idx, float* part_ml, float* part_o,
                           void* out, int* arrivals, const RollingBuffer& rb,
                           const int32_t* slot_table, hipStream_t st) {
  using S = uint16_t;
  const int G = p.group_size;
  int log2G = 0;
  while ((1 << log2G) < G) ++log2G;
  if ((1 << log2G) != G) log2G = -1;
  const uint32_t recipG = (uint32_t)((1ull << 32) / (unsigned)G + 1);  // (only read when log2G < 0)
  const float scale = p.softmax_scale != 0.f ? p.softmax_scale : 1.0f / sqrtf((float)p.head_dim);
  dim3 grid(pl.attn_splits, pl.problems), block(kAttnThreads);
  const int units = (p.n_select * p.group_size + rb.len + pl.kv_toks_per_unit - 1) / pl.kv_toks_per_unit;
  const int units_per_split = attn_units_per_split_with_buffer(pl, units);
  const bool interleave = units_per_split >= kAttnInterleaveFromSteps * kAttnUnitsPerWgStep;
  const AttnMfmaArgs a{(const S*)q, (const S*)K, (const S*)V, idx, part_ml, part_o, (S*)out, arrivals,
                       p.n_kv_heads, pl.kv_heads_per_set, pl.ctx_rows, p.n_select, G, log2G, recipG, units,
                       units_per_split, pl.attn_splits, scale * kLog2e, (const S*)rb.K, (const S*)rb.V,
                       rb.len, rb.capacity, slot_table, pl.n_groups};
  auto launch = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, block, 0, st, a); };
  if (interleave) {
    if (slot_table) launch(attn_mfma_kernel<QPK, kAttnPaged, true>);
    else if (rb.len > 0) launch(attn_mfma_kernel<QPK, kAttnRolling, true>);
    else launch(attn_mfma_kernel<QPK, kAttnPlain, true>);
  } else {
    if (slot_table) launch(attn_mfma_kernel<QPK, kAttnPaged, false>);
    else if (rb.len > 0) launch(attn_mfma_kernel<QPK, kAttnRolling, false>);
    else launch(attn_mfma_kernel<QPK, kAttnPlain, false>);
  }
  return hipGetLastError();
}

}  // namespace

bool attn_mfma_applies(const kvs_params& p, const Plan& pl) {
  return p.kv_dtype == KVS_BF16 && p.head_dim == kMfmaD && pl.kv_toks_per_unit == kTokensPerUnit &&
         pl.q_per_kv >= kAttnMfmaMinHeadsPerKv && pl.q_per_kv <= 8;
}

hipError_t launch_attn_mfma(const kvs_params& p, const Plan& pl, const void* q, const void* K,
                            const void* V, const int32_t* idx, float* part_ml, float* part_o,
                            void* out, int* arrivals, const RollingBuffer& rb,
                            const int32_t* slot_table, hipStream_t st) {
#define KVS_MFMA_CASE(n) \
  case n: return launch_mfma_qpk<n>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
  switch (pl.q_per_kv) {
    KVS_MFMA_CASE(1) KVS_MFMA_CASE(2) KVS_MFMA_CASE(3) KVS_MFMA_CASE(4)
    KVS_MFMA_CASE(5) KVS_MFMA_CASE(6) KVS_MFMA_CASE(7) KVS_MFMA_CASE(8)
  }
#undef KVS_MFMA_CASE
  return hipErrorInvalidValue;
}

}  // namespace kvs
