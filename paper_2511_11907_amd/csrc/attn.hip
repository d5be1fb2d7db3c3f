// Attention over the selected KV groups only (Sec. 3.4: the attention kernel consumes
// the groups the predictor chose; here they are gathered straight from the full
// K/V in HBM, which stands in for the paper's preload buffer).  This is the vector-ALU
// kernel, for every layout the matrix-core one (attn_mfma.hip: bf16, d = 128, three or
// more query heads per KV head) does not take: fp32 keys and values, d = 64, one or two
// heads per KV head.  launch_attn at the end of the file picks between the two.
//
// Split-K flash-decode.  A (sequence, KV head) problem owns M groups = M*G tokens;
// the token list is cut into "units" of one wave-wide 16-byte-per-lane load
// (64/LPT tokens, LPT lanes per token), units are dealt to `attn_splits`
// workgroups, and inside a workgroup to its waves.  All H_q/H_kv query heads
// that share the KV head are processed together so K and V are read once (GQA
// head packing).  A lane keeps, for its 16-byte column of the head dimension, an
// independent online-softmax state (running max, running sum, weighted V sum) per
// head for the token slot it serves; slots, waves and finally splits are merged
// with the usual log-sum-exp rescaling.  A group is G consecutive rows, i.e. one
// contiguous run of G*d elements, so with G*LPT = 64 a unit is exactly one group
// and every wave-wide load is a fully used 1 KiB burst.
//
// The final merge over the splits is done by the workgroup of a problem that finishes
// last (arrival counter in the workspace, no waiting), so the whole attention is one
// launch.
#include "device_utils.h"
#include "kernels.h"

#include "attn_merge.h"

KVS_ATTN_TRACE_ACCESSOR(kvs_debug_attn_trace)

namespace kvs {

constexpr int kAttnUnroll = kAttnUnitsPerWgStep / kAttnWaves;  // units (K load + V load each) in flight per wave

// Waves per SIMD the register budget is set for: 4 (128 registers, two workgroups per
// compute unit) wherever that compiles without spills - a spilled register is reloaded in
// order behind the loads in flight and stalls the wave for a full memory latency.
template <typename E, int QPK, int MODE>
constexpr int attn_min_waves() {
  if (MODE == kAttnPaged && E::kBytes == 2 && QPK >= 4) return 2;  // (its look-ahead needs the registers)
  if (QPK <= 4) return 4;
  if (QPK == 5 && (E::kBytes == 4 || MODE == kAttnPlain)) return 4;
  return 2;
}

template <typename E, int D, int QPK, int MODE>
__global__ __launch_bounds__(kAttnThreads, (attn_min_waves<E, QPK, MODE>())) void attn_partial_kernel(
    const typename E::storage* __restrict__ q, const typename E::storage* __restrict__ K,
    const typename E::storage* __restrict__ V, const int32_t* __restrict__ idx,
    float* part_ml, float* part_o, typename E::storage* __restrict__ out,
    int* __restrict__ arrivals, int n_kv_heads, int kv_heads_per_set, int ctx_rows, int M, int G,
    int log2G, uint32_t recipG,
    int units, int units_per_split, int n_splits, float scale_log2e,
    const typename E::storage* __restrict__ rb_K, const typename E::storage* __restrict__ rb_V,
    int rb_len, int rb_capacity, const int32_t* __restrict__ slot_table, int n_groups) {
  constexpr bool RB = MODE >= kAttnRolling;
  constexpr bool PAGED = MODE == kAttnPaged;
  constexpr int EPL = E::kPerLane;
  constexpr int LPT = D / EPL;       // lanes per token row
  constexpr int TPU = kWave / LPT;   // tokens per unit
  static_assert(LPT == 8 || LPT == 16 || LPT == 32, "row must span 8, 16 or 32 lanes");

  // per-wave partial states, merged by the whole workgroup at the end
  __shared__ AttnWaveStates<D, QPK> ws;
  __shared__ AttnMergeShared<QPK> ms;

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int split = blockIdx.x, p = blockIdx.y;
  KVS_ATTN_TRACE(0);
#ifdef KVS_ATTN_TRACE_BUILD
  if (threadIdx.x == 0)  // where the workgroup runs: XCC id (hwreg 20), HW id (hwreg 4)
    g_attn_trace[((blockIdx.y * gridDim.x + blockIdx.x) * 8 + 7) & 0xFFFF] =
        ((long long)__builtin_amdgcn_s_getreg((31 << 11) | 20) << 32) | (unsigned)__builtin_amdgcn_s_getreg((31 << 11) | 4);
#endif
  const int b = p / n_kv_heads, k = p % n_kv_heads;
  const int n_q_heads = n_kv_heads * QPK;
  const int c = lane % LPT;   // 16-byte column of the row
  const int ts = lane / LPT;  // token slot within the unit
  const int n_tok = M * G;
  // position of a token of the attended list -> which of the M selected groups it is in.
  // log2G < 0: G is not a power of two and recipG = floor(2^32 / G) + 1, which makes the
  // high half of tok * recipG equal to tok / G for every tok below 2^28 / G.
  auto group_of = [&](int tok) {
    return log2G >= 0 ? tok >> log2G : (int)__umulhi((uint32_t)tok, recipG);
  };

  // Queries of the QPK heads of this KV head.  fp32: as floats, pre-multiplied by
  // scale*log2(e).  bf16: left packed as they are stored (half the registers) and multiplied
  // against the packed keys with the two-element bf16 dot instruction, which forms the
  // products exactly in fp32; the scale is applied to the finished logit.
  constexpr bool kPackedQK = (E::kBytes == 2);
  float qr[kPackedQK ? 1 : QPK][kPackedQK ? 1 : EPL];
  uint4 qp[kPackedQK ? QPK : 1];
#pragma unroll
  for (int h = 0; h < QPK; ++h) {
    const size_t off = ((size_t)b * n_q_heads + (size_t)k * QPK + h) * D + (size_t)c * EPL;
    const uint4 v = *reinterpret_cast<const uint4*>(q + off);
    if constexpr (kPackedQK) {
      qp[h] = v;
    } else {
      unpack16<E>(v, qr[h]);
#pragma unroll
      for (int e = 0; e < EPL; ++e) qr[h][e] *= scale_log2e;
    }
  }

  float m[QPK], l[QPK], o[QPK][EPL];
#pragma unroll
  for (int h = 0; h < QPK; ++h) {
    m[h] = kNegBig;
    l[h] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[h][e] = 0.f;
  }

  const typename E::storage* Kp = PAGED ? K : K + (size_t)p * ctx_rows * D;
  const typename E::storage* Vp = PAGED ? V : V + (size_t)p * ctx_rows * D;
  const int32_t* tab = slot_table + (size_t)p * n_groups;  // (only read when PAGED)
  // rolling buffer (Sec. 3.4.1): the newest rb_len tokens follow the selected ones in the
  // token list; they are read from their own small arrays
  const typename E::storage* Kr = rb_K + (size_t)p * rb_capacity * D;
  const typename E::storage* Vr = rb_V + (size_t)p * rb_capacity * D;
  const int n_all = RB ? n_tok + rb_len : n_tok;
  // the selection of this problem's set: its own, or the one its sequence shares
  const int32_t* sel = idx + (size_t)(p / kv_heads_per_set) * M;
  const int u0 = split * units_per_split;
  // the splits partition the units of the selected tokens; the few units of the rolling
  // buffer are taken by the last split
  const int u1 = (split == n_splits - 1) ? units : min(units, u0 + units_per_split);

  // Where the selected groups of a batch are is looked up one batch ahead, while the
  // previous batch's keys and values are still on their way: a batch then costs one memory
  // latency, not two in a row.  With a mapping table the slot look-up depends on the group
  // look-up; done in the same iteration it would be waited for on the spot, together with
  // every load issued before it, so groups are found two batches ahead and slots one.
  auto locate_groups = [&](int ubase, int (&g)[kAttnUnroll]) {
#pragma unroll
    for (int u = 0; u < kAttnUnroll; ++u) {
      const int tok = (ubase + u) * TPU + ts;  // position in the attended-token list
      const bool in_cache = (ubase + u < u1) && (tok < n_tok);
      g[u] = in_cache ? sel[group_of(tok)] : 0;
    }
  };
  auto locate_slots = [&](int ubase, int (&g)[kAttnUnroll]) {  // logical group -> slot, in place
#pragma unroll
    for (int u = 0; u < kAttnUnroll; ++u) {
      const int tok = (ubase + u) * TPU + ts;
      const bool in_cache = (ubase + u < u1) && (tok < n_tok);
      g[u] = in_cache ? tab[g[u]] : 0;
    }
  };
  // request(ub, g, kv, vv): issue the K and V loads of the batch that starts at unit ub, whose
  // groups (slots) g were looked up before.  Units past the end load row 0 and are ignored.
  auto request = [&](int ub, const int (&g)[kAttnUnroll], uint4 (&kv)[kAttnUnroll], uint4 (&vv)[kAttnUnroll]) {
    size_t off[kAttnUnroll];
    bool rbf[kAttnUnroll];
#pragma unroll
    for (int u = 0; u < kAttnUnroll; ++u) {
      const int tok = (ub + u) * TPU + ts;
      const bool ok = (ub + u < u1) && (tok < n_all);
      rbf[u] = RB && ok && (tok >= n_tok);
      // (a slot index times G may not fit 32 bits: the pool is shared by all problems)
      const size_t row = rbf[u] ? (size_t)(tok - n_tok)
                                : (size_t)g[u] * (size_t)G + (size_t)(tok - group_of(tok) * G);
      off[u] = (ok ? row : 0) * D + (size_t)c * EPL;
    }
#pragma unroll
    for (int u = 0; u < kAttnUnroll; ++u)
      kv[u] = load16<true>((RB && rbf[u] ? Kr : Kp) + off[u]);  // read once: non-temporal
#pragma unroll
    for (int u = 0; u < kAttnUnroll; ++u)
      vv[u] = load16<true>((RB && rbf[u] ? Vr : Vp) + off[u]);
  };
  // consume(ub, kv, vv): online-softmax update with the batch that starts at unit ub
  auto consume = [&](int ub, const uint4 (&kv)[kAttnUnroll], const uint4 (&vv)[kAttnUnroll]) {
    bool ok[kAttnUnroll];
#pragma unroll
    for (int u = 0; u < kAttnUnroll; ++u) ok[u] = (ub + u < u1) && ((ub + u) * TPU + ts < n_all);
    // logits (already in log2 units) of this slot's token against each head
    float z[kAttnUnroll][QPK];
#pragma unroll
    for (int u = 0; u < kAttnUnroll; ++u) {
      if constexpr (kPackedQK) {
#pragma unroll
        for (int h = 0; h < QPK; ++h) {
          float acc = dot2_bf16(qp[h].x, kv[u].x, 0.f);
          acc = dot2_bf16(qp[h].y, kv[u].y, acc);
          acc = dot2_bf16(qp[h].z, kv[u].z, acc);
          acc = dot2_bf16(qp[h].w, kv[u].w, acc);
          z[u][h] = allreduce_lanes<OpSum, 1, LPT>(acc) * scale_log2e;
        }
      } else {
        float kf[EPL];
        unpack16<E>(kv[u], kf);
#pragma unroll
        for (int h = 0; h < QPK; ++h) {
          float acc = 0.f;
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc = fmaf(qr[h][e], kf[e], acc);
          z[u][h] = allreduce_lanes<OpSum, 1, LPT>(acc);
        }
      }
    }
    // online softmax update, one rescale per batch
    float pw[kAttnUnroll][QPK];
#pragma unroll
    for (int h = 0; h < QPK; ++h) {
      float mn = m[h];
#pragma unroll
      for (int u = 0; u < kAttnUnroll; ++u) mn = ok[u] ? fmaxf(mn, z[u][h]) : mn;
      const float alpha = __builtin_amdgcn_exp2f(m[h] - mn);
      m[h] = mn;
      float ls = l[h] * alpha;
#pragma unroll
      for (int u = 0; u < kAttnUnroll; ++u) {
        pw[u][h] = ok[u] ? __builtin_amdgcn_exp2f(z[u][h] - mn) : 0.f;
        ls += pw[u][h];
      }
      l[h] = ls;
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[h][e] *= alpha;
    }
#pragma unroll
    for (int u = 0; u < kAttnUnroll; ++u) {
      float vf[EPL];
      unpack16<E>(vv[u], vf);
#pragma unroll
      for (int h = 0; h < QPK; ++h)
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[h][e] = fmaf(pw[u][h], vf[e], o[h][e]);
    }
  };

  constexpr int kStep = kAttnWaves * kAttnUnroll;
  const int ub0 = u0 + wave * kAttnUnroll;
  int grp[kAttnUnroll], grp_next[kAttnUnroll], ahead[kAttnUnroll];
  uint4 kv[kAttnUnroll], vv[kAttnUnroll];
  locate_groups(ub0, grp);
  if constexpr (PAGED) {
    locate_slots(ub0, grp);
    locate_groups(ub0 + kStep, ahead);
  }
  KVS_ATTN_TRACE(1);
  for (int ub = ub0; ub < u1; ub += kStep) {
    request(ub, grp, kv, vv);
    if constexpr (PAGED) {
#pragma unroll
      for (int u = 0; u < kAttnUnroll; ++u) grp_next[u] = ahead[u];  // found an iteration ago
      locate_slots(ub + kStep, grp_next);
      locate_groups(ub + 2 * kStep, ahead);  // (past the end: nothing is read)
    } else {
      locate_groups(ub + kStep, grp_next);   // (past the end: nothing is read)
    }
    consume(ub, kv, vv);
#pragma unroll
    for (int u = 0; u < kAttnUnroll; ++u) grp[u] = grp_next[u];
  }

  KVS_ATTN_TRACE(2);
  // ---- merge the token slots of the wave (lanes with equal column c) ------------
#pragma unroll
  for (int h = 0; h < QPK; ++h) {
    const float mw = allreduce_lanes<OpMax, LPT, kWave>(m[h]);
    const float w = __builtin_amdgcn_exp2f(m[h] - mw);
    m[h] = mw;
    l[h] = allreduce_lanes<OpSum, LPT, kWave>(l[h] * w);
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[h][e] = allreduce_lanes<OpSum, LPT, kWave>(o[h][e] * w);
  }
  // ---- merge the waves of the workgroup ------------------------------------------
  if (ts == 0) {
#pragma unroll
    for (int h = 0; h < QPK; ++h) {
      if (c == 0) {
        ws.m[wave][h] = m[h];
        ws.l[wave][h] = l[h];
      }
#pragma unroll
      for (int e = 0; e < EPL; ++e) ws.o[wave][AttnWaveStates<D, QPK>::pos(h, c * EPL + e)] = o[h][e];
    }
  }
  attn_merge_and_finish<E, D, QPK>(ws, ms, part_ml, part_o,
                                   out + ((size_t)b * n_q_heads + (size_t)k * QPK) * D, arrivals, p,
                                   split, n_splits);
  KVS_ATTN_TRACE(6);
}

namespace {

template <typename E, int D, int QPK>
hipError_t launch_partial(const kvs_params& p, const Plan& pl, const void* q, const void* K,
                          const void* V, const int32_t* idx, float* part_ml, float* part_o,
                          void* out, int* arrivals, const RollingBuffer& rb, const int32_t* slot_table,
                          hipStream_t st) {
  using S = typename E::storage;
  const int G = p.group_size;
  int log2G = 0;
  while ((1 << log2G) < G) ++log2G;
  if ((1 << log2G) != G) log2G = -1;
  const uint32_t recipG = (uint32_t)((1ull << 32) / (unsigned)G + 1);  // (only read when log2G < 0)
  const float scale = p.softmax_scale != 0.f ? p.softmax_scale : 1.0f / sqrtf((float)p.head_dim);
  dim3 grid(pl.attn_splits, pl.problems), block(kAttnThreads);
  // units of the whole attended-token list: the selected tokens, then the rolling buffer
  const int units = (p.n_select * p.group_size + rb.len + pl.kv_toks_per_unit - 1) / pl.kv_toks_per_unit;
  const int units_per_split = attn_units_per_split_with_buffer(pl, units);
  auto launch = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, grid, block, 0, st, (const S*)q, (const S*)K, (const S*)V, idx, part_ml,
                       part_o, (S*)out, arrivals, p.n_kv_heads, pl.kv_heads_per_set, pl.ctx_rows,
                       p.n_select, G, log2G, recipG, units, units_per_split, pl.attn_splits,
                       scale * kLog2e, (const S*)rb.K, (const S*)rb.V, rb.len, rb.capacity,
                       slot_table, pl.n_groups);
  };
  if (slot_table) launch(attn_partial_kernel<E, D, QPK, kAttnPaged>);
  else if (rb.len > 0) launch(attn_partial_kernel<E, D, QPK, kAttnRolling>);
  else launch(attn_partial_kernel<E, D, QPK, kAttnPlain>);
  return hipGetLastError();
}

template <typename E, int D>
hipError_t launch_qpk(const kvs_params& p, const Plan& pl, const void* q, const void* K,
                      const void* V, const int32_t* idx, float* part_ml, float* part_o,
                      void* out, int* arrivals, const RollingBuffer& rb, const int32_t* slot_table,
                      hipStream_t st) {
  switch (pl.q_per_kv) {
    case 1: return launch_partial<E, D, 1>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
    case 2: return launch_partial<E, D, 2>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
    case 3: return launch_partial<E, D, 3>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
    case 4: return launch_partial<E, D, 4>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
    case 5: return launch_partial<E, D, 5>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
    case 6: return launch_partial<E, D, 6>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
    case 7: return launch_partial<E, D, 7>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
    case 8: return launch_partial<E, D, 8>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
  }
  return hipErrorInvalidValue;
}

template <typename E>
hipError_t launch_d(const kvs_params& p, const Plan& pl, const void* q, const void* K,
                    const void* V, const int32_t* idx, float* part_ml, float* part_o,
                    void* out, int* arrivals, const RollingBuffer& rb, const int32_t* slot_table,
                      hipStream_t st) {
  switch (p.head_dim) {
    case 64: return launch_qpk<E, 64>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
    case 128: return launch_qpk<E, 128>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_attn(const kvs_params& p, const Plan& pl, const void* q, const void* K,
                       const void* V, const int32_t* idx, float* part_ml, float* part_o,
                       void* out, int* arrivals, const RollingBuffer& rb, const int32_t* slot_table,
                      hipStream_t st) {
  if (attn_mfma_applies(p, pl))
    return launch_attn_mfma(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
  if (p.kv_dtype == KVS_BF16) return launch_d<BF16Elem>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
  return launch_d<F32Elem>(p, pl, q, K, V, idx, part_ml, part_o, out, arrivals, rb, slot_table, st);
}

}  // namespace kvs
