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
#include "attn_merge.h"

KVS_ATTN_TRACE_ACCESSOR(kvs_debug_attn_mfma_trace)

namespace kvs {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

constexpr int kMfmaD = 128;
constexpr int kTileTokens = 16;                       // tokens per wave batch (= kAttnUnitsPerWave units)
constexpr int kTokensPerUnit = kWave / (kMfmaD / 8);  // 4: the unit the split plan counts in
static_assert(kAttnUnitsPerWave * kTokensPerUnit == kTileTokens, "a wave batch must be one tile");

// two floats -> two bf16 in one register (round to nearest even; inputs are finite, >= 0)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)float_to_bf16_bits(lo) | ((uint32_t)float_to_bf16_bits(hi) << 16);
}

// (registers: the plain and rolling-buffer modes fit the 128 that let two workgroups share a
// compute unit; the mapping table's extra look-ahead does not, and a spilled register is
// reloaded in order behind the key loads, i.e. stalls the value loads for a full latency,
// so that mode takes what it needs)
template <int QPK, int MODE, bool INTERLEAVE>
__global__ __launch_bounds__(kAttnThreads, MODE == kAttnPaged ? 2 : 4) void attn_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    const int32_t* __restrict__ idx, float* part_ml, float* part_o, uint16_t* __restrict__ out,
    int* __restrict__ arrivals, int n_kv_heads, int kv_heads_per_set, int ctx_rows, int M, int G,
    int log2G, uint32_t recipG, int units, int units_per_split, int n_splits, float scale_log2e,
    const uint16_t* __restrict__ rb_K, const uint16_t* __restrict__ rb_V, int rb_len, int rb_capacity,
    const int32_t* __restrict__ slot_table, int n_groups) {
  constexpr bool RB = MODE >= kAttnRolling;
  constexpr bool PAGED = MODE == kAttnPaged;
  constexpr int D = kMfmaD;
  static_assert(QPK >= 1 && QPK <= 16, "the heads of a KV head are one 16-wide matrix dimension");

  __shared__ AttnWaveStates<D, QPK> ws;

  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);  // (tells the compiler it is uniform)
  const int split = blockIdx.x, p = blockIdx.y;
  KVS_ATTN_TRACE(0);
#ifdef KVS_ATTN_TRACE_BUILD
  if (threadIdx.x == 0)  // where the workgroup runs: XCC id (hwreg 20), HW id (hwreg 4)
    g_attn_trace[((blockIdx.y * gridDim.x + blockIdx.x) * 8 + 7) & 0xFFFF] =
        ((long long)__builtin_amdgcn_s_getreg((31 << 11) | 20) << 32) | (unsigned)__builtin_amdgcn_s_getreg((31 << 11) | 4);
#endif
  const int b = p / n_kv_heads, k = p % n_kv_heads;
  const int n_q_heads = n_kv_heads * QPK;
  const int c = lane & 15;  // head (logits, output), token of the tile (keys), d block (values)
  const int g = lane >> 4;  // contraction slice
  const int n_tok = M * G;
  const int n_all = RB ? n_tok + rb_len : n_tok;
  auto group_of = [&](int tok) {
    return log2G >= 0 ? tok >> log2G : (int)__umulhi((uint32_t)tok, recipG);
  };

  // Q^T operand: head c, d = 32 j + 8 g .. + 7
  uint4 qb[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    qb[j] = make_uint4(0u, 0u, 0u, 0u);
    if (c < QPK)
      qb[j] = *reinterpret_cast<const uint4*>(q + ((size_t)b * n_q_heads + (size_t)k * QPK + c) * D + 32 * j + 8 * g);
  }

  const uint16_t* Kp = PAGED ? K : K + (size_t)p * ctx_rows * D;
  const uint16_t* Vp = PAGED ? V : V + (size_t)p * ctx_rows * D;
  const int32_t* tab = slot_table + (size_t)p * n_groups;  // (only read when PAGED)
  const uint16_t* Kr = rb_K + (size_t)p * rb_capacity * D;
  const uint16_t* Vr = rb_V + (size_t)p * rb_capacity * D;
  const int32_t* sel = idx + (size_t)(p / kv_heads_per_set) * M;
  // The units of a problem go to its splits either as one contiguous range each, or - for
  // long problems - one workgroup step (a tile per wave) at a time, round-robin: every
  // workgroup then walks the whole address range of the problem, and workgroups finish
  // closer together (identical work takes a different time in different parts of a long
  // cache: 4 % on the kernel at 128K tokens, nothing at 32K).  Either way the assignment
  // is a fixed function of the launch, so results are reproducible bit for bit.
  constexpr int kWgStep = kAttnWaves * kAttnUnitsPerWave;
  const int u0 = INTERLEAVE ? split * kWgStep : split * units_per_split;
  const int u1 = (INTERLEAVE || split == n_splits - 1) ? units : min(units, u0 + units_per_split);
  const int kStep = INTERLEAVE ? n_splits * kWgStep : kWgStep;  // from one step of this workgroup to its next

  // token t of the tile that starts at unit ub is attended iff its unit belongs to this
  // split and it lies inside the list
  auto attended = [&](int ub, int t) {
    return (ub + t / kTokensPerUnit < u1) && (ub * kTokensPerUnit + t < n_all);
  };
  // Position t of the tile at unit ub in the attended-token list (positions that are not
  // attended stand for position 0, one that is), and whether it lies in the rolling buffer.
  auto position = [&](int ub, int t) { return attended(ub, t) ? ub * kTokensPerUnit + t : 0; };
  auto in_buffer = [&](int tok) { return RB && tok >= n_tok; };
  // Cache row of a position, in two steps: which selected group it falls in (a look-up in
  // the selection), then the row (through the mapping table if there is one: a second,
  // dependent look-up).  Positions in the rolling buffer look up position 0 instead and
  // ignore the result.  The look-ups are unconditional, and the choice between cache and
  // buffer is only made when the rows are requested, an iteration later: a look-up inside a
  // branch, or one that depends on another of the same iteration, is waited for on the spot,
  // together with every key and value load issued before it.
  struct Rows {
    uint32_t k, v[4];
  };
  auto cache_pos = [&](int ub, int t) {
    const int tok = position(ub, t);
    return in_buffer(tok) ? 0 : tok;
  };
  auto find_groups = [&](int ub, Rows& r) {  // -> selected group (its index in the cache)
    r.k = (uint32_t)sel[group_of(cache_pos(ub, c))];
#pragma unroll
    for (int i = 0; i < 4; ++i) r.v[i] = (uint32_t)sel[group_of(cache_pos(ub, 4 * g + i))];
  };
  auto find_rows = [&](int ub, Rows& r) {  // group -> row (in place)
    auto row = [&](uint32_t grp, int t) {
      const int tc = cache_pos(ub, t);
      if constexpr (PAGED) grp = (uint32_t)tab[grp];
      return grp * (uint32_t)G + (uint32_t)(tc - group_of(tc) * G);
    };
    r.k = row(r.k, c);
#pragma unroll
    for (int i = 0; i < 4; ++i) r.v[i] = row(r.v[i], 4 * g + i);
  };
  auto request = [&](int ub, const Rows& r, uint4 (&kv)[4], uint4 (&vv)[4]) {
    {
      const int tok = position(ub, c);
      const uint16_t* base = (in_buffer(tok) ? Kr + (size_t)(tok - n_tok) * D : Kp + (size_t)r.k * D) + 8 * g;
#pragma unroll
      for (int j = 0; j < 4; ++j) kv[j] = *reinterpret_cast<const uint4*>(base + 32 * j);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int tok = position(ub, 4 * g + i);
      vv[i] = *reinterpret_cast<const uint4*>(
          (in_buffer(tok) ? Vr + (size_t)(tok - n_tok) * D : Vp + (size_t)r.v[i] * D) + 8 * c);
    }
  };

  float m = kNegBig, l = 0.f;  // of head c, over the tokens of slice g seen so far (m: of all slices)
  f32x4_t o[8];
#pragma unroll
  for (int bb = 0; bb < 8; ++bb) o[bb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  auto consume = [&](int ub, const uint4 (&kv)[4], const uint4 (&vv)[4]) {
    f32x4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kv[j]),
                                                  __builtin_bit_cast(bf16x8_t, qb[j]), s, 0, 0, 0);
    // online softmax of head c over tokens 4g .. 4g+3 (logits in log2 units)
    bool ok[4];
    float z[4];
    float mt = kNegBig;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ok[i] = attended(ub, 4 * g + i);
      z[i] = s[i] * scale_log2e;
      mt = ok[i] ? fmaxf(mt, z[i]) : mt;
    }
    mt = fmaxf(mt, xor_lane<16>(mt));
    mt = fmaxf(mt, xor_lane<32>(mt));
    const float mn = fmaxf(m, mt);
    const float alpha = __builtin_amdgcn_exp2f(m - mn);
    float pw[4];
    float ls = l * alpha;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      pw[i] = ok[i] ? __builtin_amdgcn_exp2f(z[i] - mn) : 0.f;
      ls += pw[i];
    }
    l = ls;
    if (__builtin_amdgcn_ballot_w64(mn > m) != 0ull) {  // some head's maximum moved: rescale
#pragma unroll
      for (int bb = 0; bb < 8; ++bb) o[bb] *= alpha;
    }
    m = mn;
    uint2 pb;  // P^T operand: head c, tokens 4g .. 4g+3
    pb.x = pack_bf16x2(pw[0], pw[1]);
    pb.y = pack_bf16x2(pw[2], pw[3]);
    const uint32_t w[4][4] = {{vv[0].x, vv[0].y, vv[0].z, vv[0].w},
                              {vv[1].x, vv[1].y, vv[1].z, vv[1].w},
                              {vv[2].x, vv[2].y, vv[2].z, vv[2].w},
                              {vv[3].x, vv[3].y, vv[3].z, vv[3].w}};
#pragma unroll
    for (int bb = 0; bb < 8; ++bb) {
      // element bb of the four loaded rows: the low or the high halves of dword bb / 2
      constexpr uint32_t kLow = 0x05040100u, kHigh = 0x07060302u;  // byte selectors of v_perm_b32
      const uint32_t selb = (bb & 1) ? kHigh : kLow;
      uint2 va;
      va.x = __builtin_amdgcn_perm(w[1][bb / 2], w[0][bb / 2], selb);
      va.y = __builtin_amdgcn_perm(w[3][bb / 2], w[2][bb / 2], selb);
      o[bb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, va),
                                                        __builtin_bit_cast(s16x4_t, pb), o[bb], 0, 0, 0);
    }
  };

  const int ub0 = u0 + wave * kAttnUnitsPerWave;
  // Look-ups run ahead of the tile whose keys and values are being requested: by one tile,
  // or by two (groups) and one (mapping table) when there is a table.
  uint4 kv[4], vv[4];
  Rows rows, ahead;
  find_groups(ub0, rows);
  find_rows(ub0, rows);
  if constexpr (PAGED) find_groups(ub0 + kStep, ahead);
  KVS_ATTN_TRACE(1);
  for (int ub = ub0; ub < u1; ub += kStep) {
    request(ub, rows, kv, vv);
    if constexpr (PAGED) {
      rows = ahead;                        // groups of the next tile, found an iteration ago
      find_rows(ub + kStep, rows);         // (past the end: position 0)
      find_groups(ub + 2 * kStep, ahead);
    } else {
      find_groups(ub + kStep, ahead);
    }
    consume(ub, kv, vv);
    if constexpr (!PAGED) {
      rows = ahead;
      find_rows(ub + kStep, rows);
    }
  }

  KVS_ATTN_TRACE(2);
  // ---- this wave's state of head c: add up the four slices' denominators ----------------
  l += xor_lane<16>(l);
  l += xor_lane<32>(l);
  if (c < QPK) {
    if (g == 0) {
      ws.m[wave][c] = m;
      ws.l[wave][c] = l;
    }
#pragma unroll
    for (int bb = 0; bb < 8; ++bb)
#pragma unroll
      for (int i = 0; i < 4; ++i) ws.o[wave][AttnWaveStates<D, QPK>::pos(c, 8 * (4 * g + i) + bb)] = o[bb][i];
  }
  attn_merge_and_finish<BF16Elem, D, QPK>(ws, part_ml, part_o,
                                          out + ((size_t)b * n_q_heads + (size_t)k * QPK) * D, arrivals,
                                          p, split, n_splits);
  KVS_ATTN_TRACE(6);
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
  auto launch = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, grid, block, 0, st, (const S*)q, (const S*)K, (const S*)V, idx, part_ml,
                       part_o, (S*)out, arrivals, p.n_kv_heads, pl.kv_heads_per_set, pl.ctx_rows,
                       p.n_select, G, log2G, recipG, units, units_per_split, pl.attn_splits,
                       scale * kLog2e, (const S*)rb.K, (const S*)rb.V, rb.len, rb.capacity,
                       slot_table, pl.n_groups);
  };
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
