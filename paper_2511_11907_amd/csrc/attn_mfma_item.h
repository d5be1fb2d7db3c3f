// Attention over the selected KV groups on the matrix cores, for one split of one (sequence,
// KV head) problem, as a workgroup-level routine: the attention kernel runs it once per
// workgroup, the single-launch decode step runs it for every attention work item a workgroup
// draws.  See attn_mfma.hip for the operand layouts.
#pragma once

#include "attn_merge.h"

#ifdef KVS_WG_TRACE_BUILD
// (debug builds) the time every wave leaves its tile loop
static __device__ long long g_attn_wave_end[8192];
#endif

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

// What an attention launch is given (the same for all its work items).
struct AttnMfmaArgs {
  const uint16_t* q;
  const uint16_t* K;
  const uint16_t* V;
  const int32_t* idx;
  float* part_ml;
  float* part_o;
  uint16_t* out;
  int* arrivals;
  int n_kv_heads, kv_heads_per_set, ctx_rows, M, G, log2G;
  uint32_t recipG;
  int units, units_per_split, n_splits;
  float scale_log2e;
  const uint16_t* rb_K;
  const uint16_t* rb_V;
  int rb_len, rb_capacity;
  const int32_t* slot_table;
  int n_groups;
};

// LDS of one attention work item.  sel: the problem's selected group indices, when the
// routine is asked to look them up there (SEL_LDS) instead of in global memory.
template <int QPK, int SEL_CAP>
struct AttnMfmaShared {
  AttnWaveStates<kMfmaD, QPK> ws;
  AttnMergeShared<QPK> ms;
  int32_t sel[SEL_CAP > 0 ? SEL_CAP : 1];
};

// Split `split` of problem `p`, by all kAttnThreads lanes of the workgroup.  SEL_CAP > 0: the
// selection was written by another workgroup of the same launch; its M <= SEL_CAP indices are
// first copied into LDS with device-scope loads and every look-up goes there (the caller has
// already waited until they are published).  Returns true in the workgroup that wrote the
// problem's output.  Ends without a barrier: before its LDS is reused the caller needs one.
template <int QPK, int MODE, bool INTERLEAVE, int SEL_CAP>
__device__ __forceinline__ bool attn_mfma_item(AttnMfmaShared<QPK, SEL_CAP>& sh, const AttnMfmaArgs& a,
                                               int p, int split) {
  const uint16_t* q = as_global(a.q);
  const uint16_t* K = as_global(a.K);
  const uint16_t* V = as_global(a.V);
  const int32_t* idx = as_global(a.idx);
  float* part_ml = as_global(a.part_ml);
  float* part_o = as_global(a.part_o);
  uint16_t* out = as_global(a.out);
  int* arrivals = as_global(a.arrivals);
  const int n_kv_heads = a.n_kv_heads, kv_heads_per_set = a.kv_heads_per_set, ctx_rows = a.ctx_rows,
            M = a.M, G = a.G, log2G = a.log2G, units = a.units, units_per_split = a.units_per_split,
            n_splits = a.n_splits, rb_len = a.rb_len, rb_capacity = a.rb_capacity, n_groups = a.n_groups;
  const uint32_t recipG = a.recipG;
  const float scale_log2e = a.scale_log2e;
  const uint16_t* rb_K = as_global(a.rb_K);
  const uint16_t* rb_V = as_global(a.rb_V);
  const int32_t* slot_table = as_global(a.slot_table);
  constexpr bool SEL_LDS = SEL_CAP > 0;
  constexpr bool RB = MODE >= kAttnRolling;
  constexpr bool PAGED = MODE == kAttnPaged;
  constexpr int D = kMfmaD;
  static_assert(QPK >= 1 && QPK <= 16, "the heads of a KV head are one 16-wide matrix dimension");

  auto& ws = sh.ws;

  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);  // (tells the compiler it is uniform)
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
  const int32_t* sel_global = idx + (size_t)(p / kv_heads_per_set) * M;
  if constexpr (SEL_LDS) {
    for (int i = tid; i < M; i += kAttnThreads) sh.sel[i] = load_published(&sel_global[i]);
    lds_barrier();
  }
  auto sel_at = [&](int i) { return SEL_LDS ? sh.sel[i] : sel_global[i]; };
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
    r.k = (uint32_t)sel_at(group_of(cache_pos(ub, c)));
#pragma unroll
    for (int i = 0; i < 4; ++i) r.v[i] = (uint32_t)sel_at(group_of(cache_pos(ub, 4 * g + i)));
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
  // (keys and values are read once per step: non-temporal loads, 8-9 % faster)
  auto request = [&](int ub, const Rows& r, uint4 (&kv)[4], uint4 (&vv)[4]) {
    {
      const int tok = position(ub, c);
      const uint16_t* base = (in_buffer(tok) ? Kr + (size_t)(tok - n_tok) * D : Kp + (size_t)r.k * D) + 8 * g;
#pragma unroll
      for (int j = 0; j < 4; ++j) kv[j] = load16<true>(base + 32 * j);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int tok = position(ub, 4 * g + i);
      vv[i] = load16<true>(
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
#ifdef KVS_WG_TRACE_BUILD
  if (lane == 0) g_attn_wave_end[((blockIdx.y * gridDim.x + blockIdx.x) * kAttnWaves + wave) & 8191] = wall_clock64();
#endif
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
  const bool wrote = attn_merge_and_finish<BF16Elem, D, QPK>(
      ws, sh.ms, part_ml, part_o, out + ((size_t)b * n_q_heads + (size_t)k * QPK) * D, arrivals, p, split,
      n_splits);
  KVS_ATTN_TRACE(6);
  return wrote;
}

}  // namespace kvs
