// The streaming pass of the prediction (Sec. 3.3, Eq. 1 and "Scoring and selection") for one
// chunk of one (sequence, KV head) problem, as a workgroup-level routine: the prediction
// kernel runs it once per workgroup, the single-launch decode step runs it for every
// prediction work item a workgroup draws.  See predict.hip for what it computes and why it
// is laid out the way it is.
#pragma once

#include "device_utils.h"
#include "kernels.h"
#include "topk_block.h"

#ifndef KVS_PREDICT_TRACE
#define KVS_PREDICT_TRACE(i)  // phase timestamps, only defined by the debugging harness
#endif

namespace kvs {

static_assert(kTopkBins == kSelectHistBins && kTopkPublishedPad <= kSelectScorePad, "workspace layout and selection routine disagree");

constexpr int kPredictThreads = kPredictWgThreads;
constexpr int kPredictWaves = kPredictThreads / kWave;
constexpr int kPredictUnroll = kPredictUnitsPerWgStep / kPredictWaves;  // wave-loads in flight per wave
static_assert(kPredictUnroll * kPredictWaves == kPredictUnitsPerWgStep, "granule mismatch");
constexpr int kStepPredictThreads = 512;  // workgroup size of the single-launch step's prediction items

// Geometry of one instantiation: E metadata element, R rank, G row slots per group, UNROLL
// wave-wide loads a wave keeps in flight (4 in the prediction kernel, whose 54-64 registers
// let 32 waves share a compute unit; more where fewer waves are resident).
template <typename E, int R, int G, int UNROLL = kPredictUnroll>
struct PredictGeom {
  static constexpr int EPL = E::kPerLane;
  static constexpr int LPR = R / EPL;      // lanes per row
  static constexpr int RPU = kWave / LPR;  // rows per unit
  static_assert(LPR >= 1 && LPR <= 32 && (LPR & (LPR - 1)) == 0, "row must span 1..32 lanes");
  static constexpr bool kGroupInUnit = (G <= RPU);
  static constexpr int UPG = kGroupInUnit ? 1 : G / RPU;  // units per group otherwise
  // wave-loads in flight per wave; a group must not straddle two batches
  static constexpr int U = UPG > UNROLL ? UPG : UNROLL;
  static_assert(U % UPG == 0, "a group must not straddle two batches");
  static constexpr int kGroupsPerBatch = kGroupInUnit ? U * (RPU / G) : U / UPG;  // per wave
};

// LDS of one prediction work item.
template <typename E, int R, int G, bool HIST, int UNROLL = kPredictUnroll, int THREADS = kPredictThreads>
struct PredictShared {
  float qsum[128];
  float red[THREADS];
  float qlr[R];
  int hist[HIST ? kTopkBins : 1];
  float stage[THREADS / kWave][PredictGeom<E, R, G, UNROLL>::kGroupsPerBatch];  // group scores of a wave's batch
  int next_batch;  // WAVE_CLAIMS: the next batch of the workgroup's chunk that no wave has taken
};

// What a prediction launch is given (the same for all its work items).
struct PredictArgs {
  const void* q;
  int q_is_bf16;
  const void* K_lr;
  const float* A;
  float* gs;
  float* gs_copy;  // nullable: a second array that receives the group scores too (plain stores)
  int n_kv_heads, q_per_kv, d, n_groups, g_real, ctx_rows, units, units_per_wg, mean;
  int* hist;
  const float* qlr;
  float meta_scale;
  const float* meta_scales;  // nullable: one scale per selection set, instead of meta_scale
};

// Chunk `chunk` of problem `p`, by all kPredictThreads lanes of the workgroup.  PUBLISH: the
// group scores are written with device-scope stores, for a reader in another workgroup of
// the same launch (otherwise plain stores, complete at the end of the kernel).  The routine
// ends without a barrier: before its LDS is reused the caller needs one.
//
// WAVE_CLAIMS: the waves do not walk the chunk in lockstep order (wave w: batch w of every
// workgroup step) but take its batches of U units one at a time from a counter in LDS, the
// first one by wave index, each following one drawn while the current one's loads travel.
// Why: a compute unit serves the loads of its older waves first, so with a fixed split some
// waves finish long before others and the last ones stream alone; with claims all waves of a
// workgroup end within one batch of each other.  Which wave computes which group score
// depends on timing, the score does not.
template <typename E, int R, int G, bool HIST, bool PAD, bool PUBLISH, int UNROLL = kPredictUnroll,
          int THREADS = kPredictThreads, bool WAVE_CLAIMS = false>
__device__ __forceinline__ void predict_item(PredictShared<E, R, G, HIST, UNROLL, THREADS>& sh,
                                             const PredictArgs& a, int p, int chunk) {
  constexpr int kPredictThreads = THREADS, kPredictWaves = THREADS / kWave;  // (of this instantiation)
  using Geom = PredictGeom<E, R, G, UNROLL>;
  constexpr int EPL = Geom::EPL, LPR = Geom::LPR, RPU = Geom::RPU, UPG = Geom::UPG, U = Geom::U;
  constexpr bool kGroupInUnit = Geom::kGroupInUnit;
  constexpr int kGroupsPerBatch = Geom::kGroupsPerBatch;
  auto& s_qsum = sh.qsum;
  auto& s_red = sh.red;
  auto& s_qlr = sh.qlr;
  auto& s_hist = sh.hist;
  auto& s_stage = sh.stage;
  const void* q = as_global(a.q);
  const int q_is_bf16 = a.q_is_bf16;
  const typename E::storage* K_lr = as_global((const typename E::storage*)a.K_lr);
  const float* A = as_global(a.A);
  float* gs = as_global(a.gs);
  float* gs_copy = as_global(a.gs_copy);
  const int n_kv_heads = a.n_kv_heads, q_per_kv = a.q_per_kv, d = a.d, n_groups = a.n_groups,
            g_real = a.g_real, ctx_rows = a.ctx_rows, units = a.units, units_per_wg = a.units_per_wg,
            mean = a.mean;
  int* hist = as_global(a.hist);
  const float* qlr = as_global(a.qlr);
  const float meta_scale = a.meta_scales ? as_global(a.meta_scales)[p] : a.meta_scale;  // uniform

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int b = p / n_kv_heads, k = p % n_kv_heads;
  const int n_q_heads = n_kv_heads * q_per_kv;
  const int c = lane % LPR;   // 16-byte column of the row
  const int rl = lane / LPR;  // row within the unit

  const typename E::storage* Kp = K_lr + (size_t)p * ctx_rows * R;
  float* gsp = gs + (size_t)p * n_groups;
  const int N = n_groups * g_real;   // rows of the compressed cache
  const int n_slots = n_groups * G;  // row slots (== N unless the groups are padded)
  const int u0 = chunk * units_per_wg;
  const int u1 = min(units, u0 + units_per_wg);

  // A workgroup step covers kPredictWaves * U consecutive units; wave w takes the U
  // consecutive units starting at w * U, i.e. one contiguous run of U KiB, whose group
  // scores are U * RPU / G consecutive floats that leave in one coalesced store.
  constexpr int kStep = kPredictWaves * U;
  // (with WAVE_CLAIMS a base is that of the wave's own batch)
  const int wave_off = WAVE_CLAIMS ? 0 : wave * U;
  auto unit_of = [&](int step_base, int j) { return step_base + wave_off + j; };
  uint4 v[U];
  bool ok[U];
  auto issue = [&](int step_base) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int unit = unit_of(step_base, u);
      const int slot = unit * RPU + rl;
      size_t off;
      if constexpr (PAD) {
        const int row = (slot / G) * g_real + (slot % G);
        ok[u] = (unit < u1) && (slot < n_slots) && ((slot % G) < g_real);
        // (a slot without a row reads a valid row nearby, one its neighbours fetch anyway)
        off = (size_t)(unit < u1 ? min(row, N - 1) : 0) * R + (size_t)c * EPL;
      } else {
        ok[u] = (unit < u1) && (slot < N);
        off = (size_t)(ok[u] ? slot : 0) * R + (size_t)c * EPL;
      }
      v[u] = load16<true>(Kp + off);  // K_lr is read once: non-temporal (11-13 % faster)
    }
  };
  // Everything the prologue needs from memory is requested up front - the queries, this
  // lane's entries of the adapter, and the first batch of K_lr - so that the workgroup
  // pays one memory latency before it streams, not three in a row.
  // (the projection is done by the first 512 lanes whatever the workgroup size, so that its
  // summation order, and with it every score, is the same in all launch forms)
  constexpr int kProjectLanes = 512;
  static_assert(kPredictThreads >= kProjectLanes, "the projection needs 512 lanes");
  constexpr int NSL = kProjectLanes / R;    // slices of the d axis in the projection
  constexpr int kSpanMax = 128 / NSL;       // adapter rows per lane at d = 128
  const int pj = tid % R, psl = tid / R;
  const int span = d / NSL;
  const bool project = (qlr == nullptr);  // uniform: false when the low-rank query is given
  StridedSum qheads;
  float a_reg[kSpanMax];
  float qr[EPL];
  if (project) {
    // the query heads of this KV head, element tid of each (lanes beyond d repeat the last)
    qheads.request(q, q_is_bf16, ((size_t)b * n_q_heads + (size_t)k * q_per_kv) * d + min(tid, d - 1), d, q_per_kv);
    const float* Ak = A + (size_t)k * d * R;
#pragma unroll
    for (int i = 0; i < kSpanMax; ++i)
      a_reg[i] = psl < NSL ? Ak[(size_t)min(psl * span + i, d - 1) * R + pj] : 0.f;  // rows past the span are never used
  } else {
#pragma unroll
    for (int e = 0; e < EPL; ++e) qr[e] = qlr[(size_t)p * R + c * EPL + e] * meta_scale;
  }
  int ub = u0;  // base of the current workgroup step (WAVE_CLAIMS: of the wave's current batch)
  int drawn = 0;  // WAVE_CLAIMS: the batch this wave takes next (valid in lane 0 until broadcast)
  if constexpr (WAVE_CLAIMS) {
    ub = u0 + wave * U;
    if (tid == 0) sh.next_batch = kPredictWaves;  // (visible after the barriers of the prologue)
  }
  if (ub < u1) issue(ub);

  if constexpr (HIST) {  // this workgroup's share of the score histogram
    for (int i = tid; i < kTopkBins; i += kPredictThreads) s_hist[i] = 0;
  }

  if (project) {
    // ---- low-rank query vector of this KV head (head-summed) --------------------
    if (tid < d) s_qsum[tid] = qheads.sum(q_is_bf16, q_per_kv);
    lds_barrier();
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < kSpanMax; ++i)
      if (i < span && psl < NSL) acc = fmaf(s_qsum[psl * span + i], a_reg[i], acc);
    s_red[tid] = acc;
    lds_barrier();
    if (tid < R) {
      float tot = 0.f;
#pragma unroll 8
      for (int s = 0; s < NSL; ++s) tot += s_red[s * R + tid];
      s_qlr[tid] = tot;
    }
    lds_barrier();
#pragma unroll
    // the stored metadata is K.A / meta_scale: the factor goes into the query once
    for (int e = 0; e < EPL; ++e) qr[e] = s_qlr[c * EPL + e] * meta_scale;
  } else if constexpr (HIST || WAVE_CLAIMS) {
    lds_barrier();  // the histogram is cleared before anyone counts into it (and the batch counter set)
  }

  KVS_PREDICT_TRACE(1);
  const float inv_g = 1.0f / (float)g_real;
  const float empty = mean ? 0.f : -__builtin_huge_valf();  // score of an empty row slot

  while (ub < u1) {
    if constexpr (WAVE_CLAIMS) {  // draw the batch after this one while this one's loads travel
      if (lane == 0) drawn = atomicAdd(&sh.next_batch, 1);
    }
    float sc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float f[EPL];
      unpack16<E>(v[u], f);
      float acc = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc = fmaf(qr[e], f[e], acc);
      sc[u] = allreduce_lanes<OpSum, 1, LPR>(acc);  // token score, on all LPR lanes of the row
      if constexpr (PAD) sc[u] = ok[u] ? sc[u] : empty;
    }
    // Group representatives go through a per-wave LDS line so that they leave as one
    // coalesced store per batch (scattered 4-byte stores per unit cost ~8 % of the
    // streaming bandwidth).  Only this wave touches its line, in program order.
    if constexpr (kGroupInUnit) {
      constexpr int GPU_ = RPU / G;  // groups per unit
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float g;
        if (mean) g = allreduce_lanes<OpSum, LPR, LPR * G>(sc[u]) * inv_g;
        else g = allreduce_lanes<OpMax, LPR, LPR * G>(sc[u]);
        if ((lane % (LPR * G)) == 0) s_stage[wave][u * GPU_ + lane / (LPR * G)] = g;
      }
    } else {
#pragma unroll
      for (int u0g = 0; u0g < U; u0g += UPG) {
        float g = sc[u0g];
#pragma unroll
        for (int t = 1; t < UPG; ++t) g = mean ? g + sc[u0g + t] : fmaxf(g, sc[u0g + t]);
        if (mean) g = allreduce_lanes<OpSum, LPR, kWave>(g) * inv_g;
        else g = allreduce_lanes<OpMax, LPR, kWave>(g);
        if (lane == 0) s_stage[wave][u0g / UPG] = g;
      }
    }
    {
      // first group of this wave's batch; groups never straddle units' ends, so a group is
      // valid iff its first row is
      const int row0 = unit_of(ub, 0) * RPU;
      const int grp0 = row0 / G;
      const int row_end = min(n_slots, u1 * RPU);
#pragma unroll
      for (int t = lane; t < kGroupsPerBatch; t += kWave) {
        if ((grp0 + t) * G < row_end) {
          const float g = s_stage[wave][t];
          if constexpr (PUBLISH) {
            publish_store(&gsp[grp0 + t], g);
            if (a.gs_copy) gs_copy[(size_t)p * n_groups + grp0 + t] = g;  // uniform
          } else {
            gsp[grp0 + t] = g;
          }
          if constexpr (HIST) atomicAdd(&s_hist[score_key(g) >> kTopkLowBits], 1);
        }
      }
    }
    if constexpr (WAVE_CLAIMS) ub = u0 + __builtin_amdgcn_readfirstlane(drawn) * U;
    else ub += kStep;
    if (ub < u1) issue(ub);
    KVS_PREDICT_TRACE(2);
  }
  KVS_PREDICT_TRACE(3);

  if constexpr (HIST) {
    // add this workgroup's histogram to the problem's (only the bins it touched)
    lds_barrier();
    int* hg = hist + (size_t)p * kTopkBins;
    for (int i = tid; i < kTopkBins; i += kPredictThreads) {
      const int n = s_hist[i];
      if (n) atomicAdd(&hg[i], n);
    }
  }
}

}  // namespace kvs
