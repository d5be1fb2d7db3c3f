// Workgroup-level top-M selection (Sec. 3.3, "TopK"): the indices of the M largest fp32
// scores of one problem, ties to the lower index, written in ascending index order.
//
// Scores are compared as order-preserving 32-bit keys.  The key T of the M-th largest
// score is found MSB-first:
//   1. a 4096-bin histogram of the top 12 key bits (sign, exponent, 3 mantissa bits)
//      names the bin that holds T and how many keys lie in higher bins.  The histogram
//      is either built here or was accumulated in global memory by the kernel that
//      produced the scores.  Every wave locates the bin by itself from the per-wave
//      totals (one barrier);
//   2. the keys of that bin - a few per cent of all keys - are gathered into a list in
//      LDS, and one wave settles the remaining 20 bits with three small histograms (8, 8
//      and 4 bits) over the list entries that agree with the prefix found so far: a
//      single wave needs no barrier between the levels.  (A bin with more keys than
//      the list holds - many equal scores - is settled by the same three levels over all
//      keys, by all waves.);
//   3. one block-wide prefix sum over packed (greater, equal) counts gives every
//      selected index its final position.
// Integer work only: the result is a deterministic function of the scores.
//
// The routine is bound by the length of its dependent instruction chain, not by the
// number of keys (a few thousand per problem): it is written to keep that chain and the
// number of barriers (four when the histogram is handed in) short.
#pragma once

#include "device_utils.h"

#ifndef KVS_TOPK_TRACE
#define KVS_TOPK_TRACE(i)  // phase timestamps, only defined by the debugging harness
#endif

namespace kvs {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / kWave;
constexpr int kTopkMaxPerLane = 32;   // => at most 32768 scores per problem
constexpr int kTopkSmallPerLane = 8;  // second instantiation, for problems of at most 8192 scores
constexpr int kTopkChunk = 8;         // register slots handled (and loads in flight) per uniform branch
constexpr int kTopkBins = 4096;       // histogram over key >> kTopkLowBits
constexpr int kTopkLowBits = 20;
constexpr int kTopkPublishedPad = 2304;  // floats readable beyond the scores of a PUBLISHED call (> 4 per lane + one chunk)
constexpr int kTopkSegs = 16;          // the first histogram is searched in 16 segments of 256 bins
constexpr int kTopkBinsPerSeg = kTopkBins / kTopkSegs;
constexpr int kTopkListPerLane = 16;  // keys of one bin that step 2's wave takes into registers, per lane
constexpr int kTopkListCap = kTopkListPerLane * kWave;

constexpr int kTopkLevels = 3;        // histogram levels below the first: 8 + 8 + 4 bits
constexpr int kTopkLevelBins = 256;
static_assert(kTopkLowBits == 8 + 8 + 4, "the lower levels must cover the low bits");
static_assert(kTopkBinsPerSeg == 4 * kWave && kTopkLevelBins == 4 * kWave, "histograms are read four bins per lane");
static_assert(kTopkWaves <= 16 && kTopkSegs == 16, "prefixes over waves and segments are taken inside one row of 16 lanes");

// Histograms are stored top bin first (bin b at index size-1-b): the search runs from the
// largest keys downwards, and a lane then reads its four bins as one 16-byte piece.
constexpr int kTopkStageElems = 8192;  // scores staged through LDS per pass of a PUBLISHED call
constexpr int kTopkStageWords = kTopkStageElems + kTopkStageElems / 32;  // (one pad word per 32: conflict-free slices)
struct TopkShared {
  union {
    struct {
      alignas(16) int hist[kTopkBins];                    // top-12-bit histogram
      alignas(16) uint32_t list[kTopkListCap];            // keys of the bin that holds the M-th key
      alignas(16) int sub[kTopkLevels][kTopkLevelBins];   // histograms of the lower levels
    };
    float stage[kTopkStageWords];  // PUBLISHED calls only, before anything above is in use
  };
  uint32_t wave_tot[2][kTopkSegs];        // per-segment / per-wave totals of the block-wide prefix sums
  int n_listed;
  int sel_above;                          // hand-over of a level's result and of step 2's
  uint32_t sel_key;
};

// float -> uint32 whose unsigned order equals the float order; -0 is folded into +0
// so that equal scores have equal keys.  Keys are at least kTopkMinKey (only some NaN
// patterns with the sign bit set are raised to it; -inf and every finite score lie
// above), so that the key 0 of an unused register slot is below every key of a score and
// falls into a histogram bin that no score uses.
constexpr uint32_t kTopkMinKey = 1u << 20;
__device__ __forceinline__ uint32_t score_key(float x) {
  const uint32_t u = __float_as_uint(x + 0.0f);
  const uint32_t flip = (uint32_t)((int32_t)u >> 31) | 0x80000000u;  // all bits of a negative value, the sign bit of others
  return max(u ^ flip, kTopkMinKey);
}

// Inclusive prefix sum inside each row of 16 lanes (DPP, shifted-in lanes read as zero).
__device__ __forceinline__ int row_scan_dpp(int x) {
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, true);  // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, true);  // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, true);  // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, true);  // row_shr:8
  return x;
}

// Inclusive prefix sum over the wave (lane i gets the sum of lanes 0..i): the rows' scans,
// then the running totals of the rows are passed on with row_bcast:15 / row_bcast:31.
__device__ __forceinline__ uint32_t wave_scan_dpp(uint32_t v) {
  int x = row_scan_dpp((int)v);
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false);  // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false);  // row_bcast:31 into rows 2 and 3
  return (uint32_t)x;
}

// Exclusive prefix sum across the workgroup in thread order (one barrier).  `tot` holds one
// word per wave and must not be rewritten before the caller's next barrier.  After the
// barrier every wave adds up the totals of the waves before it inside one row of 16 lanes.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* tot) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const uint32_t incl = wave_scan_dpp(v);
  if (lane == kWave - 1) tot[wave] = incl;
  lds_barrier();
  const int w = lane & 15;  // (at most 16 waves: the waves before this one all sit in one row)
  const int before = row_scan_dpp(w < wave ? (int)tot[w] : 0);
  return (uint32_t)__builtin_amdgcn_readlane(before, 15) + incl - v;
}

// A lane's four bins `b` (top bin first) of a histogram whose bins before this lane's hold
// `above_me` keys: does the M-th key from the top fall into one of them?  If so `bin_pos`
// (position of that bin among the four) and `above` (keys in higher bins) are set.
__device__ __forceinline__ bool topk_find_in_four(const int (&b)[4], int above_me, int M, int& bin_pos, int& above) {
  bool found = false;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    if (above_me < M && M <= above_me + b[c]) found = true, bin_pos = c, above = above_me;
    above_me += b[c];
  }
  return found;
}

// One wave scans a histogram of 256 bins (top bin first, four per lane) for the bin of the
// M-th key from the top, `above` keys being above the whole histogram.  Returns the bin's
// position from the top, updates `above` and sets `in_bin` to that bin's count; wave-uniform
// results.
__device__ __forceinline__ int topk_scan_256(const int* hist_top_first, int lane, int M, int& above, int& in_bin) {
  const int4 v = *reinterpret_cast<const int4*>(hist_top_first + 4 * lane);
  const int b[4] = {v.x, v.y, v.z, v.w};
  const int tot = b[0] + b[1] + b[2] + b[3];
  const int incl = (int)wave_scan_dpp((uint32_t)tot);
  int pos = 0, mine_above = 0;
  const bool found = topk_find_in_four(b, above + incl - tot, M, pos, mine_above);
  const int mine_count = pos == 0 ? b[0] : pos == 1 ? b[1] : pos == 2 ? b[2] : b[3];
  const unsigned long long who = __ballot(found);
  // (no lane finds it only if the histogram does not belong to these scores, e.g. a
  // workspace that was never initialised: any in-range answer will do then)
  const int src = who ? (int)__builtin_ctzll(who) : 0;
  above = __builtin_amdgcn_readlane(mine_above, src);
  in_bin = __builtin_amdgcn_readlane(mine_count, src);
  return __builtin_amdgcn_readlane(4 * lane + pos, src);
}

constexpr int kTopkLevelShift[kTopkLevels] = {12, 4, 0};
constexpr int kTopkLevelBits[kTopkLevels] = {8, 8, 4};

// The keys of a source that agree with `prefix` above level LEVEL's bits are counted into
// that level's histogram.  `for_each_key(f)` calls f(key, valid) for every key of the
// source, the same number of times on all lanes of a wave.  AGGREGATE: expect many equal
// keys (a wave whose hits all fall into one bin adds them with one operation).
template <int LEVEL, bool AGGREGATE, class Source>
__device__ __forceinline__ void topk_level_count(uint32_t prefix, TopkShared& sh, Source&& for_each_key) {
  constexpr int shift = kTopkLevelShift[LEVEL], bits = kTopkLevelBits[LEVEL], nbins = 1 << bits;
  const int lane = threadIdx.x & (kWave - 1);
  const uint32_t hi = prefix >> (shift + bits);
  for_each_key([&](uint32_t key, bool valid) __attribute__((always_inline)) {
    const bool hit = valid && (key >> (shift + bits)) == hi;
    const int slot = kTopkLevelBins - 1 - (int)((key >> shift) & (uint32_t)(nbins - 1));  // top bin first
    if constexpr (!AGGREGATE) {
      if (hit) atomicAdd(&sh.sub[LEVEL][slot], 1);
      return;
    }
    const unsigned long long hits = __ballot(hit);
    if (hits != 0ull) {  // uniform
      // many equal scores would pile onto one counter: if every hit of the wave is in
      // the same bin, one lane adds them all
      const int first_hit = __builtin_ctzll(hits);
      const int slot0 = __builtin_amdgcn_readlane(slot, first_hit);
      if (__ballot(hit && slot == slot0) == hits) {
        if (lane == first_hit) atomicAdd(&sh.sub[LEVEL][slot0], __popcll(hits));
      } else if (hit) {
        atomicAdd(&sh.sub[LEVEL][slot], 1);
      }
    }
  });
}

// The scanning half of a level, by one wave: extends `prefix` by the level's bits of the
// M-th key and `above` by the keys of higher bins; returns the number of keys in the bin found.
template <int LEVEL>
__device__ __forceinline__ int topk_level_scan(uint32_t& prefix, int& above, int M, TopkShared& sh) {
  const int lane = threadIdx.x & (kWave - 1);
  int in_bin;
  const int pos = topk_scan_256(sh.sub[LEVEL], lane, M, above, in_bin);
  prefix |= (uint32_t)((kTopkLevelBins - 1 - pos) & ((1 << kTopkLevelBits[LEVEL]) - 1)) << kTopkLevelShift[LEVEL];
  return in_bin;
}

// A level run by the whole workgroup over a source that is spread over all waves: two barriers.
template <int LEVEL, class Source>
__device__ __forceinline__ void topk_level_block(uint32_t& prefix, int& above, int M, TopkShared& sh,
                                                 Source&& for_each_key) {
  topk_level_count<LEVEL, true>(prefix, sh, for_each_key);
  lds_barrier();
  if (threadIdx.x < kWave) {
    topk_level_scan<LEVEL>(prefix, above, M, sh);
    if (threadIdx.x == 0) sh.sel_key = prefix, sh.sel_above = above;
  }
  lds_barrier();
  prefix = sh.sel_key;
  above = sh.sel_above;
}

// All THREADS lanes of the workgroup must call this with the same arguments (THREADS = 1024
// in the selection kernel, 512 in the single-launch decode step).
// g: NG scores (16-byte aligned if NG is a multiple of 4); out: M indices;
// 1 <= M <= NG <= THREADS * SLOTS.
// hist_global: nullptr => the histogram of the top 12 key bits is built here, in LDS;
// otherwise it points at the problem's kTopkBins counters in global memory (bin b at
// index b), completed by an earlier kernel, and they are reset to zero on the way.
// PUBLISHED: the scores were written by other workgroups of the same launch, and the indices
// are read by other workgroups of it: both move with device-scope loads and stores.  The
// scores are then read in whole rounds of THREADS elements, the last one possibly past the
// end (ignored): g must be readable up to kTopkPublishedPad floats beyond its NG scores.
template <int SLOTS, int THREADS = kTopkThreads, bool PUBLISHED = false>
__device__ __forceinline__ void topk_block(const float* g, int32_t* __restrict__ out, int NG, int M,
                                           int* hist_global, TopkShared& sh) {
  static_assert(SLOTS % kTopkChunk == 0 && SLOTS <= kTopkMaxPerLane, "slots come in whole chunks");
  constexpr int WAVES = THREADS / kWave;
  static_assert(WAVES <= 16 && kTopkSegs % WAVES == 0, "every wave searches a whole number of histogram segments");
  constexpr int SPW = kTopkSegs / WAVES;  // histogram segments per wave
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;

  // the problem's histogram, if it was accumulated elsewhere: requested first so that
  // its latency overlaps the loads of the scores.  Histograms are handled top bin first:
  // position i stands for bin 4095 - i; a lane takes four consecutive positions of each of
  // its wave's segments.
  auto my_pos = [&](int sg) { return kTopkBinsPerSeg * (wave * SPW + sg) + 4 * lane; };
  int4 mine_raw[SPW];
#pragma unroll
  for (int sg = 0; sg < SPW; ++sg) {
    mine_raw[sg] = make_int4(0, 0, 0, 0);
    if (hist_global) mine_raw[sg] = *reinterpret_cast<const int4*>(hist_global + (kTopkBins - 4 - my_pos(sg)));
  }

  // A lane owns a contiguous slice of kpt scores (what the ordered compaction needs).
  // With NG a multiple of four the slice is a whole number of 16-byte pieces and is
  // fetched as such: a wave then touches a few cache lines per load instead of 64.
  const bool vec = (NG & 3) == 0;  // uniform
  int kpt = (NG + THREADS - 1) / THREADS;  // scores per lane
  if (vec) kpt = (kpt + 3) & ~3;
  const int first = tid * kpt;
  const int n_real = max(0, min(kpt, NG - first));  // slots of this lane that hold a score

  // Slice of this lane, as keys, fetched in chunks of kTopkChunk slots whose loads are
  // all in flight together (addresses clamped, so no lane ever branches around a load).
  // Slots beyond the slice (and beyond NG) hold key 0: below every score's key, and in a
  // bin of the histogram that stays empty, so no later step has to tell them apart.
  uint32_t key[SLOTS];
  {
    // every chunk's loads are requested before the first value is looked at, so a long
    // slice still costs one memory latency
    float x[SLOTS];
    if constexpr (PUBLISHED) {
      // Fetched with whole-wave contiguous device-scope loads (lane t takes elements t,
      // t + THREADS, ...: a few memory requests per instruction where slice-wise loads would
      // make 64, each going all the way to memory), all requested together, and handed to
      // the lanes' slices through LDS, kTopkStageElems scores per pass.
      constexpr int kPerPass = kTopkStageElems / THREADS;
      static_assert(kTopkStageElems % THREADS == 0, "a pass is a whole number of loads per lane");
      const int nk = (NG + THREADS - 1) / THREADS;  // loads per lane: uniform, <= SLOTS
      float raw[SLOTS];
#pragma unroll
      for (int k = 0; k < SLOTS; ++k) {
        raw[k] = 0.f;
        if (k < nk) raw[k] = load_published(g + k * THREADS + tid);  // (uniform; up to THREADS - 1 past the end)
      }
#pragma unroll
      for (int k = 0; k < SLOTS; ++k) asm volatile("" : "+v"(raw[k]));
#pragma unroll
      for (int j = 0; j < SLOTS; ++j) x[j] = 0.f;
#pragma unroll
      for (int h = 0; h * kPerPass < SLOTS; ++h) {
        if (h * kPerPass < nk) {  // uniform
#pragma unroll
          for (int kk = 0; kk < kPerPass; ++kk) {
            if (h * kPerPass + kk < SLOTS) {
              const int e = kk * THREADS + tid;
              sh.stage[e + (e >> 5)] = raw[h * kPerPass + kk < SLOTS ? h * kPerPass + kk : 0];
            }
          }
          lds_barrier();
#pragma unroll
          for (int j = 0; j < SLOTS; ++j) {
            const int e = first + j - h * kTopkStageElems;
            if (j < kpt && e >= 0 && e < kTopkStageElems) x[j] = sh.stage[e + (e >> 5)];
          }
          lds_barrier();  // (the staging area is reused by the next pass, then by the histograms)
        }
      }
    }
#pragma unroll
    for (int c0 = 0; c0 < SLOTS; c0 += kTopkChunk) {
      if (PUBLISHED) {  // (filled above, through LDS)
      } else if (c0 < kpt && vec) {  // uniform
#pragma unroll
        for (int j = c0; j < c0 + kTopkChunk; j += 4) {
          const float4 v = *reinterpret_cast<const float4*>(g + min(first + j, NG - 4));
          x[j] = v.x, x[j + 1] = v.y, x[j + 2] = v.z, x[j + 3] = v.w;
        }
      } else if (c0 < kpt) {  // uniform
#pragma unroll
        for (int j = c0; j < c0 + kTopkChunk; ++j) x[j] = g[min(first + j, NG - 1)];
      } else {
#pragma unroll
        for (int j = c0; j < c0 + kTopkChunk; ++j) x[j] = 0.f;
      }
    }
    // (pins every request above the first use: without it the compiler pairs each chunk's
    // loads with its conversions and waits chunk by chunk)
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) asm volatile("" : "+v"(x[j]));
#pragma unroll
    for (int c0 = 0; c0 < SLOTS; c0 += kTopkChunk) {
      if (c0 < kpt) {  // uniform
#pragma unroll
        for (int j = c0; j < c0 + kTopkChunk; ++j) key[j] = j < n_real ? score_key(x[j]) : 0u;
      } else {
#pragma unroll
        for (int j = c0; j < c0 + kTopkChunk; ++j) key[j] = 0u;
      }
    }
  }
  // every key of this lane's slice, slot by slot (skipping the unused chunks uniformly)
  auto slice_keys = [&](auto&& f) __attribute__((always_inline)) {
#pragma unroll
    for (int c0 = 0; c0 < SLOTS; c0 += kTopkChunk) {
      if (c0 < kpt) {  // uniform
#pragma unroll
        for (int j = c0; j < c0 + kTopkChunk; ++j) f(key[j], j);
      }
    }
  };

  KVS_TOPK_TRACE(1);
  // ---- 1. histogram of the top 12 bits, and the bin of the M-th key -------------------------
  for (int i = tid; i < kTopkLevels * kTopkLevelBins; i += THREADS) (&sh.sub[0][0])[i] = 0;
  if (tid == 0) sh.n_listed = 0;  // (both ordered before their use by the barrier of this step)
  int mine[SPW][4];               // this lane's bins of each of its wave's segments, top first
  // the histogram built here, in LDS, from the keys in registers (two barriers)
  auto build_here = [&]() __attribute__((always_inline)) {
    for (int i = tid; i < kTopkBins; i += THREADS) sh.hist[i] = 0;
    lds_barrier();
    slice_keys([&](uint32_t k, int j) __attribute__((always_inline)) {
      if (j < n_real) atomicAdd(&sh.hist[kTopkBins - 1 - (int)(k >> kTopkLowBits)], 1);
    });
    lds_barrier();
#pragma unroll
    for (int sg = 0; sg < SPW; ++sg) {
      const int4 v = *reinterpret_cast<const int4*>(&sh.hist[my_pos(sg)]);
      mine[sg][0] = v.x, mine[sg][1] = v.y, mine[sg][2] = v.z, mine[sg][3] = v.w;
    }
  };
  if (hist_global) {
#pragma unroll
    for (int sg = 0; sg < SPW; ++sg) {
      // (keeps the histogram load where it was written, ahead of the score loads, instead of
      // the compiler sinking it to its first use)
      asm volatile("" : "+v"(mine_raw[sg].x), "+v"(mine_raw[sg].y), "+v"(mine_raw[sg].z), "+v"(mine_raw[sg].w));
      mine[sg][0] = mine_raw[sg].w, mine[sg][1] = mine_raw[sg].z, mine[sg][2] = mine_raw[sg].y, mine[sg][3] = mine_raw[sg].x;
      *reinterpret_cast<int4*>(&sh.hist[my_pos(sg)]) = make_int4(mine[sg][0], mine[sg][1], mine[sg][2], mine[sg][3]);
    }
  } else {
    build_here();
  }
  KVS_TOPK_TRACE(2);
  uint32_t prefix;
  int above;  // keys in bins above the one that holds the M-th key
  // Every wave by itself, after one barrier: which segment of 256 bins holds the M-th key,
  // then which of those bins.  Returns the number of keys the histogram holds in all.
  auto locate = [&](uint32_t* seg_tot) __attribute__((always_inline)) {
#pragma unroll
    for (int sg = 0; sg < SPW; ++sg) {
      const uint32_t tot = (uint32_t)(mine[sg][0] + mine[sg][1] + mine[sg][2] + mine[sg][3]);
      const uint32_t incl = wave_scan_dpp(tot);
      if (lane == kWave - 1) seg_tot[wave * SPW + sg] = incl;
    }
    lds_barrier();
    const int w = lane & (kTopkSegs - 1);
    const int t_w = (int)seg_tot[w];
    const int upto_w = row_scan_dpp(t_w);  // keys in the bins of segments 0..w
    const unsigned long long reached = __ballot(upto_w >= M) & ((1ull << kTopkSegs) - 1ull);
    const int w_sel = reached ? (int)__builtin_ctzll(reached) : kTopkSegs - 1;
    above = __builtin_amdgcn_readlane(upto_w - t_w, w_sel);
    int in_bin;
    const int pos = topk_scan_256(&sh.hist[kTopkBinsPerSeg * w_sel], lane, M, above, in_bin);
    prefix = (uint32_t)(kTopkBins - 1 - (kTopkBinsPerSeg * w_sel + pos)) << kTopkLowBits;
    return __builtin_amdgcn_readlane(upto_w, kTopkSegs - 1);
  };
  const int counted = locate(sh.wave_tot[0]);
  if (hist_global && counted != NG) {  // uniform
    // The histogram handed in does not hold exactly these NG scores (it was never
    // accumulated for them, or the counters were not zero before): it is ignored and the
    // histogram is built here after all.  The barrier lets every wave finish reading the
    // old histogram before it is cleared; the per-wave totals go to the second array
    // because a wave may still be reading the first (the placement scan, which uses the
    // second array again, comes after the barriers of step 2).
    lds_barrier();
    build_here();
    locate(sh.wave_tot[1]);
  }
  const uint32_t bin = prefix >> kTopkLowBits;

  KVS_TOPK_TRACE(3);
  // ---- 2. settle the low 20 bits ---------------------------------------------------------
  // The keys of the bin go into a list in LDS (in any order: only their values matter
  // here): a lane counts its keys of the bin, a prefix sum over the wave and one atomic
  // per wave give it its place in the list.
  {
    uint32_t n_mine = 0;
    slice_keys([&](uint32_t k, int) __attribute__((always_inline)) {
      n_mine += (k >> kTopkLowBits) == bin ? 1u : 0u;
    });
    const uint32_t incl = wave_scan_dpp(n_mine);
    int wave_first = 0;
    if (lane == kWave - 1 && incl != 0u) wave_first = atomicAdd(&sh.n_listed, (int)incl);
    int at = __builtin_amdgcn_readlane(wave_first, kWave - 1) + (int)(incl - n_mine);
    slice_keys([&](uint32_t k, int) __attribute__((always_inline)) {
      if ((k >> kTopkLowBits) == bin) {
        if (at < kTopkListCap) sh.list[at] = k;
        ++at;
      }
    });
  }
  lds_barrier();
  KVS_TOPK_TRACE(4);
  const int n_listed = __builtin_amdgcn_readfirstlane(sh.n_listed);
  if (n_listed <= kTopkListCap) {  // uniform
    if (__builtin_amdgcn_readfirstlane(wave) == 0) {
      // One wave takes the list into registers and runs the levels by itself: its LDS
      // operations execute in order, so the counts of a level are complete when the same
      // wave reads them back, and no barrier is needed between the levels.
      uint32_t lk[kTopkListPerLane];
#pragma unroll
      for (int c = 0; c < kTopkListPerLane; ++c)
        lk[c] = sh.list[min(c * kWave + lane, kTopkListCap - 1)];
      auto listed_keys = [&](auto&& f) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < kTopkListPerLane; ++c)
          if (c * kWave < n_listed) f(lk[c], c * kWave + lane < n_listed);  // uniform
      };
      KVS_TOPK_TRACE(7);
      // As soon as the bin found holds a single key, that key is T.
      int settled = kTopkLevelShift[0];  // bits of `prefix` below this one are still open
      topk_level_count<0, false>(prefix, sh, listed_keys);
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      KVS_TOPK_TRACE(8);
      int in_bin = topk_level_scan<0>(prefix, above, M, sh);
      KVS_TOPK_TRACE(9);
      if (in_bin != 1) {  // uniform
        settled = kTopkLevelShift[1];
        topk_level_count<1, false>(prefix, sh, listed_keys);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        in_bin = topk_level_scan<1>(prefix, above, M, sh);
        if (in_bin != 1) {  // uniform
          settled = kTopkLevelShift[2];
          topk_level_count<2, false>(prefix, sh, listed_keys);
          __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
          topk_level_scan<2>(prefix, above, M, sh);
        }
      }
      if (settled != 0) {  // uniform
        const uint32_t want = prefix >> settled;
        listed_keys([&](uint32_t k, bool valid) __attribute__((always_inline)) {
          const unsigned long long is = __ballot(valid && (k >> settled) == want);
          if (is != 0ull) prefix = (uint32_t)__builtin_amdgcn_readlane((int)k, (int)__builtin_ctzll(is));
        });
      }
      KVS_TOPK_TRACE(10);
      if (lane == 0) sh.sel_key = prefix, sh.sel_above = above;
    }
    lds_barrier();
    prefix = sh.sel_key;
    above = sh.sel_above;
  } else {
    auto all_keys = [&](auto&& f) __attribute__((always_inline)) {
      slice_keys([&](uint32_t k, int j) __attribute__((always_inline)) { f(k, j < n_real); });
    };
    topk_level_block<0>(prefix, above, M, sh, all_keys);
    topk_level_block<1>(prefix, above, M, sh, all_keys);
    topk_level_block<2>(prefix, above, M, sh, all_keys);
  }
  KVS_TOPK_TRACE(5);
  // Selected: keys > T, plus the first `need` keys equal to T in index order.
  // (T below the smallest key of a score can only come from a histogram that does not
  // belong to these scores, e.g. a workspace that was never initialised: the unused slots
  // must stay unselected even then)
  const uint32_t T = max(prefix, kTopkMinKey);  // the M-th largest key
  const int need = M - above;  // `above` keys are greater than T

  // ---- 3. ordered compaction -------------------------------------------------------------
  uint32_t packed = 0;  // low half: keys > T, high half: keys == T
  slice_keys([&](uint32_t k, int) __attribute__((always_inline)) {
    packed += k > T ? 1u : 0u;
    packed += k == T ? 0x10000u : 0u;
  });
  const uint32_t excl = block_exclusive_scan(packed, sh.wave_tot[1]);
  KVS_TOPK_TRACE(6);
  int gt_before = (int)(excl & 0xFFFFu);
  int eq_before = (int)(excl >> 16);
  slice_keys([&](uint32_t k, int j) __attribute__((always_inline)) {
    const bool gt = k > T, eq = k == T;
    // (the bound only matters with a histogram that does not belong to these scores)
    const int pos = gt_before + min(eq_before, need);
    if ((gt || (eq && eq_before < need)) && pos < M) {
      if constexpr (PUBLISHED) publish_store(&out[pos], first + j);
      else out[pos] = first + j;
    }
    gt_before += gt ? 1 : 0;
    eq_before += eq ? 1 : 0;
  });
  if (hist_global) {  // leave the counters zero for the next call
#pragma unroll
    for (int sg = 0; sg < SPW; ++sg)
      if ((mine_raw[sg].x | mine_raw[sg].y | mine_raw[sg].z | mine_raw[sg].w) != 0)
        *reinterpret_cast<int4*>(hist_global + (kTopkBins - 4 - my_pos(sg))) = make_int4(0, 0, 0, 0);
  }
}

}  // namespace kvs
