// Workgroup-level top-M selection (Sec. 3.3, "TopK"): the indices of the M largest fp32
// scores of one problem, ties to the lower index, written in ascending index order.
//
// Scores are compared as order-preserving 32-bit keys.  The key T of the M-th largest
// score is found MSB-first:
//   1. a 4096-bin histogram of the top 12 key bits (sign, exponent, 3 mantissa bits)
//      names the bin that holds T and how many keys lie in higher bins.  The histogram
//      is either built here or was accumulated in global memory by the kernel that
//      produced the scores;
//   2. the keys of that bin - a few per cent of all keys for scores of similar
//      magnitude - are gathered in LDS, one per lane, and the remaining 20 bits are
//      settled two per round by counting, with wave ballots, how many candidates are
//      >= each of three pivots.  If the bin holds more keys than there are lanes (many
//      equal or tightly clustered scores) the same descent runs over every lane's
//      register-resident slice instead;
//   3. one block-wide prefix sum over packed (greater, equal) counts gives every
//      selected index its final position.
// Integer work only: the result is a deterministic function of the scores.
#pragma once

#include "device_utils.h"

#ifndef KVS_TOPK_TRACE
#define KVS_TOPK_TRACE(i)  // phase timestamps, only defined by the debugging harness
#endif

namespace kvs {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / kWave;
constexpr int kTopkMaxPerLane = 32;  // => at most 32768 scores per problem
constexpr int kTopkChunk = 8;        // register slots handled (and loads in flight) per uniform branch
constexpr int kTopkBins = 4096;      // histogram over key >> kTopkLowBits
constexpr int kTopkLowBits = 20;
constexpr int kTopkBinsPerLane = kTopkBins / kTopkThreads;

struct TopkShared {
  int hist[kTopkBins];              // top-12-bit histogram when it is built here
  uint32_t cand[kTopkThreads];      // keys of the bin that holds T
  int cnt[2][kTopkWaves][16];       // per-wave pivot counts, double-buffered by round
  uint32_t wave_tot[kTopkWaves];    // prefix-sum scratch
  int sel_bin, sel_above, n_cand;
};

// float -> uint32 whose unsigned order equals the float order; -0 is folded into +0
// so that equal scores have equal keys.  Every finite score maps to a key >= 1.
__device__ __forceinline__ uint32_t score_key(float x) {
  const uint32_t u = __float_as_uint(x + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inclusive prefix sum over the wave (lane i gets the sum of lanes 0..i), DPP only:
// a Hillis-Steele scan inside each row of 16 lanes (shifted-in lanes read as zero),
// then the running totals of the rows are passed on with row_bcast:15 / row_bcast:31.
__device__ __forceinline__ uint32_t wave_scan_dpp(uint32_t v) {
  int x = (int)v;
  x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, true);  // row_shr:1
  x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, true);  // row_shr:2
  x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, true);  // row_shr:4
  x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, true);  // row_shr:8
  x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false); // row_bcast:15 into rows 1 and 3
  x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false); // row_bcast:31 into rows 2 and 3
  return (uint32_t)x;
}

// Exclusive prefix sum across the workgroup in thread order (one barrier; wave_tot must
// not be rewritten before the next barrier of the caller).
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, TopkShared& sh) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const uint32_t incl = wave_scan_dpp(v);
  if (lane == kWave - 1) sh.wave_tot[wave] = incl;
  lds_barrier();
  uint32_t base = 0;
#pragma unroll
  for (int w = 0; w < kTopkWaves; ++w) base += (w < wave) ? sh.wave_tot[w] : 0u;
  return base + incl - v;
}

// One round of the descent.  c1..c3: this wave's counts of the keys it scans that are >=
// the three pivots; `base`: keys known to lie above everything that is being scanned.
// Invariant kept: at least M keys are >= prefix, and `above` (< M) keys are >= the upper
// end of the current range.  Returns true if a pivot cut off exactly M keys.
__device__ __forceinline__ bool descend(TopkShared& sh, int round, int c1, int c2, int c3, int base,
                                        int M, uint32_t p1, uint32_t p2, uint32_t p3,
                                        uint32_t& prefix, int& above) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int buf = round & 1;
  if (lane == 0) {
    sh.cnt[buf][wave][0] = c1;
    sh.cnt[buf][wave][1] = c2;
    sh.cnt[buf][wave][2] = c3;
  }
  lds_barrier();
  int C1 = base, C2 = base, C3 = base;
#pragma unroll
  for (int w = 0; w < kTopkWaves; ++w) {
    C1 += sh.cnt[buf][w][0];
    C2 += sh.cnt[buf][w][1];
    C3 += sh.cnt[buf][w][2];
  }
  int at;  // keys at or above the new lower end
  if (C3 >= M) { prefix = p3; at = C3; }
  else if (C2 >= M) { prefix = p2; above = C3; at = C2; }
  else if (C1 >= M) { prefix = p1; above = C2; at = C1; }
  else { above = C1; at = -1; }
  return at == M;
}

// All kTopkThreads lanes of the workgroup must call this with the same arguments.
// g: NG scores (16-byte aligned if NG is a multiple of 4); out: M indices;
// 1 <= M <= NG <= kTopkThreads * kTopkMaxPerLane.
// hist_global: nullptr => the histogram of the top 12 key bits is built here, in LDS;
// otherwise it points at the problem's kTopkBins counters in global memory, completed
// by an earlier kernel, and they are reset to zero on the way.
__device__ __forceinline__ void topk_block(const float* g, int32_t* __restrict__ out, int NG, int M,
                                           int* hist_global, TopkShared& sh) {
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;

  // the problem's histogram, if it was accumulated elsewhere: requested first so that
  // its latency overlaps the loads of the scores
  int mine[kTopkBinsPerLane];  // bins 4095-4*tid downwards
  if (hist_global) {
#pragma unroll
    for (int c = 0; c < kTopkBinsPerLane; ++c)
      mine[c] = hist_global[kTopkBins - 1 - (tid * kTopkBinsPerLane + c)];
  }
  // A lane owns a contiguous slice of kpt scores (what the ordered compaction needs).
  // With NG a multiple of four the slice is a whole number of 16-byte pieces and is
  // fetched as such: a wave then touches a few cache lines per load instead of 64.
  const bool vec = (NG & 3) == 0;  // uniform
  int kpt = (NG + kTopkThreads - 1) / kTopkThreads;  // scores per lane
  if (vec) kpt = (kpt + 3) & ~3;
  const int first = tid * kpt;

  // Slice of this lane, as keys, fetched in chunks of kTopkChunk slots whose loads are
  // all in flight together (addresses clamped, so no lane ever branches around a load).
  // Slots beyond the slice (and beyond NG) hold key 0, which is below the key of every
  // finite score.
  uint32_t key[kTopkMaxPerLane];
  {
    // every chunk's loads are requested before the first value is looked at, so a long
    // slice still costs one memory latency
    float x[kTopkMaxPerLane];
#pragma unroll
    for (int c0 = 0; c0 < kTopkMaxPerLane; c0 += kTopkChunk) {
      if (c0 < kpt && vec) {  // uniform
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
    for (int j = 0; j < kTopkMaxPerLane; ++j) asm volatile("" : "+v"(x[j]));
#pragma unroll
    for (int c0 = 0; c0 < kTopkMaxPerLane; c0 += kTopkChunk) {
#pragma unroll
      for (int j = c0; j < c0 + kTopkChunk; ++j)
        key[j] = (c0 < kpt && j < kpt && first + j < NG) ? score_key(x[j]) : 0u;
    }
  }

  KVS_TOPK_TRACE(1);
  if (hist_global) {
    // keep the histogram loads where they were written (ahead of the score loads) so that
    // both latencies overlap instead of the compiler sinking them to their first use
#pragma unroll
    for (int c = 0; c < kTopkBinsPerLane; ++c) asm volatile("" : "+v"(mine[c]));
  }
  // ---- 1. histogram of the top 12 bits ------------------------------------------------
  if (hist_global) {
    if (tid == 0) sh.n_cand = 0;
  } else {
    for (int i = tid; i < kTopkBins; i += kTopkThreads) sh.hist[i] = 0;
    if (tid == 0) sh.n_cand = 0;
    lds_barrier();
#pragma unroll
    for (int c0 = 0; c0 < kTopkMaxPerLane; c0 += kTopkChunk) {
      if (c0 < kpt) {  // uniform
#pragma unroll
        for (int j = c0; j < c0 + kTopkChunk; ++j)
          if (j < kpt && first + j < NG) atomicAdd(&sh.hist[key[j] >> kTopkLowBits], 1);
      }
    }
    lds_barrier();
#pragma unroll
    for (int c = 0; c < kTopkBinsPerLane; ++c)
      mine[c] = sh.hist[kTopkBins - 1 - (tid * kTopkBinsPerLane + c)];
  }
  KVS_TOPK_TRACE(2);
  {
    uint32_t tot = 0;
#pragma unroll
    for (int c = 0; c < kTopkBinsPerLane; ++c) tot += (uint32_t)mine[c];
    int above_me = (int)block_exclusive_scan(tot, sh);  // keys in bins above my first bin
#pragma unroll
    for (int c = 0; c < kTopkBinsPerLane; ++c) {
      if (above_me < M && M <= above_me + mine[c]) {
        sh.sel_bin = kTopkBins - 1 - (tid * kTopkBinsPerLane + c);
        sh.sel_above = above_me;
      }
      above_me += mine[c];
    }
  }
  lds_barrier();
  const uint32_t bin = (uint32_t)sh.sel_bin;
  uint32_t prefix = bin << kTopkLowBits;
  int above = sh.sel_above;  // keys in higher bins; the M-th key is in `bin`

  KVS_TOPK_TRACE(3);
  // ---- 2. settle the low 20 bits ----------------------------------------------------------
  // gather the keys of the bin, one slot each (order is irrelevant here): each wave
  // counts its candidates, reserves a range with one LDS atomic, then fills it
  {
    int wave_total = 0;
#pragma unroll
    for (int c0 = 0; c0 < kTopkMaxPerLane; c0 += kTopkChunk) {
      if (c0 < kpt) {  // uniform
#pragma unroll
        for (int j = c0; j < c0 + kTopkChunk; ++j)
          wave_total += __popcll(__ballot((key[j] >> kTopkLowBits) == bin));  // padding keys are 0: bin 0 only
      }
    }
    int base = 0;
    if (wave_total != 0) {  // uniform
      if (lane == 0) base = atomicAdd(&sh.n_cand, wave_total);
      base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
      for (int c0 = 0; c0 < kTopkMaxPerLane; c0 += kTopkChunk) {
        if (c0 < kpt) {  // uniform
#pragma unroll
          for (int j = c0; j < c0 + kTopkChunk; ++j) {
            const bool is_cand = (key[j] >> kTopkLowBits) == bin;
            const unsigned long long m = __ballot(is_cand);
            const int pos = base + __popcll(m & ((1ull << lane) - 1ull));
            if (is_cand && pos < kTopkThreads) sh.cand[pos] = key[j];
            base += __popcll(m);
          }
        }
      }
    }
  }
  lds_barrier();
  const int n_cand = sh.n_cand;
  KVS_TOPK_TRACE(4);
  const int bin_above = above;
  bool cut = (above + n_cand == M) && prefix != 0u;  // the whole bin is selected: nothing to settle
  if (!cut) {
    if (n_cand <= kTopkThreads) {
      // one candidate per lane; four bits per round: 15 pivots, counted with ballots,
      // summed over the waves by lanes 0..14 of every wave
      const uint32_t ck = (tid < n_cand) ? sh.cand[tid] : 0u;  // 0 is below every pivot
#pragma unroll 1
      for (int shift = kTopkLowBits - 4; shift >= 0; shift -= 4) {
        const int buf = (shift >> 2) & 1;
#pragma unroll
        for (int i = 1; i < 16; ++i) {
          const int c = __popcll(__ballot(ck >= (prefix | ((uint32_t)i << shift))));
          if (lane == 0) sh.cnt[buf][wave][i - 1] = c;
        }
        lds_barrier();
        int tot = bin_above;  // lane l (< 15): keys >= pivot l+1, counting those in higher bins
        if (lane < 15) {
#pragma unroll
          for (int w = 0; w < kTopkWaves; ++w) tot += sh.cnt[buf][w][lane];
        }
        // totals fall as the pivot rises: the pivots with >= M keys form a prefix
        const int i = __popcll(__ballot(lane < 15 && tot >= M));  // 0..15, uniform
        const int t_next = __builtin_amdgcn_readlane(tot, min(i, 14));
        const int t_here = __builtin_amdgcn_readlane(tot, max(i - 1, 0));
        if (i < 15) above = t_next;          // keys >= the next pivot lie above the new range
        if (i > 0) {
          prefix |= (uint32_t)i << shift;
          if (t_here == M) { cut = true; break; }  // uniform
        }
      }
    } else {
#pragma unroll 1
      for (int shift = kTopkLowBits - 2; shift >= 0; shift -= 2) {
        const uint32_t p1 = prefix | (1u << shift), p2 = prefix | (2u << shift), p3 = prefix | (3u << shift);
        int c1 = 0, c2 = 0, c3 = 0;
#pragma unroll
        for (int c0 = 0; c0 < kTopkMaxPerLane; c0 += kTopkChunk) {
          if (c0 < kpt) {  // uniform
#pragma unroll
            for (int j = c0; j < c0 + kTopkChunk; ++j) {
              c1 += __popcll(__ballot(key[j] >= p1));
              c2 += __popcll(__ballot(key[j] >= p2));
              c3 += __popcll(__ballot(key[j] >= p3));
            }
          }
        }
        if (descend(sh, shift >> 1, c1, c2, c3, 0, M, p1, p2, p3, prefix, above)) { cut = true; break; }
      }
    }
  }
  KVS_TOPK_TRACE(5);
  // Selected: keys > T, plus the first `need` keys equal to T in index order.
  // After a clean cut everything >= prefix is selected: T = prefix - 1 and need = 0.
  const uint32_t T = cut ? prefix - 1u : prefix;
  const int need = cut ? 0 : M - above;

  // ---- 3. ordered compaction -------------------------------------------------------------
  uint32_t packed = 0;  // low half: keys > T, high half: keys == T
#pragma unroll
  for (int c0 = 0; c0 < kTopkMaxPerLane; c0 += kTopkChunk) {
    if (c0 < kpt) {  // uniform
#pragma unroll
      for (int j = c0; j < c0 + kTopkChunk; ++j) {
        const bool real = (j < kpt) && (first + j < NG);
        packed += (real && key[j] > T) ? 1u : 0u;
        packed += (real && key[j] == T) ? 0x10000u : 0u;
      }
    }
  }
  const uint32_t excl = block_exclusive_scan(packed, sh);
  KVS_TOPK_TRACE(6);
  int gt_before = (int)(excl & 0xFFFFu);
  int eq_before = (int)(excl >> 16);
#pragma unroll
  for (int c0 = 0; c0 < kTopkMaxPerLane; c0 += kTopkChunk) {
    if (c0 < kpt) {  // uniform
#pragma unroll
      for (int j = c0; j < c0 + kTopkChunk; ++j) {
        if (j < kpt && first + j < NG) {
          const bool gt = key[j] > T, eq = key[j] == T;
          // (the bound only matters if the caller handed in a histogram that does not
          // belong to these scores, e.g. a workspace that was never initialised)
          const int pos = gt_before + min(eq_before, need);
          if ((gt || (eq && eq_before < need)) && pos < M) out[pos] = first + j;
          gt_before += gt ? 1 : 0;
          eq_before += eq ? 1 : 0;
        }
      }
    }
  }
  if (hist_global) {
#pragma unroll
    for (int c = 0; c < kTopkBinsPerLane; ++c)  // leave the counters zero for the next call
      if (mine[c]) hist_global[kTopkBins - 1 - (tid * kTopkBinsPerLane + c)] = 0;
  }
}

}  // namespace kvs
