// Workgroup-level top-M selection (Sec. 3.3, "TopK"): the indices of the M largest fp32
// scores of one problem, ties to the lower index, written in ascending index order.
//
// Scores are compared as order-preserving 32-bit keys.  The key T of the M-th largest
// score is found MSB-first:
//   1. a 4096-bin histogram of the top 12 key bits (sign, exponent, 3 mantissa bits)
//      names the bin that holds T and how many keys lie in higher bins.  The histogram
//      is either built here or was accumulated in global memory by the kernel that
//      produced the scores;
//   2. the remaining 20 bits are settled by three more, small histograms (8, 8 and 4
//      bits) in LDS, each over the keys that agree with the prefix found so far - a few
//      per cent of all keys after step 1, a handful after that - and each scanned by
//      one wave;
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

constexpr int kTopkLevels = 3;       // histogram levels below the first: 8 + 8 + 4 bits
static_assert(kTopkLowBits == 8 + 8 + 4, "the lower levels must cover the low bits");

struct TopkShared {
  int hist[kTopkBins];              // top-12-bit histogram when it is built here
  int sub[kTopkLevels][256];        // histograms of the lower levels
  uint32_t wave_tot[kTopkWaves];    // prefix-sum scratch
  int sel_bin, sel_above;
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
  if (tid < kTopkLevels * 256) (&sh.sub[0][0])[tid] = 0;  // (ordered before their use by the barriers of step 1)
  if (!hist_global) {
    for (int i = tid; i < kTopkBins; i += kTopkThreads) sh.hist[i] = 0;
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
  // ---- 2. settle the low 20 bits: three more histogram levels (8, 8 and 4 bits) ---------------
  // Only the keys that agree with the prefix found so far take part - a few per cent after
  // the first level, a handful after the second - so the LDS atomics are almost free of
  // contention; wave 0 scans the (at most 256) bins of a level from the top with one DPP
  // prefix sum.  Two barriers per level, nothing to gather, no limit on how many keys tie.
#pragma unroll
  for (int level = 0; level < kTopkLevels; ++level) {
    constexpr int kShift[kTopkLevels] = {12, 4, 0};
    constexpr int kBits[kTopkLevels] = {8, 8, 4};
    const int shift = kShift[level], bits = kBits[level], nbins = 1 << bits;
    const uint32_t hi = prefix >> (shift + bits);
#pragma unroll
    for (int c0 = 0; c0 < kTopkMaxPerLane; c0 += kTopkChunk) {
      if (c0 < kpt) {  // uniform
#pragma unroll
        for (int j = c0; j < c0 + kTopkChunk; ++j) {
          const bool real = (j < kpt) && (first + j < NG);
          const bool hit = real && (key[j] >> (shift + bits)) == hi;
          const int sub_bin = (int)((key[j] >> shift) & (uint32_t)(nbins - 1));
          const unsigned long long hits = __ballot(hit);
          if (hits != 0ull) {  // uniform
            // many equal scores would pile onto one counter: if every hit of the wave is in
            // the same bin, one lane adds them all
            const int first_hit = __builtin_ctzll(hits);
            const int bin0 = __builtin_amdgcn_readlane(sub_bin, first_hit);
            if (__ballot(hit && sub_bin == bin0) == hits) {
              if (lane == first_hit) atomicAdd(&sh.sub[level][bin0], __popcll(hits));
            } else if (hit) {
              atomicAdd(&sh.sub[level][sub_bin], 1);
            }
          }
        }
      }
    }
    lds_barrier();
    if (wave == 0) {
      int cnt[4];  // bins nbins-1-4*lane downwards
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int bin_c = nbins - 1 - (lane * 4 + c);
        cnt[c] = bin_c >= 0 ? sh.sub[level][bin_c] : 0;
      }
      const uint32_t tot = (uint32_t)(cnt[0] + cnt[1] + cnt[2] + cnt[3]);
      int above_me = above + (int)(wave_scan_dpp(tot) - tot);  // keys above my first bin
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (above_me < M && M <= above_me + cnt[c]) {
          sh.sel_bin = nbins - 1 - (lane * 4 + c);
          sh.sel_above = above_me;
        }
        above_me += cnt[c];
      }
    }
    lds_barrier();
    prefix |= (uint32_t)sh.sel_bin << shift;
    above = sh.sel_above;
  }
  KVS_TOPK_TRACE(5);
  // Selected: keys > T, plus the first `need` keys equal to T in index order.
  const uint32_t T = prefix;   // the M-th largest key
  const int need = M - above;  // `above` keys are greater than T

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
