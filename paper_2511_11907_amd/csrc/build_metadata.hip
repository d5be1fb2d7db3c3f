// Compact key metadata (Sec. 3.2): K_lr[b,k,n,:] = K[b,k,n,:] . A[k], fp32
// accumulation over the head dimension in natural order, one rounding to the
// metadata dtype.  Runs at prefill and when new groups are appended, outside the
// per-step latency.  In joint-head mode the row that is projected is the token's
// keys of all KV heads side by side, K_lr[b,n,:] = sum_k K[b,k,n,:] . A_k with A_k
// the k-th block of d rows of the single adapter: the same tile loop, run over the
// KV heads with the accumulators kept.
//
// build_metadata_mfma_kernel / build_metadata_mfma_joint_kernel (bf16 keys: the shapes the
// method is run at) put the contraction on the matrix cores and are bound by reading K;
// build_metadata_kernel (fp32 keys) is the plain fp32 FMA version described next.
//
// A workgroup owns a tile of 64 consecutive token rows of one (sequence, KV head)
// problem (of one sequence in joint-head mode).  The K tile is brought in with coalesced 16-byte loads and parked in
// LDS as fp32 (row stride d+1 words, so the 64 lanes of a wave, one row each, hit
// 64 different banks); wave w produces the w-th quarter of the r output columns
// for all 64 rows, so the adapter entries it needs are the same for every lane of
// the wave (uniform loads).
#include "device_utils.h"
#include "kernels.h"

namespace kvs {

constexpr int kMetaThreads = 256;
constexpr int kMetaRows = 64;

template <typename EK, typename EM, int RC>  // RC = r / 4 output columns per lane
__global__ __launch_bounds__(kMetaThreads) void build_metadata_kernel(
    const typename EK::storage* __restrict__ K, const float* __restrict__ A,
    typename EM::storage* __restrict__ K_lr, int n_kv_heads, int heads_per_set, int ctx_rows,
    int first_row, int row_end, int d, float meta_scale_all, const float* __restrict__ meta_scales) {
  constexpr int R = RC * 4;
  const float meta_scale = meta_scales ? meta_scales[blockIdx.y] : meta_scale_all;  // one per selection set
  extern __shared__ float s_k[];  // [kMetaRows][d + 1]
  const int tid = threadIdx.x;
  const int set = blockIdx.y;  // (b, k), or b alone when the heads are projected jointly
  const int row0 = first_row + blockIdx.x * kMetaRows;  // rows [first_row, row_end) are built
  const int ld = d + 1;
  constexpr int EPL = EK::kPerLane;
  const int lanes_per_row = d / EPL;
  const int row = tid & (kMetaRows - 1);
  const int jq = __builtin_amdgcn_readfirstlane(tid / kMetaRows);  // wave-uniform column quarter
  float acc[RC];
#pragma unroll
  for (int j = 0; j < RC; ++j) acc[j] = 0.f;

  for (int kk = 0; kk < heads_per_set; ++kk) {
    const int p = set * heads_per_set + kk;  // (b, k) problem whose keys are staged
    const int k = p % n_kv_heads;
    if (kk > 0) lds_barrier();               // everyone is done with the previous tile
    // stage the tile: 16 bytes per lane, consecutive lanes along the row
    const typename EK::storage* Kp = K + ((size_t)p * ctx_rows + row0) * d;
    for (int i = tid; i < kMetaRows * lanes_per_row; i += kMetaThreads) {
      const int r_ = i / lanes_per_row, cc = i % lanes_per_row;
      float f[EPL];
      if (row0 + r_ < row_end) {
        const uint4 v = *reinterpret_cast<const uint4*>(Kp + (size_t)r_ * d + (size_t)cc * EPL);
        unpack16<EK>(v, f);
      } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) f[e] = 0.f;
      }
#pragma unroll
      for (int e = 0; e < EPL; ++e) s_k[r_ * ld + cc * EPL + e] = f[e];
    }
    lds_barrier();
    const float* Ak = A + (size_t)k * d * R + (size_t)jq * RC;
    for (int i = 0; i < d; ++i) {
      const float kv = s_k[row * ld + i];
#pragma unroll
      for (int j = 0; j < RC; ++j) acc[j] = fmaf(kv, Ak[(size_t)i * R + j], acc[j]);
    }
  }
  if (row0 + row < row_end) {
    typename EM::storage* o = K_lr + ((size_t)set * ctx_rows + row0 + row) * R + (size_t)jq * RC;
#pragma unroll
    for (int j = 0; j < RC; ++j) {
      const float v = acc[j] / meta_scale;  // (exact when the scale is 1)
      if constexpr (EM::kBytes == 2) o[j] = float_to_bf16_bits(v);
      else if constexpr (EM::kBytes == 1) o[j] = float_to_fp8_e4m3(v);
      else o[j] = v;
    }
  }
}

// ---- matrix-core version ------------------------------------------------------------------
// K_lr^T (r x tokens) = A^T (r x d) . K^T (d x tokens), 16x16x32 bf16 MFMA tiles with fp32
// accumulation.  The keys are bf16 already.  The fp32 adapter is split into three bf16
// terms (hi + mid + lo reproduces all 24 mantissa bits), so every product is exact and the
// only rounding left is the fp32 accumulation, as in the FMA version.
//
// Operand layout of the instruction (checked on the device): lane l supplies row/column
// (l % 16) and the eight contraction indices (l / 16) * 8 .. + 7 of a 32-wide step, and
// receives output column (l % 16), rows (l / 16) * 4 .. + 3.  With tokens as the columns,
// the four lanes that share a token read 64 contiguous bytes of its key row per step
// (a 32x32 tile would leave 32: measured to be bound by the cache's tag rate at 3 TB/s),
// and a lane ends up with four consecutive rank indices of one token, i.e. one 8-byte
// store (bf16) into the row-major K_lr.  The adapter operands are laid out once per
// workgroup in LDS; each is read once per tile and used for both token blocks of the wave.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

// Exchanges between a wave's lanes for the stores (gfx950's lane-swap instructions, layouts
// checked on the device): after swap_upper_lower_half(a, b) lanes 32..63 of a hold what
// lanes 0..31 of b held and vice versa; after swap_odd_even_rows(a, b) the odd rows of 16
// lanes of a hold what the even rows of b held (row 1 <- row 0, row 3 <- row 2) and vice
// versa.
__device__ __forceinline__ void swap_upper_lower_half(uint32_t& a, uint32_t& b) {
  const auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
  a = r[0], b = r[1];
}
__device__ __forceinline__ void swap_odd_even_rows(uint32_t& a, uint32_t& b) {
  const auto r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
  a = r[0], b = r[1];
}

// 16-byte accesses of the streaming operands.  With two rank blocks per pass (r = 32) the
// kernel is faster with non-temporal keys and results (7-11 % at 16K-128K contexts); with one
// block it makes no difference and with four (r = 64, r = 128) it is 5-8 % slower, so the
// hint follows the instantiation.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
template <bool STREAM>
__device__ __forceinline__ uint4 load_keys16(const void* p) {
  if constexpr (STREAM) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
  } else {
    return *reinterpret_cast<const uint4*>(p);
  }
}
template <bool STREAM>
__device__ __forceinline__ void store_rows16(void* p, uint4 v) {
  if constexpr (STREAM) {
    const u32x4_t w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t*>(p));
  } else {
    *reinterpret_cast<uint4*>(p) = v;
  }
}

constexpr int kMfmaThreads = 256;
constexpr int kMfmaWaves = kMfmaThreads / kWave;
constexpr int kMfmaTokenBlocks = 2;                         // blocks of 16 tokens per wave
constexpr int kMfmaRowsPerWave = 16 * kMfmaTokenBlocks;
constexpr int kMfmaRowsPerTile = kMfmaWaves * kMfmaRowsPerWave;

template <typename EM, int D, int MB>  // MB blocks of 16 rank columns (r <= 16 * MB)
__global__ __launch_bounds__(kMfmaThreads) void build_metadata_mfma_kernel(
    const uint16_t* __restrict__ K, const float* __restrict__ A,
    typename EM::storage* __restrict__ K_lr, int n_kv_heads, int ctx_rows, int first_row,
    int row_end, int r, int col0, int cols, float meta_scale_all, const float* __restrict__ meta_scales) {
  const float meta_scale = meta_scales ? meta_scales[blockIdx.y] : meta_scale_all;  // one per selection set
  // this launch produces rank columns col0 .. col0 + cols - 1 (cols <= 16 * MB) of the r
  constexpr int KS = D / 32;  // contraction steps
  constexpr int TB = kMfmaTokenBlocks;
  __shared__ uint4 s_a[3][MB][KS][kWave];  // [split term][rank block][step][lane]

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int p = blockIdx.y, k_head = p % n_kv_heads;
  const int nl = lane & 15, kq = lane >> 4;

  // adapter operands: entry (mb, ks, lane) holds A[k = ks*32 + kq*8 + j][m = mb*16 + nl],
  // j = 0..7, as the hi / mid / lo bf16 terms
  {
    const float* Ak = A + (size_t)k_head * D * r;
    for (int e = tid; e < MB * KS * kWave; e += kMfmaThreads) {
      const int l = e % kWave, ks = (e / kWave) % KS, mb = e / (kWave * KS);
      const int m = mb * 16 + (l & 15), k0 = ks * 32 + (l >> 4) * 8;
      uint16_t t[3][8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float x = (m < cols) ? Ak[(size_t)(k0 + j) * r + col0 + m] : 0.f;
        const uint16_t hi = float_to_bf16_bits(x);
        const float r1 = x - bf16_bits_to_float(hi);   // exact
        const uint16_t mid = float_to_bf16_bits(r1);
        const float r2 = r1 - bf16_bits_to_float(mid);  // exact
        t[0][j] = hi, t[1][j] = mid, t[2][j] = float_to_bf16_bits(r2);
      }
#pragma unroll
      for (int sp = 0; sp < 3; ++sp)
        s_a[sp][mb][ks][l] = make_uint4(t[sp][0] | (uint32_t)t[sp][1] << 16, t[sp][2] | (uint32_t)t[sp][3] << 16,
                                        t[sp][4] | (uint32_t)t[sp][5] << 16, t[sp][6] | (uint32_t)t[sp][7] << 16);
    }
  }
  lds_barrier();

  const uint16_t* Kp = K + (size_t)p * ctx_rows * D + (size_t)kq * 8;
  typename EM::storage* Op = K_lr + (size_t)p * ctx_rows * r;
  const int n_tiles = (row_end - first_row + kMfmaRowsPerTile - 1) / kMfmaRowsPerTile;

  auto row_of = [&](int tile, int tb) {
    return first_row + tile * kMfmaRowsPerTile + wave * kMfmaRowsPerWave + tb * 16 + nl;
  };
  auto fetch = [&](int tile, uint4 (&kr)[TB][KS]) {
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      const int row = min(row_of(tile, tb), row_end - 1);  // rows past the end are computed and dropped
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        kr[tb][ks] = load_keys16<MB == 2>(Kp + (size_t)row * D + ks * 32);
    }
  };

  uint4 kcur[TB][KS], knext[TB][KS];
  int tile = blockIdx.x;
  if (tile < n_tiles) fetch(tile, kcur);
  for (; tile < n_tiles; tile += gridDim.x) {
    const int tn = tile + gridDim.x;
    if (tn < n_tiles) fetch(tn, knext);  // next tile's keys travel while this one is multiplied

    // The adapter operands are read from LDS again for every tile: kept in registers across
    // tiles (what the compiler does if it may) they cost 192 registers and leave one wave
    // per SIMD.
    asm volatile("" ::: "memory");
    f32x4_t acc[TB][MB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) acc[tb][mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#ifndef KVS_META_TERMS
#define KVS_META_TERMS 3  // (timing experiments only: fewer terms give wrong low-order bits)
#endif
#pragma unroll
    for (int sp = 0; sp < KVS_META_TERMS; ++sp)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          const bf16x8_t a = __builtin_bit_cast(bf16x8_t, s_a[sp][mb][ks][lane]);
#pragma unroll
          for (int tb = 0; tb < TB; ++tb)
            acc[tb][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                a, __builtin_bit_cast(bf16x8_t, kcur[tb][ks]), acc[tb][mb], 0, 0, 0);
        }

    // accumulator i of rank block mb is rank index mb*16 + kq*4 + i of this lane's token
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      const int row = row_of(tile, tb);
      if constexpr (EM::kBytes == 2 && (MB == 2 || MB == 4)) {
        if (cols == 16 * MB) {  // uniform: whole rank blocks, the usual case
          // The four lanes of a token hold 8 bytes of each rank block; exchanged between
          // them (rank block <-> lane group) every lane ends up with 16 or 32 consecutive
          // bytes of the row, and one or two store instructions write whole rows.
          uint32_t lo[MB], hi[MB];
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) {
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = acc[tb][mb][j] / meta_scale;
            lo[mb] = float_to_bf16_bits(v[0]) | (uint32_t)float_to_bf16_bits(v[1]) << 16;
            hi[mb] = float_to_bf16_bits(v[2]) | (uint32_t)float_to_bf16_bits(v[3]) << 16;
          }
          if constexpr (MB == 4) {
            swap_upper_lower_half(lo[0], lo[2]), swap_upper_lower_half(lo[1], lo[3]);
            swap_upper_lower_half(hi[0], hi[2]), swap_upper_lower_half(hi[1], hi[3]);
            swap_odd_even_rows(lo[0], lo[1]), swap_odd_even_rows(lo[2], lo[3]);
            swap_odd_even_rows(hi[0], hi[1]), swap_odd_even_rows(hi[2], hi[3]);
            // lane group kq now holds ranks kq*16 .. kq*16 + 15 of its token
            if (row < row_end) {
              uint4* o = reinterpret_cast<uint4*>(Op + (size_t)row * r + col0 + kq * 16);
              o[0] = make_uint4(lo[0], hi[0], lo[1], hi[1]);
              o[1] = make_uint4(lo[2], hi[2], lo[3], hi[3]);
            }
          } else {
            swap_odd_even_rows(lo[0], lo[1]), swap_odd_even_rows(hi[0], hi[1]);
            // lane group kq now holds ranks (kq & 1) * 16 + (kq & 2) * 4 .. + 7 of its token
            if (row < row_end)
              store_rows16<true>(Op + (size_t)row * r + col0 + (kq & 1) * 16 + (kq & 2) * 4,
                                 make_uint4(lo[0], hi[0], lo[1], hi[1]));
          }
          continue;
        }
      }
      if constexpr (EM::kBytes == 1 && (MB == 2 || MB == 4)) {
        if (cols == 16 * MB) {  // uniform; the same exchange with four one-byte values per rank block
          uint32_t b4[MB];
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) {
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = acc[tb][mb][j] / meta_scale;
            b4[mb] = float_to_fp8_e4m3(v[0]) | (uint32_t)float_to_fp8_e4m3(v[1]) << 8 |
                     (uint32_t)float_to_fp8_e4m3(v[2]) << 16 | (uint32_t)float_to_fp8_e4m3(v[3]) << 24;
          }
          if constexpr (MB == 4) {
            swap_upper_lower_half(b4[0], b4[2]), swap_upper_lower_half(b4[1], b4[3]);
            swap_odd_even_rows(b4[0], b4[1]), swap_odd_even_rows(b4[2], b4[3]);
            if (row < row_end)
              *reinterpret_cast<uint4*>(Op + (size_t)row * r + col0 + kq * 16) = make_uint4(b4[0], b4[1], b4[2], b4[3]);
          } else {
            swap_odd_even_rows(b4[0], b4[1]);
            if (row < row_end)
              *reinterpret_cast<uint2*>(Op + (size_t)row * r + col0 + (kq & 1) * 16 + (kq & 2) * 4) =
                  make_uint2(b4[0], b4[1]);
          }
          continue;
        }
      }
      if (row < row_end) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          const int m0 = mb * 16 + kq * 4;
          if (m0 < cols) {  // (a multiple of 16, so a quad is inside or outside as a whole)
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = acc[tb][mb][j] / meta_scale;
            typename EM::storage* o = Op + (size_t)row * r + col0 + m0;
            if constexpr (EM::kBytes == 2) {
              *reinterpret_cast<uint2*>(o) =
                  make_uint2(float_to_bf16_bits(v[0]) | (uint32_t)float_to_bf16_bits(v[1]) << 16,
                             float_to_bf16_bits(v[2]) | (uint32_t)float_to_bf16_bits(v[3]) << 16);
            } else if constexpr (EM::kBytes == 1) {
              *reinterpret_cast<uint32_t*>(o) = float_to_fp8_e4m3(v[0]) | (uint32_t)float_to_fp8_e4m3(v[1]) << 8 |
                                                (uint32_t)float_to_fp8_e4m3(v[2]) << 16 |
                                                (uint32_t)float_to_fp8_e4m3(v[3]) << 24;
            } else {
              *reinterpret_cast<float4*>(o) = make_float4(v[0], v[1], v[2], v[3]);
            }
          }
        }
      }
    }
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) kcur[tb][ks] = knext[tb][ks];
  }
}

// ---- matrix-core version, joint-head mode ---------------------------------------------------
// K_lr[b,n,:] = sum_k K[b,k,n,:] . A_k: the same tiles, with the accumulators of a wave's
// tokens kept while the KV heads go by.  The adapter block of one head at a time lives in
// LDS (all H_kv blocks would not fit), so a workgroup restages it per head and amortises
// that over the 256 token rows it owns per pass; the keys of the head are requested first
// and travel while the block is staged.
constexpr int kMfmaJointTokenBlocks = 4;  // blocks of 16 tokens per wave
constexpr int kMfmaJointRowsPerWave = 16 * kMfmaJointTokenBlocks;
constexpr int kMfmaJointRowsPerTile = kMfmaWaves * kMfmaJointRowsPerWave;

template <typename EM, int D, int MB>
__global__ __launch_bounds__(kMfmaThreads) void build_metadata_mfma_joint_kernel(
    const uint16_t* __restrict__ K, const float* __restrict__ A,
    typename EM::storage* __restrict__ K_lr, int n_kv_heads, int ctx_rows, int first_row,
    int row_end, int r, int col0, int cols, float meta_scale_all, const float* __restrict__ meta_scales) {
  const float meta_scale = meta_scales ? meta_scales[blockIdx.y] : meta_scale_all;  // one per selection set
  constexpr int KS = D / 32;
  constexpr int TB = kMfmaJointTokenBlocks;
  __shared__ uint4 s_a[3][MB][KS][kWave];

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int b = blockIdx.y;
  const int nl = lane & 15, kq = lane >> 4;
  typename EM::storage* Op = K_lr + (size_t)b * ctx_rows * r;
  const int n_tiles = (row_end - first_row + kMfmaJointRowsPerTile - 1) / kMfmaJointRowsPerTile;

  for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const int row0 = first_row + tile * kMfmaJointRowsPerTile + wave * kMfmaJointRowsPerWave + nl;
    f32x4_t acc[TB][MB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) acc[tb][mb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    for (int kh = 0; kh < n_kv_heads; ++kh) {
      // this head's keys of the wave's tokens: requested before the adapter block is staged
      const uint16_t* Kp = K + ((size_t)b * n_kv_heads + kh) * ctx_rows * D + (size_t)kq * 8;
      uint4 kr[TB][KS];
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        const int row = min(row0 + tb * 16, row_end - 1);  // rows past the end are computed and dropped
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          kr[tb][ks] = *reinterpret_cast<const uint4*>(Kp + (size_t)row * D + ks * 32);  // (non-temporal: slower here)
      }
      lds_barrier();  // everyone is done with the previous head's block
      {
        const float* Ak = A + (size_t)kh * D * r;
        for (int e = tid; e < MB * KS * kWave; e += kMfmaThreads) {
          const int l = e % kWave, ks = (e / kWave) % KS, mb = e / (kWave * KS);
          const int m = mb * 16 + (l & 15), k0 = ks * 32 + (l >> 4) * 8;
          uint16_t t[3][8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float x = (m < cols) ? Ak[(size_t)(k0 + j) * r + col0 + m] : 0.f;
            const uint16_t hi = float_to_bf16_bits(x);
            const float r1 = x - bf16_bits_to_float(hi);   // exact
            const uint16_t mid = float_to_bf16_bits(r1);
            const float r2 = r1 - bf16_bits_to_float(mid);  // exact
            t[0][j] = hi, t[1][j] = mid, t[2][j] = float_to_bf16_bits(r2);
          }
#pragma unroll
          for (int sp = 0; sp < 3; ++sp)
            s_a[sp][mb][ks][l] = make_uint4(t[sp][0] | (uint32_t)t[sp][1] << 16, t[sp][2] | (uint32_t)t[sp][3] << 16,
                                            t[sp][4] | (uint32_t)t[sp][5] << 16, t[sp][6] | (uint32_t)t[sp][7] << 16);
        }
      }
      lds_barrier();
#pragma unroll
      for (int sp = 0; sp < 3; ++sp)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) {
            const bf16x8_t a = __builtin_bit_cast(bf16x8_t, s_a[sp][mb][ks][lane]);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
              acc[tb][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                  a, __builtin_bit_cast(bf16x8_t, kr[tb][ks]), acc[tb][mb], 0, 0, 0);
          }
    }

#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
      const int row = row0 + tb * 16;
      if (row < row_end) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          const int m0 = mb * 16 + kq * 4;
          if (m0 < cols) {
            float v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = acc[tb][mb][j] / meta_scale;
            typename EM::storage* o = Op + (size_t)row * r + col0 + m0;
            if constexpr (EM::kBytes == 2) {
              *reinterpret_cast<uint2*>(o) =
                  make_uint2(float_to_bf16_bits(v[0]) | (uint32_t)float_to_bf16_bits(v[1]) << 16,
                             float_to_bf16_bits(v[2]) | (uint32_t)float_to_bf16_bits(v[3]) << 16);
            } else if constexpr (EM::kBytes == 1) {
              *reinterpret_cast<uint32_t*>(o) = float_to_fp8_e4m3(v[0]) | (uint32_t)float_to_fp8_e4m3(v[1]) << 8 |
                                                (uint32_t)float_to_fp8_e4m3(v[2]) << 16 |
                                                (uint32_t)float_to_fp8_e4m3(v[3]) << 24;
            } else {
              *reinterpret_cast<float4*>(o) = make_float4(v[0], v[1], v[2], v[3]);
            }
          }
        }
      }
    }
  }
}

namespace {

template <typename EK, typename EM, int RC>
hipError_t launch_one(const kvs_params& p, const Plan& pl, const void* K, const float* A,
                      void* K_lr, int first_row, int n_rows, hipStream_t st) {
  dim3 grid((n_rows + kMetaRows - 1) / kMetaRows, pl.sets), block(kMetaThreads);
  const size_t lds = (size_t)kMetaRows * (p.head_dim + 1) * sizeof(float);
  hipLaunchKernelGGL((build_metadata_kernel<EK, EM, RC>), grid, block, lds, st,
                     (const typename EK::storage*)K, A, (typename EM::storage*)K_lr, p.n_kv_heads,
                     pl.kv_heads_per_set, pl.ctx_rows, first_row, first_row + n_rows, p.head_dim,
                     p.meta_scale != 0.f ? p.meta_scale : 1.0f, p.meta_scales);
  return hipGetLastError();
}

template <typename EK, typename EM>
hipError_t launch_r(const kvs_params& p, const Plan& pl, const void* K, const float* A,
                    void* K_lr, int first_row, int n_rows, hipStream_t st) {
  switch (p.rank) {
    case 16: return launch_one<EK, EM, 4>(p, pl, K, A, K_lr, first_row, n_rows, st);
    case 32: return launch_one<EK, EM, 8>(p, pl, K, A, K_lr, first_row, n_rows, st);
    case 64: return launch_one<EK, EM, 16>(p, pl, K, A, K_lr, first_row, n_rows, st);
    case 128: return launch_one<EK, EM, 32>(p, pl, K, A, K_lr, first_row, n_rows, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_build_metadata(const kvs_params& p, const Plan& pl, const void* K,
                                 const float* A, void* K_lr, int first_row, int n_rows,
                                 hipStream_t st) {
  if (n_rows <= 0) return hipSuccess;
  const bool kb = p.kv_dtype == KVS_BF16, mbf = p.meta_dtype == KVS_BF16;
  if (kb) {  // matrix-core paths (r = 128: two passes of 64 columns)
    const bool joint = pl.kv_heads_per_set > 1;
    const int rows_per_tile = joint ? kMfmaJointRowsPerTile : kMfmaRowsPerTile;
    const int tiles = (n_rows + rows_per_tile - 1) / rows_per_tile;
    int wgs = (kMetaMfmaTargetWgs + pl.sets - 1) / pl.sets;   // enough workgroups to fill the chip,
    wgs = wgs < 1 ? 1 : (wgs > tiles ? tiles : wgs);          // each walking several tiles
    dim3 grid(wgs, pl.sets), block(kMfmaThreads);
    const float scale = p.meta_scale != 0.f ? p.meta_scale : 1.0f;
    auto go = [&](auto kernel, auto* out) {
      for (int col0 = 0; col0 < p.rank; col0 += 64) {
        const int cols = p.rank - col0 < 64 ? p.rank - col0 : 64;
        hipLaunchKernelGGL(kernel, grid, block, 0, st, (const uint16_t*)K, A, out, p.n_kv_heads,
                           pl.ctx_rows, first_row, first_row + n_rows, p.rank, col0, cols, scale, p.meta_scales);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
      }
      return hipSuccess;
    };
    const int mb = p.rank >= 64 ? 4 : p.rank / 16;  // 1, 2 or 4 rank blocks per pass
    const bool d128 = p.head_dim == 128;
#define KVS_MFMA_PICK(KERNEL, EM, T)                                                                  \
  if (d128) return mb == 4 ? go(KERNEL<EM, 128, 4>, (T*)K_lr)                                        \
                 : mb == 2 ? go(KERNEL<EM, 128, 2>, (T*)K_lr)                                        \
                           : go(KERNEL<EM, 128, 1>, (T*)K_lr);                                       \
  return mb == 4 ? go(KERNEL<EM, 64, 4>, (T*)K_lr)                                                   \
       : mb == 2 ? go(KERNEL<EM, 64, 2>, (T*)K_lr)                                                   \
                 : go(KERNEL<EM, 64, 1>, (T*)K_lr);
#define KVS_MFMA_CASE(EM, T)                                                                          \
  if (joint) { KVS_MFMA_PICK(build_metadata_mfma_joint_kernel, EM, T) }                              \
  KVS_MFMA_PICK(build_metadata_mfma_kernel, EM, T)
    if (p.meta_dtype == KVS_FP8_E4M3) { KVS_MFMA_CASE(FP8Elem, uint8_t) }
    if (mbf) { KVS_MFMA_CASE(BF16Elem, uint16_t) }
    KVS_MFMA_CASE(F32Elem, float)
#undef KVS_MFMA_CASE
#undef KVS_MFMA_PICK
  }
  if (p.meta_dtype == KVS_FP8_E4M3) {
    if (kb) return launch_r<BF16Elem, FP8Elem>(p, pl, K, A, K_lr, first_row, n_rows, st);
    return launch_r<F32Elem, FP8Elem>(p, pl, K, A, K_lr, first_row, n_rows, st);
  }
  const bool mb = mbf;
  if (kb && mb) return launch_r<BF16Elem, BF16Elem>(p, pl, K, A, K_lr, first_row, n_rows, st);
  if (kb && !mb) return launch_r<BF16Elem, F32Elem>(p, pl, K, A, K_lr, first_row, n_rows, st);
  if (!kb && mb) return launch_r<F32Elem, BF16Elem>(p, pl, K, A, K_lr, first_row, n_rows, st);
  return launch_r<F32Elem, F32Elem>(p, pl, K, A, K_lr, first_row, n_rows, st);
}

// A completed group leaves the rolling buffer (Sec. 3.4.1): the first G rows of every
// (b, kv head)'s buffer become cache rows N .. N+G-1.  16 bytes per lane, one workgroup
// per problem (G*d elements of K and of V: a few KiB).
__global__ __launch_bounds__(256) void append_rows_kernel(const uint4* __restrict__ rb_K,
                                                          const uint4* __restrict__ rb_V,
                                                          uint4* __restrict__ K, uint4* __restrict__ V,
                                                          size_t rb_stride16, size_t cache_stride16,
                                                          size_t dst_off16, int n16) {
  const size_t p = blockIdx.x;
  for (int i = threadIdx.x; i < n16; i += blockDim.x) {
    K[p * cache_stride16 + dst_off16 + i] = rb_K[p * rb_stride16 + i];
    V[p * cache_stride16 + dst_off16 + i] = rb_V[p * rb_stride16 + i];
  }
}

hipError_t launch_append_rows(const kvs_params& p, const Plan& pl, const RollingBuffer& rb,
                              void* K, void* V, hipStream_t st) {
  const size_t row16 = (size_t)p.head_dim * (p.kv_dtype == KVS_BF16 ? 2 : 4) / 16;  // 16-byte pieces per row
  hipLaunchKernelGGL(append_rows_kernel, dim3(pl.problems), dim3(256), 0, st, (const uint4*)rb.K,
                     (const uint4*)rb.V, (uint4*)K, (uint4*)V, (size_t)rb.capacity * row16,
                     (size_t)pl.ctx_rows * row16, (size_t)p.ctx_len * row16,
                     (int)(p.group_size * row16));
  return hipGetLastError();
}

}  // namespace kvs
