// Device-side helpers shared by the kvswap_hip kernels (gfx950, wave64 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvs {

constexpr int kWave = 64;

// A pointer to device (global) memory whose address space the compiler can no longer see -
// because it was read back from a structure in memory - marked as such again: without this
// every access through it becomes a flat access, which also waits on the LDS counter.
template <class T>
__device__ __forceinline__ T* as_global(T* p) {
  typedef T __attribute__((address_space(1))) * global_ptr;
  global_ptr g = (global_ptr)p;
  asm volatile("" : "+s"(g));  // (uniform pointers only; keeps the two casts from cancelling)
  return (T*)g;
}

// ---- storage element traits ------------------------------------------------
// A lane always moves 16 bytes per load: 4 fp32, 8 bf16 or 16 fp8 values.
struct F32Elem {
  using storage = float;
  static constexpr int kBytes = 4;
  static constexpr int kPerLane = 4;
};
struct BF16Elem {
  using storage = uint16_t;
  static constexpr int kBytes = 2;
  static constexpr int kPerLane = 8;
};

// 8-bit float, OCP E4M3 (finite-only): metadata only.  gfx950's packed conversions
// implement exactly this format (checked on the device for all 256 codes).
struct FP8Elem {
  using storage = uint8_t;
  static constexpr int kBytes = 1;
  static constexpr int kPerLane = 16;
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}

// fp32 -> bf16 bits, round-to-nearest-even (finite inputs).
__device__ __forceinline__ uint16_t float_to_bf16_bits(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename E>
__device__ __forceinline__ void unpack16(const uint4& v, float (&f)[E::kPerLane]);

template <>
__device__ __forceinline__ void unpack16<F32Elem>(const uint4& v, float (&f)[4]) {
  f[0] = __uint_as_float(v.x);
  f[1] = __uint_as_float(v.y);
  f[2] = __uint_as_float(v.z);
  f[3] = __uint_as_float(v.w);
}

template <>
__device__ __forceinline__ void unpack16<BF16Elem>(const uint4& v, float (&f)[8]) {
  // element 2i is the low half of dword i, element 2i+1 the high half
  f[0] = __uint_as_float(v.x << 16);
  f[1] = __uint_as_float(v.x & 0xFFFF0000u);
  f[2] = __uint_as_float(v.y << 16);
  f[3] = __uint_as_float(v.y & 0xFFFF0000u);
  f[4] = __uint_as_float(v.z << 16);
  f[5] = __uint_as_float(v.z & 0xFFFF0000u);
  f[6] = __uint_as_float(v.w << 16);
  f[7] = __uint_as_float(v.w & 0xFFFF0000u);
}

template <>
__device__ __forceinline__ void unpack16<FP8Elem>(const uint4& v, float (&f)[16]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {  // bytes 0,1 and 2,3 of each dword, two values per conversion
    const auto lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);
    const auto hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);
    f[4 * i + 0] = lo[0];
    f[4 * i + 1] = lo[1];
    f[4 * i + 2] = hi[0];
    f[4 * i + 3] = hi[1];
  }
}

// fp32 -> E4M3 code, round-to-nearest-even, magnitudes beyond 448 saturate (the
// hardware conversion would turn them into NaN).
__device__ __forceinline__ uint8_t float_to_fp8_e4m3(float x) {
  const float c = fminf(fmaxf(x, -448.0f), 448.0f);
  return (uint8_t)(__builtin_amdgcn_cvt_pk_fp8_f32(c, c, 0, false) & 0xFF);
}

// a.lo*b.lo + a.hi*b.hi + c over two packed bf16 pairs, products and sum in fp32.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

// Sum over `count` (<= kMaxSummed) elements base[first + j * stride] as fp32, in two halves:
// request() issues all the loads, sum() adds them up.  Written as a loop that adds as it
// goes, every load would be waited for on its own, one memory latency after the other; and
// with other requests placed between the two halves this latency overlaps theirs.
constexpr int kMaxSummed = 8;
struct StridedSum {
  uint32_t raw[kMaxSummed];
  __device__ __forceinline__ void request(const void* base, int is_bf16, size_t first, size_t stride, int count) {
    if (is_bf16) {  // uniform
#pragma unroll
      for (int j = 0; j < kMaxSummed; ++j)
        raw[j] = ((const uint16_t*)base)[first + (size_t)min(j, count - 1) * stride];
    } else {
#pragma unroll
      for (int j = 0; j < kMaxSummed; ++j)
        raw[j] = ((const uint32_t*)base)[first + (size_t)min(j, count - 1) * stride];
    }
  }
  __device__ __forceinline__ float sum(int is_bf16, int count) const {
    float total = 0.f;
#pragma unroll
    for (int j = 0; j < kMaxSummed; ++j) {
      const float v = is_bf16 ? bf16_bits_to_float(raw[j]) : __uint_as_float(raw[j]);
      total += (j < count) ? v : 0.f;
    }
    return total;
  }
};

// ---- workgroup barrier for LDS traffic only ----------------------------------------------
// __syncthreads() also waits for every outstanding global load and store of the wave,
// which serialises the memory latency the kernels work to overlap (prefetched tiles,
// scattered result stores).  Wherever only LDS contents have to be ordered, this barrier
// is used instead: it waits for the wave's LDS operations alone.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- cross-lane exchange -----------------------------------------------------
// xor_lane<M>(x): value of x held by lane (lane ^ M).  DPP where the ISA has a
// matching pattern (no LDS traffic), the LDS crossbar otherwise.
template <int MASK>
__device__ __forceinline__ float xor_lane(float x) {
  static_assert(MASK == 1 || MASK == 2 || MASK == 4 || MASK == 8 || MASK == 16 || MASK == 32,
                "power-of-two lane mask below 64");
  const int xi = __float_as_int(x);
  int r;
  if constexpr (MASK == 1) {
    r = __builtin_amdgcn_update_dpp(xi, xi, 0xB1, 0xF, 0xF, false);  // quad_perm:[1,0,3,2]
  } else if constexpr (MASK == 2) {
    r = __builtin_amdgcn_update_dpp(xi, xi, 0x4E, 0xF, 0xF, false);  // quad_perm:[2,3,0,1]
  } else if constexpr (MASK == 8) {
    r = __builtin_amdgcn_update_dpp(xi, xi, 0x128, 0xF, 0xF, false); // row_ror:8 == xor 8 in a row of 16
  } else if constexpr (MASK == 4 || MASK == 16) {
    r = __builtin_amdgcn_ds_swizzle(xi, (MASK << 10) | 0x1F);        // bit mode: and 0x1f, or 0, xor MASK
  } else {
    r = __shfl_xor(xi, 32, kWave);
  }
  return __int_as_float(r);
}

struct OpSum {
  static __device__ __forceinline__ float apply(float a, float b) { return a + b; }
};
struct OpMax {
  static __device__ __forceinline__ float apply(float a, float b) { return fmaxf(a, b); }
};

// All-reduce over the lanes whose ids differ only in the bits LO <= bit-mask < HI
// (LO, HI powers of two; LO == HI is a no-op).  Every participating lane ends
// with the combined value.
template <typename Op, int LO, int HI>
__device__ __forceinline__ float allreduce_lanes(float x) {
  if constexpr (LO < HI) {
    if constexpr (LO == 4 && HI >= 16) {
      // strides 4 and 8 inside a row of 16: two rotations cover {l, l+4, l+8, l+12}
      const int x0 = __float_as_int(x);
      x = Op::apply(x, __int_as_float(__builtin_amdgcn_update_dpp(x0, x0, 0x124, 0xF, 0xF, false)));  // row_ror:4
      const int x1 = __float_as_int(x);
      x = Op::apply(x, __int_as_float(__builtin_amdgcn_update_dpp(x1, x1, 0x128, 0xF, 0xF, false)));  // row_ror:8
      return allreduce_lanes<Op, 16, HI>(x);
    } else {
      x = Op::apply(x, xor_lane<LO>(x));
      return allreduce_lanes<Op, LO * 2, HI>(x);
    }
  }
  return x;
}

// ---- handing results to another workgroup ----------------------------------------------
// The streaming kernels finish a problem in whichever workgroup arrives last at a
// per-problem counter.  Workgroups of one problem run on different XCDs, whose L2
// caches are not coherent with each other, and a device-scope fence costs a sweep of
// the whole L2 per workgroup (measured: it multiplies the kernel time).  So the few
// values that cross workgroups are moved with device-scope accesses instead, which go
// past the non-coherent cache levels: the publisher writes them with device-scope
// stores (and device-scope atomics), waits until the memory system has acknowledged
// them, and only then bumps the arrival counter; the last workgroup reads them with
// device-scope loads.  No cache is flushed or invalidated, and nobody ever waits on
// another workgroup.

__device__ __forceinline__ void publish_store(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void publish_store(int* p, int v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float load_published(const float* p) {
  return __hip_atomic_load(const_cast<float*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ int load_published(const int* p) {
  return __hip_atomic_load(const_cast<int*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Every lane calls this after its last publish_store / device-scope atomic: all of
// this lane's outstanding memory operations have completed, then a workgroup barrier.
// After it, one lane may bump the arrival counter.
// The wait and the barrier are hardware ordering; towards the compiler they are no memory
// barriers for global memory, so a compiler-only fence on either side keeps it from moving
// a publish_store below the wait or a later access above it (no instruction is emitted).
__device__ __forceinline__ void publish_complete_and_barrier() {
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0) expcnt(0) lgkmcnt(0)
  __atomic_signal_fence(__ATOMIC_SEQ_CST);
  lds_barrier();
}

// Placed between learning (from an arrival counter or a flag) that another workgroup's
// values are published and the first load_published of them: keeps the compiler from
// hoisting those loads above the point where the arrival is known (no instruction is
// emitted; the hardware returns the loads of a wave in order).
__device__ __forceinline__ void consume_fence() { __atomic_signal_fence(__ATOMIC_SEQ_CST); }

// A 16-byte global load, optionally with the non-temporal hint (data that is read once).
typedef uint32_t kvs_u32x4 __attribute__((ext_vector_type(4)));
template <bool STREAM>
__device__ __forceinline__ uint4 load16(const void* p) {
  if constexpr (STREAM) {
    const kvs_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const kvs_u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
  } else {
    return *reinterpret_cast<const uint4*>(p);
  }
}

}  // namespace kvs
