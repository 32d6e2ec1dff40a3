// Device-side helpers shared by the gfx950 kernels: 128-bit vector access for float32 and
// bfloat16 storage, wave64 reductions, and launch utilities.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tempo.h"

namespace tempo {

constexpr int kWave = 64;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// Round two floats to bfloat16 (nearest even, hardware v_cvt_pk_bf16_f32) and pack lo|hi<<16.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return as_f32(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return as_f32(w & 0xFFFF0000u); }
// Value a float takes after a round trip through bfloat16 storage.
__device__ __forceinline__ float round_bf16(float v) {
  return as_f32(pack_bf16(v, 0.0f) << 16);
}

// Storage traits.  A "chunk" is 8 consecutive elements: one 16-byte access for bfloat16, two
// for float32.  All chunk accesses need 16-byte (bf16) / 32-byte-pair (f32) aligned addresses,
// which holds when the base pointer is 16-byte aligned and the element offset is a multiple
// of 8.
template <typename T>
struct Store;

template <>
struct Store<float> {
  static constexpr int kBytes = 4;
  __device__ static __forceinline__ void load8(const float* p, float (&v)[8]) {
    const f32x4 a = *reinterpret_cast<const f32x4*>(p);
    const f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  __device__ static __forceinline__ void store8(float* p, const float (&v)[8]) {
    f32x4 a = {v[0], v[1], v[2], v[3]};
    f32x4 b = {v[4], v[5], v[6], v[7]};
    *reinterpret_cast<f32x4*>(p) = a;
    *reinterpret_cast<f32x4*>(p + 4) = b;
  }
  __device__ static __forceinline__ float load1(const float* p) { return *p; }
  __device__ static __forceinline__ void store1(float* p, float v) { *p = v; }
  __device__ static __forceinline__ float round(float v) { return v; }
};

template <>
struct Store<bf16_t> {
  static constexpr int kBytes = 2;
  __device__ static __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
    const u32x4 w = *reinterpret_cast<const u32x4*>(p);
    v[0] = bf16_lo(w.x); v[1] = bf16_hi(w.x);
    v[2] = bf16_lo(w.y); v[3] = bf16_hi(w.y);
    v[4] = bf16_lo(w.z); v[5] = bf16_hi(w.z);
    v[6] = bf16_lo(w.w); v[7] = bf16_hi(w.w);
  }
  __device__ static __forceinline__ void store8(bf16_t* p, const float (&v)[8]) {
    u32x4 w = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]),
               pack_bf16(v[6], v[7])};
    *reinterpret_cast<u32x4*>(p) = w;
  }
  __device__ static __forceinline__ float load1(const bf16_t* p) {
    return as_f32(static_cast<uint32_t>(p->bits) << 16);
  }
  __device__ static __forceinline__ void store1(bf16_t* p, float v) {
    p->bits = static_cast<uint16_t>(pack_bf16(v, 0.0f) & 0xFFFFu);
  }
  __device__ static __forceinline__ float round(float v) { return round_bf16(v); }
};

// Guarded chunk access: elements at or beyond `n_left` (counted from p) are absent.
template <typename T>
__device__ __forceinline__ void load8_guarded(const T* p, int64_t n_left, float (&v)[8], float fill) {
  if (n_left >= 8) {
    Store<T>::load8(p, v);
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (i < n_left) ? Store<T>::load1(p + i) : fill;
  }
}
template <typename T>
__device__ __forceinline__ void store8_guarded(T* p, int64_t n_left, const float (&v)[8]) {
  if (n_left >= 8) {
    Store<T>::store8(p, v);
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (i < n_left) Store<T>::store1(p + i, v[i]);
  }
}

// Butterfly reductions over groups of LANES consecutive lanes of a wave (LANES a power of
// two <= 64); every lane of the group ends with the result.
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int m = LANES / 2; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}
template <int LANES>
__device__ __forceinline__ float group_max(float v) {
#pragma unroll
  for (int m = LANES / 2; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
  return v;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace tempo
