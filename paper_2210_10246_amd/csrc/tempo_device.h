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

// Storage traits.  All bulk traffic moves in 16-byte "pieces": 8 consecutive bfloat16 or 4
// consecutive float32 elements.  Kernels are laid out so that the 64 lanes of a wave touch 64
// adjacent pieces with one instruction (1 KiB contiguous): a lane that instead owned 32
// adjacent bytes of float32 (two accesses, each strided by 32 bytes across the wave) was
// measured at 4.0 TB/s where the contiguous form reaches 6.2 TB/s.
// A piece needs a 16-byte aligned address: base pointers are checked on the host and element
// offsets are multiples of the piece length.
template <typename T>
struct Store;

template <>
struct Store<float> {
  static constexpr int kVec = 4;  // elements per piece
  __device__ static __forceinline__ float load1(const float* p) { return *p; }
  __device__ static __forceinline__ void store1(float* p, float v) { *p = v; }
  __device__ static __forceinline__ float round(float v) { return v; }
  __device__ static __forceinline__ void unpack(const u32x4 w, float (&v)[4]) {
    v[0] = as_f32(w.x); v[1] = as_f32(w.y); v[2] = as_f32(w.z); v[3] = as_f32(w.w);
  }
  __device__ static __forceinline__ u32x4 pack(const float (&v)[4]) {
    return u32x4{as_u32(v[0]), as_u32(v[1]), as_u32(v[2]), as_u32(v[3])};
  }
  __device__ static __forceinline__ u32x4 neg_inf_piece() {
    return u32x4{0xFF800000u, 0xFF800000u, 0xFF800000u, 0xFF800000u};
  }
};

template <>
struct Store<bf16_t> {
  static constexpr int kVec = 8;
  __device__ static __forceinline__ float load1(const bf16_t* p) {
    return as_f32(static_cast<uint32_t>(p->bits) << 16);
  }
  __device__ static __forceinline__ void store1(bf16_t* p, float v) {
    p->bits = static_cast<uint16_t>(pack_bf16(v, 0.0f) & 0xFFFFu);
  }
  __device__ static __forceinline__ float round(float v) { return round_bf16(v); }
  __device__ static __forceinline__ void unpack(const u32x4 w, float (&v)[8]) {
    v[0] = bf16_lo(w.x); v[1] = bf16_hi(w.x);
    v[2] = bf16_lo(w.y); v[3] = bf16_hi(w.y);
    v[4] = bf16_lo(w.z); v[5] = bf16_hi(w.z);
    v[6] = bf16_lo(w.w); v[7] = bf16_hi(w.w);
  }
  __device__ static __forceinline__ u32x4 pack(const float (&v)[8]) {
    return u32x4{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]),
                 pack_bf16(v[6], v[7])};
  }
  __device__ static __forceinline__ u32x4 neg_inf_piece() {
    return u32x4{0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u, 0xFF80FF80u};
  }
};

// Streaming (non-temporal) 16-byte accesses for data that is touched exactly once.
__device__ __forceinline__ u32x4 ldg_stream(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
__device__ __forceinline__ void stg_stream(void* p, u32x4 v) {
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
}
template <typename T>
__device__ __forceinline__ void load_piece(const T* p, float (&v)[Store<T>::kVec]) {
  Store<T>::unpack(ldg_stream(p), v);
}
template <typename T>
__device__ __forceinline__ void store_piece(T* p, const float (&v)[Store<T>::kVec]) {
  stg_stream(p, Store<T>::pack(v));
}
// float32 parameters (gamma, beta, LDS tables): plain cached accesses of kVec floats
template <int V>
__device__ __forceinline__ void load_floats(const float* p, float (&v)[V]) {
  static_assert(V == 4 || V == 8, "piece length");
  const f32x4 a = *reinterpret_cast<const f32x4*>(p);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
  if constexpr (V == 8) {
    const f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
}
template <int V>
__device__ __forceinline__ void store_floats(float* p, const float (&v)[V]) {
  static_assert(V == 4 || V == 8, "piece length");
  *reinterpret_cast<f32x4*>(p) = f32x4{v[0], v[1], v[2], v[3]};
  if constexpr (V == 8) *reinterpret_cast<f32x4*>(p + 4) = f32x4{v[4], v[5], v[6], v[7]};
}

// Raw (still packed) piece, so rows fetched ahead cost 4 registers per piece.
template <typename T>
struct Raw {
  u32x4 a;
  __device__ __forceinline__ void load(const T* p) { a = ldg_stream(p); }
  __device__ __forceinline__ void unpack(float (&v)[Store<T>::kVec]) const {
    Store<T>::unpack(a, v);
  }
};

// Guarded piece access: elements at or beyond `n_left` (counted from p) are absent.
template <typename T>
__device__ __forceinline__ void load_piece_guarded(const T* p, int64_t n_left,
                                                   float (&v)[Store<T>::kVec], float fill) {
  constexpr int V = Store<T>::kVec;
  if (n_left >= V) {
    load_piece<T>(p, v);
  } else {
#pragma unroll
    for (int i = 0; i < V; ++i) v[i] = (i < n_left) ? Store<T>::load1(p + i) : fill;
  }
}
template <typename T>
__device__ __forceinline__ void store_piece_guarded(T* p, int64_t n_left,
                                                    const float (&v)[Store<T>::kVec]) {
  constexpr int V = Store<T>::kVec;
  if (n_left >= V) {
    store_piece<T>(p, v);
  } else {
#pragma unroll
    for (int i = 0; i < V; ++i)
      if (i < n_left) Store<T>::store1(p + i, v[i]);
  }
}

// Cross-lane moves inside a row of 16 lanes through DPP (data-parallel primitives: the source
// lane is selected by the instruction itself, no LDS round trip).  The four controls below
// pair every lane with lane^1, lane^2 (quad permutes), then mirror 8 and 16 lanes, which for
// values already equal inside a quad / half row acts like lane^4 and lane^8.
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // row_half_mirror
constexpr int kDppMirror = 0x140;      // row_mirror
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return static_cast<uint32_t>(
      __builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return as_f32(dpp_u32<CTRL>(as_u32(v)));
}

// Butterfly reductions over groups of LANES consecutive lanes of a wave (LANES a power of
// two, 4 <= LANES <= 64, groups aligned to LANES); every lane of the group ends with the
// result.  Steps inside a 16-lane row use DPP, the steps across rows go through ds_bpermute.
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(LANES >= 4 && LANES <= 64, "group size");
  v += dpp_f32<kDppXor1>(v);
  v += dpp_f32<kDppXor2>(v);
  if (LANES >= 8) v += dpp_f32<kDppHalfMirror>(v);
  if (LANES >= 16) v += dpp_f32<kDppMirror>(v);
  if (LANES >= 32) v += __shfl_xor(v, 16, kWave);
  if (LANES >= 64) v += __shfl_xor(v, 32, kWave);
  return v;
}
template <int LANES>
__device__ __forceinline__ float group_max(float v) {
  static_assert(LANES >= 4 && LANES <= 64, "group size");
  v = fmaxf(v, dpp_f32<kDppXor1>(v));
  v = fmaxf(v, dpp_f32<kDppXor2>(v));
  if (LANES >= 8) v = fmaxf(v, dpp_f32<kDppHalfMirror>(v));
  if (LANES >= 16) v = fmaxf(v, dpp_f32<kDppMirror>(v));
  if (LANES >= 32) v = fmaxf(v, __shfl_xor(v, 16, kWave));
  if (LANES >= 64) v = fmaxf(v, __shfl_xor(v, 32, kWave));
  return v;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits until the wave's
// outstanding global loads and stores have completed (s_waitcnt vmcnt(0)): behind a batch of
// stores that is microseconds, and in a loop it also waits for the rows fetched ahead.  No
// kernel here passes data between the waves of a workgroup through global memory.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Row reductions for rows owned by LANES consecutive threads of a workgroup.  A row inside
// one wave: butterflies.  A row spread over LANES/64 waves: butterfly per wave, then one
// exchange through `slots` (one entry per wave of the workgroup) behind a workgroup barrier, so
// every thread of the workgroup has to make the call; consecutive calls must alternate between
// two slot arrays (a fast wave may already write its next value while a slow one still reads).
// Every lane of the row ends with the same result.
template <int LANES, bool MAX>
__device__ __forceinline__ float row_reduce(float v, float* slots) {
  if constexpr (LANES <= kWave) {
    return MAX ? group_max<LANES>(v) : group_sum<LANES>(v);
  } else {
    v = MAX ? group_max<kWave>(v) : group_sum<kWave>(v);
    if ((threadIdx.x & (kWave - 1)) == 0) slots[threadIdx.x / kWave] = v;
    lds_barrier();
    constexpr int W = LANES / kWave;
    const int w0 = (threadIdx.x / LANES) * W;
    float r = slots[w0];
#pragma unroll
    for (int k = 1; k < W; ++k) r = MAX ? fmaxf(r, slots[w0 + k]) : r + slots[w0 + k];
    return r;
  }
}

// Two sums at once (one barrier for both); slots holds two floats per wave of the workgroup.
template <int LANES>
__device__ __forceinline__ void row_sum2(float& a, float& b, float2* slots) {
  if constexpr (LANES <= kWave) {
    a = group_sum<LANES>(a);
    b = group_sum<LANES>(b);
  } else {
    a = group_sum<kWave>(a);
    b = group_sum<kWave>(b);
    if ((threadIdx.x & (kWave - 1)) == 0) slots[threadIdx.x / kWave] = make_float2(a, b);
    lds_barrier();
    constexpr int W = LANES / kWave;
    const int w0 = (threadIdx.x / LANES) * W;
    float2 r = slots[w0];
#pragma unroll
    for (int k = 1; k < W; ++k) {
      r.x += slots[w0 + k].x;
      r.y += slots[w0 + k].y;
    }
    a = r.x;
    b = r.y;
  }
}

// Merge the per-piece mask bits of the lanes that share a 32-bit mask word: 4 lanes with 8 bits
// each (bfloat16 pieces) or 8 lanes with 4 bits each (float32 pieces).  `lane` is the index of
// the lane's piece within its row/tile (only its low bits matter).  Every lane of the sharing
// group returns the whole word.
template <int V>
__device__ __forceinline__ uint32_t merge_mask_word(uint32_t bits, int lane) {
  static_assert(V == 4 || V == 8, "piece length");
  constexpr int kLanes = 32 / V;
  uint32_t w = bits << (V * (lane & (kLanes - 1)));
  w |= dpp_u32<kDppXor1>(w);
  w |= dpp_u32<kDppXor2>(w);
  if (V == 4) w |= dpp_u32<kDppHalfMirror>(w);
  return w;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace tempo
