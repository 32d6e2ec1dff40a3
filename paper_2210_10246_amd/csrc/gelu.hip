// In-place GELU for gfx950: forward writes y and a 1-bit "side of the minimum" mask, backward
// evaluates GELU'(GELU*^-1(y, m)) from the stored output (Sec. 3.1; App. E.1 eq. 1-2; App. F.1).
//
// Both kernels are streaming: every lane owns chunks of 8 consecutive elements (one 16-byte
// access in bf16, two in f32); the 8 mask bits of a chunk are merged over 4 adjacent lanes so
// the mask is written and read as whole 32-bit words.  The piecewise-cubic tables live in LDS
// (one 16-byte row per piece, fetched with a single ds_read_b128 per element).
#include "tempo_device.h"
#include "tempo_host.h"

#define TEMPO_TABLE_QUAL __device__
#include "gelu_tables.inc"

namespace tempo {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 2;  // chunks in flight per lane and loop trip

template <int KIND>
struct GeluConst;
template <>
struct GeluConst<TEMPO_GELU_ERF> {
  static constexpr uint32_t xstar = TEMPO_GELU_ERF_XSTAR_F32;
  static constexpr uint32_t ys_hi = TEMPO_GELU_ERF_YSTAR_HI;
  static constexpr uint32_t ys_lo = TEMPO_GELU_ERF_YSTAR_LO;
  __device__ static const uint32_t (*bwd_table())[4] { return tempo_gelu_bwd_table_erf; }
};
template <>
struct GeluConst<TEMPO_GELU_TANH> {
  static constexpr uint32_t xstar = TEMPO_GELU_TANH_XSTAR_F32;
  static constexpr uint32_t ys_hi = TEMPO_GELU_TANH_YSTAR_HI;
  static constexpr uint32_t ys_lo = TEMPO_GELU_TANH_YSTAR_LO;
  __device__ static const uint32_t (*bwd_table())[4] { return tempo_gelu_bwd_table_tanh; }
};

__device__ __forceinline__ float cubic(const f32x4 c, float z) {
  return fmaf(fmaf(fmaf(c.w, z, c.z), z, c.y), z, c.x);
}

// GELU(x), erf form: cubic pieces of width 1/16 on [-8, 8); x outside is x (right) or -0.
__device__ __forceinline__ float gelu_erf_value(float x, const f32x4* tab) {
  const float t = x * static_cast<float>(TEMPO_GELU_FWD_PER_UNIT);
  const float lo = TEMPO_GELU_FWD_LO * TEMPO_GELU_FWD_PER_UNIT;
  const float hi = TEMPO_GELU_FWD_HI * TEMPO_GELU_FWD_PER_UNIT - 0.0078125f;
  const float fl = floorf(fminf(fmaxf(t, lo), hi));
  const float z = t - fl;  // exact inside the table range; NaN stays NaN
  const int idx = static_cast<int>(fl) - static_cast<int>(lo);
  float y = cubic(tab[idx], z);
  y = (x >= TEMPO_GELU_FWD_HI) ? x : y;
  y = (x < TEMPO_GELU_FWD_LO) ? -0.0f : y;
  return y;
}

// GELU(x), tanh form written as x * sigmoid(2u): no cancellation on the left tail.
__device__ __forceinline__ float gelu_tanh_value(float x) {
  const float k = 0.7978845608028654f;      // sqrt(2/pi)
  const float ka = 0.7978845608028654f * 0.044715f;
  const float m2log2e = -2.0f * 1.4426950408889634f;
  const float inner = fmaf(x * x, ka, k);
  const float e = __builtin_amdgcn_exp2f(m2log2e * x * inner);  // exp(-2u)
  return x * __builtin_amdgcn_rcpf(1.0f + e);
}

// d(y, m) = GELU'(GELU*^-1(y, m)).
template <int KIND>
__device__ __forceinline__ float gelu_composite(float y, bool right, const f32x4* tab) {
  const float ys_hi = as_f32(GeluConst<KIND>::ys_hi);
  const float ys_lo = as_f32(GeluConst<KIND>::ys_lo);
  const float t = fmaxf((y - ys_hi) - ys_lo, 0.0f);
  const float s = __builtin_amdgcn_sqrtf(t);
  const float c = right ? static_cast<float>(TEMPO_GELU_CR) : static_cast<float>(TEMPO_GELU_CL);
  const float umax = right ? (TEMPO_GELU_NR - 0.00001f) : (TEMPO_GELU_NL - 0.00001f);
  const int base = right ? 0 : TEMPO_GELU_NR;
  const float u = fminf(s * c, umax);
  const float fl = floorf(u);
  const float z_s = u - fl;
  const int idx_s = static_cast<int>(fl) + base;
  // left tail: quarter-octaves of -y below 2^TAIL_TOP_EXP
  const float ny = -y;
  const uint32_t bits = as_u32(ny);
  constexpr int kRem = 23 - TEMPO_GELU_TAIL_SUB_BITS;
  constexpr uint32_t kTop =
      ((127u + TEMPO_GELU_TAIL_TOP_EXP - 1u) << TEMPO_GELU_TAIL_SUB_BITS) |
      ((1u << TEMPO_GELU_TAIL_SUB_BITS) - 1u);
  const uint32_t it = min(kTop - (bits >> kRem), static_cast<uint32_t>(TEMPO_GELU_NT - 1));
  const float z_t = static_cast<float>(bits & ((1u << kRem) - 1u));
  const bool tail = !right && (ny < 0.0625f);
  static_assert(TEMPO_GELU_TAIL_TOP_EXP == -4, "tail threshold literal");
  const int idx = tail ? static_cast<int>(it) + (TEMPO_GELU_NR + TEMPO_GELU_NL) : idx_s;
  const float z = tail ? z_t : z_s;
  float d = cubic(tab[idx], z);
  return (y != y) ? y : d;
}

template <int ROWS>
__device__ __forceinline__ void load_table(f32x4* lds, const uint32_t (*src)[4]) {
  for (int i = threadIdx.x; i < ROWS; i += kThreads) {
    const u32x4 r = *reinterpret_cast<const u32x4*>(src[i]);
    f32x4 f = {as_f32(r.x), as_f32(r.y), as_f32(r.z), as_f32(r.w)};
    lds[i] = f;
  }
  __syncthreads();
}

// Merge the 8-bit chunk masks of 4 adjacent lanes into the 32-bit word they share.
__device__ __forceinline__ uint32_t merge_quad_bytes(uint32_t byte, int lane_in_quad) {
  uint32_t w = byte << (8 * lane_in_quad);
  w |= __shfl_xor(w, 1, kWave);
  w |= __shfl_xor(w, 2, kWave);
  return w;
}

template <typename T, int KIND>
__global__ __launch_bounds__(kThreads) void gelu_fwd_kernel(const T* x, T* y,  // may alias
                                                            uint32_t* __restrict__ mask,
                                                            int64_t n) {
  __shared__ f32x4 tab[KIND == TEMPO_GELU_ERF ? TEMPO_GELU_FWD_ROWS : 1];
  if (KIND == TEMPO_GELU_ERF) load_table<TEMPO_GELU_FWD_ROWS>(tab, tempo_gelu_fwd_table_erf);
  const float xstar = as_f32(GeluConst<KIND>::xstar);
  const int64_t n_chunks = (n + 7) >> 3;
  const int64_t threads = static_cast<int64_t>(gridDim.x) * kThreads;
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t gtid = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  // trip count is uniform over a wave: lanes past the end run with everything guarded off
  for (int64_t q0 = gtid; q0 - lane < n_chunks; q0 += threads * kUnroll) {
    float v[kUnroll][8];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t q = q0 + u * threads;
      const int64_t left = n - q * 8;
      if (left > 0) {
        load8_guarded<T>(x + q * 8, left, v[u], -1.0e30f);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[u][i] = -1.0e30f;
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t q = q0 + u * threads;
      const int64_t left = n - q * 8;
      uint32_t byte = 0;
      float r[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float xv = v[u][i];
        byte |= (xv >= xstar ? 1u : 0u) << i;
        r[i] = (KIND == TEMPO_GELU_ERF) ? gelu_erf_value(xv, tab) : gelu_tanh_value(xv);
      }
      const uint32_t word = merge_quad_bytes(byte, lane & 3);
      if (left > 0) store8_guarded<T>(y + q * 8, left, r);
      if ((lane & 3) == 0 && left > 0) mask[q >> 2] = word;
    }
  }
}

template <typename T, int KIND>
__global__ __launch_bounds__(kThreads) void gelu_bwd_kernel(const T* dy,  // may alias dx
                                                            const T* __restrict__ y,
                                                            const uint32_t* __restrict__ mask,
                                                            T* dx, int64_t n) {
  __shared__ f32x4 tab[TEMPO_GELU_BWD_ROWS];
  load_table<TEMPO_GELU_BWD_ROWS>(tab, GeluConst<KIND>::bwd_table());
  const int64_t n_chunks = (n + 7) >> 3;
  const int64_t threads = static_cast<int64_t>(gridDim.x) * kThreads;
  const int64_t gtid = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  for (int64_t q0 = gtid; q0 < n_chunks; q0 += threads * kUnroll) {
    float g[kUnroll][8], o[kUnroll][8];
    uint32_t w[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t q = q0 + u * threads;
      const int64_t left = n - q * 8;
      w[u] = 0;
      if (left > 0) {
        load8_guarded<T>(dy + q * 8, left, g[u], 0.0f);
        load8_guarded<T>(y + q * 8, left, o[u], 0.0f);
        w[u] = mask[q >> 2];
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t q = q0 + u * threads;
      const int64_t left = n - q * 8;
      if (left <= 0) continue;
      const uint32_t byte = w[u] >> (8 * static_cast<int>(q & 3));
      float r[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const bool right = (byte >> i) & 1u;
        r[i] = g[u][i] * gelu_composite<KIND>(o[u][i], right, tab);
      }
      store8_guarded<T>(dx + q * 8, left, r);
    }
  }
}

int stream_grid(int64_t n, int blocks_per_cu) {
  const int64_t n_chunks = (n + 7) / 8;
  const int64_t want = (n_chunks + kThreads * kUnroll - 1) / (kThreads * kUnroll);
  const int64_t cap = static_cast<int64_t>(compute_units()) * blocks_per_cu;
  return static_cast<int>(want < cap ? want : cap);
}

}  // namespace

tempo_status launch_gelu_fwd(const void* x, void* y, uint32_t* mask, int64_t n, tempo_dtype dt,
                             tempo_gelu_kind kind, hipStream_t st) {
  const int grid = stream_grid(n, tune_get(kTuneGeluFwdBlocksPerCu));
#define TEMPO_LAUNCH(T, K)                                                                   \
  hipLaunchKernelGGL((gelu_fwd_kernel<T, K>), dim3(grid), dim3(kThreads), 0, st,             \
                     static_cast<const T*>(x), static_cast<T*>(y), mask, n)
  if (dt == TEMPO_F32) {
    if (kind == TEMPO_GELU_ERF) TEMPO_LAUNCH(float, TEMPO_GELU_ERF);
    else TEMPO_LAUNCH(float, TEMPO_GELU_TANH);
  } else {
    if (kind == TEMPO_GELU_ERF) TEMPO_LAUNCH(bf16_t, TEMPO_GELU_ERF);
    else TEMPO_LAUNCH(bf16_t, TEMPO_GELU_TANH);
  }
#undef TEMPO_LAUNCH
  return launch_status();
}

tempo_status launch_gelu_bwd(const void* dy, const void* y, const uint32_t* mask, void* dx,
                             int64_t n, tempo_dtype dt, tempo_gelu_kind kind, hipStream_t st) {
  const int grid = stream_grid(n, tune_get(kTuneGeluBwdBlocksPerCu));
#define TEMPO_LAUNCH(T, K)                                                                   \
  hipLaunchKernelGGL((gelu_bwd_kernel<T, K>), dim3(grid), dim3(kThreads), 0, st,             \
                     static_cast<const T*>(dy), static_cast<const T*>(y), mask,              \
                     static_cast<T*>(dx), n)
  if (dt == TEMPO_F32) {
    if (kind == TEMPO_GELU_ERF) TEMPO_LAUNCH(float, TEMPO_GELU_ERF);
    else TEMPO_LAUNCH(float, TEMPO_GELU_TANH);
  } else {
    if (kind == TEMPO_GELU_ERF) TEMPO_LAUNCH(bf16_t, TEMPO_GELU_ERF);
    else TEMPO_LAUNCH(bf16_t, TEMPO_GELU_TANH);
  }
#undef TEMPO_LAUNCH
  return launch_status();
}

}  // namespace tempo
