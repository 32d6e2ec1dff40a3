// In-place GELU for gfx950: forward writes y and a 1-bit "side of the minimum" mask, backward
// evaluates GELU'(GELU*^-1(y, m)) from the stored output (Sec. 3.1; App. E.1 eq. 1-2; App. F.1).
// The same kernels serve SiLU, x * sigmoid(x), which also has a single minimum: the general
// recipe for in-place elementwise layers (Sec. 5.1) with another table set.  KIND is
// TEMPO_GELU_ERF, TEMPO_GELU_TANH or kActSilu.
//
// Both kernels are streaming: every lane owns 16-byte pieces (8 bf16 or 4 f32 elements); the
// mask bits of a piece are merged over the 4 (bf16) or 8 (f32) adjacent lanes that share a
// word, so the mask is written and read as whole 32-bit words.  float32 forward evaluates the
// activation directly (exp2 and rcp), float32 backward piecewise cubics whose coefficient rows
// live in LDS (one ds_read_b128 per element); bfloat16 looks the function value up per bit
// pattern.
#include <type_traits>

#include "tempo_device.h"
#include "tempo_host.h"

#define TEMPO_TABLE_QUAL __device__
#include "gelu_tables.inc"

namespace tempo {
namespace {

template <int KIND>
struct GeluConst;
// Per activation: the minimum (x* as compared in float32, y* split hi + lo), the number of
// right-branch and left-near pieces of the backward table, the rows of that table, and how many
// bf16 patterns lower the left branch's lookup window starts.
#define TEMPO_ACT_CONST(KIND, UPPER, lower)                                                  \
  template <>                                                                                \
  struct GeluConst<KIND> {                                                                   \
    static constexpr uint32_t xstar = TEMPO_GELU_##UPPER##_XSTAR_F32;                        \
    static constexpr uint32_t ys_hi = TEMPO_GELU_##UPPER##_YSTAR_HI;                         \
    static constexpr uint32_t ys_lo = TEMPO_GELU_##UPPER##_YSTAR_LO;                         \
    static constexpr int NR = TEMPO_GELU_##UPPER##_NR;                                       \
    static constexpr int NL = TEMPO_GELU_##UPPER##_NL;                                       \
    static constexpr int kBwdRows = TEMPO_GELU_##UPPER##_BWD_ROWS;                           \
    static constexpr int kLutLeftShift = TEMPO_GELU_##UPPER##_LUT_LEFT_SHIFT;                \
    __device__ static const uint32_t (*bwd_table())[4] { return tempo_gelu_bwd_table_##lower; } \
    __device__ static const uint32_t* lut_fwd() { return tempo_gelu_lut_fwd_##lower; }       \
    __device__ static const uint32_t* lut_bwd() { return tempo_gelu_lut_bwd_##lower; }       \
  };
TEMPO_ACT_CONST(TEMPO_GELU_ERF, ERF, erf)
TEMPO_ACT_CONST(TEMPO_GELU_TANH, TANH, tanh)
TEMPO_ACT_CONST(kActSilu, SILU, silu)
#undef TEMPO_ACT_CONST

__device__ __forceinline__ float cubic(const f32x4 c, float z) {
  return fmaf(fmaf(fmaf(c.w, z, c.z), z, c.y), z, c.x);
}

// GELU(x) = x Phi(x), erf form.  Phi(x) = 1/2 erfc(-x / sqrt 2); for z >= 0,
// erfc(z) = exp(-z^2) erfcx(z), and 1/2 erfcx(z) (1 + z/2) is one polynomial of degree 8 in
// t = 1 / (1 + z/2) (relative error 9e-8 up to |x| = 9; beyond, the exponential has long made
// Phi 0 or 1).  With w = |x| sqrt(log2(e)/2) the exponential is exp2(-w^2).  x < 0 takes the
// small value itself, so the left tail keeps its relative accuracy, and the product with x comes
// last, so the zero at x = 0 is exact.  No table: the kernel needs no LDS.
__device__ __forceinline__ float gelu_erf_value(float x) {
  const float w = fabsf(x) * as_f32(TEMPO_GELU_ERFC_W_SCALE);
  const float t = __builtin_amdgcn_rcpf(fmaf(w, as_f32(TEMPO_GELU_ERFC_T_FACTOR), 1.0f));
  const float u = fmaf(t, as_f32(TEMPO_GELU_ERFC_UA), as_f32(TEMPO_GELU_ERFC_UB));
  static_assert(TEMPO_GELU_ERFC_DEG == 8, "Horner chain below");
  float q = as_f32(TEMPO_GELU_ERFC_Q8);
  q = fmaf(q, u, as_f32(TEMPO_GELU_ERFC_Q7));
  q = fmaf(q, u, as_f32(TEMPO_GELU_ERFC_Q6));
  q = fmaf(q, u, as_f32(TEMPO_GELU_ERFC_Q5));
  q = fmaf(q, u, as_f32(TEMPO_GELU_ERFC_Q4));
  q = fmaf(q, u, as_f32(TEMPO_GELU_ERFC_Q3));
  q = fmaf(q, u, as_f32(TEMPO_GELU_ERFC_Q2));
  q = fmaf(q, u, as_f32(TEMPO_GELU_ERFC_Q1));
  q = fmaf(q, u, as_f32(TEMPO_GELU_ERFC_Q0));
  const float half_erfc = t * q * __builtin_amdgcn_exp2f(-(w * w));  // 1/2 erfc(|x| / sqrt 2)
  const float phi = (x < 0.0f) ? half_erfc : 1.0f - half_erfc;
  return x * phi;  // NaN stays NaN
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

// SiLU(x) = x * sigmoid(x); exp overflows to +inf on the far left, which gives -0.
__device__ __forceinline__ float silu_value(float x) {
  const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * x);  // exp(-x)
  return x * __builtin_amdgcn_rcpf(1.0f + e);
}

template <int KIND>
__device__ __forceinline__ float act_value(float x) {
  if constexpr (KIND == TEMPO_GELU_ERF) return gelu_erf_value(x);
  else if constexpr (KIND == TEMPO_GELU_TANH) return gelu_tanh_value(x);
  else return silu_value(x);
}

// d(y, m) = GELU'(GELU*^-1(y, m)).
template <int KIND>
__device__ __forceinline__ float gelu_composite(float y, bool right, const f32x4* tab) {
  const float ys_hi = as_f32(GeluConst<KIND>::ys_hi);
  const float ys_lo = as_f32(GeluConst<KIND>::ys_lo);
  const float t = fmaxf((y - ys_hi) - ys_lo, 0.0f);
  const float s = __builtin_amdgcn_sqrtf(t);
  const float c = right ? static_cast<float>(TEMPO_GELU_CR) : static_cast<float>(TEMPO_GELU_CL);
  constexpr int NR = GeluConst<KIND>::NR, NL = GeluConst<KIND>::NL;
  const float umax = right ? (NR - 0.00001f) : (NL - 0.00001f);
  const int base = right ? 0 : NR;
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
  const int idx = tail ? static_cast<int>(it) + (NR + NL) : idx_s;
  const float z = tail ? z_t : z_s;
  float d = cubic(tab[idx], z);
  return (y != y) ? y : d;
}

template <int ROWS, int THREADS>
__device__ __forceinline__ void load_table(f32x4* lds, const uint32_t (*src)[4]) {
  for (int i = threadIdx.x; i < ROWS; i += THREADS) {
    const u32x4 r = *reinterpret_cast<const u32x4*>(src[i]);
    f32x4 f = {as_f32(r.x), as_f32(r.y), as_f32(r.z), as_f32(r.w)};
    lds[i] = f;
  }
  __syncthreads();
}


// ---- float32 storage: piecewise cubics ------------------------------------------------------
// Work decomposition: workgroup b owns the contiguous tile of THREADS*K pieces (4 floats each)
// starting at piece b*THREADS*K; piece k of lane t is tile_base + k*THREADS + t, so each
// access of a wave is one contiguous 1 KiB run, workgroups are short-lived, and the whole grid
// sweeps memory front to back.  8 lanes share a 32-bit mask word.
// Workgroup size: the memory system moves the most for workgroups of a single wave with one
// piece per lane (a plain copy gains 3-6 % over four waves).  The forward kernels stage no
// table and take exactly that shape (5 % faster than four waves of four pieces).  The
// backward kernels stage a table of 13-17 KiB, paid once per workgroup, and do best with four
// waves of two pieces (two waves measured 5 % slower for SiLU's table).  In the backward all
// of a lane's loads are issued before the table is staged into LDS, so the latencies overlap.
template <int KIND, int K, int THREADS>
__global__ __launch_bounds__(THREADS) void gelu_fwd_kernel(const float* x, float* y,  // may alias
                                                           uint32_t* __restrict__ mask,
                                                           int64_t n) {
  const float xstar = as_f32(GeluConst<KIND>::xstar);
  const int64_t q_base = static_cast<int64_t>(blockIdx.x) * (THREADS * K) + threadIdx.x;
  float v[K][4];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int64_t q = q_base + k * THREADS;
    const int64_t left = n - q * 4;
    if (left > 0) {
      load_piece_guarded<float>(x + q * 4, left, v[k], -1.0e30f);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) v[k][i] = -1.0e30f;  // absent: mask bit 0
    }
  }
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int64_t q = q_base + k * THREADS;
    const int64_t left = n - q * 4;
    uint32_t bits = 0;
    float r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float xv = v[k][i];
      bits |= (xv >= xstar ? 1u : 0u) << i;
      r[i] = act_value<KIND>(xv);
    }
    // every lane of the wave takes part in the merge; absent pieces contribute zero bits
    const uint32_t word = merge_mask_word<4>(bits, threadIdx.x);
    if (left > 0) store_piece_guarded<float>(y + q * 4, left, r);
    if ((threadIdx.x & 7) == 0 && left > 0) mask[q >> 3] = word;
  }
}

template <int KIND, int K, int THREADS>
__global__ __launch_bounds__(THREADS) void gelu_bwd_kernel(const float* dy,  // may alias dx
                                                           const float* __restrict__ y,
                                                           const uint32_t* __restrict__ mask,
                                                           float* dx, int64_t n) {
  __shared__ f32x4 tab[GeluConst<KIND>::kBwdRows];
  const int64_t q_base = static_cast<int64_t>(blockIdx.x) * (THREADS * K) + threadIdx.x;
  float g[K][4], o[K][4];
  uint32_t w[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int64_t q = q_base + k * THREADS;
    const int64_t left = n - q * 4;
    w[k] = 0;
    if (left > 0) {
      load_piece_guarded<float>(dy + q * 4, left, g[k], 0.0f);
      load_piece_guarded<float>(y + q * 4, left, o[k], 0.0f);
      w[k] = __builtin_nontemporal_load(mask + (q >> 3));
    }
  }
  load_table<GeluConst<KIND>::kBwdRows, THREADS>(tab, GeluConst<KIND>::bwd_table());
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int64_t q = q_base + k * THREADS;
    const int64_t left = n - q * 4;
    if (left <= 0) continue;
    const uint32_t bits = w[k] >> (4 * static_cast<int>(q & 7));
    float r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool right = (bits >> i) & 1u;
      r[i] = g[k][i] * gelu_composite<KIND>(o[k][i], right, tab);
    }
    store_piece_guarded<float>(dx + q * 4, left, r);
  }
}

// ---- bfloat16 storage: per-pattern lookup ------------------------------------------------
// A bf16 value has 2^16 bit patterns, so GELU ("Phi" factor) and the backward composite are
// tabulated per pattern (tables generated offline, float32 entries) and staged into LDS:
// 16 KiB forward, 32 KiB backward.  Per element this leaves a handful of integer ops, one
// ds_read_b32 and one multiply, which keeps the vector ALU far below the memory time (the
// cubic path above costs ~40 VALU ops per element, more than a bf16 element's share of HBM
// time).  Workgroups of 1024 lanes own contiguous tiles of K pieces
// per lane.
constexpr int kLutBwdThreads = 1024;  // 512 is 2-5 % slower

template <int WORDS, int THREADS>
__device__ __forceinline__ void stage_lut(uint32_t* lds, const uint32_t* src) {
  static_assert(WORDS % (4 * THREADS) == 0, "whole 16-byte pieces per lane");
#pragma unroll
  for (int i = 0; i < WORDS / (4 * THREADS); ++i) {
    const int j = (i * THREADS + threadIdx.x) * 4;
    *reinterpret_cast<u32x4*>(lds + j) = *reinterpret_cast<const u32x4*>(src + j);
  }
  __syncthreads();
}

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef short i16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t lds_word(const uint32_t* lut, uint32_t byte_offset) {
  return *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(lut) + byte_offset);
}

// LDS byte offsets of the forward entries of the two bf16 values packed in w (packed 16-bit
// integer ops: one instruction serves both halves).  Entry index = key | sign << 11 with
// key = clamp(pattern(|x|) - LUT_LO, 0, LUT_N - 1).
__device__ __forceinline__ uint32_t lut_fwd_offsets(uint32_t w) {
  const u16x2 lo = {TEMPO_GELU_LUT_LO, TEMPO_GELU_LUT_LO};
  const u16x2 top = {TEMPO_GELU_LUT_N - 1, TEMPO_GELU_LUT_N - 1};
  u16x2 k = __builtin_bit_cast(u16x2, w & 0x7FFF7FFFu);
  k = __builtin_elementwise_min(__builtin_elementwise_sub_sat(k, lo), top);
  const uint32_t idx = ((w >> 4) & 0x08000800u) | __builtin_bit_cast(uint32_t, k);
  const u16x2 two = {2, 2};
  return __builtin_bit_cast(uint32_t, static_cast<u16x2>(__builtin_bit_cast(u16x2, idx) << two));
}

// Same for the backward entries; mm holds the two mask bits at bit 0 and bit 16.  The left
// branch (mask bit 0) looks SHIFT patterns lower.  Index = m << 12 | sign << 11 | key.
template <int SHIFT>
__device__ __forceinline__ uint32_t lut_bwd_offsets(uint32_t w, uint32_t mm) {
  constexpr short lo_r = TEMPO_GELU_LUT_LO;  // window of the right branch
  const i16x2 shift = {SHIFT, SHIFT};
  const i16x2 lo = {lo_r, lo_r};
  const i16x2 hi = {lo_r + TEMPO_GELU_LUT_N - 1, lo_r + TEMPO_GELU_LUT_N - 1};
  const i16x2 one = {1, 1};
  // a + (1 - m) * shift, then the right branch's window
  i16x2 a = __builtin_bit_cast(i16x2, w & 0x7FFF7FFFu);
  a = a + (one - __builtin_bit_cast(i16x2, mm)) * shift;
  a = __builtin_elementwise_min(__builtin_elementwise_max(a, lo), hi) - lo;
  const uint32_t idx = ((w >> 4) & 0x08000800u) | (mm << 12) | __builtin_bit_cast(uint32_t, a);
  const u16x2 two = {2, 2};
  return __builtin_bit_cast(uint32_t, static_cast<u16x2>(__builtin_bit_cast(u16x2, idx) << two));
}

// One chunk (8 bf16 in 4 words) of the forward: y words and the 8 mask bits.
__device__ __forceinline__ void gelu_fwd_lut_chunk(const u32x4 w, const uint32_t* lut, u32x4& yw,
                                                   uint32_t& byte) {
  const uint32_t in[4] = {w.x, w.y, w.z, w.w};
  uint32_t out[4];
  uint32_t acc = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t off = lut_fwd_offsets(in[j]);
    const uint32_t e0 = lds_word(lut, off & 0xFFFFu);
    const uint32_t e1 = lds_word(lut, off >> 16);
    // shift the mask bit (entry LSB) of each element into the top of acc
    acc = __builtin_amdgcn_alignbit(e0, acc, 1);
    acc = __builtin_amdgcn_alignbit(e1, acc, 1);
    out[j] = pack_bf16(bf16_lo(in[j]) * as_f32(e0), bf16_hi(in[j]) * as_f32(e1));
  }
  yw = u32x4{out[0], out[1], out[2], out[3]};
  byte = acc >> 24;
}

template <int SHIFT>
__device__ __forceinline__ u32x4 gelu_bwd_lut_chunk(const u32x4 wy, const u32x4 wd, uint32_t byte,
                                                    const uint32_t* lut) {
  const uint32_t iy[4] = {wy.x, wy.y, wy.z, wy.w};
  const uint32_t id[4] = {wd.x, wd.y, wd.z, wd.w};
  uint32_t out[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t mm = (((byte >> (2 * j)) & 3u) * 0x8001u) & 0x00010001u;
    const uint32_t off = lut_bwd_offsets<SHIFT>(iy[j], mm);
    const float y0 = bf16_lo(iy[j]), y1 = bf16_hi(iy[j]);
    float d0 = as_f32(lds_word(lut, off & 0xFFFFu));
    float d1 = as_f32(lds_word(lut, off >> 16));
    d0 = (y0 != y0) ? y0 : d0;  // NaN in y propagates
    d1 = (y1 != y1) ? y1 : d1;
    out[j] = pack_bf16(bf16_lo(id[j]) * d0, bf16_hi(id[j]) * d1);
  }
  return u32x4{out[0], out[1], out[2], out[3]};
}

// Partial chunk at the very end of the tensor: gather / scatter element by element.
__device__ __forceinline__ u32x4 load_tail_bf16(const bf16_t* p, int64_t left, uint32_t fill) {
  uint32_t t[4] = {fill, fill, fill, fill};
  for (int i = 0; i < left; ++i) {
    const uint32_t b = p[i].bits;
    t[i >> 1] = (i & 1) ? ((t[i >> 1] & 0x0000FFFFu) | (b << 16)) : ((t[i >> 1] & 0xFFFF0000u) | b);
  }
  return u32x4{t[0], t[1], t[2], t[3]};
}
__device__ __forceinline__ void store_tail_bf16(bf16_t* p, int64_t left, const u32x4 v) {
  const uint32_t t[4] = {v.x, v.y, v.z, v.w};
  for (int i = 0; i < left; ++i)
    p[i].bits = static_cast<uint16_t>((i & 1) ? (t[i >> 1] >> 16) : (t[i >> 1] & 0xFFFFu));
}

constexpr uint32_t kAbsentX = 0xF149F149u;  // two bf16 of about -2.5e30: mask bit 0

// THREADS lanes per workgroup: 1024, or 512 with half the pieces per lane for large tensors
// (2-4 % faster from 130 MB of traffic up, 20 % slower at 70 MB).
template <int KIND, int K, int THREADS>
__global__ __launch_bounds__(THREADS) void gelu_fwd_lut_kernel(const bf16_t* x, bf16_t* y,
                                                                   uint32_t* __restrict__ mask,
                                                                   int64_t n) {
  __shared__ uint32_t lut[2 * TEMPO_GELU_LUT_N];
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t q_base = static_cast<int64_t>(blockIdx.x) * (THREADS * K) + threadIdx.x;
  const bool full = (static_cast<int64_t>(blockIdx.x) + 1) * (THREADS * K) * 8 <= n;
  u32x4 w[K];
  if (full) {  // whole tile inside the tensor: straight-line loads
#pragma unroll
    for (int k = 0; k < K; ++k) w[k] = ldg_stream(x + (q_base + k * THREADS) * 8);
  } else {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int64_t q = q_base + k * THREADS;
      const int64_t left = n - q * 8;
      w[k] = u32x4{kAbsentX, kAbsentX, kAbsentX, kAbsentX};
      if (left >= 8) w[k] = ldg_stream(x + q * 8);
      else if (left > 0) w[k] = load_tail_bf16(x + q * 8, left, kAbsentX);
    }
  }
  stage_lut<2 * TEMPO_GELU_LUT_N, THREADS>(lut, GeluConst<KIND>::lut_fwd());
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int64_t q = q_base + k * THREADS;
    u32x4 yw;
    uint32_t byte;
    gelu_fwd_lut_chunk(w[k], lut, yw, byte);
    // every lane of the wave takes part in the merge; absent chunks contribute zero bits
    const uint32_t word = merge_mask_word<8>(byte, lane);
    if (full) {
      stg_stream(y + q * 8, yw);
      if ((lane & 3) == 0) mask[q >> 2] = word;
    } else {
      const int64_t left = n - q * 8;
      if (left >= 8) stg_stream(y + q * 8, yw);
      else if (left > 0) store_tail_bf16(y + q * 8, left, yw);
      if ((lane & 3) == 0 && left > 0) mask[q >> 2] = word;
    }
  }
}

template <int KIND, int K>
__global__ __launch_bounds__(kLutBwdThreads) void gelu_bwd_lut_kernel(const bf16_t* dy,
                                                                   const bf16_t* __restrict__ y,
                                                                   const uint32_t* __restrict__ mask,
                                                                   bf16_t* dx, int64_t n) {
  __shared__ uint32_t lut[4 * TEMPO_GELU_LUT_N];
  const int64_t q_base = static_cast<int64_t>(blockIdx.x) * (kLutBwdThreads * K) + threadIdx.x;
  const bool full = (static_cast<int64_t>(blockIdx.x) + 1) * (kLutBwdThreads * K) * 8 <= n;
  u32x4 wy[K], wd[K];
  uint32_t mw[K];
  if (full) {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int64_t q = q_base + k * kLutBwdThreads;
      wd[k] = ldg_stream(dy + q * 8);
      wy[k] = ldg_stream(y + q * 8);
      mw[k] = __builtin_nontemporal_load(mask + (q >> 2));
    }
  } else {
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int64_t q = q_base + k * kLutBwdThreads;
      const int64_t left = n - q * 8;
      wy[k] = wd[k] = u32x4{0u, 0u, 0u, 0u};
      mw[k] = 0;
      if (left >= 8) {
        wd[k] = ldg_stream(dy + q * 8);
        wy[k] = ldg_stream(y + q * 8);
      } else if (left > 0) {
        wd[k] = load_tail_bf16(dy + q * 8, left, 0u);
        wy[k] = load_tail_bf16(y + q * 8, left, 0u);
      }
      if (left > 0) mw[k] = mask[q >> 2];
    }
  }
  stage_lut<4 * TEMPO_GELU_LUT_N, kLutBwdThreads>(lut, GeluConst<KIND>::lut_bwd());
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int64_t q = q_base + k * kLutBwdThreads;
    const uint32_t byte = mw[k] >> (8 * static_cast<int>(q & 3));
    const u32x4 r = gelu_bwd_lut_chunk<GeluConst<KIND>::kLutLeftShift>(wy[k], wd[k], byte, lut);
    if (full) {
      stg_stream(dx + q * 8, r);
    } else {
      const int64_t left = n - q * 8;
      if (left >= 8) stg_stream(dx + q * 8, r);
      else if (left > 0) store_tail_bf16(dx + q * 8, left, r);
    }
  }
}

int lut_grid(int64_t n, int k, int threads) {
  const int64_t n_chunks = (n + 7) / 8;
  const int64_t per_block = static_cast<int64_t>(threads) * k;
  return static_cast<int>((n_chunks + per_block - 1) / per_block);
}


int tile_grid(int64_t n, int k, int threads) {  // float32 pieces of 4 elements
  const int64_t n_pieces = (n + 3) / 4;
  const int64_t per_block = static_cast<int64_t>(threads) * k;
  return static_cast<int>((n_pieces + per_block - 1) / per_block);
}

int pick_k(int tuned) { return tuned >= 4 ? 4 : (tuned >= 2 ? 2 : 1); }

}  // namespace

// Shape of the float32 kernels: lanes per workgroup and pieces per lane.  Knob 15 at 1: the
// measured optimum (see gelu_fwd_kernel: one wave of one piece forward, four waves of two pieces
// backward); else that many lanes with the pieces of knobs 0 / 1.
struct F32Shape {
  int threads;
  int k;
};
static F32Shape f32_shape(bool forward, int kind) {
  const int forced = tune_get(kTuneGeluF32Threads);
  (void)kind;
  if (forced == 1) return forward ? F32Shape{64, 1} : F32Shape{256, 2};
  const int k = pick_k(tune_get(forward ? kTuneGeluFwdChunks : kTuneGeluBwdChunks));
  return {forced >= 256 ? 256 : (forced >= 128 ? 128 : 64), k};
}
template <typename F>
static void with_f32_threads(int threads, F&& f) {
  if (threads == 64) f(std::integral_constant<int, 64>{});
  else if (threads == 128) f(std::integral_constant<int, 128>{});
  else f(std::integral_constant<int, 256>{});
}

// Launch KERNEL<KIND, K> for the run-time (kind, k); THREADS lanes per workgroup.
template <int KIND, typename F>
static void with_k(int k, F&& f) {
  if (k == 1) f(std::integral_constant<int, KIND>{}, std::integral_constant<int, 1>{});
  else if (k == 2) f(std::integral_constant<int, KIND>{}, std::integral_constant<int, 2>{});
  else f(std::integral_constant<int, KIND>{}, std::integral_constant<int, 4>{});
}
template <typename F>
static void with_kind_k(int kind, int k, F&& f) {
  if (kind == TEMPO_GELU_ERF) with_k<TEMPO_GELU_ERF>(k, f);
  else if (kind == TEMPO_GELU_TANH) with_k<TEMPO_GELU_TANH>(k, f);
  else with_k<kActSilu>(k, f);
}

tempo_status launch_gelu_fwd(const void* x, void* y, uint32_t* mask, int64_t n, tempo_dtype dt,
                             int kind, hipStream_t st) {
  const int k = pick_k(tune_get(kTuneGeluFwdChunks));
  if (dt == TEMPO_BF16) {
    // large tensors: half-size workgroups with half the pieces per lane
    const bool small_groups = n >= tune_get(kTuneGeluFwdSmallGroupsFrom) * int64_t{1048576} && k >= 2;
    with_kind_k(kind, small_groups ? k / 2 : k, [&](auto kd, auto kk) {
      constexpr int KD = decltype(kd)::value, KK = decltype(kk)::value;
      if (small_groups)
        hipLaunchKernelGGL((gelu_fwd_lut_kernel<KD, KK, 512>), dim3(lut_grid(n, KK, 512)), dim3(512),
                           0, st, static_cast<const bf16_t*>(x), static_cast<bf16_t*>(y), mask, n);
      else
        hipLaunchKernelGGL((gelu_fwd_lut_kernel<KD, KK, 1024>), dim3(lut_grid(n, KK, 1024)),
                           dim3(1024), 0, st, static_cast<const bf16_t*>(x),
                           static_cast<bf16_t*>(y), mask, n);
    });
    return launch_status();
  }
  const F32Shape sh = f32_shape(true, kind);
  with_kind_k(kind, sh.k, [&](auto kd, auto kk) {
    with_f32_threads(sh.threads, [&](auto th) {
      constexpr int TH = decltype(th)::value;
      hipLaunchKernelGGL((gelu_fwd_kernel<decltype(kd)::value, decltype(kk)::value, TH>),
                         dim3(tile_grid(n, sh.k, TH)), dim3(TH), 0, st, static_cast<const float*>(x),
                         static_cast<float*>(y), mask, n);
    });
  });
  return launch_status();
}

tempo_status launch_gelu_bwd(const void* dy, const void* y, const uint32_t* mask, void* dx,
                             int64_t n, tempo_dtype dt, int kind, hipStream_t st) {
  const int k = pick_k(tune_get(kTuneGeluBwdChunks));
  if (dt == TEMPO_BF16) {
    with_kind_k(kind, k, [&](auto kd, auto kk) {
      hipLaunchKernelGGL((gelu_bwd_lut_kernel<decltype(kd)::value, decltype(kk)::value>),
                         dim3(lut_grid(n, k, kLutBwdThreads)), dim3(kLutBwdThreads), 0, st,
                         static_cast<const bf16_t*>(dy), static_cast<const bf16_t*>(y), mask,
                         static_cast<bf16_t*>(dx), n);
    });
    return launch_status();
  }
  const F32Shape sh = f32_shape(false, kind);
  with_kind_k(kind, sh.k, [&](auto kd, auto kk) {
    with_f32_threads(sh.threads, [&](auto th) {
      constexpr int TH = decltype(th)::value;
      hipLaunchKernelGGL((gelu_bwd_kernel<decltype(kd)::value, decltype(kk)::value, TH>),
                         dim3(tile_grid(n, sh.k, TH)), dim3(TH), 0, st, static_cast<const float*>(dy),
                         static_cast<const float*>(y), mask, static_cast<float*>(dx), n);
    });
  });
  return launch_status();
}

}  // namespace tempo
