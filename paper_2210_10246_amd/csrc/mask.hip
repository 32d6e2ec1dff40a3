// Conversions between the 1-bit keep/branch masks of this library and 1-byte-per-element masks
// (the form the paper's own implementation stores, Sec. 3.3, and the layout of a framework's
// boolean tensor).  Bit e of the packed mask is bit (e & 31) of word e >> 5.
#include "tempo_device.h"
#include "tempo_host.h"

namespace tempo {
namespace {

constexpr int kThreads = 256;

// 4 mask bits -> 4 bytes of 0/1: the multiplier copies the nibble to bit offsets 0, 7, 14 and
// 21, which puts bit j at bit 8j; no two partial products share a bit position.
__device__ __forceinline__ uint32_t spread4(uint32_t nibble) {
  return ((nibble & 0xFu) * 0x00204081u) & 0x01010101u;
}

// 4 bytes -> 4 bits (byte != 0): fold each byte onto its bit 0, then gather bits 0, 8, 16, 24
// into bits 24..27 with one multiply.
__device__ __forceinline__ uint32_t gather4(uint32_t v) {
  v |= v >> 4;
  v |= v >> 2;
  v |= v >> 1;
  v &= 0x01010101u;
  return ((v * 0x01020408u) >> 24) & 0xFu;
}

// One lane per 16 elements: half a mask word in, one 16-byte store out.
__global__ __launch_bounds__(kThreads) void bits_to_bytes_kernel(const uint32_t* __restrict__ bits,
                                                                uint8_t* __restrict__ bytes,
                                                                int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  const int64_t e0 = i * 16;
  if (e0 >= n) return;
  const uint32_t half = (bits[i >> 1] >> (16 * static_cast<int>(i & 1))) & 0xFFFFu;
  if (e0 + 16 <= n) {
    u32x4 out;
    out.x = spread4(half);
    out.y = spread4(half >> 4);
    out.z = spread4(half >> 8);
    out.w = spread4(half >> 12);
    stg_stream(reinterpret_cast<u32x4*>(bytes + e0), out);
  } else {
    for (int k = 0; e0 + k < n; ++k) bytes[e0 + k] = (half >> k) & 1u;
  }
}

// One lane per 16 elements; lanes 2k and 2k+1 hold the two halves of word k and the even lane
// writes it.  No lane leaves early: the pair exchange needs both.  Bits past n are written 0.
__global__ __launch_bounds__(kThreads) void bytes_to_bits_kernel(const uint8_t* __restrict__ bytes,
                                                                uint32_t* __restrict__ bits,
                                                                int64_t n) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  const int64_t e0 = i * 16;
  uint32_t half = 0;
  if (e0 + 16 <= n) {
    const u32x4 in = ldg_stream(reinterpret_cast<const u32x4*>(bytes + e0));
    half = gather4(in.x) | (gather4(in.y) << 4) | (gather4(in.z) << 8) | (gather4(in.w) << 12);
  } else if (e0 < n) {
    for (int k = 0; e0 + k < n; ++k) half |= (bytes[e0 + k] != 0 ? 1u : 0u) << k;
  }
  uint32_t word = half << (16 * static_cast<int>(i & 1));
  word |= dpp_u32<kDppXor1>(word);
  if ((i & 1) == 0 && e0 < n) bits[i >> 1] = word;
}

}  // namespace

tempo_status launch_mask_bits_to_bytes(const uint32_t* bits, uint8_t* bytes, int64_t n,
                                       hipStream_t st) {
  const int64_t blocks = ((n + 15) / 16 + kThreads - 1) / kThreads;
  if (blocks > INT32_MAX) return TEMPO_ERR_INVALID_ARG;
  hipLaunchKernelGGL(bits_to_bytes_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0,
                     st, bits, bytes, n);
  return launch_status();
}

tempo_status launch_mask_bytes_to_bits(const uint8_t* bytes, uint32_t* bits, int64_t n,
                                       hipStream_t st) {
  const int64_t blocks = ((n + 15) / 16 + kThreads - 1) / kThreads;
  if (blocks > INT32_MAX) return TEMPO_ERR_INVALID_ARG;
  hipLaunchKernelGGL(bytes_to_bits_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0,
                     st, bytes, bits, n);
  return launch_status();
}

}  // namespace tempo
