// C ABI of libtempo: argument validation, then one launcher per entry point.
#include <atomic>
#include <cmath>

#include "tempo_device.h"
#include "tempo_host.h"

namespace tempo {

static std::atomic<int> g_tune[kTuneCount] = {
    {4},      // gelu fwd: chunks per lane
    {2},      // gelu bwd: chunks per lane
    {3},      // layernorm fwd: workgroups per CU (beyond that they loop with prefetch)
    {4},      // layernorm bwd: rows per lane group
    {65536},  // attention fwd: workgroups per CU (65536 = one row per lane group)
    {65536},  // attention bwd: workgroups per CU
    {2},      // attention fwd: rows per lane group
    {2},      // layernorm fwd: rows per lane group
    {4},      // attention fwd: most pieces per lane of a one-wave row
    {4},      // attention bwd: the same
    {4},      // layernorm fwd: the same
    {3},      // layernorm bwd: the same (3: rows of 4 pieces per lane would keep their parameters in LDS)
    {1},      // layernorm bwd: workgroups per CU beyond which they loop with prefetch
    {24},     // bf16 gelu/silu fwd: Mi elements from which workgroups have 512 lanes
    {128},    // attention fwd / bwd: lanes per workgroup
    {1},      // float32 gelu/silu: lanes per workgroup (1: chosen per kernel)
};

int tune_get(TuneKey k) { return g_tune[k].load(std::memory_order_relaxed); }

int compute_units() {
  static std::atomic<int> cached{0};
  int v = cached.load(std::memory_order_relaxed);
  if (v > 0) return v;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess ||
      prop.multiProcessorCount <= 0) {
    (void)hipGetLastError();
    return 256;
  }
  cached.store(prop.multiProcessorCount, std::memory_order_relaxed);
  return prop.multiProcessorCount;
}

static bool dtype_ok(tempo_dtype dt) { return dt == TEMPO_F32 || dt == TEMPO_BF16; }
static bool kind_ok(tempo_gelu_kind k) { return k == TEMPO_GELU_ERF || k == TEMPO_GELU_TANH; }
static bool prob_ok(float p) { return p >= 0.0f && p < 1.0f; }  // false for NaN

// A tensor has at most 2^40 elements (terabytes: far beyond device memory), so that no product
// of sizes and no grid computed from one can overflow.  Sizes are known to be >= 0 here.
constexpr int64_t kMaxElements = int64_t{1} << 40;
static bool count_ok(int64_t a, int64_t b = 1, int64_t c = 1, int64_t d = 1) {
  int64_t n = a;
  for (int64_t f : {b, c, d}) {
    if (f != 0 && n > kMaxElements / f) return false;
    n *= f;
  }
  return n <= kMaxElements;
}

// Workgroups of the yardstick kernels are single waves: measured on 1 GiB tensors, one-wave
// workgroups move 3.5 % (one read, one write) to 6 % (two and two) more than four-wave ones.
constexpr int kCopyThreads = kWave;

// Plain streaming copy, 16 bytes per lane and access: the reference point for what the memory
// system delivers to a kernel that does nothing else, and the known-size kernel against which
// hardware byte counters are calibrated.
__global__ __launch_bounds__(kCopyThreads) void copy_kernel(const u32x4* __restrict__ src,
                                                            u32x4* __restrict__ dst, int64_t n16) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kCopyThreads;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kCopyThreads + threadIdx.x; i < n16;
       i += stride)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// The same with several streams: reads NR tensors, combines them (XOR, so that no load can be
// dropped) and writes NW tensors, one 16-byte piece per lane and stream, a full grid of
// short-lived workgroups.  What the memory system delivers depends on the mix of read and
// write streams (two reads and two writes reach less than one and one), so each layer kernel
// is held against the plain kernel of its own mix.
template <int NR, int NW>
__global__ __launch_bounds__(kCopyThreads) void copy_streams_kernel(const u32x4* r0, const u32x4* r1,
                                                           const u32x4* r2, u32x4* w0, u32x4* w1,
                                                           int64_t n16) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kCopyThreads + threadIdx.x;
  if (i >= n16) return;
  u32x4 v = __builtin_nontemporal_load(r0 + i);
  if constexpr (NR >= 2) v ^= __builtin_nontemporal_load(r1 + i);
  if constexpr (NR >= 3) v ^= __builtin_nontemporal_load(r2 + i);
  __builtin_nontemporal_store(v, w0 + i);
  if constexpr (NW >= 2) __builtin_nontemporal_store(v + 1u, w1 + i);
}

}  // namespace tempo

using namespace tempo;

extern "C" {

const char* tempo_status_string(tempo_status s) {
  switch (s) {
    case TEMPO_OK: return "ok";
    case TEMPO_ERR_INVALID_ARG: return "invalid argument";
    case TEMPO_ERR_UNSUPPORTED: return "unsupported (pointer not 16-byte aligned)";
    case TEMPO_ERR_WORKSPACE: return "workspace too small";
    case TEMPO_ERR_LAUNCH: return "kernel launch failed";
  }
  return "unknown status";
}

int tempo_version(void) { return 100; }

TEMPO_API int tempo_set_launch_param(int key, int value) {
  if (key < 0 || key >= kTuneCount || value < 1 || value > 65536) return TEMPO_ERR_INVALID_ARG;
  g_tune[key].store(value, std::memory_order_relaxed);
  return TEMPO_OK;
}

TEMPO_API int tempo_get_launch_param(int key) {
  if (key < 0 || key >= kTuneCount) return -1;
  return tune_get(static_cast<TuneKey>(key));
}

tempo_status tempo_copy(const void* src, void* dst, int64_t nbytes, int blocks_per_cu,
                        void* hip_stream) {
  if (nbytes < 0 || (nbytes & 15) != 0 || blocks_per_cu < 1) return TEMPO_ERR_INVALID_ARG;
  if (nbytes == 0) return TEMPO_OK;
  if (!src || !dst) return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(src) || !aligned16(dst)) return TEMPO_ERR_UNSUPPORTED;
  const int64_t n16 = nbytes / 16;
  const int64_t want = (n16 + kCopyThreads - 1) / kCopyThreads;
  const int64_t cap = static_cast<int64_t>(compute_units()) * blocks_per_cu;
  hipLaunchKernelGGL(copy_kernel, dim3(static_cast<unsigned>(want < cap ? want : cap)),
                     dim3(kCopyThreads), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<const u32x4*>(src),
                     static_cast<u32x4*>(dst), n16);
  return launch_status();
}

tempo_status tempo_copy_streams(const void* const* reads, int n_reads, void* const* writes,
                                int n_writes, int64_t nbytes, void* hip_stream) {
  if (nbytes < 0 || (nbytes & 15) != 0 || n_reads < 1 || n_reads > 3 || n_writes < 1 ||
      n_writes > 2 || nbytes / 16 > (int64_t{1} << 31) * kCopyThreads)
    return TEMPO_ERR_INVALID_ARG;
  if (nbytes == 0) return TEMPO_OK;
  if (!reads || !writes) return TEMPO_ERR_INVALID_ARG;
  const u32x4* r[3] = {nullptr, nullptr, nullptr};
  u32x4* w[2] = {nullptr, nullptr};
  for (int i = 0; i < n_reads; ++i) {
    if (!reads[i]) return TEMPO_ERR_INVALID_ARG;
    if (!aligned16(reads[i])) return TEMPO_ERR_UNSUPPORTED;
    r[i] = static_cast<const u32x4*>(reads[i]);
  }
  for (int i = 0; i < n_writes; ++i) {
    if (!writes[i]) return TEMPO_ERR_INVALID_ARG;
    if (!aligned16(writes[i])) return TEMPO_ERR_UNSUPPORTED;
    w[i] = static_cast<u32x4*>(writes[i]);
  }
  const int64_t n16 = nbytes / 16;
  const dim3 grid(static_cast<unsigned>((n16 + kCopyThreads - 1) / kCopyThreads));
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
#define TEMPO_LAUNCH(NR, NW)                                                                 \
  hipLaunchKernelGGL((copy_streams_kernel<NR, NW>), grid, dim3(kCopyThreads), 0, st, r[0], r[1], \
                     r[2], w[0], w[1], n16)
  switch (n_reads * 10 + n_writes) {
    case 11: TEMPO_LAUNCH(1, 1); break;
    case 12: TEMPO_LAUNCH(1, 2); break;
    case 21: TEMPO_LAUNCH(2, 1); break;
    case 22: TEMPO_LAUNCH(2, 2); break;
    case 31: TEMPO_LAUNCH(3, 1); break;
    default: TEMPO_LAUNCH(3, 2); break;
  }
#undef TEMPO_LAUNCH
  return launch_status();
}

tempo_status tempo_gelu_fwd(const void* x, void* y, uint32_t* mask, int64_t n, tempo_dtype dt,
                            tempo_gelu_kind kind, void* hip_stream) {
  if (n < 0 || !count_ok(n) || !dtype_ok(dt) || !kind_ok(kind)) return TEMPO_ERR_INVALID_ARG;
  if (n == 0) return TEMPO_OK;
  if (!x || !y || !mask) return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(y) || !aligned16(mask)) return TEMPO_ERR_UNSUPPORTED;
  return launch_gelu_fwd(x, y, mask, n, dt, kind, static_cast<hipStream_t>(hip_stream));
}

tempo_status tempo_gelu_bwd(const void* dy, const void* y, const uint32_t* mask, void* dx,
                            int64_t n, tempo_dtype dt, tempo_gelu_kind kind, void* hip_stream) {
  if (n < 0 || !count_ok(n) || !dtype_ok(dt) || !kind_ok(kind)) return TEMPO_ERR_INVALID_ARG;
  if (n == 0) return TEMPO_OK;
  if (!dy || !y || !mask || !dx) return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(dy) || !aligned16(y) || !aligned16(mask) || !aligned16(dx))
    return TEMPO_ERR_UNSUPPORTED;
  return launch_gelu_bwd(dy, y, mask, dx, n, dt, kind, static_cast<hipStream_t>(hip_stream));
}

tempo_status tempo_silu_fwd(const void* x, void* y, uint32_t* mask, int64_t n, tempo_dtype dt,
                            void* hip_stream) {
  if (n < 0 || !count_ok(n) || !dtype_ok(dt)) return TEMPO_ERR_INVALID_ARG;
  if (n == 0) return TEMPO_OK;
  if (!x || !y || !mask) return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(y) || !aligned16(mask)) return TEMPO_ERR_UNSUPPORTED;
  return launch_gelu_fwd(x, y, mask, n, dt, kActSilu, static_cast<hipStream_t>(hip_stream));
}

tempo_status tempo_silu_bwd(const void* dy, const void* y, const uint32_t* mask, void* dx,
                            int64_t n, tempo_dtype dt, void* hip_stream) {
  if (n < 0 || !count_ok(n) || !dtype_ok(dt)) return TEMPO_ERR_INVALID_ARG;
  if (n == 0) return TEMPO_OK;
  if (!dy || !y || !mask || !dx) return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(dy) || !aligned16(y) || !aligned16(mask) || !aligned16(dx))
    return TEMPO_ERR_UNSUPPORTED;
  return launch_gelu_bwd(dy, y, mask, dx, n, dt, kActSilu, static_cast<hipStream_t>(hip_stream));
}

tempo_status tempo_layernorm_fwd(const void* x, const float* gamma, const float* beta, void* y,
                                 float* rstd, float* mean, int64_t N, int64_t M, float eps,
                                 tempo_dtype dt, void* hip_stream) {
  if (N < 0 || M < 0 || !dtype_ok(dt) || !(eps >= 0.0f) || M > INT32_MAX || !count_ok(N, M))
    return TEMPO_ERR_INVALID_ARG;
  if (N == 0 || M == 0) return TEMPO_OK;
  if (!x || !gamma || !beta || !y || !rstd) return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(gamma) || !aligned16(beta) || !aligned16(y) ||
      !aligned16(rstd) || !aligned16(mean))
    return TEMPO_ERR_UNSUPPORTED;
  return launch_layernorm_fwd(x, gamma, beta, y, rstd, mean, N, M, eps, dt,
                              static_cast<hipStream_t>(hip_stream));
}

size_t tempo_layernorm_bwd_workspace_bytes(int64_t N, int64_t M) {
  if (N <= 0 || M <= 0 || M > INT32_MAX || !count_ok(N, M)) return 0;
  // the larger of the two dtypes' needs, so one query serves both
  const size_t a = layernorm_bwd_workspace_bytes(N, M, TEMPO_F32);
  const size_t b = layernorm_bwd_workspace_bytes(N, M, TEMPO_BF16);
  return a > b ? a : b;
}

tempo_status tempo_layernorm_bwd(const void* dy, const void* y, const float* gamma,
                                 const float* beta, const float* rstd, void* dx, float* dgamma,
                                 float* dbeta, void* workspace, size_t workspace_bytes, int64_t N,
                                 int64_t M, tempo_dtype dt, void* hip_stream) {
  if (N < 0 || M < 0 || !dtype_ok(dt) || M > INT32_MAX || !count_ok(N, M))
    return TEMPO_ERR_INVALID_ARG;
  if (N == 0 || M == 0) return TEMPO_OK;
  if (!dy || !y || !gamma || !beta || !rstd || !dx || !dgamma || !dbeta || !workspace)
    return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(dy) || !aligned16(y) || !aligned16(gamma) || !aligned16(beta) ||
      !aligned16(rstd) || !aligned16(dx) || !aligned16(dgamma) || !aligned16(dbeta) ||
      !aligned16(workspace))
    return TEMPO_ERR_UNSUPPORTED;
  return launch_layernorm_bwd(dy, y, gamma, beta, rstd, dx, dgamma, dbeta,
                              static_cast<float*>(workspace), workspace_bytes, N, M, dt,
                              static_cast<hipStream_t>(hip_stream));
}

tempo_status tempo_layernorm_bwd_static(const void* dy, const void* y, const float* gamma,
                                        const float* beta, const float* rstd, void* dx,
                                        float* dgamma, float* dbeta, int64_t N, int64_t M,
                                        tempo_dtype dt, void* hip_stream) {
  if (N < 0 || M < 0 || !dtype_ok(dt) || M > INT32_MAX || !count_ok(N, M))
    return TEMPO_ERR_INVALID_ARG;
  if (N == 0 || M == 0) return TEMPO_OK;
  if (!dy || !y || !gamma || !beta || !rstd || !dx || !dgamma || !dbeta)
    return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(dy) || !aligned16(y) || !aligned16(gamma) || !aligned16(beta) ||
      !aligned16(rstd) || !aligned16(dx) || !aligned16(dgamma) || !aligned16(dbeta))
    return TEMPO_ERR_UNSUPPORTED;
  void* ptr = nullptr;
  const tempo_status got = static_scratch(&ptr);
  if (got != TEMPO_OK) return got;
  // the launcher checks the plan's need against the array's size before it launches anything
  return launch_layernorm_bwd(dy, y, gamma, beta, rstd, dx, dgamma, dbeta,
                              static_cast<float*>(ptr), TEMPO_STATIC_SCRATCH_BYTES, N, M, dt,
                              static_cast<hipStream_t>(hip_stream));
}

tempo_status tempo_attn_softmax_dropout_fwd(const void* scores, const int32_t* key_len, int causal,
                                            void* probs, void* out, uint32_t* keep_bits, int64_t B,
                                            int64_t A, int64_t Sq, int64_t Sk, float p,
                                            uint64_t seed, uint64_t offset, tempo_dtype dt,
                                            void* hip_stream) {
  if (B < 0 || A < 0 || Sq < 0 || Sk < 0 || !dtype_ok(dt) || !prob_ok(p) || Sq > INT32_MAX ||
      Sk > INT32_MAX || !count_ok(B, A, Sq, Sk) || B * A > INT32_MAX)
    return TEMPO_ERR_INVALID_ARG;
  if (B == 0 || A == 0 || Sq == 0 || Sk == 0) return TEMPO_OK;
  if (!scores || !probs || !keep_bits) return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(scores) || !aligned16(probs) || !aligned16(out) || !aligned16(keep_bits))
    return TEMPO_ERR_UNSUPPORTED;
  return launch_attn_fwd(scores, key_len, causal, probs, out, keep_bits, B, A, Sq, Sk, p, seed,
                         offset, dt, static_cast<hipStream_t>(hip_stream));
}

tempo_status tempo_attn_softmax_dropout_bwd(const void* dout, const void* probs,
                                            const uint32_t* keep_bits, void* dscores,
                                            void* out_recomputed, int64_t B, int64_t A, int64_t Sq,
                                            int64_t Sk, float p, tempo_dtype dt, void* hip_stream) {
  if (B < 0 || A < 0 || Sq < 0 || Sk < 0 || !dtype_ok(dt) || !prob_ok(p) || Sq > INT32_MAX ||
      Sk > INT32_MAX || !count_ok(B, A, Sq, Sk) || B * A > INT32_MAX)
    return TEMPO_ERR_INVALID_ARG;
  if (B == 0 || A == 0 || Sq == 0 || Sk == 0) return TEMPO_OK;
  if (!dout || !probs || !keep_bits || !dscores) return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(dout) || !aligned16(probs) || !aligned16(keep_bits) || !aligned16(dscores) ||
      !aligned16(out_recomputed))
    return TEMPO_ERR_UNSUPPORTED;
  return launch_attn_bwd(dout, probs, keep_bits, dscores, out_recomputed, B, A, Sq, Sk, p, dt,
                         static_cast<hipStream_t>(hip_stream));
}

tempo_status tempo_attn_softmax_dropout_bwd_bytemask(const void* dout, const void* probs,
                                                     const uint8_t* keep_bytes, void* dscores,
                                                     void* out_recomputed, int64_t B, int64_t A,
                                                     int64_t Sq, int64_t Sk, float p,
                                                     tempo_dtype dt, void* hip_stream) {
  if (B < 0 || A < 0 || Sq < 0 || Sk < 0 || !dtype_ok(dt) || !prob_ok(p) || Sq > INT32_MAX ||
      Sk > INT32_MAX || !count_ok(B, A, Sq, Sk) || B * A > INT32_MAX)
    return TEMPO_ERR_INVALID_ARG;
  if (B == 0 || A == 0 || Sq == 0 || Sk == 0) return TEMPO_OK;
  if (!dout || !probs || !keep_bytes || !dscores) return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(dout) || !aligned16(probs) || !aligned16(keep_bytes) || !aligned16(dscores) ||
      !aligned16(out_recomputed))
    return TEMPO_ERR_UNSUPPORTED;
  return launch_attn_bwd_bytemask(dout, probs, keep_bytes, dscores, out_recomputed, B, A, Sq, Sk,
                                  p, dt, static_cast<hipStream_t>(hip_stream));
}

tempo_status tempo_attn_softmax_dropout_bwd_regen(const void* dout, const void* probs,
                                                  void* dscores, void* out_recomputed, int64_t B,
                                                  int64_t A, int64_t Sq, int64_t Sk, float p,
                                                  uint64_t seed, uint64_t offset, tempo_dtype dt,
                                                  void* hip_stream) {
  if (B < 0 || A < 0 || Sq < 0 || Sk < 0 || !dtype_ok(dt) || !prob_ok(p) || Sq > INT32_MAX ||
      Sk > INT32_MAX || !count_ok(B, A, Sq, Sk) || B * A > INT32_MAX)
    return TEMPO_ERR_INVALID_ARG;
  if (B == 0 || A == 0 || Sq == 0 || Sk == 0) return TEMPO_OK;
  if (!dout || !probs || !dscores) return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(dout) || !aligned16(probs) || !aligned16(dscores) || !aligned16(out_recomputed))
    return TEMPO_ERR_UNSUPPORTED;
  return launch_attn_bwd_regen(dout, probs, dscores, out_recomputed, B, A, Sq, Sk, p, seed,
                               offset, dt, static_cast<hipStream_t>(hip_stream));
}

tempo_status tempo_mask_bits_to_bytes(const uint32_t* bits, uint8_t* bytes, int64_t n,
                                      void* hip_stream) {
  if (n < 0 || !count_ok(n)) return TEMPO_ERR_INVALID_ARG;
  if (n == 0) return TEMPO_OK;
  if (!bits || !bytes) return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(bits) || !aligned16(bytes)) return TEMPO_ERR_UNSUPPORTED;
  return launch_mask_bits_to_bytes(bits, bytes, n, static_cast<hipStream_t>(hip_stream));
}

tempo_status tempo_mask_bytes_to_bits(const uint8_t* bytes, uint32_t* bits, int64_t n,
                                      void* hip_stream) {
  if (n < 0 || !count_ok(n)) return TEMPO_ERR_INVALID_ARG;
  if (n == 0) return TEMPO_OK;
  if (!bits || !bytes) return TEMPO_ERR_INVALID_ARG;
  if (!aligned16(bits) || !aligned16(bytes)) return TEMPO_ERR_UNSUPPORTED;
  return launch_mask_bytes_to_bits(bytes, bits, n, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
