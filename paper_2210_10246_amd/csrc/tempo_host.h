// Host-side declarations shared by the launchers and the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tempo.h"
#include "../../include/tempo_tune.h"

namespace tempo {

// Launch-shape knobs.
enum TuneKey {
  kTuneGeluFwdChunks = 0,       // 8-element chunks per lane (1, 2 or 4)
  kTuneGeluBwdChunks = 1,
  kTuneLnFwdBlocksPerCu = 2,    // cap on workgroups per compute unit
  kTuneLnBwdRowsPerGroup = 3,   // rows each lane group walks (sets the grid and the workspace)
  kTuneAttnFwdBlocksPerCu = 4,  // cap on workgroups per compute unit
  kTuneAttnBwdBlocksPerCu = 5,
  kTuneAttnFwdRows = 6,         // rows a lane group of attn fwd fetches at once (1 or 2)
  kTuneLnFwdRows = 7,           // layernorm_fwd: 1 = one row per lane group at a time, else 2 or 4 by shape
  kTuneAttnFwdMaxPieces = 8,    // attn fwd: pieces per lane above which a row takes 2-4 waves
  kTuneAttnBwdMaxPieces = 9,    // the same for attn bwd
  kTuneLnFwdMaxPieces = 10,     // the same for layernorm_fwd
  kTuneLnBwdMaxPieces = 11,     // and layernorm_bwd
  kTuneLnBwdLoopBlocksPerCu = 12,  // layernorm_bwd: workgroups per CU beyond which they loop
  kTuneGeluFwdSmallGroupsFrom = 13,  // bf16 gelu/silu fwd: Mi elements from which 512-lane groups
  kTuneAttnThreads = 14,        // attn fwd / bwd: lanes per workgroup (64, 128 or 256; at least one row's)
  kTuneGeluF32Threads = 15,     // float32 gelu/silu: lanes per workgroup (64, 128, 256; 1 = per kernel)
  kTuneCount = 16
};
int tune_get(TuneKey k);
int compute_units();

inline tempo_status launch_status() {
  return hipGetLastError() == hipSuccess ? TEMPO_OK : TEMPO_ERR_LAUNCH;
}

// kind: TEMPO_GELU_ERF, TEMPO_GELU_TANH or kActSilu (the activation kernels serve all three).
constexpr int kActSilu = 2;
tempo_status launch_gelu_fwd(const void* x, void* y, uint32_t* mask, int64_t n, tempo_dtype dt,
                             int kind, hipStream_t st);
tempo_status launch_gelu_bwd(const void* dy, const void* y, const uint32_t* mask, void* dx,
                             int64_t n, tempo_dtype dt, int kind, hipStream_t st);
tempo_status launch_layernorm_fwd(const void* x, const float* gamma, const float* beta, void* y,
                                  float* rstd, float* mean, int64_t N, int64_t M, float eps,
                                  tempo_dtype dt, hipStream_t st);
size_t layernorm_bwd_workspace_bytes(int64_t N, int64_t M, tempo_dtype dt);
// TEMPO_ERR_WORKSPACE if workspace_bytes is less than this call's launch plan needs.
tempo_status launch_layernorm_bwd(const void* dy, const void* y, const float* gamma,
                                  const float* beta, const float* rstd, void* dx, float* dgamma,
                                  float* dbeta, float* workspace, size_t workspace_bytes,
                                  int64_t N, int64_t M, tempo_dtype dt, hipStream_t st);

// Device address of the current device's static scratch array (TEMPO_STATIC_SCRATCH_BYTES).
tempo_status static_scratch(void** ptr);
tempo_status launch_attn_fwd(const void* scores, const int32_t* key_len, int causal, void* probs,
                             void* out, uint32_t* keep_bits, int64_t B, int64_t A, int64_t Sq,
                             int64_t Sk, float p, uint64_t seed, uint64_t offset, tempo_dtype dt,
                             hipStream_t st);
tempo_status launch_attn_bwd(const void* dout, const void* probs, const uint32_t* keep_bits,
                             void* dscores, void* out_re, int64_t B, int64_t A, int64_t Sq,
                             int64_t Sk, float p, tempo_dtype dt, hipStream_t st);
tempo_status launch_attn_bwd_bytemask(const void* dout, const void* probs,
                                      const uint8_t* keep_bytes, void* dscores, void* out_re,
                                      int64_t B, int64_t A, int64_t Sq, int64_t Sk, float p,
                                      tempo_dtype dt, hipStream_t st);
tempo_status launch_attn_bwd_regen(const void* dout, const void* probs, void* dscores,
                                   void* out_re, int64_t B, int64_t A, int64_t Sq, int64_t Sk,
                                   float p, uint64_t seed, uint64_t offset, tempo_dtype dt,
                                   hipStream_t st);
tempo_status launch_mask_bits_to_bytes(const uint32_t* bits, uint8_t* bytes, int64_t n,
                                       hipStream_t st);
tempo_status launch_mask_bytes_to_bits(const uint8_t* bytes, uint32_t* bits, int64_t n,
                                       hipStream_t st);

}  // namespace tempo
