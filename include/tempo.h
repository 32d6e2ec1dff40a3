/*
 * libtempo: memory-reduced forward/backward of three Transformer layers on gfx950 (MI355X),
 * after "Tempo: Accelerating Transformer-Based Model Training through Memory Footprint
 * Reduction" (arXiv 2210.10246).
 *
 * Conventions shared by every entry point
 *   Pointers   All data pointers are DEVICE pointers, owned by the caller; the library
 *              allocates nothing, never frees, and keeps no state between calls (the
 *              launch-shape knobs of tempo_tune.h, a separate interface for tuning and
 *              benchmarking, are the one exception and are not needed to use the layers).
 *              Every base pointer must be 16-byte aligned (TEMPO_ERR_UNSUPPORTED otherwise).
 *   Stream     hip_stream is a hipStream_t passed as void* (NULL = the default stream).  Work
 *              is enqueued on it and the call returns without synchronising.  Every entry point
 *              only launches kernels (no allocation, copy or memset), so a call may be recorded
 *              into a HIP graph by stream capture, a process's first call included.
 *   Layout     Contiguous row-major.  Activations are float32 (TEMPO_F32) or bfloat16
 *              (TEMPO_BF16); gamma, beta, dgamma, dbeta, rstd and mean are always float32.
 *   Bit masks  Element e (flat row-major index) is bit (e mod 32) of 32-bit word (e div 32).
 *              1 = "input at or right of the minimum" (GELU) / "kept" (dropout).  The caller
 *              sizes a mask ceil(n/32) words; unused bits of the last word are written 0.
 *   In place   Only the aliasing named per function is allowed; nothing else may overlap.
 *   Errors     A status code is returned; nothing is thrown and nothing aborts.
 *              INVALID_ARG: NULL required pointer, negative size, a tensor of more than 2^40
 *              elements, a row length (M, Sq, Sk) or a slice count B*A above 2^31 - 1, bad
 *              enum, p outside [0,1) or NaN, eps < 0 or NaN.  UNSUPPORTED: misaligned pointer.  WORKSPACE: workspace too
 *              small.  LAUNCH: the HIP runtime reported an error at launch.  Sizes of zero
 *              return TEMPO_OK without launching.
 */
#ifndef TEMPO_H_
#define TEMPO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Every entry point below is exported from libtempo.so with default visibility. */
#define TEMPO_API __attribute__((visibility("default")))

typedef enum {
  TEMPO_OK = 0,
  TEMPO_ERR_INVALID_ARG = 1,
  TEMPO_ERR_UNSUPPORTED = 2,
  TEMPO_ERR_WORKSPACE = 3,
  TEMPO_ERR_LAUNCH = 4
} tempo_status;

typedef enum { TEMPO_F32 = 0, TEMPO_BF16 = 1 } tempo_dtype;

/* GELU(x) = x Phi(x) (ERF) or 0.5 x (1 + tanh(sqrt(2/pi)(x + 0.044715 x^3))) (TANH). */
typedef enum { TEMPO_GELU_ERF = 0, TEMPO_GELU_TANH = 1 } tempo_gelu_kind;

/* Static, human-readable name of a status code. */
TEMPO_API const char* tempo_status_string(tempo_status s);

/* Library version as major*10000 + minor*100 + patch. */
TEMPO_API int tempo_version(void);

/*
 * In-place GELU forward, (y, m) = GELU*(x)            [Sec. 3.1; App. E.1 eq. (1); App. F.1]
 *   x    [n] in   activations (dt)
 *   y    [n] out  GELU(x) (dt); may alias x (the input need not survive)
 *   mask [ceil(n/32)] out  bit e = 1 iff x[e] >= x*, x* the location of GELU's single minimum
 *        (erf: -0.75179..., tanh form: -0.75246...) rounded to float32.
 */
TEMPO_API tempo_status tempo_gelu_fwd(const void* x, void* y, uint32_t* mask, int64_t n,
                            tempo_dtype dt, tempo_gelu_kind kind, void* hip_stream);

/*
 * In-place GELU backward, dx = dy * GELU'(GELU*^-1(y, m))      [App. E.1 eq. (2); App. F.1]
 * computed from the stored OUTPUT and the mask, never from x.  The composite is evaluated by
 * piecewise cubics in sqrt(y - y*) (and in -y on the left tail), max abs error ~2e-7.
 *   dy, y [n] in (dt); mask [ceil(n/32)] in; dx [n] out (dt), may alias dy.
 * y below the minimum value y* gives 0; left branch with y >= 0 gives 0; NaN in y propagates.
 */
TEMPO_API tempo_status tempo_gelu_bwd(const void* dy, const void* y, const uint32_t* mask, void* dx,
                            int64_t n, tempo_dtype dt, tempo_gelu_kind kind, void* hip_stream);

/*
 * In-place SiLU: the in-place recipe for elementwise layers on another activation with a
 * single minimum                                            [Sec. 5.1 (extending In-place GELU)]
 *   SiLU(x) = x sigmoid(x) has its only minimum at x* = -(1 + W(1/e)) = -1.27846...,
 *   y* = -0.27846...; on each side of x* it is one-to-one, so the steps of Sec. 5.1 apply as
 *   for GELU: forward folds the side indicator m = [x >= x*] (x* rounded to float32) into the
 *   kernel, backward evaluates dx = dy SiLU'(SiLU*^-1(y, m)) from the stored output.
 *   Arguments, layouts, aliasing and edge-case readings as tempo_gelu_fwd / tempo_gelu_bwd.
 */
TEMPO_API tempo_status tempo_silu_fwd(const void* x, void* y, uint32_t* mask, int64_t n,
                            tempo_dtype dt, void* hip_stream);
TEMPO_API tempo_status tempo_silu_bwd(const void* dy, const void* y, const uint32_t* mask, void* dx,
                            int64_t n, tempo_dtype dt, void* hip_stream);

/*
 * In-place LayerNorm forward                                              [App. D.2; Sec. 3.2]
 *   mu_i = mean_j x_ij, sigma_i^2 = mean_j (x_ij - mu_i)^2 (biased),
 *   rstd_i = 1/sqrt(sigma_i^2 + eps), y_ij = gamma_j (x_ij - mu_i) rstd_i + beta_j.
 *   x [N,M] in (dt); gamma, beta [M] in (f32); y [N,M] out (dt), may alias x;
 *   rstd [N] out (f32): the only per-row side information backward needs;
 *   mean [N] out (f32), may be NULL.
 */
TEMPO_API tempo_status tempo_layernorm_fwd(const void* x, const float* gamma, const float* beta,
                                 void* y, float* rstd, float* mean,
                                 int64_t N, int64_t M, float eps,
                                 tempo_dtype dt, void* hip_stream);

/* Bytes of device workspace tempo_layernorm_bwd needs for an [N,M] problem (partial column
 * sums of dgamma/dbeta, one slot per workgroup; written and read inside the call). */
TEMPO_API size_t tempo_layernorm_bwd_workspace_bytes(int64_t N, int64_t M);

/*
 * In-place LayerNorm backward, all gradients from the OUTPUT                [App. D.3]
 *   xhat_ij = (y_ij - beta_j)/gamma_j   (requires gamma_j != 0; not checked)
 *   dgamma_j = sum_i dy_ij xhat_ij,  dbeta_j = sum_i dy_ij,
 *   dx_ij = rstd_i [ dy_ij gamma_j - xhat_ij (1/M) sum_k dy_ik gamma_k xhat_ik
 *                                  - (1/M) sum_k dy_ik gamma_k ].
 *   dy, y [N,M] in (dt); gamma, beta [M], rstd [N] in (f32);
 *   dx [N,M] out (dt), may alias dy; dgamma, dbeta [M] out (f32), summed in a fixed order
 *   (bit-reproducible run to run); workspace: device memory of at least
 *   tempo_layernorm_bwd_workspace_bytes(N, M) bytes, 16-byte aligned.
 */
TEMPO_API tempo_status tempo_layernorm_bwd(const void* dy, const void* y, const float* gamma,
                                 const float* beta, const float* rstd,
                                 void* dx, float* dgamma, float* dbeta,
                                 void* workspace, size_t workspace_bytes,
                                 int64_t N, int64_t M, tempo_dtype dt, void* hip_stream);

/*
 * tempo_layernorm_bwd for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and bit-identical results, but the partial column sums go to a scratch array of
 * TEMPO_STATIC_SCRATCH_BYTES that lives in the library's code object (one copy per GPU, held
 * until the process ends) instead of a caller's workspace.  The call allocates nothing and
 * frees nothing.  Nothing in the array has to be zero between calls (every slot that is read
 * is written first by the same call).
 *   TEMPO_ERR_WORKSPACE: the problem needs more scratch than the array holds.  With the default
 *   launch shapes every M <= 4096 that is a multiple of 8 (bfloat16) or 4 (float32) fits for any
 *   N; longer rows up to 8192 columns (multiples of 8 in bfloat16, of 4 in float32) fit while
 *   N * 8 * M bytes do; other M fit while min(N, 1024) * 8 * M bytes do.
 *   TEMPO_ERR_LAUNCH: the array's device address could not be obtained.  It is looked up on the
 *   first call on each GPU: make that call before a stream capture begins.
 * All calls on one GPU share that GPU's array: calls that may run at the same time on one GPU
 * (different streams, or graphs replayed concurrently) race on it and must be serialised by the
 * caller; calls on different GPUs are independent.
 */
#define TEMPO_STATIC_SCRATCH_BYTES (8u << 20)
TEMPO_API tempo_status tempo_layernorm_bwd_static(const void* dy, const void* y, const float* gamma,
                                 const float* beta, const float* rstd,
                                 void* dx, float* dgamma, float* dbeta,
                                 int64_t N, int64_t M, tempo_dtype dt, void* hip_stream);

/*
 * Attention softmax -> dropout forward, keeping only P and a bit mask  [Sec. 3.3, 3.4; App. E.3, E.4]
 *   scores [B,A,Sq,Sk] in (dt), already scaled by 1/sqrt(d).
 *   key_len [B] int32 in, may be NULL: key column j >= key_len[b] is masked (treated as -inf).
 *   causal != 0: column j > i + (Sk - Sq) is masked.
 *   probs [B,A,Sq,Sk] out (dt): P = softmax over the unmasked columns, 0 where masked (a row
 *        with no unmasked column is all 0).  This is the tensor to keep for backward.
 *   out  [B,A,Sq,Sk] out (dt): P K / (1-p), computed from the STORED (rounded) P; transient
 *        input of the P.V product, not needed by backward.  May be NULL.
 *   keep_bits [ceil(B A Sq Sk / 32)] out: K, independent of the masking.
 *   Dropout contract (reproducible, independent of launch geometry): element e belongs to group
 *   g = e >> 3; Philox4x32-10 with counter (g_lo, g_hi, offset_lo, offset_hi) and key
 *   (seed_lo, seed_hi) gives words w0..w3; r = (w[(e & 7) >> 1] >> (16 (e & 1))) & 0xFFFF;
 *   kept iff r < T16, T16 = floor((1 - (double)p) 65536 + 0.5).  p == 0 keeps everything.
 *   (The words of group g are what rocRAND's philox4x32_10 engine returns when it is seeded
 *   with (seed, subsequence = offset, offset = 4 g).)
 *   probs may alias scores.
 */
TEMPO_API tempo_status tempo_attn_softmax_dropout_fwd(const void* scores, const int32_t* key_len, int causal,
                                            void* probs, void* out, uint32_t* keep_bits,
                                            int64_t B, int64_t A, int64_t Sq, int64_t Sk,
                                            float p, uint64_t seed, uint64_t offset,
                                            tempo_dtype dt, void* hip_stream);

/*
 * Attention softmax -> dropout backward from (dOut, P, K)             [Sec. 3.3, 3.4; App. E.3, E.4]
 *   dP = dOut K/(1-p);  dS_ij = P_ij (dP_ij - sum_k dP_ik P_ik)   (softmax gradient from its
 *   output alone);  out_recomputed = P K/(1-p), bit-identical to the forward's out: the
 *   dropout output is recomputed by one mask multiply instead of being stored.
 *   dout, probs [B,A,Sq,Sk] in (dt); keep_bits in; dscores out (dt), may alias dout;
 *   out_recomputed out (dt), may be NULL.
 */
TEMPO_API tempo_status tempo_attn_softmax_dropout_bwd(const void* dout, const void* probs,
                                            const uint32_t* keep_bits, void* dscores,
                                            void* out_recomputed,
                                            int64_t B, int64_t A, int64_t Sq, int64_t Sk, float p,
                                            tempo_dtype dt, void* hip_stream);

/*
 * The same backward with no stored mask                                   [Sec. 3.3; App. E.4]
 *   Sec. 3.3 weighs keeping the dropout mask against producing it again.  Because the keep
 *   decision of element e is a pure function of (seed, offset, e) (the dropout contract of the
 *   forward above), backward can draw the bits again: pass the p, seed and offset of the forward
 *   call and keep no mask at all (forward's keep_bits output still has to be a valid buffer; it
 *   can be a transient).  Results are bit-identical to tempo_attn_softmax_dropout_bwd on the
 *   forward's mask.  Costs one generator call per 8 elements instead of 1/8 byte of traffic.
 *   Arguments as above.
 */
TEMPO_API tempo_status tempo_attn_softmax_dropout_bwd_regen(const void* dout, const void* probs,
                                            void* dscores, void* out_recomputed,
                                            int64_t B, int64_t A, int64_t Sq, int64_t Sk, float p,
                                            uint64_t seed, uint64_t offset,
                                            tempo_dtype dt, void* hip_stream);

/*
 * The same backward reading a mask of one byte per element            [Sec. 3.3 (8-bit masks)]
 *   The paper's implementation keeps the dropout mask as 8-bit booleans.  This entry point
 *   consumes such a mask directly (no conversion pass): keep_bytes [B A Sq Sk] device bytes,
 *   element e kept iff keep_bytes[e] != 0.  Everything else as
 *   tempo_attn_softmax_dropout_bwd, with which it agrees bit for bit on the same mask.
 *   Costs one byte instead of one bit of mask traffic per element.
 */
TEMPO_API tempo_status tempo_attn_softmax_dropout_bwd_bytemask(const void* dout, const void* probs,
                                            const uint8_t* keep_bytes, void* dscores,
                                            void* out_recomputed,
                                            int64_t B, int64_t A, int64_t Sq, int64_t Sk, float p,
                                            tempo_dtype dt, void* hip_stream);

/*
 * Mask layout conversion: packed bits <-> one byte per element        [Sec. 3.3 (8-bit masks)]
 *   The paper's implementation keeps the dropout mask as one byte per element; this library
 *   keeps one bit (bit e & 31 of word e >> 5).  These two calls convert between the layouts,
 *   e.g. to hand a mask to, or take one from, code that expects boolean bytes.
 *   bits  [ceil(n/32)] device words;  bytes [n] device bytes, both 16-byte aligned.
 *   bits_to_bytes writes 0 or 1 per element.  bytes_to_bits sets bit e iff bytes[e] != 0 and
 *   writes 0 into the unused high bits of the last word.  n == 0 is a no-op.
 */
TEMPO_API tempo_status tempo_mask_bits_to_bytes(const uint32_t* bits, uint8_t* bytes, int64_t n,
                                            void* hip_stream);
TEMPO_API tempo_status tempo_mask_bytes_to_bits(const uint8_t* bytes, uint32_t* bits, int64_t n,
                                            void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TEMPO_H_ */
