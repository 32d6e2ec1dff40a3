/*
 * libtempo, tuning and benchmarking interface.  Nothing here is needed to use the layers of
 * tempo.h: these calls exist so that launch shapes can be swept and a streaming kernel can be
 * held against a plain copy on the same GPU.  They are the only part of the library with
 * process-wide state.
 */
#ifndef TEMPO_TUNE_H_
#define TEMPO_TUNE_H_

#include "tempo.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Launch-shape knobs (process-wide, not needed for correctness).  Every entry point of tempo.h
 * reads the knobs it depends on once per call, so its workspace check and its launch always
 * agree; a knob changed between tempo_layernorm_bwd_workspace_bytes and the call can at worst
 * make that call return TEMPO_ERR_WORKSPACE.
 *   key 0 / 1: 16-byte pieces per lane in gelu_fwd / gelu_bwd (1, 2 or 4; float32: see key 15);
 *   key 13: tensor size in Mi elements from which the bfloat16 gelu/silu forward uses workgroups
 *   of 512 lanes with half the pieces per lane (65536: never);
 *   key 2, 4, 5: cap on workgroups per compute unit of layernorm_fwd, attn fwd, attn bwd
 *   (rows beyond the cap are walked in a loop);
 *   key 6, 7: rows a lane group of attn fwd / layernorm_fwd fetches at once (1, or 2 and more:
 *   layernorm_fwd then takes 4 rows of one piece per lane, 2 of two pieces);
 *   key 8, 9, 10, 11: attn fwd / attn bwd / layernorm_fwd / layernorm_bwd: 16-byte pieces per
 *   lane above which a row is spread over 2 or 4 waves instead of one (16 or more: never);
 *   key 15: lanes per workgroup of the float32 gelu / silu kernels (64, 128 or 256, with the
 *   pieces per lane of keys 0 / 1; 1, the default: one wave of one piece per lane forward, four
 *   waves of two pieces backward);
 *   key 14: lanes per workgroup of attn fwd / bwd (64, 128 or 256; never fewer than a row's);
 *   key 3: rows each lane group of layernorm_bwd walks; key 12: workgroups per compute unit
 *   beyond which its workgroups loop over the rows; keys 3, 11 and 12 set its grid and the
 *   size of its workspace, so query tempo_layernorm_bwd_workspace_bytes after changing them.
 * Results never depend on these except the summation order of dgamma/dbeta and of the softmax
 * denominator and the other row sums (keys 8-11).  value in
 * [1, 65536].  tempo_set_launch_param returns TEMPO_OK or TEMPO_ERR_INVALID_ARG; the getter
 * returns -1 for an unknown key.
 */
TEMPO_API int tempo_set_launch_param(int key, int value);
TEMPO_API int tempo_get_launch_param(int key);

/*
 * Plain device-to-device copy of nbytes (a multiple of 16) with 16-byte accesses, at most
 * blocks_per_cu workgroups per compute unit.  Not part of the method: it is the yardstick for
 * the bandwidth a pure streaming kernel reaches on this GPU and the known-size kernel used to
 * calibrate hardware byte counters.  src and dst must not overlap.
 */
TEMPO_API tempo_status tempo_copy(const void* src, void* dst, int64_t nbytes, int blocks_per_cu,
                                  void* hip_stream);

/*
 * The same yardstick for a given mix of streams: reads n_reads (1..3) tensors of nbytes each,
 * combines them and writes n_writes (1..2) tensors of nbytes each, one 16-byte access per lane
 * and tensor.  The bandwidth a streaming kernel can reach on this GPU depends on how many
 * tensors it reads and writes at once; this is the plain kernel to hold a layer kernel against
 * (GELU forward and LayerNorm forward: 1 read 1 write; their backwards: 2 and 1; attention
 * forward: 1 and 2; attention backward: 2 and 2).  reads / writes are HOST arrays of device
 * pointers; no tensor may overlap another.  nbytes a multiple of 16.
 */
TEMPO_API tempo_status tempo_copy_streams(const void* const* reads, int n_reads,
                                          void* const* writes, int n_writes, int64_t nbytes,
                                          void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TEMPO_TUNE_H_ */
