"""Thin ctypes binding of libtempo.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA tensors (PyTorch supplies device memory and the stream; every step
of the layers runs in the HIP kernels).  Outputs are written into tensors the caller passes.
There is no CPU fallback: if the shared library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtempo.so")

TEMPO_OK = 0
TEMPO_F32, TEMPO_BF16 = 0, 1
TEMPO_GELU_ERF, TEMPO_GELU_TANH = 0, 1
_DT = {torch.float32: TEMPO_F32, torch.bfloat16: TEMPO_BF16}
_KIND = {"erf": TEMPO_GELU_ERF, "tanh": TEMPO_GELU_TANH}

_vp, _i64, _u64 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64
_int, _f32, _sz = ctypes.c_int, ctypes.c_float, ctypes.c_size_t

_SIGNATURES = {
    "tempo_status_string": (ctypes.c_char_p, [_int]),
    "tempo_version": (_int, []),
    "tempo_set_launch_param": (_int, [_int, _int]),
    "tempo_get_launch_param": (_int, [_int]),
    "tempo_copy": (_int, [_vp, _vp, _i64, _int, _vp]),
    "tempo_copy_streams": (_int, [_vp, _int, _vp, _int, _i64, _vp]),
    "tempo_gelu_fwd": (_int, [_vp, _vp, _vp, _i64, _int, _int, _vp]),
    "tempo_gelu_bwd": (_int, [_vp, _vp, _vp, _vp, _i64, _int, _int, _vp]),
    "tempo_silu_fwd": (_int, [_vp, _vp, _vp, _i64, _int, _vp]),
    "tempo_silu_bwd": (_int, [_vp, _vp, _vp, _vp, _i64, _int, _vp]),
    "tempo_layernorm_fwd": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _f32, _int, _vp]),
    "tempo_layernorm_bwd_workspace_bytes": (_sz, [_i64, _i64]),
    "tempo_layernorm_bwd": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _i64, _i64,
                                   _int, _vp]),
    "tempo_layernorm_bwd_static": (_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _int,
                                          _vp]),
    "tempo_attn_softmax_dropout_fwd": (_int, [_vp, _vp, _int, _vp, _vp, _vp, _i64, _i64, _i64,
                                              _i64, _f32, _u64, _u64, _int, _vp]),
    "tempo_attn_softmax_dropout_bwd": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64,
                                              _f32, _int, _vp]),
    "tempo_attn_softmax_dropout_bwd_bytemask": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64,
                                                       _i64, _f32, _int, _vp]),
    "tempo_attn_softmax_dropout_bwd_regen": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _i64,
                                                    _f32, _u64, _u64, _int, _vp]),
    "tempo_mask_bits_to_bytes": (_int, [_vp, _vp, _i64, _vp]),
    "tempo_mask_bytes_to_bits": (_int, [_vp, _vp, _i64, _vp]),
}

_lib = None


class TempoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def load() -> ctypes.CDLL:
    """Load libtempo.so (built in-tree by build.py); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} not found: build it with `python -m paper_2210_10246_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().tempo_status_string(status).decode()


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous CUDA tensors")
    return t.data_ptr()


def _want(name: str, t: Optional[torch.Tensor], dtype, numel: Optional[int] = None,
          at_least: Optional[int] = None):
    """The C ABI reads raw bytes: a tensor of another dtype or size would be misread, or read
    out of bounds, on the device.  None is let through (optional arguments)."""
    if t is None:
        return
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"{name} must have {numel} elements, got {t.numel()}")
    if at_least is not None and t.numel() < at_least:
        raise ValueError(f"{name} must have at least {at_least} elements, got {t.numel()}")


def _act_dtype(name: str, t: torch.Tensor) -> int:
    if t.dtype not in _DT:
        raise ValueError(f"{name} must be float32 or bfloat16, got {t.dtype}")
    return _DT[t.dtype]


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _check(status: int, where: str):
    if status != TEMPO_OK:
        raise TempoError(status, where)


def mask_words(n: int) -> int:
    return (n + 31) // 32


def tempo_set_launch_param(key: int, value: int):
    _check(load().tempo_set_launch_param(key, value), "tempo_set_launch_param")


def tempo_get_launch_param(key: int) -> int:
    return load().tempo_get_launch_param(key)


def tempo_copy(src, dst, blocks_per_cu=16, stream=None):
    """Plain streaming copy of src into dst (same byte size, multiple of 16)."""
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    _check(load().tempo_copy(_ptr(src), _ptr(dst), nbytes, blocks_per_cu, _stream(stream)),
           "tempo_copy")


def tempo_copy_streams(reads, writes, stream=None):
    """Plain streaming kernel over len(reads) input and len(writes) output tensors of one size."""
    nbytes = reads[0].numel() * reads[0].element_size()
    for t in list(reads) + list(writes):
        if t.numel() * t.element_size() != nbytes:
            raise ValueError("all tensors must have the same size in bytes")
    r = (ctypes.c_void_p * len(reads))(*[_ptr(t) for t in reads])
    w = (ctypes.c_void_p * len(writes))(*[_ptr(t) for t in writes])
    _check(load().tempo_copy_streams(r, len(reads), w, len(writes), nbytes, _stream(stream)),
           "tempo_copy_streams")


def tempo_gelu_fwd(x, y, mask, kind="erf", stream=None):
    """(y, mask) = GELU*(x); y may be x."""
    n = x.numel()
    dt = _act_dtype("x", x)
    _want("y", y, x.dtype, n)
    _want("mask", mask, torch.int32, at_least=mask_words(n))
    _check(load().tempo_gelu_fwd(_ptr(x), _ptr(y), _ptr(mask), n, dt,
                                 _KIND[kind], _stream(stream)), "tempo_gelu_fwd")


def tempo_gelu_bwd(dy, y, mask, dx, kind="erf", stream=None):
    """dx = dy * GELU'(GELU*^-1(y, mask)); dx may be dy."""
    n = y.numel()
    dt = _act_dtype("y", y)
    _want("dy", dy, y.dtype, n)
    _want("dx", dx, y.dtype, n)
    _want("mask", mask, torch.int32, at_least=mask_words(n))
    _check(load().tempo_gelu_bwd(_ptr(dy), _ptr(y), _ptr(mask), _ptr(dx), n, dt,
                                 _KIND[kind], _stream(stream)), "tempo_gelu_bwd")


def tempo_silu_fwd(x, y, mask, stream=None):
    """(y, mask) = SiLU*(x); y may be x."""
    n = x.numel()
    dt = _act_dtype("x", x)
    _want("y", y, x.dtype, n)
    _want("mask", mask, torch.int32, at_least=mask_words(n))
    _check(load().tempo_silu_fwd(_ptr(x), _ptr(y), _ptr(mask), n, dt,
                                 _stream(stream)), "tempo_silu_fwd")


def tempo_silu_bwd(dy, y, mask, dx, stream=None):
    """dx = dy * SiLU'(SiLU*^-1(y, mask)); dx may be dy."""
    n = y.numel()
    dt = _act_dtype("y", y)
    _want("dy", dy, y.dtype, n)
    _want("dx", dx, y.dtype, n)
    _want("mask", mask, torch.int32, at_least=mask_words(n))
    _check(load().tempo_silu_bwd(_ptr(dy), _ptr(y), _ptr(mask), _ptr(dx), n, dt,
                                 _stream(stream)), "tempo_silu_bwd")


def tempo_layernorm_fwd(x, gamma, beta, y, rstd, mean=None, eps=1e-5, stream=None):
    M = x.shape[-1]
    N = x.numel() // M if M else 0
    dt = _act_dtype("x", x)
    _want("y", y, x.dtype, x.numel())
    _want("gamma", gamma, torch.float32, M)
    _want("beta", beta, torch.float32, M)
    _want("rstd", rstd, torch.float32, N)
    _want("mean", mean, torch.float32, N)
    _check(load().tempo_layernorm_fwd(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(rstd),
                                      _ptr(mean), N, M, eps, dt, _stream(stream)),
           "tempo_layernorm_fwd")


def tempo_layernorm_bwd_workspace_bytes(N: int, M: int) -> int:
    return load().tempo_layernorm_bwd_workspace_bytes(N, M)


def tempo_layernorm_bwd(dy, y, gamma, beta, rstd, dx, dgamma, dbeta, workspace, stream=None):
    M = y.shape[-1]
    N = y.numel() // M if M else 0
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    dt = _act_dtype("y", y)
    _want("dy", dy, y.dtype, y.numel())
    _want("dx", dx, y.dtype, y.numel())
    _want("gamma", gamma, torch.float32, M)
    _want("beta", beta, torch.float32, M)
    _want("rstd", rstd, torch.float32, N)
    _want("dgamma", dgamma, torch.float32, M)
    _want("dbeta", dbeta, torch.float32, M)
    _check(load().tempo_layernorm_bwd(_ptr(dy), _ptr(y), _ptr(gamma), _ptr(beta), _ptr(rstd),
                                      _ptr(dx), _ptr(dgamma), _ptr(dbeta), _ptr(workspace),
                                      ws_bytes, N, M, dt, _stream(stream)),
           "tempo_layernorm_bwd")


def tempo_layernorm_bwd_static(dy, y, gamma, beta, rstd, dx, dgamma, dbeta, stream=None):
    """tempo_layernorm_bwd with the library's static scratch array as workspace."""
    M = y.shape[-1]
    N = y.numel() // M if M else 0
    dt = _act_dtype("y", y)
    _want("dy", dy, y.dtype, y.numel())
    _want("dx", dx, y.dtype, y.numel())
    _want("gamma", gamma, torch.float32, M)
    _want("beta", beta, torch.float32, M)
    _want("rstd", rstd, torch.float32, N)
    _want("dgamma", dgamma, torch.float32, M)
    _want("dbeta", dbeta, torch.float32, M)
    _check(load().tempo_layernorm_bwd_static(_ptr(dy), _ptr(y), _ptr(gamma), _ptr(beta), _ptr(rstd),
                                             _ptr(dx), _ptr(dgamma), _ptr(dbeta), N, M, dt,
                                             _stream(stream)), "tempo_layernorm_bwd_static")


def tempo_attn_softmax_dropout_fwd(scores, key_len, causal, probs, out, keep_bits, p, seed, offset,
                                   stream=None):
    B, A, Sq, Sk = scores.shape
    n = scores.numel()
    dt = _act_dtype("scores", scores)
    _want("key_len", key_len, torch.int32, B)
    _want("probs", probs, scores.dtype, n)
    _want("out", out, scores.dtype, n)
    _want("keep_bits", keep_bits, torch.int32, at_least=mask_words(n))
    _check(load().tempo_attn_softmax_dropout_fwd(
        _ptr(scores), _ptr(key_len), int(bool(causal)), _ptr(probs), _ptr(out), _ptr(keep_bits),
        B, A, Sq, Sk, p, seed, offset, dt, _stream(stream)),
        "tempo_attn_softmax_dropout_fwd")


def tempo_attn_softmax_dropout_bwd(dout, probs, keep_bits, dscores, out_recomputed, p, stream=None):
    B, A, Sq, Sk = probs.shape
    n = probs.numel()
    dt = _act_dtype("probs", probs)
    _want("dout", dout, probs.dtype, n)
    _want("dscores", dscores, probs.dtype, n)
    _want("out_recomputed", out_recomputed, probs.dtype, n)
    _want("keep_bits", keep_bits, torch.int32, at_least=mask_words(n))
    _check(load().tempo_attn_softmax_dropout_bwd(
        _ptr(dout), _ptr(probs), _ptr(keep_bits), _ptr(dscores), _ptr(out_recomputed),
        B, A, Sq, Sk, p, dt, _stream(stream)),
        "tempo_attn_softmax_dropout_bwd")


def tempo_attn_softmax_dropout_bwd_bytemask(dout, probs, keep_bytes, dscores, out_recomputed, p,
                                            stream=None):
    """Backward reading a mask of one byte per element (uint8 or bool tensor; non-zero = kept)."""
    B, A, Sq, Sk = probs.shape
    n = probs.numel()
    dt = _act_dtype("probs", probs)
    _want("dout", dout, probs.dtype, n)
    _want("dscores", dscores, probs.dtype, n)
    _want("out_recomputed", out_recomputed, probs.dtype, n)
    if keep_bytes.dtype not in (torch.uint8, torch.bool) or keep_bytes.numel() != n:
        raise ValueError(f"keep_bytes must be uint8 or bool with {n} elements, got "
                         f"{keep_bytes.dtype} with {keep_bytes.numel()}")
    _check(load().tempo_attn_softmax_dropout_bwd_bytemask(
        _ptr(dout), _ptr(probs), _ptr(keep_bytes), _ptr(dscores), _ptr(out_recomputed),
        B, A, Sq, Sk, p, dt, _stream(stream)), "tempo_attn_softmax_dropout_bwd_bytemask")


def tempo_attn_softmax_dropout_bwd_regen(dout, probs, dscores, out_recomputed, p, seed, offset,
                                         stream=None):
    B, A, Sq, Sk = probs.shape
    n = probs.numel()
    dt = _act_dtype("probs", probs)
    _want("dout", dout, probs.dtype, n)
    _want("dscores", dscores, probs.dtype, n)
    _want("out_recomputed", out_recomputed, probs.dtype, n)
    _check(load().tempo_attn_softmax_dropout_bwd_regen(
        _ptr(dout), _ptr(probs), _ptr(dscores), _ptr(out_recomputed), B, A, Sq, Sk, p, seed,
        offset, dt, _stream(stream)), "tempo_attn_softmax_dropout_bwd_regen")


def tempo_mask_bits_to_bytes(bits, bytes_, n, stream=None):
    _want("bits", bits, torch.int32, at_least=mask_words(n))
    _want("bytes", bytes_, torch.uint8, at_least=n)
    _check(load().tempo_mask_bits_to_bytes(_ptr(bits), _ptr(bytes_), n, _stream(stream)),
           "tempo_mask_bits_to_bytes")


def tempo_mask_bytes_to_bits(bytes_, bits, n, stream=None):
    _want("bits", bits, torch.int32, at_least=mask_words(n))
    _want("bytes", bytes_, torch.uint8, at_least=n)
    _check(load().tempo_mask_bytes_to_bits(_ptr(bytes_), _ptr(bits), n, _stream(stream)),
           "tempo_mask_bytes_to_bits")
