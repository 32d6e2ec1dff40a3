"""Host logic of the C ABI that needs no GPU: symbols, status strings, argument validation."""
import ctypes
import os
import re

import pytest

from paper_2210_10246_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    import glob
    text = "".join(open(h).read() for h in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))))
    return sorted(set(re.findall(r"TEMPO_API\s+[\w\s\*]+?\b(tempo_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert len(names) >= 11 and "tempo_attn_softmax_dropout_bwd" in names
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(B._SIGNATURES) == set(names)


def test_status_strings():
    assert B.status_string(0) == "ok"
    assert len({B.status_string(i) for i in range(5)}) == 5


def test_invalid_arguments_are_rejected_before_any_launch():
    lib = B.load()
    INVALID, UNSUPPORTED = 1, 2
    # negative size, bad enums
    assert lib.tempo_gelu_fwd(16, 16, 16, -1, 0, 0, None) == INVALID
    assert lib.tempo_gelu_fwd(16, 16, 16, 8, 7, 0, None) == INVALID
    assert lib.tempo_gelu_fwd(16, 16, 16, 8, 0, 9, None) == INVALID
    assert lib.tempo_gelu_bwd(16, 16, 16, 16, 8, 1, 2, None) == INVALID
    # null pointers
    assert lib.tempo_gelu_fwd(None, 16, 16, 8, 0, 0, None) == INVALID
    assert lib.tempo_gelu_bwd(16, 16, None, 16, 8, 0, 0, None) == INVALID
    assert lib.tempo_layernorm_fwd(16, 16, 16, 16, None, None, 2, 8, 1e-5, 0, None) == INVALID
    assert lib.tempo_layernorm_bwd(16, 16, 16, 16, 16, 16, 16, 16, None, 0, 2, 8, 0, None) == INVALID
    # misaligned pointers
    assert lib.tempo_gelu_fwd(20, 16, 16, 8, 0, 0, None) == UNSUPPORTED
    assert lib.tempo_layernorm_fwd(16, 16, 16, 16, 16, 4, 2, 8, 1e-5, 0, None) == UNSUPPORTED
    # eps < 0 / NaN, p outside [0, 1) / NaN
    assert lib.tempo_layernorm_fwd(16, 16, 16, 16, 16, None, 2, 8, -1.0, 0, None) == INVALID
    assert lib.tempo_layernorm_fwd(16, 16, 16, 16, 16, None, 2, 8, float("nan"), 0, None) == INVALID
    for p in (-0.1, 1.0, 1.5, float("nan")):
        assert lib.tempo_attn_softmax_dropout_fwd(16, None, 0, 16, 16, 16, 1, 1, 8, 8, p, 0, 0, 0, None) == INVALID
        assert lib.tempo_attn_softmax_dropout_bwd(16, 16, 16, 16, None, 1, 1, 8, 8, p, 0, None) == INVALID
        assert lib.tempo_attn_softmax_dropout_bwd_regen(16, 16, 16, None, 1, 1, 8, 8, p, 0, 0, 0, None) == INVALID
    assert lib.tempo_attn_softmax_dropout_bwd_regen(16, None, 16, None, 1, 1, 8, 8, 0.1, 0, 0, 0, None) == INVALID
    assert lib.tempo_attn_softmax_dropout_bwd_regen(16, 16, 24, None, 1, 1, 8, 8, 0.1, 0, 0, 0, None) == UNSUPPORTED
    assert lib.tempo_mask_bits_to_bytes(16, 16, -1, None) == INVALID
    assert lib.tempo_attn_softmax_dropout_bwd_bytemask(16, 16, None, 16, None, 1, 1, 8, 8, 0.1, 0, None) == INVALID
    assert lib.tempo_attn_softmax_dropout_bwd_bytemask(16, 16, 24, 16, None, 1, 1, 8, 8, 0.1, 0, None) == UNSUPPORTED
    assert lib.tempo_attn_softmax_dropout_bwd_bytemask(16, 16, 16, 16, None, 1, 1, 8, 8, 1.0, 0, None) == INVALID
    assert lib.tempo_attn_softmax_dropout_bwd_bytemask(None, None, None, None, None, 0, 1, 8, 8, 0.1, 0, None) == 0
    assert lib.tempo_silu_fwd(16, 16, 16, -1, 0, None) == INVALID
    assert lib.tempo_silu_fwd(16, 16, 16, 8, 5, None) == INVALID
    assert lib.tempo_silu_bwd(16, 16, None, 16, 8, 0, None) == INVALID
    assert lib.tempo_silu_bwd(16, 24, 16, 16, 8, 0, None) == UNSUPPORTED
    assert lib.tempo_mask_bits_to_bytes(None, 16, 5, None) == INVALID
    assert lib.tempo_mask_bytes_to_bits(16, None, 5, None) == INVALID
    assert lib.tempo_mask_bytes_to_bits(17, 16, 5, None) == UNSUPPORTED
    assert lib.tempo_attn_softmax_dropout_fwd(16, None, 0, 16, 16, 16, 1, -1, 8, 8, 0.1, 0, 0, 0, None) == INVALID
    # sizes whose products would overflow, or that no device memory can hold
    big = 1 << 62
    assert lib.tempo_gelu_fwd(16, 16, 16, (1 << 40) + 1, 0, 0, None) == INVALID
    assert lib.tempo_silu_bwd(16, 16, 16, 16, big, 0, None) == INVALID
    assert lib.tempo_layernorm_fwd(16, 16, 16, 16, 16, None, big, 8, 1e-5, 0, None) == INVALID
    assert lib.tempo_layernorm_fwd(16, 16, 16, 16, 16, None, 2, 1 << 31, 1e-5, 0, None) == INVALID
    assert lib.tempo_layernorm_bwd(16, 16, 16, 16, 16, 16, 16, 16, 16, 1 << 40, 1 << 33, 1 << 20, 0, None) == INVALID
    assert lib.tempo_layernorm_bwd_workspace_bytes(1 << 33, 1 << 20) == 0
    assert lib.tempo_attn_softmax_dropout_fwd(16, None, 0, 16, 16, 16, 1 << 31, 1 << 31, 8, 8, 0.1, 0, 0, 0, None) == INVALID
    assert lib.tempo_attn_softmax_dropout_fwd(16, None, 0, 16, 16, 16, 1 << 16, 1 << 16, 1, 8, 0.1, 0, 0, 0, None) == INVALID
    assert lib.tempo_attn_softmax_dropout_bwd(16, 16, 16, 16, None, 1 << 20, 1 << 10, 1 << 10, 1 << 10, 0.1, 0, None) == INVALID
    assert lib.tempo_attn_softmax_dropout_bwd_regen(16, 16, 16, None, 1, 1, 1 << 31, 8, 0.1, 0, 0, 0, None) == INVALID
    assert lib.tempo_mask_bytes_to_bits(16, 16, big, None) == INVALID
    # workspace too small
    need = lib.tempo_layernorm_bwd_workspace_bytes(64, 128)
    assert need >= 2 * 128 * 4
    assert lib.tempo_layernorm_bwd(16, 16, 16, 16, 16, 16, 16, 16, 16, need - 1, 64, 128, 0, None) == 3


def test_zero_sizes_return_ok_without_pointers():
    lib = B.load()
    assert lib.tempo_gelu_fwd(None, None, None, 0, 0, 0, None) == 0
    assert lib.tempo_gelu_bwd(None, None, None, None, 0, 1, 1, None) == 0
    assert lib.tempo_layernorm_fwd(None, None, None, None, None, None, 0, 768, 1e-5, 0, None) == 0
    assert lib.tempo_layernorm_bwd(None, None, None, None, None, None, None, None, None, 0, 0, 8, 0, None) == 0
    assert lib.tempo_attn_softmax_dropout_fwd(None, None, 0, None, None, None, 0, 12, 128, 128, 0.1, 0, 0, 0, None) == 0
    assert lib.tempo_attn_softmax_dropout_bwd(None, None, None, None, None, 2, 12, 0, 128, 0.1, 0, None) == 0
    assert lib.tempo_attn_softmax_dropout_bwd_regen(None, None, None, None, 2, 0, 8, 128, 0.1, 1, 2, 0, None) == 0
    assert lib.tempo_mask_bits_to_bytes(None, None, 0, None) == 0
    assert lib.tempo_silu_fwd(None, None, None, 0, 0, None) == 0
    assert lib.tempo_silu_bwd(None, None, None, None, 0, 1, None) == 0
    assert lib.tempo_mask_bytes_to_bits(None, None, 0, None) == 0
    assert lib.tempo_layernorm_bwd_workspace_bytes(0, 8) == 0


def test_launch_params():
    lib = B.load()
    old = B.tempo_get_launch_param(3)
    B.tempo_set_launch_param(3, 1)
    assert B.tempo_get_launch_param(3) == 1
    a = lib.tempo_layernorm_bwd_workspace_bytes(512, 512)      # 8 rows per workgroup: 64 slots
    B.tempo_set_launch_param(3, 2)
    b = lib.tempo_layernorm_bwd_workspace_bytes(512, 512)      # still 64: never fewer workgroups than CUs
    assert a == b == 64 * 2 * 512 * 4                           # one [2, M] float slot per workgroup
    assert lib.tempo_layernorm_bwd_workspace_bytes(1 << 20, 1024) <= 4096 * 2 * 1024 * 4
    B.tempo_set_launch_param(3, old)
    assert lib.tempo_set_launch_param(99, 1) == 1 and lib.tempo_set_launch_param(0, 0) == 1
    assert lib.tempo_get_launch_param(-1) == -1


def test_workloads_are_seeded_and_storage_exact():
    import numpy as np
    import torch
    from paper_2210_10246_amd import workloads as W
    cfg = W.config(0)
    a = W.layernorm_inputs(cfg, rows=4)
    b = W.layernorm_inputs(cfg, rows=4)
    assert all(torch.equal(a[k], b[k]) for k in a)
    assert a["x"].dtype == torch.float32 and a["x"].shape == (4, 768)
    c1 = W.attention_inputs(W.config(1), batch=3)
    assert c1["scores"].dtype == torch.bfloat16 and c1["scores"].shape == (3, 16, 128, 128)
    assert c1["key_len"].dtype == torch.int32 and int(c1["key_len"].min()) >= 64 and int(c1["key_len"].max()) <= 128
    assert W.attention_inputs(W.config(3), batch=1)["causal"] is True
    g = W.gelu_inputs(W.config(4), rows=64)
    x = W.as_f64(g["x"])
    assert np.abs(x).max() > 8.0            # the 1 % outliers x20 are there
    assert np.array_equal(x, W.as_f64(g["x"].to(torch.bfloat16)))   # already bf16-exact
