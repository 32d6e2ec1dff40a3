"""Host-side checks of bench.py that need no GPU: argument contract, the algorithmic byte
counts it prices bandwidth with, and the activation-byte inventory against the oracle's closed
form."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from oracle import tempo_oracle as O  # noqa: E402
from paper_2210_10246_amd import workloads as W  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line that could be mistaken for a result


@pytest.mark.parametrize("index", range(5))
def test_algorithmic_bytes_per_element(index):
    cfg = W.config(index)
    e = cfg.elem_bytes
    key_len = W.attention_inputs(cfg)["key_len"] if index in (0, 1) else None
    key_len = None if key_len is None else key_len.tolist()
    a = bench.algorithmic_bytes(cfg, key_len)
    n_g = cfg.tokens * cfg.ffn
    n_a = cfg.batch * cfg.heads * cfg.seq * cfg.seq
    # reads of every input and writes of every output, masks at one bit per element
    assert a["gelu_fwd"] == n_g * (2 * e + 0.125)
    assert a["gelu_bwd"] == n_g * (3 * e + 0.125)
    assert a["attn_fwd_dense"] == n_a * (3 * e + 0.125)
    # masked scores are not counted as read: padding beyond key_len[b], or above the diagonal
    if cfg.mask == "causal":
        frac = (cfg.seq + 1) / (2 * cfg.seq)
    elif key_len is not None:
        frac = sum(key_len) / (len(key_len) * cfg.seq)
        assert 0.5 <= frac < 1.0
    else:
        frac = 1.0
    assert a["attn_fwd"] == pytest.approx(n_a * ((2 + frac) * e + 0.125), rel=1e-12)
    assert a["attn_bwd"] == n_a * (4 * e + 0.125)
    assert a["attn_bwd_regen"] == n_a * 4 * e
    assert a["attn_bwd_bytemask"] == n_a * (4 * e + 1)
    assert a["layernorm_fwd"] == cfg.tokens * (cfg.hidden * 2 * e + 4) + 8 * cfg.hidden
    assert a["layernorm_bwd"] == cfg.tokens * (cfg.hidden * 3 * e + 4) + 16 * cfg.hidden


@pytest.mark.parametrize("index", range(5))
def test_activation_bytes_saved_equal_the_closed_form(index):
    cfg = W.config(index)
    saved = bench.activation_bytes_saved(cfg)
    ref = O.activation_bytes_saved_bitmask(cfg.hidden, cfg.heads, cfg.seq, cfg.elem_bytes)
    assert saved["gelu"] == ref["gelu"]
    assert saved["layernorm"] == ref["layernorm"]
    assert saved["attention"] == ref["dropout"] + ref["softmax"]
