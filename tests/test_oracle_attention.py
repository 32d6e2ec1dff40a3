"""Pins for the oracle's softmax -> dropout sublayer (Sec. 3.3, 3.4; App. E.3, E.4)."""
import numpy as np
import pytest
import torch

from oracle import tempo_oracle as O


def _scores(seed, shape=(2, 3, 5, 8)):
    return np.random.default_rng(seed).normal(size=shape)


@pytest.mark.parametrize("mode", ["none", "padding", "causal", "both"])
def test_softmax_against_library_and_rows_sum_to_one(mode):
    s = _scores(0)
    B, A, Sq, Sk = s.shape
    key_len = np.array([8, 5]) if mode in ("padding", "both") else None
    causal = mode in ("causal", "both")
    P, out, K = O.attn_softmax_dropout_fwd(s, key_len, causal, 0.0, 1, 0, "f32")
    valid = O.attention_valid(B, A, Sq, Sk, key_len, causal)
    ref = torch.softmax(torch.from_numpy(np.where(valid, s, -np.inf)), dim=-1).numpy()
    np.testing.assert_allclose(P, ref, rtol=0, atol=6e-8)
    np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-6)
    assert np.all(P[~valid] == 0)
    assert K.all() and np.array_equal(out, P)      # p = 0: nothing dropped, scale 1


def test_causal_mask_is_lower_triangular_with_offset():
    v = O.attention_valid(1, 1, 3, 5, None, True)[0, 0]
    assert v.astype(int).tolist() == [[1, 1, 1, 0, 0], [1, 1, 1, 1, 0], [1, 1, 1, 1, 1]]
    v = O.attention_valid(1, 1, 4, 4, None, True)[0, 0]
    assert np.array_equal(v, np.tril(np.ones((4, 4), bool)))


def test_shift_invariance_and_large_scores():
    s = _scores(1) * 30
    P0, _, _ = O.attn_softmax_dropout_fwd(s, None, False, 0.0, 1, 0, "f32")
    P1, _, _ = O.attn_softmax_dropout_fwd(s + 1000.0, None, False, 0.0, 1, 0, "f32")
    np.testing.assert_allclose(P0, P1, rtol=0, atol=1e-7)
    assert np.isfinite(P1).all()


def test_fully_masked_row_is_zero():
    s = _scores(2, (1, 1, 2, 4))
    P, out, _ = O.attn_softmax_dropout_fwd(s, np.array([0]), False, 0.1, 1, 0, "f32")
    assert np.all(P == 0) and np.all(out == 0)
    dS, _ = O.attn_softmax_dropout_bwd(np.ones_like(s), P, np.ones(s.shape, bool), 0.1, "f32")
    assert np.all(dS == 0)


def test_dropout_definition():
    # Sec. 3.3: dropped entries are zero, survivors are scaled by 1/(1-p)
    s = _scores(3, (2, 2, 16, 32))
    p = 0.25
    P, out, K = O.attn_softmax_dropout_fwd(s, None, False, p, 7, 3, "f32")
    assert np.all(out[~K] == 0)
    np.testing.assert_allclose(out[K], P[K] / (1 - p), rtol=1e-6)
    assert 0.6 < K.mean() < 0.9
    # mask depends on (seed, offset) only
    _, _, K2 = O.attn_softmax_dropout_fwd(s * 2, None, True, p, 7, 3, "f32")
    assert np.array_equal(K, K2)
    _, _, K3 = O.attn_softmax_dropout_fwd(s, None, False, p, 7, 4, "f32")
    assert not np.array_equal(K, K3)


@pytest.mark.parametrize("mode", ["none", "padding", "causal"])
def test_backward_against_library_autograd(mode):
    s = _scores(4, (2, 2, 6, 8))
    B, A, Sq, Sk = s.shape
    key_len = np.array([6, 8]) if mode == "padding" else None
    causal = mode == "causal"
    p = 0.1
    valid = O.attention_valid(B, A, Sq, Sk, key_len, causal)
    # float64 P (not rounded) so the comparison is free of storage rounding
    st = torch.from_numpy(np.where(valid, s, -np.inf)).requires_grad_(True)
    Pt = torch.softmax(st, dim=-1)
    K = O.dropout_keep(s.size, p, 11, 0).reshape(s.shape)
    scale = float(np.float32(1) / (np.float32(1) - np.float32(p)))
    outt = Pt * torch.from_numpy(K.astype(np.float64)) * scale
    dout = np.random.default_rng(5).normal(size=s.shape)
    (ref,) = torch.autograd.grad(outt, st, torch.from_numpy(dout))
    dS, out_re = O.attn_softmax_dropout_bwd(dout, Pt.detach().numpy(), K, p, "f32")
    np.testing.assert_allclose(dS, ref.numpy(), rtol=2e-7, atol=1e-7)
    np.testing.assert_allclose(out_re, outt.detach().numpy(), rtol=2e-7, atol=0)
    np.testing.assert_allclose(dS.sum(-1), 0, atol=1e-6)     # softmax gradient rows sum to zero
    assert np.all(dS[~valid] == 0)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_recomputed_output_is_bit_identical(dt):
    # Sec. 3.3: backward recomputes the discarded dropout output by one mask multiply
    s = O.round_to_dtype(_scores(6, (1, 2, 8, 16)), dt)
    P, out, K = O.attn_softmax_dropout_fwd(s, None, False, 0.1, 5, 0, dt)
    _, out_re = O.attn_softmax_dropout_bwd(np.zeros_like(s), P, K, 0.1, dt)
    assert np.array_equal(out, out_re)
    assert np.array_equal(O.round_to_dtype(P, dt), P) and np.array_equal(O.round_to_dtype(out, dt), out)
