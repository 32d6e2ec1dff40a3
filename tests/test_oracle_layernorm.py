"""Pins for the oracle's In-place LayerNorm (Sec. 3.2; App. D.2, D.3)."""
import numpy as np
import pytest
import torch

from oracle import tempo_oracle as O


def _case(seed, N=7, M=24, shift=0.0):
    rng = np.random.default_rng(seed)
    x = rng.normal(size=(N, M)) + shift
    gamma = 1.0 + 0.1 * rng.normal(size=M)
    beta = 0.1 * rng.normal(size=M)
    dy = rng.normal(size=(N, M))
    return x, gamma, beta, dy


def _fwd64(x, gamma, beta, eps):
    """Unrounded float64 forward (the stored y of the oracle is rounded to dt)."""
    M = x.shape[-1]
    mu = x.mean(-1, keepdims=True)
    var = ((x - mu) ** 2).sum(-1, keepdims=True) / M
    rstd = 1 / np.sqrt(var + eps)
    return gamma * (x - mu) * rstd + beta, rstd[:, 0], mu[:, 0]


@pytest.mark.parametrize("eps", [1e-12, 1e-5])
def test_forward_against_library(eps):
    x, gamma, beta, _ = _case(0, shift=3.0)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (x.shape[1],), torch.from_numpy(gamma),
                                         torch.from_numpy(beta), eps).numpy()
    y, rstd, mean = O.layernorm_fwd(x, gamma, beta, eps, "f32")
    np.testing.assert_allclose(y, ref, rtol=0, atol=4e-7)
    np.testing.assert_allclose(mean, x.mean(-1), rtol=1e-7)
    np.testing.assert_allclose(rstd, 1 / np.sqrt(x.var(-1) + eps), rtol=1e-7)


def test_forward_invariants():
    # before the affine map every row has mean 0 and variance sigma^2 / (sigma^2 + eps)
    x, gamma, beta, _ = _case(1, N=5, M=64)
    eps = 1e-5
    y, rstd, mean = _fwd64(x, gamma, beta, eps)
    xhat = (y - beta) / gamma
    np.testing.assert_allclose(xhat.mean(-1), 0, atol=1e-14)
    var = x.var(-1)
    np.testing.assert_allclose(xhat.var(-1), var / (var + eps), rtol=1e-12)
    # constant row: variance 0, y = beta
    yc, rc, mc = O.layernorm_fwd(np.full((1, 8), 2.5), np.ones(8), np.zeros(8), 1e-5, "f32")
    assert np.all(yc == 0) and mc[0] == 2.5 and rc[0] == pytest.approx(1 / np.sqrt(1e-5), rel=1e-7)


@pytest.mark.parametrize("eps", [1e-12, 1e-5])
def test_output_based_gradient_equals_input_based(eps):
    # the claim of App. D.3: gradients from the output alone equal the standard ones
    x, gamma, beta, dy = _case(2)
    y, rstd, _ = _fwd64(x, gamma, beta, eps)
    dx, dg, db = O.layernorm_bwd(dy, y, gamma, beta, rstd, "f32")
    rx, rg, rb = O.layernorm_bwd_from_input(dy, x, gamma, eps)
    np.testing.assert_allclose(dx, rx, rtol=2e-7, atol=2e-7)
    np.testing.assert_allclose(dg, rg, rtol=2e-7, atol=1e-7)
    np.testing.assert_allclose(db, rb, rtol=2e-7, atol=1e-7)


def test_gradients_against_library_autograd():
    x, gamma, beta, dy = _case(3, N=9, M=40)
    eps = 1e-5
    xt = torch.from_numpy(x).requires_grad_(True)
    gt = torch.from_numpy(gamma).requires_grad_(True)
    bt = torch.from_numpy(beta).requires_grad_(True)
    yt = torch.nn.functional.layer_norm(xt, (x.shape[1],), gt, bt, eps)
    rx, rg, rb = torch.autograd.grad(yt, (xt, gt, bt), torch.from_numpy(dy))
    y, rstd, _ = _fwd64(x, gamma, beta, eps)
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=0, atol=1e-13)
    dx, dg, db = O.layernorm_bwd(dy, y, gamma, beta, rstd, "f32")
    np.testing.assert_allclose(dx, rx.numpy(), rtol=2e-7, atol=2e-7)
    np.testing.assert_allclose(dg, rg.numpy(), rtol=2e-7, atol=2e-7)
    np.testing.assert_allclose(db, rb.numpy(), rtol=2e-7, atol=2e-7)
    ix, ig, ib = O.layernorm_bwd_from_input(dy, x, gamma, eps)
    np.testing.assert_allclose(ix, rx.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(ig, rg.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(ib, rb.numpy(), rtol=1e-11, atol=1e-13)


def test_gradient_against_finite_differences():
    x, gamma, beta, dy = _case(4, N=3, M=10)
    eps = 1e-5
    y, rstd, _ = _fwd64(x, gamma, beta, eps)
    dx, dg, db = O.layernorm_bwd(dy, y, gamma, beta, rstd, "f32")
    loss = lambda xx, gg, bb: float((_fwd64(xx, gg, bb, eps)[0] * dy).sum())
    h = 1e-6
    for (i, j) in [(0, 0), (1, 3), (2, 9)]:
        xp, xm = x.copy(), x.copy()
        xp[i, j] += h
        xm[i, j] -= h
        assert dx[i, j] == pytest.approx((loss(xp, gamma, beta) - loss(xm, gamma, beta)) / (2 * h), abs=2e-6)
    for j in (0, 5):
        gp, gm = gamma.copy(), gamma.copy()
        gp[j] += h
        gm[j] -= h
        assert dg[j] == pytest.approx((loss(x, gp, beta) - loss(x, gm, beta)) / (2 * h), abs=2e-6)
        bp, bm = beta.copy(), beta.copy()
        bp[j] += h
        bm[j] -= h
        assert db[j] == pytest.approx((loss(x, gamma, bp) - loss(x, gamma, bm)) / (2 * h), abs=2e-6)


def test_backward_row_invariants():
    # textbook LayerNorm-gradient facts: dx is orthogonal to 1 and to xhat in every row
    x, gamma, beta, dy = _case(5, N=6, M=48)
    y, rstd, _ = _fwd64(x, gamma, beta, 1e-12)
    xhat = (y - beta) / gamma
    M = x.shape[1]
    g = dy * gamma
    dx64 = rstd[:, None] * (g - xhat * (g * xhat).sum(-1, keepdims=True) / M - g.sum(-1, keepdims=True) / M)
    dx, _, _ = O.layernorm_bwd(dy, y, gamma, beta, rstd, "f32")
    np.testing.assert_allclose(dx, dx64, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(dx64.sum(-1), 0, atol=1e-12)
    # exactly rstd c1 eps/(sigma^2+eps): zero up to the eps term
    np.testing.assert_allclose((dx64 * xhat).sum(-1), 0, atol=1e-9)


def test_zero_gamma_is_rejected():
    x, gamma, beta, dy = _case(6)
    gamma[3] = 0.0
    with pytest.raises(ValueError):
        O.layernorm_bwd(dy, x, gamma, beta, np.ones(x.shape[0]), "f32")
