"""Pins for the oracle's In-place GELU (Sec. 3.1; App. E.1 eq. 1-2; App. F.1) and for the same
recipe applied to SiLU (Sec. 5.1)."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import tempo_oracle as O

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))
KINDS = ["erf", "tanh", "silu"]


def _torch_gelu(x, kind):
    if kind == "silu":
        return torch.nn.functional.silu(x)
    return torch.nn.functional.gelu(x, approximate="none" if kind == "erf" else "tanh")


def test_silu_minimum_in_closed_form():
    # SiLU'(x) = sigma(x) (1 + x sigma(-x)) = 0  <=>  x = -(1 + W(1/e)), and then y = -W(1/e)
    from scipy.special import lambertw
    w = float(lambertw(1.0 / np.e).real)
    assert O.GELU_XSTAR["silu"] == pytest.approx(-(1.0 + w), abs=1e-14)
    assert O.GELU_YSTAR["silu"] == pytest.approx(-w, abs=1e-15)
    # extremes of SiLU': SiLU'' = sigma(x) sigma(-x) (2 + x (1 - 2 sigma(x))) vanishes at +-2.3994
    x = np.linspace(-20, 20, 400001)
    d = O.gelu_derivative(x, "silu")
    assert d.max() == pytest.approx(1.0998393, abs=1e-6) and d.min() == pytest.approx(-0.0998393, abs=1e-6)
    assert abs(x[np.argmax(d)] - 2.3994) < 1e-3 and abs(x[np.argmin(d)] + 2.3994) < 1e-3


def test_minimum_location_matches_paper():
    g = GOLD["gelu_minimum_x"]
    assert round(O.GELU_XSTAR["erf"], g["digits"]) == g["value"]
    # closed form: Phi(x*) + x* phi(x*) = 0, evaluated with the math module only
    import math
    xs = O.GELU_XSTAR["erf"]
    phi = math.exp(-0.5 * xs * xs) / math.sqrt(2 * math.pi)
    Phi = 0.5 * math.erfc(-xs / math.sqrt(2))
    assert abs(Phi + xs * phi) < 1e-15


@pytest.mark.parametrize("kind", KINDS)
def test_single_extremum_two_monotone_branches(kind):
    # Sec. 3.1: one extremum, so each side of it is one-to-one
    xs = O.GELU_XSTAR[kind]
    left = np.linspace(-12.0, xs, 20001)
    right = np.linspace(xs, 12.0, 20001)
    assert np.all(np.diff(O.gelu_value(left, kind)) < 0)
    assert np.all(np.diff(O.gelu_value(right, kind)) > 0)
    assert O.gelu_value(np.float64(xs), kind) == pytest.approx(O.GELU_YSTAR[kind], abs=1e-16)


@pytest.mark.parametrize("kind", KINDS)
def test_forward_against_library_gelu(kind):
    x = np.concatenate([np.random.default_rng(1).normal(size=4000) * 3, [0.0, -0.0, 30.0, -30.0]])
    ref = _torch_gelu(torch.from_numpy(x), kind).numpy()
    got = O.gelu_value(x, kind)
    # the library's erf form 0.5 x (1 + erf) cancels in the left tail: absolute floor there
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=5e-16)
    assert O.gelu_value(np.float64(0.0), kind) == 0.0


@pytest.mark.parametrize("kind", KINDS)
def test_mask_is_side_of_minimum(kind):
    xs32 = np.float32(O.GELU_XSTAR[kind])
    assert O.GELU_XSTAR_F32[kind] == float(xs32)
    x = np.array([np.nextafter(xs32, np.float32(-np.inf)), xs32, np.nextafter(xs32, np.float32(np.inf)),
                  -5.0, 0.0, 3.0], dtype=np.float64)
    _, m = O.gelu_fwd(x, kind, "f32")
    assert m.tolist() == [False, True, True, False, True, True]


@pytest.mark.parametrize("kind", KINDS)
def test_inverse_recovers_input(kind):
    # App. E.1 eq. 1: GELU*^-1(GELU(x), m) = x
    x = np.random.default_rng(2).normal(size=5000) * 2.5
    x = x[np.abs(x - O.GELU_XSTAR[kind]) > 1e-3]
    y = O.gelu_value(x, kind)
    m = x >= O.GELU_XSTAR_F32[kind]
    np.testing.assert_allclose(O.gelu_inverse(y, m, kind), x, rtol=0, atol=2e-10)


@pytest.mark.parametrize("kind", KINDS)
def test_backward_equals_library_autograd(kind):
    # the output-based gradient must equal the standard input-based one (App. E.1 eq. 2)
    rng = np.random.default_rng(3)
    x = rng.normal(size=6000) * 2.0
    dy = rng.normal(size=x.size)
    xt = torch.from_numpy(x).requires_grad_(True)
    yt = _torch_gelu(xt, kind)
    (ref,) = torch.autograd.grad(yt, xt, torch.from_numpy(dy))
    m = x >= O.GELU_XSTAR_F32[kind]
    # unrounded float64 y: no storage rounding between forward and backward
    got = O.gelu_bwd(dy, yt.detach().numpy(), m, kind, "f32")
    # dx is rounded to f32 on store; near the minimum d ~ sqrt(y - y*) amplifies 1e-16 in y
    np.testing.assert_allclose(got, ref.numpy(), rtol=1e-6, atol=2e-7)
    np.testing.assert_allclose(O.gelu_bwd_from_input(dy, x, kind), ref.numpy(), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("kind", KINDS)
def test_derivative_against_finite_differences(kind):
    x = np.linspace(-6, 6, 241)
    h = 1e-5
    fd = (O.gelu_value(x + h, kind) - O.gelu_value(x - h, kind)) / (2 * h)
    np.testing.assert_allclose(O.gelu_derivative(x, kind), fd, rtol=0, atol=1e-9)


def test_derivative_closed_form_extremes():
    # GELU'' = phi(x)(2 - x^2) vanishes at +-sqrt(2): the extremes of GELU'
    s2 = np.sqrt(2.0)
    assert float(O.gelu_derivative(np.float64(s2), "erf")) == pytest.approx(1.128904145, abs=1e-9)
    assert float(O.gelu_derivative(np.float64(-s2), "erf")) == pytest.approx(-0.128904145, abs=1e-9)
    x = np.linspace(-8, 8, 4001)
    d = O.gelu_derivative(x, "erf")
    assert d.max() <= 1.128904146 and d.min() >= -0.128904146


@pytest.mark.parametrize("kind", KINDS)
def test_backward_readings_at_the_edges(kind):
    ys = O.GELU_YSTAR[kind]
    dy = np.ones(7)
    y = np.array([ys - 1e-3, 0.0, -0.0, 0.0, np.inf, np.nan, 1e-30])
    m = np.array([1, 0, 0, 1, 1, 1, 0], dtype=bool)
    d = O.gelu_bwd(dy, y, m, kind, "f32")
    assert d[0] == 0.0            # stored y below the true minimum
    assert d[1] == 0.0 and d[2] == 0.0   # left branch underflowed to zero
    assert d[3] == 0.5            # right branch, y = 0 -> x = 0
    assert d[4] == 1.0            # saturated
    assert np.isnan(d[5])
    assert d[6] == 0.0            # left branch with positive y cannot come from a forward
    # left tail: d -> 0-, right tail: d -> 1
    tail = O.gelu_bwd(np.ones(2), np.array([-1e-30, 20.0]), np.array([0, 1], bool), kind, "f32")
    assert -1e-25 < tail[0] <= 0.0 and tail[1] == 1.0


@pytest.mark.parametrize("kind", KINDS)
def test_composite_monotone_on_right_branch_up_to_peak(kind):
    # d(y, m=1) rises from 0 at the minimum to the peak of GELU'
    xs = O.GELU_XSTAR[kind]
    x = np.linspace(xs, 1.3, 500)
    y = O.gelu_value(x, kind)
    d = O.gelu_bwd(np.ones_like(y), y, np.ones(y.size, bool), kind, "f32")
    assert np.all(np.diff(d) >= -1e-7) and d[0] == 0.0


def test_storage_rounding_bf16():
    a = np.array([1.00390625, 1.01171875, -0.16997, 3.0e38 * 1.2, 0.0, -0.0, np.inf, np.nan])
    r = O.round_to_dtype(a, "bf16")
    ref = torch.from_numpy(a).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(r, ref)
    rnd = np.random.default_rng(5).normal(size=20000) * np.exp(np.random.default_rng(6).normal(size=20000) * 8)
    got = O.round_to_dtype(rnd, "bf16")
    # one rounding from float64; torch rounds f64 -> f32 -> bf16, equal except on double-rounding ties
    ref = torch.from_numpy(rnd).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.mean(got != ref) < 1e-3
    assert np.all(np.abs(got - rnd) <= np.abs(rnd) * 2.0 ** -8)
