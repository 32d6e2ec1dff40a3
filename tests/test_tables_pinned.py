"""Pins the COMMITTED kernel tables (csrc/gelu_tables.inc) to PyTorch's float64 gelu / silu and
their autograd, independently of the generator that wrote them and of the oracle.

Nothing here inverts a function.  The backward tables (d as a function of the stored OUTPUT y
and the side bit m, App. E.1 eq. 2) are checked by forward sampling: for a dense float64 grid of
inputs x, torch gives y(x) and, by autograd, d(x) = dy/dx; on each side of the minimum y is
monotone in x, so a table entry keyed by some y must lie between the d of the two samples
whose y bracket the key.  The last test regenerates the file and compares it byte for byte.
"""
import math
import os
import re
import subprocess
import sys

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INC = os.path.join(ROOT, "paper_2210_10246_amd", "csrc", "gelu_tables.inc")
GEN = os.path.join(ROOT, "paper_2210_10246_amd", "csrc", "gen_gelu_tables.py")
KINDS = ("erf", "tanh", "silu")


def _parse():
    text = open(INC).read()
    arrays = {}
    for m in re.finditer(r"const uint32_t (\w+)\[(\d+)\](\[4\])? = \{(.*?)\};", text, re.S):
        vals = np.array([int(v, 16) for v in re.findall(r"0x([0-9A-Fa-f]{8})u", m.group(4))],
                        dtype=np.uint32)
        assert vals.size == int(m.group(2)) * (4 if m.group(3) else 1), m.group(1)
        arrays[m.group(1)] = vals
    defs = {}
    for name, val in re.findall(r"^#define (TEMPO_GELU_\w+) (\S+)$", text, re.M):
        val = val.strip("()")
        if val.endswith("u") and val.startswith("0x"):
            defs[name] = int(val[:-1], 16)
        elif val.endswith("f"):
            defs[name] = float(val[:-1])
        else:
            defs[name] = int(val, 0)
    return arrays, defs


ARR, DEF = _parse()


def f32(words):
    return np.asarray(words, dtype=np.uint32).view(np.float32).astype(np.float64)


def bf16_value(pattern):
    return (np.asarray(pattern, dtype=np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def act(x, kind):
    """(y, dy/dx) from torch float64 and its autograd."""
    t = torch.tensor(np.asarray(x, dtype=np.float64), requires_grad=True)
    if kind == "silu":
        y = torch.nn.functional.silu(t)
    else:
        y = torch.nn.functional.gelu(t, approximate="none" if kind == "erf" else "tanh")
    (d,) = torch.autograd.grad(y.sum(), t)
    return y.detach().numpy(), d.numpy()


@pytest.fixture(scope="module", params=KINDS)
def sampled(request):
    """Dense forward samples of one activation, split at the sample of smallest y."""
    kind = request.param
    x = np.linspace(-31.0, 17.5, 8_000_001)
    y, d = act(x, kind)
    i = int(np.argmin(y))
    # left branch from the minimum outwards, as far as y stays clear of the rounding noise of
    # torch's 0.5 x (1 + erf): below the smallest key of any table
    j = int(np.argmax(y[: i + 1] < -4e-9))
    return kind, (x[j : i + 1][::-1], y[j : i + 1][::-1], d[j : i + 1][::-1]), (x[i:], y[i:], d[i:]), y[i]


def _bracket(branch, keys):
    """d of the two samples whose y bracket each key (y increases along both branches as given:
    the left one is stored from the minimum outwards)."""
    _, y, d = branch
    assert np.all(np.diff(y) >= 0)
    j = np.searchsorted(y, keys)
    assert j.min() >= 1 and j.max() < y.size, "samples do not cover the keys"
    lo = np.minimum(d[j - 1], d[j])
    hi = np.maximum(d[j - 1], d[j])
    return lo, hi


def test_forward_lookup_entries_are_the_activation_over_x(sampled):
    kind = sampled[0]
    n, lo_pat = DEF["TEMPO_GELU_LUT_N"], DEF["TEMPO_GELU_LUT_LO"]
    words = ARR[f"tempo_gelu_lut_fwd_{kind}"].reshape(2, n)
    mag = bf16_value(lo_pat + np.arange(n))
    assert mag[0] == 2.0 ** -12 and mag[-1] < 16.0 and bf16_value(lo_pat + n) == 16.0
    flips = {}
    for sign, x in ((0, mag), (1, -mag)):
        y, d = act(x, kind)
        entry = f32(words[sign] & np.uint32(0xFFFFFFFE))
        # the entry is a float32 whose last bit carries the mask: 2^-23 relative; torch's own
        # 0.5 x (1 + erf) / (1 + tanh) cancels on the far left: 2^-52 |x| absolute
        assert np.all(np.abs(x * entry - y) <= 2.5e-7 * np.abs(y) + 4e-15), (kind, sign)
        flips[sign] = (words[sign] & 1).astype(bool)
    assert flips[0].all()                                   # x > 0: right of the minimum
    m = flips[1]                                            # x = -mag, mag increasing
    k = int(np.argmin(m))                                   # first pattern left of the minimum
    assert m[:k].all() and not m[k:].any(), "mask bit is not a single step"
    # the step sits at the minimum: the slope changes sign between the two patterns around it
    _, d = act(-mag[k - 1 : k + 1], kind)
    assert d[0] > 1e-6 and d[1] < -1e-6
    xstar = f32([DEF[f"TEMPO_GELU_{kind.upper()}_XSTAR_F32"]])[0]
    assert -mag[k] < xstar <= -mag[k - 1]
    if kind == "erf":
        assert abs(xstar - (-0.75179)) < 5e-6               # the minimum printed in Sec. 3.1


def test_backward_lookup_entries_lie_between_bracketing_samples(sampled):
    kind, left, right, ymin = sampled
    n, lo_pat = DEF["TEMPO_GELU_LUT_N"], DEF["TEMPO_GELU_LUT_LO"]
    shift = DEF[f"TEMPO_GELU_{kind.upper()}_LUT_LEFT_SHIFT"]
    table = f32(ARR[f"tempo_gelu_lut_bwd_{kind}"]).reshape(2, 2, n)     # [m][sign of y][key]
    mag = bf16_value(lo_pat + np.arange(n))
    tol = lambda lo, hi: 1.5e-7 * np.maximum(np.abs(lo), np.abs(hi)) + 1e-12

    def check(entries, branch, keys, what):
        lo, hi = _bracket(branch, keys)
        t = tol(lo, hi)
        bad = (entries < lo - t) | (entries > hi + t)
        assert not bad.any(), (kind, what, keys[bad][:4], entries[bad][:4], lo[bad][:4], hi[bad][:4])
        return float(np.max(hi - lo))

    # m = 1, y >= 0
    w = check(table[1, 0], right, mag, "right, y > 0")
    assert w < 2e-5                                          # the brackets are tight
    # m = 1, y < 0: between the minimum value and 0; at or below the minimum value the entry is 0
    above = -mag > ymin
    assert above.any() and (~above).any()
    check(table[1, 1][above], right, -mag[above], "right, y < 0")
    assert np.all(table[1, 1][~above] == 0.0)
    # m = 0, y < 0, key window `shift` patterns lower
    magl = bf16_value(lo_pat - shift + np.arange(n))
    above = -magl > ymin
    check(table[0, 1][above], left, -magl[above], "left")
    assert np.all(table[0, 1][~above] == 0.0)
    assert np.all(table[0, 0] == 0.0)                        # left of the minimum with y >= 0: none
    # the window's ends stand in for everything beyond them
    assert abs(table[1, 0][-1] - 1.0) < 1e-5 and abs(table[1, 0][0] - 0.5) < 1e-3
    assert abs(table[0, 1][0]) < 1e-4 and table[0, 1][0] <= 0.0


def _eval_backward_cubics(kind, y, right):
    """The float32 backward table as the kernel indexes it (csrc/gelu.hip, gelu_composite),
    evaluated in float64 at arbitrary float64 y."""
    K = kind.upper()
    rows = f32(ARR[f"tempo_gelu_bwd_table_{kind}"]).reshape(-1, 4)
    nr, nl, nt = DEF[f"TEMPO_GELU_{K}_NR"], DEF[f"TEMPO_GELU_{K}_NL"], DEF["TEMPO_GELU_NT"]
    assert rows.shape[0] == DEF[f"TEMPO_GELU_{K}_BWD_ROWS"] == nr + nl + nt
    ystar = f32([DEF[f"TEMPO_GELU_{K}_YSTAR_HI"]])[0] + f32([DEF[f"TEMPO_GELU_{K}_YSTAR_LO"]])[0]
    s = np.sqrt(np.maximum(y - ystar, 0.0))
    if right:
        u = np.minimum(s * DEF["TEMPO_GELU_CR"], nr - 1e-5)
        idx, z = np.floor(u).astype(int), u - np.floor(u)
    else:
        u = np.minimum(s * DEF["TEMPO_GELU_CL"], nl - 1e-5)
        idx, z = nr + np.floor(u).astype(int), u - np.floor(u)
        sub, top = DEF["TEMPO_GELU_TAIL_SUB_BITS"], DEF["TEMPO_GELU_TAIL_TOP_EXP"]
        tail = -y < 2.0 ** top
        mant, ex = np.frexp(np.where(tail, -y, 1.0))        # -y = mant 2^ex, mant in [0.5, 1)
        frac = (2.0 * mant - 1.0) * (1 << sub)              # mantissa fraction in quarter units
        piece = (top - ex) * (1 << sub) + ((1 << sub) - 1 - np.floor(frac).astype(int))
        piece = np.minimum(piece, nt - 1)
        zt = (frac - np.floor(frac)) * float(1 << (23 - sub))
        idx, z = np.where(tail, nr + nl + piece, idx), np.where(tail, zt, z)
    c = rows[idx]
    return ((c[:, 3] * z + c[:, 2]) * z + c[:, 1]) * z + c[:, 0]


def test_backward_cubic_rows_follow_forward_samples(sampled):
    kind, left, right, ymin = sampled
    worst = 0.0
    for branch, is_right in ((right, True), (left, False)):
        x, y, d = branch
        sel = slice(None, None, 7)                           # a million samples per branch
        ys, ds = y[sel], d[sel]
        got = _eval_backward_cubics(kind, ys, is_right)
        err = np.abs(got - ds)
        # the fit's ~3e-8 plus the float32 rounding of the coefficients.  Within 1e-9 of the
        # minimum value (less than a tenth of y's float32 spacing there) d ~ sqrt(y - y*) turns
        # the 2^-53 rounding of torch's y and of the table's two-float y* into ~1e-6: those few
        # samples only have to be as small as d is there
        near = ys - ymin < 1e-9
        assert err[~near].max() <= 2e-7, (kind, is_right, float(ys[~near][np.argmax(err[~near])]),
                                          float(err[~near].max()))
        assert np.all(np.abs(got[near]) <= 5e-5) and np.all(np.abs(ds[near]) <= 5e-5)
        worst = max(worst, float(err.max()))
    assert worst > 0.0


def test_forward_erfc_polynomial_gives_the_normal_distribution_function():
    """The float32 erf forward has no table: it evaluates 1/2 erfc(|x|/sqrt 2) as
    t h(u) exp2(-w^2) (csrc/gelu.hip, gelu_erf_value) from the constants in the table file.
    The same steps in numpy float32 arithmetic, against torch's float64 erfc."""
    f = np.float32
    one = lambda name: f32([DEF[name]])[0].astype(f)
    q = [one(f"TEMPO_GELU_ERFC_Q{i}") for i in range(DEF["TEMPO_GELU_ERFC_DEG"] + 1)]
    x = np.concatenate([np.linspace(-9.0, 9.0, 2_000_001),
                        [0.0, 1e-30, -1e-30, 1e-12, -1e-12, 1e-6, -1e-6, 12.0, -12.0]]).astype(f)
    w = np.abs(x) * one("TEMPO_GELU_ERFC_W_SCALE")
    t = f(1) / (w * one("TEMPO_GELU_ERFC_T_FACTOR") + f(1))
    u = t * one("TEMPO_GELU_ERFC_UA") + one("TEMPO_GELU_ERFC_UB")
    h = np.full_like(u, q[-1])
    for c in q[-2::-1]:
        h = h * u + c
    with np.errstate(under="ignore"):
        half_erfc = t * h * np.exp2(-(w * w)).astype(f)
    phi = np.where(x < 0, half_erfc, f(1) - half_erfc).astype(np.float64)
    x64 = x.astype(np.float64)
    ref = 0.5 * torch.special.erfc(torch.tensor(-x64 / math.sqrt(2.0))).numpy()   # Phi(x), no cancellation
    rel = np.abs(phi - ref) / ref
    # float32 steps: ~1e-6 where GELU matters; on the far left tail the rounding of w^2 in the
    # exponent grows with w^2 (|GELU| < 1e-5 there)
    assert rel[x >= -4.0].max() <= 2.5e-6 and rel[x >= -9.0].max() <= 1e-5
    y, _ = act(x64, "erf")
    assert np.all(np.abs(x64 * phi - y) <= 2.5e-6 * np.abs(y) + 1e-9)
    tiny = (np.abs(x64) <= 1e-3) & (x64 != 0)              # next to the zero of GELU: truly relative
    assert np.all(np.abs(x64 * phi - y)[tiny] <= 5e-7 * np.abs(y)[tiny])
    assert np.all(np.sign(x64 * phi)[tiny] == np.sign(x64)[tiny])
    # beyond the fitted range the exponential decides: 1 on the right, still the tail on the left
    assert phi[x == 12.0][0] == 1.0 and abs(phi[x == -12.0][0] / ref[x == -12.0][0] - 1.0) < 1e-3


def test_committed_tables_equal_a_fresh_run_of_the_generator(tmp_path):
    out = tmp_path / "gelu_tables.inc"
    subprocess.run([sys.executable, GEN, str(out)], check=True, capture_output=True, timeout=600)
    assert out.read_bytes() == open(INC, "rb").read()
