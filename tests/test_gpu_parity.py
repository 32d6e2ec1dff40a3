"""Parity of the HIP path (through the C ABI) against the float64 oracle, element by element.

Backward kernels are fed the oracle's stored forward results (rounded to the storage dtype),
so that both sides consume identical bits.  Masks must match bit for bit; floating-point
results within helpers.TOL under helpers.rel_err.
"""
import numpy as np
import pytest
import torch

from helpers import TOL, rel_err
from oracle import tempo_oracle as O
from paper_2210_10246_amd import workloads as W

pytestmark = pytest.mark.gpu

TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2210_10246_amd import binding
    binding.load()
    return binding


def dev(a, dt):
    """float64 array (already representable in dt) -> CUDA tensor of dtype dt."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(TDT[dt]).cuda()


def host(t):
    return t.detach().cpu().to(torch.float64).numpy()


def words(t):
    return t.detach().cpu().numpy().view(np.uint32)


def stored(rng, shape, dt, scale=1.0):
    return O.round_to_dtype(rng.standard_normal(shape) * scale, dt)


# ------------------------------------------------------------------ GELU (and SiLU, Sec. 5.1)
GELU_SIZES = [1, 7, 8, 31, 32, 33, 1000, 4099, 2 * 128 * 3072, 1_000_003]
ACT_KINDS = ["erf", "tanh", "silu"]


def act_fwd(B, kind, x, y, mask):
    if kind == "silu":
        B.tempo_silu_fwd(x, y, mask)
    else:
        B.tempo_gelu_fwd(x, y, mask, kind)


def act_bwd(B, kind, dy, y, mask, dx):
    if kind == "silu":
        B.tempo_silu_bwd(dy, y, mask, dx)
    else:
        B.tempo_gelu_bwd(dy, y, mask, dx, kind)


@pytest.mark.parametrize("kind", ACT_KINDS)
@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("n", GELU_SIZES)
def test_gelu_fwd(B, n, dt, kind):
    rng = np.random.default_rng(n)
    x = stored(rng, n, dt, 1.5)
    if n >= 1000:  # a few exact branch points, far tails and signed zeros
        xs32 = np.float32(O.GELU_XSTAR[kind])
        edge = [xs32, np.nextafter(xs32, np.float32(-9)), np.nextafter(xs32, np.float32(9)),
                0.0, -0.0, 7.99, 8.0, 9.5, -7.99, -8.0, -9.5, 30.0, -30.0, 15.9, 16.0, 17.0,
                -15.9, -16.0, -17.0, -60.0, -87.0, -90.0, -200.0, 200.0]
        x[: len(edge)] = O.round_to_dtype(np.array(edge, dtype=np.float64), dt)
    y_ref, m_ref = O.gelu_fwd(x, kind, dt)
    xd = dev(x, dt)
    yd = torch.full_like(xd, 7.0)
    md = torch.full((B.mask_words(n),), -1, dtype=torch.int32, device="cuda")
    act_fwd(B, kind, xd, yd, md)
    torch.cuda.synchronize()
    assert np.array_equal(words(md), O.pack_bits(m_ref)), "mask differs"
    assert rel_err(host(yd), y_ref) <= TOL[dt]
    # in place: the input's storage need not survive
    md2 = torch.zeros_like(md)
    act_fwd(B, kind, xd, xd, md2)
    torch.cuda.synchronize()
    assert torch.equal(xd, yd) and torch.equal(md, md2)


@pytest.mark.parametrize("kind", ACT_KINDS)
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_gelu_fwd_next_to_its_zero(B, dt, kind):
    """x = 0 is a plain zero of the activation, not a cancellation point: for |x| from 1e-12 to
    1e-3 the error is held relative to the value itself (no RMS floor), the sign must be that
    of x, and +-0 map to +-0."""
    mag = np.logspace(-12, -3, 1000)
    x = O.round_to_dtype(np.concatenate([mag, -mag, [0.0, -0.0]]), dt)
    y_ref, m_ref = O.gelu_fwd(x, kind, dt)
    xd = dev(x, dt)
    yd = torch.full_like(xd, 7.0)
    md = torch.empty(B.mask_words(x.size), dtype=torch.int32, device="cuda")
    act_fwd(B, kind, xd, yd, md)
    torch.cuda.synchronize()
    got = host(yd)
    assert np.array_equal(words(md), O.pack_bits(m_ref))
    assert np.array_equal(np.signbit(got), np.signbit(x))
    assert got[-2] == 0.0 and got[-1] == 0.0
    nz = x != 0
    assert np.max(np.abs(got[nz] - y_ref[nz]) / np.abs(y_ref[nz])) <= TOL[dt]


@pytest.mark.parametrize("kind", ACT_KINDS)
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_activation_does_not_depend_on_launch_shape(B, dt, kind):
    """Knobs 0, 1 (pieces per lane), 13 (bf16 forward workgroup size) and 15 (float32 lanes per
    workgroup): every shape gives bit-identical y, mask and dx, equal to the default's."""
    n = 300_007
    rng = np.random.default_rng(15)
    xd, dyd = dev(stored(rng, n, dt, 1.5), dt), dev(stored(rng, n, dt), dt)
    keys = (0, 1, 13, 15)
    old = [B.tempo_get_launch_param(k) for k in keys]
    results = []
    try:
        shapes = [tuple(old)] + [(k0, k1, g, t) for k0 in (1, 2, 4) for k1 in (1, 2, 4)
                                 for g, t in ((1, 64), (65536, 128), (old[2], 256), (old[2], 1))]
        for shape in shapes:
            for k, v in zip(keys, shape):
                B.tempo_set_launch_param(k, v)
            yd = torch.full_like(xd, 7.0)
            md = torch.zeros(B.mask_words(n), dtype=torch.int32, device="cuda")
            dxd = torch.full_like(xd, 7.0)
            act_fwd(B, kind, xd, yd, md)
            act_bwd(B, kind, dyd, yd, md, dxd)
            torch.cuda.synchronize()
            results.append((yd, md, dxd))
    finally:
        for k, v in zip(keys, old):
            B.tempo_set_launch_param(k, v)
    for r in results[1:]:
        assert all(torch.equal(a, b) for a, b in zip(results[0], r))


@pytest.mark.parametrize("kind", ACT_KINDS)
@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("n", [1, 9, 33, 4099, 300_000])
def test_gelu_bwd(B, n, dt, kind):
    rng = np.random.default_rng(100 + n)
    x = stored(rng, n, dt, 1.7)
    if n >= 4099:
        lo, hi = (-45.0, 22.0) if kind == "silu" else (-14.0, 8.0)
        x[:2000] = O.round_to_dtype(rng.uniform(lo, hi, 2000), dt)                  # both tails
        x[2000:3000] = O.round_to_dtype(O.GELU_XSTAR[kind] + rng.normal(size=1000) * 1e-2, dt)
    y, m = O.gelu_fwd(x, kind, dt)
    dy = stored(rng, n, dt)
    ref = O.gelu_bwd(dy, y, m, kind, dt)
    dyd, yd = dev(dy, dt), dev(y, dt)
    md = torch.from_numpy(O.pack_bits(m).view(np.int32)).cuda()
    dxd = torch.empty_like(dyd)
    act_bwd(B, kind, dyd, yd, md, dxd)
    torch.cuda.synchronize()
    assert rel_err(host(dxd), ref) <= TOL[dt]
    act_bwd(B, kind, dyd, yd, md, dyd)     # dx may alias dy
    torch.cuda.synchronize()
    assert torch.equal(dyd, dxd)


@pytest.mark.parametrize("kind", ACT_KINDS)
def test_gelu_bwd_edge_values(B, kind):
    ys = O.GELU_YSTAR[kind]
    y = np.array([ys - 1e-3, ys, 0.0, -0.0, 0.0, np.inf, np.nan, 1e-30, -1e-30, -1e-45, 20.0, 6.5,
                  -0.0625, -0.06249, -0.1, 1e-20, 17.5, 18.5, 40.0, 0.9 * ys, 0.9 * ys, 0.999 * ys,
                  0.999 * ys, -1e-8, -1e-10], dtype=np.float64)
    y = O.round_to_dtype(y, "f32")
    m = np.array([1, 1, 0, 0, 1, 1, 1, 0, 0, 0, 1, 1, 0, 0, 0, 1, 1, 1, 1, 0, 1, 0, 1, 0, 0],
                 dtype=bool)
    dy = np.ones_like(y)
    ref = O.gelu_bwd(dy, y, m, kind, "f32")
    dxd = torch.empty(y.size, dtype=torch.float32, device="cuda")
    md = torch.from_numpy(O.pack_bits(m).view(np.int32)).cuda()
    act_bwd(B, kind, dev(dy, "f32"), dev(y, "f32"), md, dxd)
    got = host(dxd)
    assert np.isnan(got[6]) and np.isnan(ref[6])
    ok = ~np.isnan(ref)
    np.testing.assert_allclose(got[ok], ref[ok], rtol=0, atol=5e-7)


@pytest.mark.parametrize("kind", ["erf", "silu"])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_gelu_round_trip_against_input_based_gradient(B, dt, kind):
    # fwd then bwd on the GPU vs dy * GELU'(x): the lossy part is only the storage of y
    rng = np.random.default_rng(7)
    n = 200_000
    x = stored(rng, n, dt, 1.5)
    dy = stored(rng, n, dt)
    xd, dyd = dev(x, dt), dev(dy, dt)
    yd = torch.empty_like(xd)
    md = torch.empty(B.mask_words(n), dtype=torch.int32, device="cuda")
    dxd = torch.empty_like(xd)
    act_fwd(B, kind, xd, yd, md)
    act_bwd(B, kind, dyd, yd, md, dxd)
    ref = O.gelu_bwd_from_input(dy, x, kind)
    err = np.abs(host(dxd) - ref)
    # the square-root singularity at the minimum amplifies the rounding of y: |dd| ~ sqrt(ulp)
    assert err.max() <= (5e-3 if dt == "f32" else 0.15) * max(1.0, np.abs(dy).max())
    assert np.sqrt(np.mean(err**2)) <= (2e-6 if dt == "f32" else 6e-3)


# ------------------------------------------------------------------ LayerNorm
LN_SHAPES = [(256, 768), (5, 1024), (37, 768), (3, 8), (9, 64), (7, 100), (4, 4096), (3, 2048),
             (2, 4104), (1, 1), (6, 1536), (300, 1024), (3, 3072), (1030, 256),
             # beyond 4096 columns: register-resident up to 8192 (float32 with 6 or 8 pieces per
             # lane), the any-shape kernels beyond and for rows that are not whole pieces
             (5, 8192), (70, 6144), (300, 5120), (2, 8200), (3, 8190), (600, 7168),
             # any-shape backward: column sums in registers (up to 2048 and up to 5120 columns) / in memory
             (1500, 1001), (2000, 4100), (3, 9300)]


@pytest.mark.parametrize("eps", [1e-12, 1e-5])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", LN_SHAPES)
def test_layernorm_fwd(B, shape, dt, eps):
    N, M = shape
    rng = np.random.default_rng(N * 10007 + M)
    x = stored(rng, shape, dt) + O.round_to_dtype(rng.normal(size=(N, 1)), dt)
    x = O.round_to_dtype(x, dt)
    gamma = O.round_to_dtype(1 + 0.1 * rng.standard_normal(M), "f32")
    beta = O.round_to_dtype(0.1 * rng.standard_normal(M), "f32")
    if M == 1:
        eps = 1e-5
    y_ref, rstd_ref, mean_ref = O.layernorm_fwd(x, gamma, beta, eps, dt)
    xd, gd, bd = dev(x, dt), dev(gamma, "f32"), dev(beta, "f32")
    yd = torch.empty_like(xd)
    rd = torch.empty(N, dtype=torch.float32, device="cuda")
    md = torch.empty(N, dtype=torch.float32, device="cuda")
    B.tempo_layernorm_fwd(xd, gd, bd, yd, rd, md, eps)
    torch.cuda.synchronize()
    assert rel_err(host(yd), y_ref) <= TOL[dt]
    assert rel_err(host(rd), rstd_ref) <= TOL["f32"]
    assert rel_err(host(md), mean_ref) <= TOL["f32"]
    rd2 = torch.empty_like(rd)
    B.tempo_layernorm_fwd(xd, gd, bd, xd, rd2, None, eps)     # in place, no mean
    torch.cuda.synchronize()
    assert torch.equal(xd, yd) and torch.equal(rd, rd2)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", LN_SHAPES)
def test_layernorm_bwd(B, shape, dt):
    N, M = shape
    eps = 1e-5      # M == 1: every row is its own mean, so xhat = 0, dx = 0 and dgamma = 0 exactly
    rng = np.random.default_rng(N * 7919 + M)
    x = stored(rng, shape, dt)
    gamma = O.round_to_dtype(1 + 0.1 * rng.standard_normal(M), "f32")
    beta = O.round_to_dtype(0.1 * rng.standard_normal(M), "f32")
    dy = stored(rng, shape, dt)
    y, rstd, _ = O.layernorm_fwd(x, gamma, beta, eps, dt)
    dx_ref, dg_ref, db_ref = O.layernorm_bwd(dy, y, gamma, beta, rstd, dt)
    dyd, yd = dev(dy, dt), dev(y, dt)
    gd, bd, rd = dev(gamma, "f32"), dev(beta, "f32"), dev(rstd, "f32")
    dxd = torch.empty_like(dyd)
    dgd = torch.empty(M, dtype=torch.float32, device="cuda")
    dbd = torch.empty(M, dtype=torch.float32, device="cuda")
    ws = torch.empty(max(B.tempo_layernorm_bwd_workspace_bytes(N, M), 16), dtype=torch.uint8, device="cuda")
    B.tempo_layernorm_bwd(dyd, yd, gd, bd, rd, dxd, dgd, dbd, ws)
    torch.cuda.synchronize()
    if M == 1:
        # dx is nothing but the cancellation dy*gamma - dy*gamma (the stored y differs from beta
        # only by its rounding): the error is measured against the terms that cancel
        terms = np.abs(dy * gamma * rstd[:, None]).max()
        assert np.abs(host(dxd) - dx_ref).max() <= 4 * 2.0 ** -24 * terms
    else:
        assert rel_err(host(dxd), dx_ref) <= TOL[dt]
    assert rel_err(host(dgd), dg_ref) <= TOL["f32"]
    assert rel_err(host(dbd), db_ref) <= TOL["f32"]
    dg2, db2 = torch.empty_like(dgd), torch.empty_like(dbd)
    B.tempo_layernorm_bwd(dyd, yd, gd, bd, rd, dyd, dg2, db2, ws)    # dx may alias dy
    torch.cuda.synchronize()
    assert torch.equal(dyd, dxd)
    assert torch.equal(dg2, dgd) and torch.equal(db2, dbd)          # fixed summation order
    with pytest.raises(B.TempoError):
        B.tempo_layernorm_bwd(dyd, yd, gd, bd, rd, dxd, dgd, dbd, ws[:2 * M * 4 - 1])   # under one slot


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(37, 2048), (5, 3072), (9, 4096), (3, 1032), (600, 1536)])
def test_layernorm_row_over_one_or_several_waves(B, shape, dt):
    """Long rows: the same results whether one wave or 2-4 waves own a row (knobs 10, 11),
    with row counts that leave lane groups without a row in the last batch."""
    N, M = shape
    eps = 1e-5
    rng = np.random.default_rng(N * 31 + M)
    x = stored(rng, shape, dt)
    gamma = O.round_to_dtype(1 + 0.1 * rng.standard_normal(M), "f32")
    beta = O.round_to_dtype(0.1 * rng.standard_normal(M), "f32")
    dy = stored(rng, shape, dt)
    y, rstd, mean = O.layernorm_fwd(x, gamma, beta, eps, dt)
    dx_ref, dg_ref, db_ref = O.layernorm_bwd(dy, y, gamma, beta, rstd, dt)
    xd, dyd, yd0 = dev(x, dt), dev(dy, dt), dev(y, dt)
    gd, bd, rd0 = dev(gamma, "f32"), dev(beta, "f32"), dev(rstd, "f32")
    old = B.tempo_get_launch_param(10), B.tempo_get_launch_param(11)
    try:
        for max_pieces in (1, 2, 4, 16):
            B.tempo_set_launch_param(10, max_pieces)
            B.tempo_set_launch_param(11, max_pieces)
            yd = torch.full_like(xd, 3.0)
            rd = torch.full((N,), 3.0, dtype=torch.float32, device="cuda")
            md = torch.full((N,), 3.0, dtype=torch.float32, device="cuda")
            B.tempo_layernorm_fwd(xd, gd, bd, yd, rd, md, eps)
            torch.cuda.synchronize()
            assert rel_err(host(yd), y) <= TOL[dt], max_pieces
            assert rel_err(host(rd), rstd) <= TOL["f32"], max_pieces
            assert rel_err(host(md), mean) <= TOL["f32"], max_pieces
            dxd = torch.full_like(dyd, 3.0)
            dgd = torch.full((M,), 3.0, dtype=torch.float32, device="cuda")
            dbd = torch.full((M,), 3.0, dtype=torch.float32, device="cuda")
            ws = torch.empty(B.tempo_layernorm_bwd_workspace_bytes(N, M), dtype=torch.uint8, device="cuda")
            B.tempo_layernorm_bwd(dyd, yd0, gd, bd, rd0, dxd, dgd, dbd, ws)
            torch.cuda.synchronize()
            assert rel_err(host(dxd), dx_ref) <= TOL[dt], max_pieces
            assert rel_err(host(dgd), dg_ref) <= TOL["f32"], max_pieces
            assert rel_err(host(dbd), db_ref) <= TOL["f32"], max_pieces
    finally:
        B.tempo_set_launch_param(10, old[0])
        B.tempo_set_launch_param(11, old[1])


def test_layernorm_bwd_grid_of_more_than_4096_workgroups(B):
    """Knob 12 raised so that the backward does not loop: one workgroup per batch of rows,
    here 4100 of them, and every row has to be covered (dx written, dgamma/dbeta complete)."""
    N, M, dt = 64 * 4100 - 5, 64, "bf16"
    rng = np.random.default_rng(4100)
    x = stored(rng, (N, M), dt)
    gamma = O.round_to_dtype(1 + 0.1 * rng.standard_normal(M), "f32")
    beta = O.round_to_dtype(0.1 * rng.standard_normal(M), "f32")
    dy = stored(rng, (N, M), dt)
    y, rstd, _ = O.layernorm_fwd(x, gamma, beta, 1e-5, dt)
    dx_ref, dg_ref, db_ref = O.layernorm_bwd(dy, y, gamma, beta, rstd, dt)
    dyd, yd = dev(dy, dt), dev(y, dt)
    gd, bd, rd = dev(gamma, "f32"), dev(beta, "f32"), dev(rstd, "f32")
    old = B.tempo_get_launch_param(12)
    try:
        B.tempo_set_launch_param(12, 64)
        need = B.tempo_layernorm_bwd_workspace_bytes(N, M)
        assert need > 4096 * 2 * M * 4            # more than 4096 partial slots
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        dxd = torch.full_like(dyd, 3.0)
        dgd = torch.full((M,), 3.0, dtype=torch.float32, device="cuda")
        dbd = torch.full((M,), 3.0, dtype=torch.float32, device="cuda")
        B.tempo_layernorm_bwd(dyd, yd, gd, bd, rd, dxd, dgd, dbd, ws)
        torch.cuda.synchronize()
    finally:
        B.tempo_set_launch_param(12, old)
    assert rel_err(host(dxd), dx_ref) <= TOL[dt]
    assert rel_err(host(dgd), dg_ref) <= TOL["f32"]
    assert rel_err(host(dbd), db_ref) <= TOL["f32"]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(3001, 768), (2100, 2048), (1101, 4096), (4099, 256)])
def test_layernorm_fwd_looping_workgroups(B, shape, dt):
    """More row batches than workgroups: workgroups walk the batches, prefetching the next."""
    N, M = shape
    rng = np.random.default_rng(N + M)
    x = stored(rng, shape, dt)
    gamma = O.round_to_dtype(1 + 0.1 * rng.standard_normal(M), "f32")
    beta = O.round_to_dtype(0.1 * rng.standard_normal(M), "f32")
    y, rstd, mean = O.layernorm_fwd(x, gamma, beta, 1e-5, dt)
    xd, gd, bd = dev(x, dt), dev(gamma, "f32"), dev(beta, "f32")
    old = B.tempo_get_launch_param(2), B.tempo_get_launch_param(10)
    try:
        for cap, max_pieces in ((1, 16), (1, 2), (65536, 16)):
            B.tempo_set_launch_param(2, cap)
            B.tempo_set_launch_param(10, max_pieces)
            yd = torch.full_like(xd, 3.0)
            rd = torch.full((N,), 3.0, dtype=torch.float32, device="cuda")
            md = torch.full((N,), 3.0, dtype=torch.float32, device="cuda")
            B.tempo_layernorm_fwd(xd, gd, bd, yd, rd, md, 1e-5)
            torch.cuda.synchronize()
            assert rel_err(host(yd), y) <= TOL[dt], (cap, max_pieces)
            assert rel_err(host(rd), rstd) <= TOL["f32"], (cap, max_pieces)
            assert rel_err(host(md), mean) <= TOL["f32"], (cap, max_pieces)
    finally:
        B.tempo_set_launch_param(2, old[0])
        B.tempo_set_launch_param(10, old[1])


# ------------------------------------------------------------------ attention softmax -> dropout
ATTN_CASES = [
    # B, A, Sq, Sk, mask, p
    (2, 12, 128, 128, "none", 0.1),
    (3, 2, 128, 128, "padding", 0.1),
    (2, 2, 512, 512, "padding", 0.1),
    (1, 2, 1024, 1024, "causal", 0.1),
    (1, 2, 5, 40, "none", 0.1),        # rows end inside a mask word: byte stores
    (2, 1, 7, 100, "padding", 0.25),   # rows not a multiple of 8: scalar path
    (1, 1, 3, 8, "causal", 0.5),
    (1, 3, 4, 64, "causal", 0.1),      # Sq != Sk
    (2, 2, 16, 96, "zero_len", 0.1),   # one sequence fully masked
    (1, 2, 33, 2048, "causal", 0.1),
    (1, 1, 9, 3072, "padding", 0.1),
    (1, 1, 5, 4104, "none", 0.1),      # longer than the register path in float32
    (1, 2, 7, 8192, "causal", 0.1),    # longest row of the register path in bfloat16
    (2, 1, 5, 1544, "padding", 0.1),   # long row ending inside a mask word
    (2, 2, 64, 160, "padding", 0.0),   # p = 0: everything kept
    (1, 1, 70, 1, "none", 0.1),
    # rows of any length held in registers by one wave (4, 16 or 32 chunks of 64 elements), the
    # keep bits of 448 elements drawn together; and the any-length kernels beyond 2048
    (1, 1, 70, 449, "none", 0.3),
    (2, 1, 5, 1001, "causal", 0.1),
    (1, 2, 3, 1543, "padding", 0.1),
    (1, 1, 3, 2055, "none", 0.1),
]


def _attn_inputs(case, dt, rng):
    Bn, A, Sq, Sk, mask, p = case
    s = stored(rng, (Bn, A, Sq, Sk), dt, 0.125 if Sk >= 128 else 1.0)
    key_len, causal = None, False
    if mask == "padding":
        key_len = rng.integers(max(1, Sk // 2), Sk + 1, size=Bn).astype(np.int32)
    elif mask == "zero_len":
        key_len = np.array([0] + [Sk - 3] * (Bn - 1), dtype=np.int32)
    elif mask == "causal":
        causal = True
    return s, key_len, causal, np.float32(p)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("case", ATTN_CASES, ids=lambda c: "x".join(map(str, c)))
def test_attn_fwd(B, case, dt):
    rng = np.random.default_rng(hash(case[:4]) % (1 << 31))
    s, key_len, causal, p = _attn_inputs(case, dt, rng)
    seed, offset = 0x5EED0000ABCD1234, (1 << 33) + 17
    P_ref, out_ref, K_ref = O.attn_softmax_dropout_fwd(s, key_len, causal, p, seed, offset, dt)
    sd = dev(s, dt)
    kd = None if key_len is None else torch.from_numpy(key_len).cuda()
    Pd = torch.full_like(sd, 3.0)
    od = torch.full_like(sd, 3.0)
    n = s.size
    md = torch.full((B.mask_words(n),), -1, dtype=torch.int32, device="cuda")
    B.tempo_attn_softmax_dropout_fwd(sd, kd, causal, Pd, od, md, float(p), seed, offset)
    torch.cuda.synchronize()
    assert np.array_equal(words(md), O.pack_bits(K_ref)), "keep mask differs"
    assert rel_err(host(Pd), P_ref) <= TOL[dt]
    assert rel_err(host(od), out_ref) <= TOL[dt]
    valid = O.attention_valid(*s.shape, key_len, causal)
    assert np.all(host(Pd)[~valid] == 0) and np.all(host(od)[~K_ref] == 0)
    # out is optional; P may overwrite the scores
    md2 = torch.zeros_like(md)
    B.tempo_attn_softmax_dropout_fwd(sd, kd, causal, sd, None, md2, float(p), seed, offset)
    torch.cuda.synchronize()
    assert torch.equal(sd, Pd) and torch.equal(md, md2)
    # backward's recomputed dropout output is bit-identical to the forward's (same stored P)
    dod = dev(stored(rng, s.shape, dt), dt)
    dsd, ord_ = torch.empty_like(sd), torch.empty_like(sd)
    B.tempo_attn_softmax_dropout_bwd(dod, Pd, md, dsd, ord_, float(p))
    torch.cuda.synchronize()
    assert torch.equal(ord_.view(torch.int16 if dt == "bf16" else torch.int32),
                       od.view(torch.int16 if dt == "bf16" else torch.int32))


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("case", ATTN_CASES, ids=lambda c: "x".join(map(str, c)))
def test_attn_bwd(B, case, dt):
    rng = np.random.default_rng(hash(case[:4]) % (1 << 31) + 1)
    s, key_len, causal, p = _attn_inputs(case, dt, rng)
    seed, offset = 99, 5
    P, _, K = O.attn_softmax_dropout_fwd(s, key_len, causal, p, seed, offset, dt)
    dout = stored(rng, s.shape, dt)
    dS_ref, out_re_ref = O.attn_softmax_dropout_bwd(dout, P, K, p, dt)
    dod, Pd = dev(dout, dt), dev(P, dt)
    md = torch.from_numpy(O.pack_bits(K).view(np.int32)).cuda()
    dsd, ord_ = torch.empty_like(dod), torch.empty_like(dod)
    B.tempo_attn_softmax_dropout_bwd(dod, Pd, md, dsd, ord_, float(p))
    torch.cuda.synchronize()
    assert rel_err(host(dsd), dS_ref) <= TOL[dt]
    assert rel_err(host(ord_), out_re_ref) <= TOL[dt]
    B.tempo_attn_softmax_dropout_bwd(dod, Pd, md, dod, None, float(p))   # in place, no Out
    torch.cuda.synchronize()
    assert torch.equal(dod, dsd)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("case", ATTN_CASES, ids=lambda c: "x".join(map(str, c)))
def test_attn_bwd_without_stored_mask(B, case, dt):
    """Backward that draws the keep bits again from (seed, offset) against the oracle's backward
    on the oracle's mask, and bit for bit against the mask-reading backward."""
    rng = np.random.default_rng(hash(case[:4]) % (1 << 31) + 2)
    s, key_len, causal, p = _attn_inputs(case, dt, rng)
    seed, offset = 0xC0FFEE0000000001, (1 << 40) + 3
    P, _, K = O.attn_softmax_dropout_fwd(s, key_len, causal, p, seed, offset, dt)
    dout = stored(rng, s.shape, dt)
    dS_ref, out_re_ref = O.attn_softmax_dropout_bwd(dout, P, K, p, dt)
    dod, Pd = dev(dout, dt), dev(P, dt)
    dsd, ord_ = torch.empty_like(dod), torch.empty_like(dod)
    B.tempo_attn_softmax_dropout_bwd_regen(dod, Pd, dsd, ord_, float(p), seed, offset)
    torch.cuda.synchronize()
    assert rel_err(host(dsd), dS_ref) <= TOL[dt]
    assert rel_err(host(ord_), out_re_ref) <= TOL[dt]
    assert np.array_equal(host(ord_) != 0, (K & (P != 0)))
    md = torch.from_numpy(O.pack_bits(K).view(np.int32)).cuda()
    ds2, or2 = torch.empty_like(dod), torch.empty_like(dod)
    B.tempo_attn_softmax_dropout_bwd(dod, Pd, md, ds2, or2, float(p))
    torch.cuda.synchronize()
    assert torch.equal(dsd, ds2) and torch.equal(ord_, or2)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("case", ATTN_CASES, ids=lambda c: "x".join(map(str, c)))
def test_attn_bwd_with_a_mask_of_one_byte_per_element(B, case, dt):
    """Backward fed the paper's mask layout (8-bit booleans, Sec. 3.3) against the oracle, and bit
    for bit against the backward that reads packed bits; any non-zero byte means kept."""
    rng = np.random.default_rng(hash(case[:4]) % (1 << 31) + 3)
    s, key_len, causal, p = _attn_inputs(case, dt, rng)
    seed, offset = 7, 9
    P, _, K = O.attn_softmax_dropout_fwd(s, key_len, causal, p, seed, offset, dt)
    dout = stored(rng, s.shape, dt)
    dS_ref, out_re_ref = O.attn_softmax_dropout_bwd(dout, P, K, p, dt)
    dod, Pd = dev(dout, dt), dev(P, dt)
    md = torch.from_numpy(O.pack_bits(K).view(np.int32)).cuda()
    ds0, or0 = torch.empty_like(dod), torch.empty_like(dod)
    B.tempo_attn_softmax_dropout_bwd(dod, Pd, md, ds0, or0, float(p))
    n = s.size
    pad = (-n) % 16
    for marks in (np.ones(n, dtype=np.uint8), rng.integers(1, 256, n).astype(np.uint8)):
        kb = torch.zeros(n + pad, dtype=torch.uint8, device="cuda")
        kb[:n] = torch.from_numpy(K.reshape(-1).astype(np.uint8) * marks).cuda()
        dsd, ord_ = torch.full_like(dod, 3.0), torch.full_like(dod, 3.0)
        B.tempo_attn_softmax_dropout_bwd_bytemask(dod, Pd, kb[:n], dsd, ord_, float(p))
        torch.cuda.synchronize()
        assert rel_err(host(dsd), dS_ref) <= TOL[dt]
        assert rel_err(host(ord_), out_re_ref) <= TOL[dt]
        assert torch.equal(dsd, ds0) and torch.equal(ord_, or0)
    kbool = torch.from_numpy(K.reshape(-1)).cuda()                     # a torch.bool tensor as it is
    B.tempo_attn_softmax_dropout_bwd_bytemask(dod, Pd, kbool, dod, None, float(p))   # in place, no Out
    torch.cuda.synchronize()
    assert torch.equal(dod, ds0)


@pytest.mark.parametrize("n", [1, 15, 16, 17, 31, 32, 33, 4096, 100_003, 3_000_000])
def test_mask_layout_conversion(B, n):
    rng = np.random.default_rng(n)
    K = rng.random(n) < 0.9
    bits = torch.from_numpy(O.pack_bits(K).view(np.int32)).cuda()
    pad = (-n) % 16
    bytes_d = torch.full((n + pad,), 7, dtype=torch.uint8, device="cuda")
    B.tempo_mask_bits_to_bytes(bits, bytes_d, n)
    torch.cuda.synchronize()
    got = bytes_d.cpu().numpy()
    assert np.array_equal(got[:n], K.astype(np.uint8))
    assert np.all(got[n:] == 7), "wrote past n"
    # and back; any non-zero byte counts as kept
    src = K.astype(np.uint8) * rng.integers(1, 256, n).astype(np.uint8)
    src_d = torch.from_numpy(src).cuda()
    back = torch.full((B.mask_words(n) + 4,), -1, dtype=torch.int32, device="cuda")
    B.tempo_mask_bytes_to_bits(src_d, back, n)
    torch.cuda.synchronize()
    w = words(back)
    assert np.array_equal(w[:B.mask_words(n)], O.pack_bits(K))
    assert np.all(w[B.mask_words(n):] == 0xFFFFFFFF), "wrote past the last word"


def test_byte_mask_from_forward_feeds_backward(B):
    """A mask kept as bytes (the paper's layout) converts back to the bits backward reads."""
    rng = np.random.default_rng(77)
    s = stored(rng, (2, 3, 48, 96), "bf16")
    sd = dev(s, "bf16")
    Pd, od = torch.empty_like(sd), torch.empty_like(sd)
    n = s.size
    md = torch.empty(B.mask_words(n), dtype=torch.int32, device="cuda")
    B.tempo_attn_softmax_dropout_fwd(sd, None, False, Pd, od, md, 0.1, 11, 12)
    kept = torch.empty(n, dtype=torch.uint8, device="cuda")
    B.tempo_mask_bits_to_bytes(md, kept, n)
    K = O.dropout_keep(n, np.float32(0.1), 11, 12)
    assert np.array_equal(kept.cpu().numpy(), K.astype(np.uint8))
    md2 = torch.zeros_like(md)
    B.tempo_mask_bytes_to_bits(kept, md2, n)
    assert torch.equal(md, md2)


def test_mask_does_not_depend_on_launch_shape(B):
    rng = np.random.default_rng(5)
    s = stored(rng, (2, 2, 64, 256), "bf16")
    sd = dev(s, "bf16")
    masks = []
    old = B.tempo_get_launch_param(4)
    for cap in (1, 3, 16):
        B.tempo_set_launch_param(4, cap)
        md = torch.zeros(B.mask_words(s.size), dtype=torch.int32, device="cuda")
        B.tempo_attn_softmax_dropout_fwd(sd, None, False, torch.empty_like(sd), None, md, 0.1, 42, 0)
        masks.append(md.cpu())
    B.tempo_set_launch_param(4, old)
    assert torch.equal(masks[0], masks[1]) and torch.equal(masks[0], masks[2])
    assert np.array_equal(words(masks[0]), O.pack_bits(O.dropout_keep(s.size, 0.1, 42, 0)))


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_attn_row_over_one_or_several_waves(B, dt):
    """Long rows: the same result whether one wave or 2-4 waves own a row (knob 8); the second
    lane group of the last row set has no row when Sq is odd."""
    rng = np.random.default_rng(8)
    s = stored(rng, (1, 2, 5, 1024), dt, 0.125)
    key_len = np.array([1000], dtype=np.int32)
    P_ref, out_ref, K_ref = O.attn_softmax_dropout_fwd(s, key_len, False, np.float32(0.1), 3, 4, dt)
    sd, kd = dev(s, dt), torch.from_numpy(key_len).cuda()
    old = B.tempo_get_launch_param(8)
    try:
        for max_pieces in (1, 2, 4, 16):
            B.tempo_set_launch_param(8, max_pieces)
            Pd, od = torch.full_like(sd, 3.0), torch.full_like(sd, 3.0)
            md = torch.full((B.mask_words(s.size),), -1, dtype=torch.int32, device="cuda")
            B.tempo_attn_softmax_dropout_fwd(sd, kd, False, Pd, od, md, 0.1, 3, 4)
            torch.cuda.synchronize()
            assert np.array_equal(words(md), O.pack_bits(K_ref)), max_pieces
            assert rel_err(host(Pd), P_ref) <= TOL[dt], max_pieces
            assert rel_err(host(od), out_ref) <= TOL[dt], max_pieces
    finally:
        B.tempo_set_launch_param(8, old)
    # backward, knob 9
    dout = stored(rng, s.shape, dt)
    dS_ref, out_re_ref = O.attn_softmax_dropout_bwd(dout, P_ref, K_ref, np.float32(0.1), dt)
    dod, Pd = dev(dout, dt), dev(P_ref, dt)
    md = torch.from_numpy(O.pack_bits(K_ref).view(np.int32)).cuda()
    old = B.tempo_get_launch_param(9)
    try:
        for max_pieces in (1, 2, 4, 16):
            B.tempo_set_launch_param(9, max_pieces)
            for regen in (False, True):
                dsd, ord_ = torch.full_like(dod, 3.0), torch.full_like(dod, 3.0)
                if regen:
                    B.tempo_attn_softmax_dropout_bwd_regen(dod, Pd, dsd, ord_, 0.1, 3, 4)
                else:
                    B.tempo_attn_softmax_dropout_bwd(dod, Pd, md, dsd, ord_, 0.1)
                torch.cuda.synchronize()
                assert rel_err(host(dsd), dS_ref) <= TOL[dt], (max_pieces, regen)
                assert rel_err(host(ord_), out_re_ref) <= TOL[dt], (max_pieces, regen)
    finally:
        B.tempo_set_launch_param(9, old)


def test_non_default_stream(B):
    st = torch.cuda.Stream()
    rng = np.random.default_rng(6)
    x = stored(rng, 5000, "f32")
    xd = dev(x, "f32")
    yd = torch.empty_like(xd)
    md = torch.empty(B.mask_words(x.size), dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        B.tempo_gelu_fwd(xd, yd, md, "erf")
    st.synchronize()
    y_ref, m_ref = O.gelu_fwd(x, "erf", "f32")
    assert rel_err(host(yd), y_ref) <= TOL["f32"] and np.array_equal(words(md), O.pack_bits(m_ref))


@pytest.mark.parametrize("N", [64, 40_000])       # 40 000 rows: the LayerNorm kernels loop
def test_hip_graph_replays_match_eager(B, N):
    """The benchmark replays captured HIP graphs: every replay must reproduce the eagerly
    launched results, with the program's own eager work and synchronisations in between."""
    rng = np.random.default_rng(11)
    dt = "bf16"
    M, n = 1024, 64 * 4096
    x = dev(stored(rng, n, dt), dt)
    dy = dev(stored(rng, n, dt), dt)
    lx = dev(stored(rng, (N, M), dt), dt)
    ldy = dev(stored(rng, (N, M), dt), dt)
    gamma = dev(O.round_to_dtype(1 + 0.1 * rng.standard_normal(M), "f32"), "f32")
    beta = dev(O.round_to_dtype(0.1 * rng.standard_normal(M), "f32"), "f32")
    s = dev(stored(rng, (2, 2, 128, 128), dt, 0.125), dt)
    do = dev(stored(rng, (2, 2, 128, 128), dt), dt)
    kl = torch.tensor([100, 128], dtype=torch.int32, device="cuda")
    ws = torch.empty(B.tempo_layernorm_bwd_workspace_bytes(N, M), dtype=torch.uint8, device="cuda")

    def fresh():
        return dict(y=torch.empty_like(x), m=torch.empty(B.mask_words(n), dtype=torch.int32, device="cuda"),
                    dx=torch.empty_like(x), ly=torch.empty_like(lx), rstd=torch.empty(N, device="cuda"),
                    ldx=torch.empty_like(lx), dg=torch.empty(M, device="cuda"), db=torch.empty(M, device="cuda"),
                    P=torch.empty_like(s), out=torch.empty_like(s), k=torch.empty(B.mask_words(s.numel()), dtype=torch.int32, device="cuda"),
                    dS=torch.empty_like(s), ore=torch.empty_like(s))

    def run(o):
        B.tempo_gelu_fwd(x, o["y"], o["m"], "erf")
        B.tempo_gelu_bwd(dy, o["y"], o["m"], o["dx"], "erf")
        B.tempo_layernorm_fwd(lx, gamma, beta, o["ly"], o["rstd"], None, 1e-12)
        B.tempo_layernorm_bwd(ldy, o["ly"], gamma, beta, o["rstd"], o["ldx"], o["dg"], o["db"], ws)
        B.tempo_attn_softmax_dropout_fwd(s, kl, False, o["P"], o["out"], o["k"], 0.1, 77, 3)
        B.tempo_attn_softmax_dropout_bwd(do, o["P"], o["k"], o["dS"], o["ore"], 0.1)

    eager = fresh()
    run(eager)
    torch.cuda.synchronize()
    captured = fresh()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run(captured)
    for rep in range(4):
        for t in captured.values():
            t.zero_() if t.dtype != torch.int32 else t.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        scratch = fresh()
        run(scratch)                      # eager work between replays
        torch.cuda.synchronize()
        for name in eager:
            assert torch.equal(captured[name].view(torch.uint8), eager[name].view(torch.uint8)), (rep, name)


# ------------------------------------------------------------------ degenerate inputs
@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("p", [0.9, 0.999, 0.99999])
def test_attn_with_almost_everything_dropped(B, p, dt):
    # keep thresholds of 6554, 66 and 1 out of 65536; scales of 10, 1e3 and 1e5
    rng = np.random.default_rng(int(p * 1e6))
    shape = (2, 4, 128, 128)
    s = stored(rng, shape, dt, 0.125)
    p = np.float32(p)
    seed, offset = 77, 5                                    # keeps 12959, 132 and 3 elements
    P_ref, out_ref, K_ref = O.attn_softmax_dropout_fwd(s, None, False, p, seed, offset, dt)
    assert 0 < K_ref.sum() < K_ref.size // 5
    sd = dev(s, dt)
    Pd, od = torch.empty_like(sd), torch.empty_like(sd)
    md = torch.empty(B.mask_words(s.size), dtype=torch.int32, device="cuda")
    B.tempo_attn_softmax_dropout_fwd(sd, None, False, Pd, od, md, float(p), seed, offset)
    assert np.array_equal(words(md), O.pack_bits(K_ref))
    assert rel_err(host(Pd), P_ref) <= TOL[dt]
    assert rel_err(host(od), out_ref) <= TOL[dt]
    dout = stored(rng, shape, dt)
    dS_ref, _ = O.attn_softmax_dropout_bwd(dout, P_ref, K_ref, p, dt)
    dsd = torch.empty_like(sd)
    B.tempo_attn_softmax_dropout_bwd(dev(dout, dt), dev(P_ref, dt), md, dsd, None, float(p))
    assert rel_err(host(dsd), dS_ref) <= TOL[dt]
    dsd2 = torch.empty_like(sd)
    B.tempo_attn_softmax_dropout_bwd_regen(dev(dout, dt), dev(P_ref, dt), dsd2, None, float(p), seed, offset)
    assert torch.equal(dsd, dsd2)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("Sk", [128, 1000, 2048])
def test_attn_scores_with_minus_infinity_and_large_magnitudes(B, Sk, dt):
    # scores that already carry an additive mask: -inf entries, one row of nothing but -inf,
    # and magnitudes for which exp overflows without the max subtraction
    rng = np.random.default_rng(Sk)
    shape = (1, 2, 9, Sk)
    s = stored(rng, shape, dt, 60.0)
    s[rng.random(shape) < 0.1] = -np.inf
    s[0, 1, 4, :] = -np.inf
    s[0, 0, 2, :] = -300.0
    s[0, 0, 2, 5] = 300.0
    p, seed, offset = np.float32(0.1), 9, 0
    with np.errstate(invalid="ignore"):
        P_ref, out_ref, K_ref = O.attn_softmax_dropout_fwd(s, None, False, p, seed, offset, dt)
    assert np.all(P_ref[0, 1, 4] == 0) and P_ref[0, 0, 2, 5] == 1.0
    sd = dev(s, dt)
    Pd, od = torch.empty_like(sd), torch.empty_like(sd)
    md = torch.empty(B.mask_words(s.size), dtype=torch.int32, device="cuda")
    B.tempo_attn_softmax_dropout_fwd(sd, None, False, Pd, od, md, float(p), seed, offset)
    assert np.array_equal(words(md), O.pack_bits(K_ref))
    assert rel_err(host(Pd), P_ref) <= TOL[dt]
    assert rel_err(host(od), out_ref) <= TOL[dt]
    assert np.all(host(Pd)[0, 1, 4] == 0)


@pytest.mark.parametrize("eps", [1e-12, 1e-5])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("M", [64, 768, 1024, 4104, 6152])
def test_layernorm_constant_rows(B, M, dt, eps):
    # zero variance: rstd = 1/sqrt(eps), y = beta exactly (the constants are chosen so that the
    # float32 row sums are exact), and backward from y = beta
    rng = np.random.default_rng(M)
    consts = np.array([0.0, 1.0, -2.5, 1024.0, -0.0078125, 3.0])
    N = consts.size
    x = np.repeat(consts[:, None], M, axis=1)
    gamma = O.round_to_dtype(1 + 0.1 * rng.standard_normal(M), "f32")
    beta = O.round_to_dtype(0.1 * rng.standard_normal(M), "f32")
    y_ref, rstd_ref, mean_ref = O.layernorm_fwd(x, gamma, beta, eps, dt)
    assert np.array_equal(y_ref, O.round_to_dtype(np.broadcast_to(beta, x.shape), dt))
    xd, gd, bd = dev(x, dt), dev(gamma, "f32"), dev(beta, "f32")
    yd = torch.empty_like(xd)
    rd = torch.empty(N, dtype=torch.float32, device="cuda")
    md = torch.empty(N, dtype=torch.float32, device="cuda")
    B.tempo_layernorm_fwd(xd, gd, bd, yd, rd, md, eps)
    assert np.array_equal(host(yd), y_ref)
    assert rel_err(host(rd), rstd_ref) <= TOL["f32"]
    assert np.array_equal(host(md), mean_ref)
    dy = stored(rng, (N, M), dt)
    dx_ref, dg_ref, db_ref = O.layernorm_bwd(dy, y_ref, gamma, beta, host(rd), dt)
    dxd = torch.empty_like(xd)
    dgd = torch.empty(M, dtype=torch.float32, device="cuda")
    dbd = torch.empty(M, dtype=torch.float32, device="cuda")
    ws = torch.empty(B.tempo_layernorm_bwd_workspace_bytes(N, M), dtype=torch.uint8, device="cuda")
    B.tempo_layernorm_bwd(dev(dy, dt), yd, gd, bd, rd, dxd, dgd, dbd, ws)
    assert rel_err(host(dxd), dx_ref) <= TOL[dt]
    assert rel_err(host(dbd), db_ref) <= TOL["f32"]
    # dgamma = sum dy * xhat with xhat = 0 up to the rounding of y = beta to the storage dtype
    assert np.abs(host(dgd) - dg_ref).max() <= 1e-5 * max(1.0, np.abs(dy).max()) * N


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 3, 70, 128), (1, 2, 37, 512), (1, 1, 9, 2048), (1, 2, 5, 4104)])
def test_attention_does_not_depend_on_workgroup_size(B, shape, dt):
    """Knob 14: one, two or four waves per workgroup (never fewer lanes than a row takes) give
    bit-identical P, Out, mask, dS and recomputed Out, equal to the default choice."""
    rng = np.random.default_rng(sum(shape))
    sd = dev(stored(rng, shape, dt, 0.125), dt)
    dod = dev(stored(rng, shape, dt), dt)
    n = sd.numel()
    kl = torch.tensor([shape[3] - 3] * shape[0], dtype=torch.int32, device="cuda")
    results = []
    old = B.tempo_get_launch_param(14)
    try:
        for threads in (old, 64, 128, 256):
            B.tempo_set_launch_param(14, threads)
            Pd, od = torch.full_like(sd, 3.0), torch.full_like(sd, 3.0)
            md = torch.zeros(B.mask_words(n), dtype=torch.int32, device="cuda")
            B.tempo_attn_softmax_dropout_fwd(sd, kl, True, Pd, od, md, 0.1, 5, 6)
            dsd, ord_ = torch.full_like(sd, 3.0), torch.full_like(sd, 3.0)
            B.tempo_attn_softmax_dropout_bwd(dod, Pd, md, dsd, ord_, 0.1)
            torch.cuda.synchronize()
            results.append((Pd, od, md, dsd, ord_))
    finally:
        B.tempo_set_launch_param(14, old)
    view = torch.int16 if dt == "bf16" else torch.int32
    for r in results[1:]:
        for a, b in zip(results[0], r):
            assert torch.equal(a.view(view) if a.dtype != torch.int32 else a,
                               b.view(view) if b.dtype != torch.int32 else b)
    assert torch.equal(results[0][1].view(view), results[0][4].view(view))   # Out recomputed


@pytest.mark.parametrize("nr,nw", [(1, 1), (2, 1), (1, 2), (2, 2), (3, 2)])
def test_copy_streams_yardstick(B, nr, nw):
    """The plain multi-stream kernel bench.py holds the layer kernels against: every write
    tensor is the XOR of the read tensors (the second one plus one per 32-bit word)."""
    n = 256 * 1000 + 16            # int32 words; a ragged last workgroup
    g = torch.Generator(device="cuda").manual_seed(nr * 10 + nw)
    reads = [torch.randint(-2**31, 2**31 - 1, (n,), dtype=torch.int32, device="cuda", generator=g)
             for _ in range(nr)]
    writes = [torch.zeros(n, dtype=torch.int32, device="cuda") for _ in range(nw)]
    B.tempo_copy_streams(reads, writes)
    torch.cuda.synchronize()
    want = reads[0].clone()
    for r in reads[1:]:
        want ^= r
    assert torch.equal(writes[0], want)
    if nw == 2:
        assert torch.equal(writes[1], want + 1)       # wraps like the kernel's unsigned add
