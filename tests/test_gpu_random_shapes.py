"""Seeded random shapes through every entry point against the oracle: ragged sizes, row lengths on
both sides of every kernel-shape boundary (pieces per lane, lanes per row, rows over several
waves, the scalar fall-back paths), both dtypes, all mask forms."""
import numpy as np
import pytest
import torch

from helpers import TOL, rel_err
from oracle import tempo_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2210_10246_amd import binding
    binding.load()
    return binding


def dev(a, dt):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dt == "bf16" else t


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def words(t):
    return t.detach().cpu().numpy().view(np.uint32)


def stored(rng, shape, dt, scale=1.0):
    return O.round_to_dtype(rng.standard_normal(shape) * scale, dt)


def _row_lengths(rng, count, top):
    """Row lengths spread over the whole range, with boundaries of the kernel shapes mixed in."""
    edges = [8, 16, 24, 32, 64, 96, 128, 192, 256, 264, 384, 448, 512, 520, 768, 896, 1024, 1032,
             1536, 2048, 2056, 3072, 4096, 5120, 6144, 8192]
    picks = [int(x) for x in rng.integers(1, top, count // 2)]
    picks += [int(e + d) for e, d in zip(rng.choice(edges, count - count // 2),
                                         rng.choice([-8, -1, 0, 0, 1, 8], count - count // 2))]
    return [min(max(p, 1), top) for p in picks if p <= top + 8]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_layernorm_random_shapes(B, dt):
    rng = np.random.default_rng(1234)
    for M in _row_lengths(rng, 40, 8300):
        # mostly a few rows; now and then enough for workgroups that loop
        N = int(rng.integers(1, 70)) if rng.random() < 0.75 else int(rng.integers(300, 1200))
        x = stored(rng, (N, M), dt) * rng.uniform(0.5, 3.0) + rng.normal()
        x = O.round_to_dtype(x, dt)
        gamma = O.round_to_dtype(1 + 0.1 * rng.standard_normal(M), "f32")
        beta = O.round_to_dtype(0.1 * rng.standard_normal(M), "f32")
        dy = stored(rng, (N, M), dt)
        y, rstd, mean = O.layernorm_fwd(x, gamma, beta, 1e-5, dt)
        xd, gd, bd = dev(x, dt), dev(gamma, "f32"), dev(beta, "f32")
        yd = torch.full_like(xd, 3.0)
        rd = torch.full((N,), 3.0, dtype=torch.float32, device="cuda")
        B.tempo_layernorm_fwd(xd, gd, bd, yd, rd, None, 1e-5)
        assert rel_err(host(yd), y) <= TOL[dt], (N, M)
        assert rel_err(host(rd), rstd) <= TOL["f32"], (N, M)
        if M == 1:
            continue
        dx_ref, dg_ref, db_ref = O.layernorm_bwd(dy, y, gamma, beta, rstd, dt)
        dxd = torch.full_like(xd, 3.0)
        dgd = torch.full((M,), 3.0, dtype=torch.float32, device="cuda")
        dbd = torch.full((M,), 3.0, dtype=torch.float32, device="cuda")
        ws = torch.empty(max(B.tempo_layernorm_bwd_workspace_bytes(N, M), 16), dtype=torch.uint8,
                         device="cuda")
        B.tempo_layernorm_bwd(dev(dy, dt), dev(y, dt), gd, bd, dev(rstd, "f32"), dxd, dgd, dbd, ws)
        assert rel_err(host(dxd), dx_ref) <= TOL[dt], (N, M)
        assert rel_err(host(dgd), dg_ref) <= TOL["f32"], (N, M)
        assert rel_err(host(dbd), db_ref) <= TOL["f32"], (N, M)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_attention_random_shapes(B, dt):
    rng = np.random.default_rng(4321)
    for Sk in _row_lengths(rng, 40, 4200):
        Bn, A = int(rng.integers(1, 3)), int(rng.integers(1, 3))
        Sq = int(rng.integers(1, 40))
        mask = rng.choice(["none", "padding", "causal", "both"])
        key_len = None
        if mask in ("padding", "both"):
            key_len = rng.integers(0, Sk + 1, size=Bn).astype(np.int32)
        causal = mask in ("causal", "both")
        p = np.float32(rng.choice([0.0, 0.1, 0.3]))
        seed, offset = int(rng.integers(0, 2**62)), int(rng.integers(0, 2**40))
        s = stored(rng, (Bn, A, Sq, Sk), dt, 0.5)
        P_ref, out_ref, K_ref = O.attn_softmax_dropout_fwd(s, key_len, causal, p, seed, offset, dt)
        sd = dev(s, dt)
        kd = None if key_len is None else torch.from_numpy(key_len).cuda()
        Pd, od = torch.full_like(sd, 3.0), torch.full_like(sd, 3.0)
        md = torch.full((B.mask_words(s.size),), -1, dtype=torch.int32, device="cuda")
        B.tempo_attn_softmax_dropout_fwd(sd, kd, causal, Pd, od, md, float(p), seed, offset)
        case = (Bn, A, Sq, Sk, mask, float(p))
        assert np.array_equal(words(md), O.pack_bits(K_ref)), case
        assert rel_err(host(Pd), P_ref) <= TOL[dt], case
        assert rel_err(host(od), out_ref) <= TOL[dt], case
        dout = stored(rng, s.shape, dt)
        dS_ref, out_re_ref = O.attn_softmax_dropout_bwd(dout, P_ref, K_ref, p, dt)
        dod, Pd2 = dev(dout, dt), dev(P_ref, dt)
        for regen in (False, True):
            dsd, ord_ = torch.full_like(sd, 3.0), torch.full_like(sd, 3.0)
            if regen:
                B.tempo_attn_softmax_dropout_bwd_regen(dod, Pd2, dsd, ord_, float(p), seed, offset)
            else:
                B.tempo_attn_softmax_dropout_bwd(dod, Pd2, md, dsd, ord_, float(p))
            assert rel_err(host(dsd), dS_ref) <= TOL[dt], (case, regen)
            assert rel_err(host(ord_), out_re_ref) <= TOL[dt], (case, regen)


@pytest.mark.parametrize("kind", ["erf", "tanh", "silu"])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_activation_random_sizes(B, dt, kind):
    rng = np.random.default_rng(99)
    sizes = [int(x) for x in rng.integers(1, 200_000, 10)] + [8192 * 4 - 1, 8192 * 4, 8192 * 4 + 1,
                                                            1024 * 8 * 4 * 3 + 5]
    for n in sizes:
        x = stored(rng, n, dt, rng.uniform(0.5, 4.0))
        dy = stored(rng, n, dt)
        y_ref, m_ref = O.gelu_fwd(x, kind, dt)
        dx_ref = O.gelu_bwd(dy, y_ref, m_ref, kind, dt)
        xd = dev(x, dt)
        yd = torch.full_like(xd, 7.0)
        md = torch.full((B.mask_words(n),), -1, dtype=torch.int32, device="cuda")
        dxd = torch.full_like(xd, 7.0)
        if kind == "silu":
            B.tempo_silu_fwd(xd, yd, md)
            B.tempo_silu_bwd(dev(dy, dt), dev(y_ref, dt), md, dxd)
        else:
            B.tempo_gelu_fwd(xd, yd, md, kind)
            B.tempo_gelu_bwd(dev(dy, dt), dev(y_ref, dt), md, dxd, kind)
        assert np.array_equal(words(md), O.pack_bits(m_ref)), n
        assert rel_err(host(yd), y_ref) <= TOL[dt], n
        assert rel_err(host(dxd), dx_ref) <= TOL[dt], n
