"""Tensors of more than 2^32 elements: element indices beyond 32 bits, byte offsets beyond 2^33.

The float64 oracle cannot walk such tensors, so the inputs are drawn on the device (seeded),
and the oracle is run on sampled elements / whole sampled rows copied back from the device:
the ends of the tensor, the neighbourhood of element 2^31 and 2^32, and a random sample.
Properties that hold for the whole tensor (mask population, zeros under the padding mask,
bit-identical recomputed dropout output, column sums) are checked on the device.
"""
import numpy as np
import pytest
import torch

from helpers import TOL, rel_err
from oracle import tempo_oracle as O
from paper_2210_10246_amd import workloads as W

pytestmark = pytest.mark.gpu

CHUNK = 1 << 28


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2210_10246_amd import binding
    binding.load()
    return binding


def _normal(n, std, seed):
    """bfloat16 N(0, std^2) drawn on the device, chunk by chunk."""
    gen = torch.Generator(device="cuda").manual_seed(seed)
    t = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    for i in range(0, n, CHUNK):
        t[i:i + CHUNK].normal_(0.0, std, generator=gen)
    return t


def _take(t, idx):
    return W.as_f64(t.reshape(-1)[torch.from_numpy(idx).cuda()])


def _mask_bits(md, idx):
    words = md[torch.from_numpy(idx >> 5).cuda()].cpu().numpy().view(np.uint32)
    return ((words >> (idx & 31).astype(np.uint32)) & 1).astype(bool)


def test_gelu_beyond_2_32_elements(B):
    dt = "bf16"
    n = (1 << 32) + 8 * 1024 * 4 * 3 + 5                  # ragged last tile, ragged last mask word
    x = _normal(n, 1.5, 1)
    y = torch.empty_like(x)
    md = torch.empty(B.mask_words(n), dtype=torch.int32, device="cuda")
    B.tempo_gelu_fwd(x, y, md, "erf")
    rng = np.random.default_rng(1)
    idx = np.unique(np.concatenate([
        rng.integers(0, n, 200_000), np.arange(4096), np.arange(n - 5000, n),
        np.arange((1 << 31) - 4096, (1 << 31) + 4096), np.arange((1 << 32) - 4096, (1 << 32) + 4096)]))
    x_s = _take(x, idx)
    y_ref, m_ref = O.gelu_fwd(x_s, "erf", dt)
    y_gpu = _take(y, idx)
    assert rel_err(y_gpu, y_ref) <= TOL[dt]
    assert np.array_equal(_mask_bits(md, idx), m_ref)
    # whole tensor: the mask holds exactly the elements at or right of the minimum, pad bits 0
    xstar = float(O.GELU_XSTAR_F32["erf"])
    right = sum(int((x[i:i + CHUNK].float() >= xstar).sum()) for i in range(0, n, CHUNK))
    words = md.cpu().numpy().view(np.uint32)
    assert int(np.bitwise_count(words).sum(dtype=np.int64)) == right
    assert int(words[-1]) >> (n & 31) == 0
    del x
    dy = _normal(n, 1.0, 2)
    dx = torch.empty_like(dy)
    B.tempo_gelu_bwd(dy, y, md, dx, "erf")
    ref = O.gelu_bwd(_take(dy, idx), y_gpu, m_ref, "erf", dt)
    assert rel_err(_take(dx, idx), ref) <= TOL[dt]
    B.tempo_gelu_bwd(dy, y, md, dy, "erf")                 # in place
    torch.cuda.synchronize()
    assert all(torch.equal(dy[i:i + CHUNK], dx[i:i + CHUNK]) for i in range(0, n, CHUNK))


def _sample_rows(rng, rows, row_len, extra=()):
    cross = (1 << 32) // row_len                           # the row that holds element 2^32
    cross31 = (1 << 31) // row_len
    pick = np.concatenate([rng.integers(0, rows, 150), [0, 1, rows - 2, rows - 1],
                           np.arange(cross - 2, cross + 3), np.arange(cross31 - 1, cross31 + 2),
                           np.asarray(extra, dtype=np.int64)])
    return np.unique(pick[(pick >= 0) & (pick < rows)])


@pytest.mark.parametrize("M", [4096, 4100])       # register-resident rows / the any-length kernels
def test_layernorm_beyond_2_32_elements(B, M):
    dt = "bf16"
    N = (1 << 20) + 3
    assert N * M > 1 << 32
    x = _normal(N * M, 1.0, 3).view(N, M)
    rng = np.random.default_rng(3)
    gamma = torch.from_numpy((1.0 + 0.1 * rng.standard_normal(M)).astype(np.float32))
    beta = torch.from_numpy((0.1 * rng.standard_normal(M)).astype(np.float32))
    gd, bd = gamma.cuda(), beta.cuda()
    y = torch.empty_like(x)
    rstd = torch.empty(N, dtype=torch.float32, device="cuda")
    mean = torch.empty(N, dtype=torch.float32, device="cuda")
    B.tempo_layernorm_fwd(x, gd, bd, y, rstd, mean, 1e-12)
    rows = _sample_rows(rng, N, M)
    ri = torch.from_numpy(rows).cuda()
    g64, b64 = W.as_f64(gamma), W.as_f64(beta)
    y_ref, rstd_ref, mean_ref = O.layernorm_fwd(W.as_f64(x[ri]), g64, b64, 1e-12, dt)
    assert rel_err(W.as_f64(y[ri]), y_ref) <= TOL[dt]
    assert rel_err(W.as_f64(rstd[ri]), rstd_ref) <= TOL["f32"]
    assert np.abs(W.as_f64(mean[ri]) - mean_ref).max() <= 1e-6
    del x
    dy = _normal(N * M, 1.0, 4).view(N, M)
    dx = torch.empty_like(dy)
    dg = torch.empty(M, dtype=torch.float32, device="cuda")
    db = torch.empty(M, dtype=torch.float32, device="cuda")
    ws = torch.empty(B.tempo_layernorm_bwd_workspace_bytes(N, M), dtype=torch.uint8, device="cuda")
    B.tempo_layernorm_bwd(dy, y, gd, bd, rstd, dx, dg, db, ws)
    dx_ref, _, _ = O.layernorm_bwd(W.as_f64(dy[ri]), W.as_f64(y[ri]), g64, b64, W.as_f64(rstd[ri]), dt)
    assert rel_err(W.as_f64(dx[ri]), dx_ref) <= TOL[dt]
    # column sums over all rows: float64 sums on the device, 64 Ki rows at a time
    dg64 = torch.zeros(M, dtype=torch.float64, device="cuda")
    db64 = torch.zeros(M, dtype=torch.float64, device="cuda")
    for i in range(0, N, 1 << 16):
        d = dy[i:i + (1 << 16)].double()
        xhat = (y[i:i + (1 << 16)].double() - bd.double()) / gd.double()
        dg64 += (d * xhat).sum(0)
        db64 += d.sum(0)
    assert rel_err(W.as_f64(dg), W.as_f64(dg64)) <= TOL["f32"]
    assert rel_err(W.as_f64(db), W.as_f64(db64)) <= TOL["f32"]


@pytest.mark.parametrize("Sk", [4128, 4100])      # register-resident rows / the any-length kernels
def test_attention_beyond_2_32_elements(B, Sk):
    dt = "bf16"
    Bn, A, Sq = 2, 16, 32768
    rows, n = Bn * A * Sq, Bn * A * Sq * Sk
    assert n > 1 << 32
    p, seed, offset = 0.1, 0x5EED0000FEEDBEEF, (1 << 40) + 3
    key_len = np.array([Sk, 3001], dtype=np.int32)
    kd = torch.from_numpy(key_len).cuda()
    s = _normal(n, 0.125, 5).view(Bn, A, Sq, Sk)
    P, out = torch.empty_like(s), torch.empty_like(s)
    md = torch.empty(B.mask_words(n), dtype=torch.int32, device="cuda")
    B.tempo_attn_softmax_dropout_fwd(s, kd, False, P, out, md, p, seed, offset)
    dout = _normal(n, 1.0, 6).view(Bn, A, Sq, Sk)
    dS, out_re = torch.empty_like(s), torch.empty_like(s)
    B.tempo_attn_softmax_dropout_bwd(dout, P, md, dS, out_re, p)
    torch.cuda.synchronize()
    # whole tensor: recomputed output bit-identical, nothing under the padding mask
    assert all(torch.equal(out[b, a].view(torch.int16), out_re[b, a].view(torch.int16))
               for b in range(Bn) for a in range(A))
    assert all(int(torch.count_nonzero(P[1, a, :, 3001:])) == 0 for a in range(A))
    assert all(int(torch.count_nonzero(dS[1, a, :, 3001:])) == 0 for a in range(A))
    # sampled rows against the oracle, keep bits taken at the row's offset in the flat tensor
    rng = np.random.default_rng(5)
    picked = _sample_rows(rng, rows, Sk, extra=[A * Sq - 1, A * Sq])
    s2, P2, o2, do2, dS2 = (t.view(rows, Sk) for t in (s, P, out, dout, dS))
    words = md.cpu().numpy().view(np.uint32)
    scale = float(np.float32(1.0) / (np.float32(1.0) - np.float32(p)))
    for b in range(Bn):
        sel = picked[(picked // (A * Sq)) == b]
        ri = torch.from_numpy(sel).cuda()
        shape = (1, 1, len(sel), Sk)
        P_ref, _, _ = O.attn_softmax_dropout_fwd(W.as_f64(s2[ri]).reshape(shape), key_len[b:b + 1],
                                                 False, 0.0, seed, offset, dt)
        K_ref = np.stack([O.dropout_keep(Sk, p, seed, offset, start=int(r) * Sk) for r in sel])
        for k, r in enumerate(sel):
            start = int(r) * Sk
            w0, w1 = start >> 5, (start + Sk + 31) >> 5
            bits = O.unpack_bits(words[w0:w1], (w1 - w0) * 32)[start - w0 * 32:][:Sk]
            assert np.array_equal(bits, K_ref[k]), (b, r)
        P_gpu = W.as_f64(P2[ri]).reshape(shape)
        assert rel_err(P_gpu, P_ref) <= TOL[dt]
        out_ref = O.round_to_dtype(P_ref * K_ref.reshape(shape) * scale, dt)
        assert rel_err(W.as_f64(o2[ri]).reshape(shape), out_ref) <= TOL[dt]
        dS_ref, _ = O.attn_softmax_dropout_bwd(W.as_f64(do2[ri]).reshape(shape), P_gpu,
                                               K_ref.reshape(shape), p, dt)
        assert rel_err(W.as_f64(dS2[ri]).reshape(shape), dS_ref) <= TOL[dt]
    # the backward that draws the bits again gives the same gradient
    dS_b = torch.empty_like(s)
    B.tempo_attn_softmax_dropout_bwd_regen(dout, P, dS_b, None, p, seed, offset)
    torch.cuda.synchronize()
    assert all(torch.equal(dS[b, a], dS_b[b, a]) for b in range(Bn) for a in range(A))
