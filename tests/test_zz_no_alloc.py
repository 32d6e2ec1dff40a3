"""The entry point that allocates nothing: tempo_layernorm_bwd_static against
tempo_layernorm_bwd (same kernels, caller's workspace) through the C ABI, bit for bit, on calls
in a row that share the static scratch array, each smaller than the one before, so that stale
partial sums of a larger call lie behind the slots a smaller call uses."""
import numpy as np
import pytest
import torch

from helpers import TOL, rel_err
from oracle import tempo_oracle as O

pytestmark = pytest.mark.gpu

TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2210_10246_amd import binding
    binding.load()
    return binding


def _case(B, N, M, dt, seed, check_oracle):
    rng = np.random.default_rng(seed)
    x = O.round_to_dtype(rng.standard_normal((N, M)), dt)
    gamma = O.round_to_dtype(1 + 0.1 * rng.standard_normal(M), "f32")
    beta = O.round_to_dtype(0.1 * rng.standard_normal(M), "f32")
    dy = O.round_to_dtype(rng.standard_normal((N, M)), dt)
    y, rstd, _ = O.layernorm_fwd(x, gamma, beta, 1e-5, dt)
    t = lambda a, d: torch.from_numpy(np.ascontiguousarray(a)).to(TDT[d]).cuda()
    dyd, yd = t(dy, dt), t(y, dt)
    gd, bd, rd = t(gamma, "f32"), t(beta, "f32"), t(rstd, "f32")
    ws = torch.empty(max(B.tempo_layernorm_bwd_workspace_bytes(N, M), 16), dtype=torch.uint8, device="cuda")
    dx0 = torch.empty_like(dyd)
    dg0 = torch.empty(M, dtype=torch.float32, device="cuda")
    db0 = torch.empty(M, dtype=torch.float32, device="cuda")
    B.tempo_layernorm_bwd(dyd, yd, gd, bd, rd, dx0, dg0, db0, ws)
    dx1 = torch.full_like(dyd, 3.0)
    dg1 = torch.full((M,), 3.0, dtype=torch.float32, device="cuda")
    db1 = torch.full((M,), 3.0, dtype=torch.float32, device="cuda")
    before = torch.cuda.memory_allocated()
    B.tempo_layernorm_bwd_static(dyd, yd, gd, bd, rd, dx1, dg1, db1)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    view = torch.int16 if dt == "bf16" else torch.int32
    assert torch.equal(dx0.view(view), dx1.view(view)), (N, M, dt)
    assert torch.equal(dg0.view(torch.int32), dg1.view(torch.int32)), (N, M, dt)
    assert torch.equal(db0.view(torch.int32), db1.view(torch.int32)), (N, M, dt)
    if check_oracle:
        dx_ref, dg_ref, db_ref = O.layernorm_bwd(dy, y, gamma, beta, rstd, dt)
        h = lambda a: a.detach().cpu().to(torch.float64).numpy()
        assert rel_err(h(dx1), dx_ref) <= TOL[dt]
        assert rel_err(h(dg1), dg_ref) <= TOL["f32"]
        assert rel_err(h(db1), db_ref) <= TOL["f32"]


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_static_scratch_matches_workspace_entry_point_on_shrinking_calls(B, dt):
    # looping grid (every slot of a 256-workgroup grid), then smaller and smaller problems whose
    # grids use a prefix of those slots, a row of 8192 columns (register-resident in bfloat16, the
    # any-M kernel in float32), a row length of the any-M kernel, and one row
    for i, (N, M) in enumerate([(9000, 1024), (100, 8192), (700, 1024), (300, 768), (37, 4096), (65, 100), (1, 8)]):
        _case(B, N, M, dt, 1000 + i, check_oracle=True)


def test_static_scratch_rejects_problems_beyond_the_array(B):
    N, M = 5000, 8200                     # any-M kernel: min(N, 1024) slots of 8*M bytes > 8 MiB
    assert B.tempo_layernorm_bwd_workspace_bytes(N, M) > (8 << 20)
    z = torch.zeros(N, M, dtype=torch.float32, device="cuda")
    g = torch.ones(M, dtype=torch.float32, device="cuda")
    r = torch.ones(N, dtype=torch.float32, device="cuda")
    with pytest.raises(B.TempoError) as e:
        B.tempo_layernorm_bwd_static(z, z, g, g, r, torch.empty_like(z), torch.empty_like(g), torch.empty_like(g))
    assert e.value.status == 3            # TEMPO_ERR_WORKSPACE
    # zero-size calls need no pointers and no scratch
    assert B.load().tempo_layernorm_bwd_static(None, None, None, None, None, None, None, None, 0, 8, 0, None) == 0


def test_static_scratch_under_graph_capture(B):
    # the callers it is for: captured once (after one ordinary call on this GPU, so that the
    # array's address is already known), replayed with new inputs, with eager work in between
    N, M, dt = 3000, 1024, "bf16"
    rng = np.random.default_rng(77)
    t = lambda a, d: torch.from_numpy(np.ascontiguousarray(a)).to(TDT[d]).cuda()
    gd = t(O.round_to_dtype(1 + 0.1 * rng.standard_normal(M), "f32"), "f32")
    bd = t(O.round_to_dtype(0.1 * rng.standard_normal(M), "f32"), "f32")
    dyd, yd = t(rng.standard_normal((N, M)), dt), t(rng.standard_normal((N, M)), dt)
    rd = t(0.5 + rng.random(N), "f32")
    ws = torch.empty(B.tempo_layernorm_bwd_workspace_bytes(N, M), dtype=torch.uint8, device="cuda")
    out = lambda: (torch.empty_like(dyd), torch.empty(M, device="cuda"), torch.empty(M, device="cuda"))
    warm = out()
    B.tempo_layernorm_bwd_static(dyd, yd, gd, bd, rd, *warm)
    torch.cuda.synchronize()
    cap = out()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.tempo_layernorm_bwd_static(dyd, yd, gd, bd, rd, *cap)
    for rep in range(3):
        dyd.copy_(t(rng.standard_normal((N, M)), dt))
        yd.copy_(t(rng.standard_normal((N, M)), dt))
        for o in cap:
            o.fill_(3.0)
        torch.cuda.synchronize()
        g.replay()
        ref = out()
        B.tempo_layernorm_bwd(dyd, yd, gd, bd, rd, *ref, ws)     # eager work between replays
        torch.cuda.synchronize()
        for a, b in zip(cap, ref):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), rep
