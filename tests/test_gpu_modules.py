"""The drop-in PyTorch layers (App. F of the paper) against stock PyTorch layers: same outputs,
same gradients, fewer bytes kept for backward."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import tempo_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def M():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2210_10246_amd import binding, modules
    binding.load()
    return modules


def reference_layer(layer, x, key_len, keep):
    """The same encoder layer from stock PyTorch ops, sharing `layer`'s parameters; `keep` is the
    dropout keep mask [B, A, S, S] (float 0/1) or None for no dropout."""
    Bn, S, H = x.shape
    A = layer.heads
    d = H // A
    q, k, v = layer.qkv(x).view(Bn, S, 3, A, d).permute(2, 0, 3, 1, 4)
    scores = torch.matmul(q, k.transpose(-1, -2)) * (1.0 / math.sqrt(d))
    if key_len is not None:
        j = torch.arange(S, device=x.device)[None, None, None, :]
        scores = scores.masked_fill(j >= key_len.view(Bn, 1, 1, 1), float("-inf"))
    probs = torch.softmax(scores, dim=-1)
    if keep is not None:
        scale = float(np.float32(1.0) / (np.float32(1.0) - np.float32(layer.core.p)))
        probs = probs * keep * scale
    ctxt = torch.matmul(probs, v).permute(0, 2, 1, 3).reshape(Bn, S, H)
    x = F.layer_norm(x + layer.proj(ctxt), (H,), layer.ln1.weight, layer.ln1.bias, layer.ln1.eps)
    return F.layer_norm(x + layer.fc2(F.gelu(layer.fc1(x))), (H,), layer.ln2.weight, layer.ln2.bias,
                        layer.ln2.eps)


def grads(out, params, dout):
    return torch.autograd.grad(out, params, dout, retain_graph=False)


@pytest.mark.parametrize("p", [0.0, 0.1])
def test_encoder_layer_matches_stock_pytorch(M, p):
    torch.manual_seed(0)
    Bn, S, H, A = 3, 64, 256, 4
    layer = M.TempoEncoderLayer(H, A, 4 * H, p_attn=p, eps=1e-5).cuda().train()
    with torch.no_grad():
        for ln in (layer.ln1, layer.ln2):
            ln.weight.add_(0.1 * torch.randn_like(ln.weight))
            ln.bias.add_(0.1 * torch.randn_like(ln.bias))
    x = torch.randn(Bn, S, H, device="cuda", requires_grad=True)
    key_len = torch.tensor([64, 40, 17], dtype=torch.int32, device="cuda")
    dout = torch.randn(Bn, S, H, device="cuda")
    params = [x] + list(layer.parameters())

    layer.core.offset = 6
    out = layer(x, key_len)                       # uses offset 7
    g = grads(out, params, dout)

    keep = None
    if p > 0:
        K = O.dropout_keep(Bn * A * S * S, p, layer.core.seed, 7).reshape(Bn, A, S, S)
        keep = torch.from_numpy(K.astype(np.float32)).cuda()
    ref = reference_layer(layer, x, key_len, keep)
    gr = grads(ref, params, dout)

    def close(a, b, tol):
        scale = b.abs().max().clamp_min(1e-6)
        return ((a - b).abs().max() / scale).item() <= tol

    assert close(out, ref, 2e-5)
    for a, b in zip(g, gr):
        assert close(a, b, 2e-4), (a.shape, ((a - b).abs().max() / b.abs().max()).item())


def _stashed_bytes(fn):
    """Bytes of distinct storages autograd keeps for backward while fn() runs."""
    seen = {}

    def pack(t):
        if t.is_cuda:
            seen[t.untyped_storage().data_ptr()] = t.untyped_storage().nbytes()
        return t

    with torch.autograd.graph.saved_tensors_hooks(pack, lambda t: t):
        out = fn()
    return sum(seen.values()), out


def test_encoder_layer_keeps_fewer_activation_bytes(M):
    torch.manual_seed(1)
    Bn, S, H, A = 4, 128, 512, 8
    layer = M.TempoEncoderLayer(H, A, 4 * H, p_attn=0.1, eps=1e-5).cuda().train()
    x = torch.randn(Bn, S, H, device="cuda", requires_grad=True)
    keep = (torch.rand(Bn, A, S, S, device="cuda") < 0.9).float()
    tempo_bytes, _ = _stashed_bytes(lambda: layer(x))
    stock_bytes, _ = _stashed_bytes(lambda: reference_layer(layer, x, None, keep))
    tokens, e = Bn * S, 4
    # what the three layers drop per token: the 4H GELU input (minus a bit mask), both
    # LayerNorm inputs, and the dropout output of the attention sublayer
    expected = tokens * ((4 * H * e - 4 * H // 8) + 2 * H * e + A * S * e)
    saved = stock_bytes - tempo_bytes
    assert saved >= 0.85 * expected, (stock_bytes, tempo_bytes, expected)
    print(f"stashed bytes per token: stock {stock_bytes / tokens:.0f}, tempo {tempo_bytes / tokens:.0f}, "
          f"saved {saved / tokens:.0f} (expected >= {0.85 * expected / tokens:.0f})")


def test_encoder_layer_holds_less_device_memory_between_forward_and_backward(M):
    """The same saving as the allocator sees it: bytes allocated once forward has returned
    (output and autograd stash alive), stock layer against the memory-reduced one."""
    torch.manual_seed(5)
    Bn, S, H, A = 8, 128, 512, 8
    layer = M.TempoEncoderLayer(H, A, 4 * H, p_attn=0.1, eps=1e-5).cuda().train()
    x = torch.randn(Bn, S, H, device="cuda", requires_grad=True)
    keep = (torch.rand(Bn, A, S, S, device="cuda") < 0.9).float()

    def held(fn):
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        torch.cuda.reset_peak_memory_stats()
        out = fn()
        torch.cuda.synchronize()
        after = torch.cuda.memory_allocated()
        out.sum().backward()
        torch.cuda.synchronize()
        peak = torch.cuda.max_memory_allocated() - before
        del out
        return after - before, peak

    held(lambda: layer(x))                       # warm the allocator and the library
    tempo_held, tempo_peak = held(lambda: layer(x))
    stock_held, stock_peak = held(lambda: reference_layer(layer, x, None, keep))
    tokens, e = Bn * S, 4
    expected = tokens * ((4 * H * e - 4 * H // 8) + 2 * H * e + A * S * e)
    saved = stock_held - tempo_held
    print(f"held after forward per token: stock {stock_held / tokens:.0f} B, tempo {tempo_held / tokens:.0f} B, "
          f"saved {saved / tokens:.0f} B (expected >= {0.85 * expected / tokens:.0f}); "
          f"peak over forward+backward: stock {stock_peak / tokens:.0f} B, tempo {tempo_peak / tokens:.0f} B")
    assert saved >= 0.85 * expected, (stock_held, tempo_held, expected)
    assert tempo_peak <= stock_peak


def test_attention_core_without_stored_mask(M):
    """store_mask=False: same gradients bit for bit, and the mask leaves the stash."""
    torch.manual_seed(3)
    Bn, A, S, d = 2, 4, 96, 32
    scores = torch.randn(Bn, A, S, S, device="cuda", requires_grad=True)
    v = torch.randn(Bn, A, S, d, device="cuda", requires_grad=True)
    dctx = torch.randn(Bn, A, S, d, device="cuda")
    res = {}
    for store in (True, False):
        core = M.TempoAttentionCore(0.1, seed=5, store_mask=store).cuda().train()
        stash, out = _stashed_bytes(lambda: core(scores, v))
        res[store] = (stash, out, torch.autograd.grad(out, (scores, v), dctx))
    assert torch.equal(res[True][1], res[False][1])
    for a, b in zip(res[True][2], res[False][2]):
        assert torch.equal(a, b)
    assert res[True][0] - res[False][0] == scores.numel() // 8


def test_inplace_silu_module(M):
    torch.manual_seed(4)
    act = M.InplaceSiLU().cuda()
    x = torch.randn(64, 1000, device="cuda", requires_grad=True) * 2
    x.retain_grad()
    dout = torch.randn(64, 1000, device="cuda")
    stash, y = _stashed_bytes(lambda: act(x))
    y.backward(dout)
    xr = x.detach().clone().requires_grad_(True)
    yr = F.silu(xr)
    yr.backward(dout)
    assert (y - yr).abs().max().item() <= 1e-5 * yr.abs().max().item()
    # float32 y a few ulp above the minimum: d ~ sqrt(y - y*) amplifies its rounding
    assert (x.grad - xr.grad).abs().max().item() <= 5e-3 * dout.abs().max().item()
    assert ((x.grad - xr.grad) ** 2).mean().sqrt().item() <= 2e-6
    assert stash == x.numel() * 4 + x.numel() // 8       # y and one bit per element


def test_modules_in_bf16(M):
    torch.manual_seed(2)
    gelu = M.InplaceGELU().cuda()
    ln = M.InplaceLayerNorm(768).cuda()
    x = torch.randn(16, 128, 768, device="cuda", dtype=torch.bfloat16, requires_grad=True)
    dout = torch.randn(16, 128, 768, device="cuda", dtype=torch.bfloat16)
    y = ln(gelu(x))
    y.backward(dout)
    xr = x.detach().clone().requires_grad_(True)
    yr = F.layer_norm(F.gelu(xr.float()), (768,), ln.weight, ln.bias, ln.eps)
    yr.backward(dout.float())
    assert (y.float() - yr).abs().max().item() <= 0.05
    rel = (x.grad.float() - xr.grad.float()).abs().max() / xr.grad.float().abs().max()
    # two bf16 roundings in between (y of GELU, dy into GELU backward) and the sqrt-shaped
    # sensitivity of the composite at the GELU minimum
    assert rel.item() <= 0.05
