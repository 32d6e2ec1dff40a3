"""Drop-in PyTorch layers over the C ABI (the way the paper ships its kernels: App. F).

Only what is stashed for backward differs from the stock layers:
  InplaceGELU        keeps the output (which the next Linear keeps anyway) and a 1-bit mask
  InplaceSiLU        the same for SiLU (Sec. 5.1)
  InplaceLayerNorm   keeps the output and one float per row
  TempoAttentionCore softmax -> dropout -> (. @ V) keeping the softmax output P and a 1-bit
                     mask; the dropout output is a transient in forward and is recomputed by
                     the backward kernel for the gradient of V (Sec. 3.3).
Every arithmetic step of the three layers runs in the HIP kernels; the two matrix products
around the attention sublayer are ordinary library GEMMs (torch.matmul).
"""
from __future__ import annotations

import math

import torch
from torch import nn

from . import binding as B


def _words(n: int, device) -> torch.Tensor:
    return torch.empty(B.mask_words(n), dtype=torch.int32, device=device)


class _InplaceGELUFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, kind):
        x = x.contiguous()
        y = torch.empty_like(x)
        mask = _words(x.numel(), x.device)
        if kind == "silu":
            B.tempo_silu_fwd(x, y, mask)
        else:
            B.tempo_gelu_fwd(x, y, mask, kind)
        ctx.kind = kind
        ctx.save_for_backward(y, mask)
        return y

    @staticmethod
    def backward(ctx, dy):
        y, mask = ctx.saved_tensors
        dy = dy.contiguous()
        dx = torch.empty_like(dy)
        if ctx.kind == "silu":
            B.tempo_silu_bwd(dy, y, mask, dx)
        else:
            B.tempo_gelu_bwd(dy, y, mask, dx, ctx.kind)
        return dx, None


class InplaceGELU(nn.Module):
    """GELU whose backward needs the output and one bit per element (Sec. 3.1)."""

    def __init__(self, approximate: str = "none"):
        super().__init__()
        self.kind = {"none": "erf", "tanh": "tanh"}[approximate]

    def forward(self, x):
        return _InplaceGELUFn.apply(x, self.kind)


class InplaceSiLU(nn.Module):
    """SiLU with the same stash as InplaceGELU: the in-place recipe for elementwise layers
    (Sec. 5.1) on another activation with a single minimum."""

    def forward(self, x):
        return _InplaceGELUFn.apply(x, "silu")


class _InplaceLayerNormFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, gamma, beta, eps):
        x = x.contiguous()
        M = x.shape[-1]
        N = x.numel() // M
        y = torch.empty_like(x)
        rstd = torch.empty(N, dtype=torch.float32, device=x.device)
        B.tempo_layernorm_fwd(x, gamma, beta, y, rstd, None, eps)
        ctx.save_for_backward(y, gamma, beta, rstd)
        return y

    @staticmethod
    def backward(ctx, dy):
        y, gamma, beta, rstd = ctx.saved_tensors
        dy = dy.contiguous()
        M = y.shape[-1]
        N = y.numel() // M
        dx = torch.empty_like(dy)
        dgamma = torch.empty_like(gamma)
        dbeta = torch.empty_like(beta)
        ws = torch.empty(B.tempo_layernorm_bwd_workspace_bytes(N, M), dtype=torch.uint8,
                         device=y.device)
        B.tempo_layernorm_bwd(dy, y, gamma, beta, rstd, dx, dgamma, dbeta, ws)
        return dx, dgamma, dbeta, None


class InplaceLayerNorm(nn.Module):
    """LayerNorm over the last dimension whose backward needs the output and rstd (Sec. 3.2).
    Parameters are float32 whatever the activation dtype; gamma must stay non-zero."""

    def __init__(self, hidden: int, eps: float = 1e-5):
        super().__init__()
        self.weight = nn.Parameter(torch.ones(hidden, dtype=torch.float32))
        self.bias = nn.Parameter(torch.zeros(hidden, dtype=torch.float32))
        self.eps = eps

    def _apply(self, fn, recurse=True):
        # .bfloat16() / .half() / .to(dtype) on a model must not narrow gamma and beta: the
        # kernels read them as float32.  Follow the device of the cast, keep the values.
        def keep_float32(t):
            out = fn(t)
            if t.dtype == torch.float32 and out.dtype != torch.float32:
                out = t.to(device=out.device)
            return out
        return super()._apply(keep_float32, recurse)

    def forward(self, x):
        w, b = self.weight, self.bias
        if w.dtype != torch.float32 or b.dtype != torch.float32:   # parameters replaced by hand
            w, b = w.float(), b.float()
        return _InplaceLayerNormFn.apply(x, w, b, self.eps)


class _AttentionCoreFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, scores, v, key_len, causal, p, seed, offset, store_mask):
        scores = scores.contiguous()
        probs = torch.empty_like(scores)
        out = torch.empty_like(scores)          # transient: freed when forward returns
        keep = _words(scores.numel(), scores.device)
        B.tempo_attn_softmax_dropout_fwd(scores, key_len, causal, probs, out, keep, p, seed, offset)
        ctx.rng = (p, seed, offset)
        ctx.store_mask = store_mask
        if store_mask:
            ctx.save_for_backward(probs, v, keep)
        else:                                   # the mask is a transient too: drawn again later
            ctx.save_for_backward(probs, v)
        return torch.matmul(out, v)

    @staticmethod
    def backward(ctx, dctx):
        probs, v = ctx.saved_tensors[:2]
        dout = torch.matmul(dctx, v.transpose(-1, -2)).contiguous()
        out_re = torch.empty_like(probs)
        dscores = torch.empty_like(probs)
        p, seed, offset = ctx.rng
        if ctx.store_mask:
            B.tempo_attn_softmax_dropout_bwd(dout, probs, ctx.saved_tensors[2], dscores, out_re, p)
        else:
            B.tempo_attn_softmax_dropout_bwd_regen(dout, probs, dscores, out_re, p, seed, offset)
        dv = torch.matmul(out_re.transpose(-1, -2), dctx)
        return dscores, dv, None, None, None, None, None, None


class TempoAttentionCore(nn.Module):
    """context = dropout(softmax(mask(scores))) @ V for scores [B, A, Sq, Sk] already scaled by
    1/sqrt(d).  Each forward in training mode draws a fresh mask: the counter offset advances.
    store_mask=False keeps no mask for backward, which then draws the same bits again."""

    def __init__(self, p: float = 0.1, seed: int = 0x5EED, store_mask: bool = True):
        super().__init__()
        self.p, self.seed, self.offset, self.store_mask = p, seed, 0, store_mask

    def forward(self, scores, v, key_len=None, causal=False):
        p = self.p if self.training else 0.0
        self.offset += 1
        return _AttentionCoreFn.apply(scores, v, key_len, causal, p, self.seed, self.offset,
                                      self.store_mask)


class TempoEncoderLayer(nn.Module):
    """A post-LN BERT encoder layer built from the three memory-reduced layers (Fig. 1 of the
    paper); hidden-state dropouts are left out (they are not part of the method)."""

    def __init__(self, hidden: int, heads: int, ffn: int, p_attn: float = 0.1, eps: float = 1e-12,
                 dtype=torch.float32):
        super().__init__()
        self.heads = heads
        self.qkv = nn.Linear(hidden, 3 * hidden, dtype=dtype)
        self.proj = nn.Linear(hidden, hidden, dtype=dtype)
        self.fc1 = nn.Linear(hidden, ffn, dtype=dtype)
        self.fc2 = nn.Linear(ffn, hidden, dtype=dtype)
        self.ln1 = InplaceLayerNorm(hidden, eps)
        self.ln2 = InplaceLayerNorm(hidden, eps)
        self.act = InplaceGELU()
        self.core = TempoAttentionCore(p_attn)

    def forward(self, x, key_len=None):
        Bn, S, H = x.shape
        d = H // self.heads
        q, k, v = self.qkv(x).view(Bn, S, 3, self.heads, d).permute(2, 0, 3, 1, 4)
        scores = torch.matmul(q, k.transpose(-1, -2)) * (1.0 / math.sqrt(d))
        ctxt = self.core(scores, v.contiguous(), key_len)
        ctxt = ctxt.permute(0, 2, 1, 3).reshape(Bn, S, H)
        x = self.ln1(x + self.proj(ctxt))
        return self.ln2(x + self.fc2(self.act(self.fc1(x))))
