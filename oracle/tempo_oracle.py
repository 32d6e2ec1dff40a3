"""Plain float64 CPU oracle for the three memory-reduced Tempo layers.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
CPU-baseline leg.  It shares no code with the HIP library and never imports it.

Every function takes float64 arrays whose values the caller has already rounded to
the storage dtype ("f32" or "bf16"), does its arithmetic in float64 in the order the
paper states it, and rounds only where a tensor is *stored* in the storage dtype.

What is pinned and by what (tests/test_oracle_*.py):
  gelu_fwd            library erf-GELU / tanh-GELU of PyTorch CPU float64; GELU(0)=0;
                      minimum location printed in Sec. 3.1 (x ~ -0.75179)
  gelu_bwd            autograd of PyTorch's float64 GELU on the unrounded output;
                      central finite differences; closed-form extremes of GELU'
  kind "silu"         (the same recipe on another single-minimum activation, Sec. 5.1)
                      PyTorch float64 silu + autograd; the minimum in closed form through
                      the Lambert W function: x* = -(1 + W(1/e)), y* = -W(1/e)
  layernorm_fwd/bwd   PyTorch float64 layer_norm + autograd; the output-based gradient of
                      App. D.3 against the input-based twin; finite differences;
                      row invariants (sum dx = 0, sum dx*xhat = 0)
  attn_softmax_dropout_fwd/bwd
                      PyTorch float64 softmax autograd with this oracle's keep bits;
                      rows sum to one; shift invariance; sum dS = 0
  activation_bytes_*  the twelve percentages of App. H (Fig. 10) and the 56 % / 17 %
                      statements of Sec. 2.1
  philox4x32_10       rocRAND's Philox4x32-10 engine run on the host (an independent
                      implementation; same blocks for 64-bit seeds, counters and offsets),
                      plus the closed forms of the two Weyl key increments, the bijectivity
                      of the round function (explicit inverse) and avalanche
  dropout_keep        the same engine's 16-bit lanes under the threshold rule; keep rate, bit
                      balance, lag correlations
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erfc  # library primitive: complementary error function

_SQRT2 = math.sqrt(2.0)
_SQRT_2_OVER_PI = math.sqrt(2.0 / math.pi)
_INV_SQRT_2PI = 1.0 / math.sqrt(2.0 * math.pi)
_TANH_CUBIC = 0.044715

GELU_KINDS = ("erf", "tanh")
#: every activation the in-place recipe is applied to: the two GELU forms and SiLU
ACT_KINDS = GELU_KINDS + ("silu",)
DTYPES = ("f32", "bf16")


# --------------------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------------------
def round_to_dtype(a, dt: str) -> np.ndarray:
    """Round float64 values to the storage dtype (round-to-nearest-even), return float64.

    f32: IEEE binary32.  bf16: 8 significant bits, binary32's exponent range; rounded
    directly from float64 (one rounding), quantum 2^(e-7) with e clamped at -126.
    """
    a = np.asarray(a, dtype=np.float64)
    if dt == "f32":
        with np.errstate(over="ignore"):
            return a.astype(np.float32).astype(np.float64)
    if dt != "bf16":
        raise ValueError(f"unknown dtype {dt!r}")
    out = a.copy()
    fin = np.isfinite(a) & (a != 0.0)
    if np.any(fin):
        v = a[fin]
        _, ex = np.frexp(v)  # v = m * 2^ex, 0.5 <= |m| < 1  ->  floor(log2|v|) = ex - 1
        e = np.maximum(ex.astype(np.int64) - 1, -126)
        q = np.ldexp(1.0, (e - 7).astype(np.int64))
        r = np.rint(v / q) * q  # v / q is exact (power of two); rint is ties-to-even
        big = np.abs(r) >= math.ldexp(1.0, 128)
        r = np.where(big, np.copysign(np.inf, r), r)
        out[fin] = r
    return out


# --------------------------------------------------------------------------------------
# In-place GELU  (Sec. 3.1; App. E.1 eq. 1-2; App. F.1)
# --------------------------------------------------------------------------------------
def gelu_value(x, kind: str) -> np.ndarray:
    """GELU(x).  erf kind: x * Phi(x).  tanh kind: x * sigmoid(2u), which equals
    0.5 x (1 + tanh u) with u = sqrt(2/pi) (x + 0.044715 x^3).
    silu kind (Sec. 5.1 applied to SiLU): x * sigmoid(x)."""
    x = np.asarray(x, dtype=np.float64)
    if kind == "erf":
        return x * (0.5 * erfc(-x / _SQRT2))
    if kind == "silu":
        with np.errstate(over="ignore"):
            return x / (1.0 + np.exp(-x))
    if kind == "tanh":
        u = _SQRT_2_OVER_PI * (x + _TANH_CUBIC * x**3)
        with np.errstate(over="ignore"):
            return x / (1.0 + np.exp(-2.0 * u))
    raise ValueError(f"unknown GELU kind {kind!r}")


def gelu_derivative(x, kind: str) -> np.ndarray:
    """GELU'(x) in terms of the INPUT.  erf: Phi(x) + x phi(x).
    silu: sigma(x) (1 + x (1 - sigma(x))), with 1 - sigma(x) taken as sigma(-x)."""
    x = np.asarray(x, dtype=np.float64)
    if kind == "erf":
        return 0.5 * erfc(-x / _SQRT2) + x * np.exp(-0.5 * x * x) * _INV_SQRT_2PI
    if kind == "silu":
        with np.errstate(over="ignore"):
            sg = 1.0 / (1.0 + np.exp(-x))
            sn = 1.0 / (1.0 + np.exp(x))
        return sg * (1.0 + x * sn)
    if kind == "tanh":
        u = _SQRT_2_OVER_PI * (x + _TANH_CUBIC * x**3)
        du = _SQRT_2_OVER_PI * (1.0 + 3.0 * _TANH_CUBIC * x * x)
        with np.errstate(over="ignore"):
            sg = 1.0 / (1.0 + np.exp(-2.0 * u))
        return sg + x * sg * (1.0 - sg) * 2.0 * du
    raise ValueError(f"unknown GELU kind {kind!r}")


def _solve_minimum(kind: str) -> float:
    """Location of the activation's single minimum: the root of its derivative in
    [-1, -0.5] (GELU) or [-2, -1] (SiLU), by bisection."""
    # GELU'(-1) < 0 < GELU'(-0.5) for both GELU kinds; SiLU'(-2) < 0 < SiLU'(-1)
    lo, hi = (-2.0, -1.0) if kind == "silu" else (-1.0, -0.5)
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if float(gelu_derivative(np.float64(mid), kind)) < 0.0:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


#: x* (float64) where GELU has its minimum, per kind (Sec. 3.1 prints -0.75179 for erf)
GELU_XSTAR = {k: _solve_minimum(k) for k in ACT_KINDS}
#: y* = GELU(x*)
GELU_YSTAR = {k: float(gelu_value(np.float64(GELU_XSTAR[k]), k)) for k in ACT_KINDS}
#: the branch point as compared by the forward pass: x* rounded to binary32
GELU_XSTAR_F32 = {k: float(np.float32(GELU_XSTAR[k])) for k in ACT_KINDS}


def gelu_fwd(x, kind: str, dt: str):
    """(y, m) = GELU*(x)  (App. E.1 eq. 1; App. F.1).

    y is stored in dt; m[e] = 1 iff x[e] >= x* ("greater than or equal to the point at
    which the minimum occurs"), with x* taken at binary32 precision.
    Returns (y float64 holding dt values, m bool array of x's shape).
    """
    x = np.asarray(x, dtype=np.float64)
    y = round_to_dtype(gelu_value(x, kind), dt)
    m = x >= GELU_XSTAR_F32[kind]
    return y, m


def gelu_inverse(y, m, kind: str) -> np.ndarray:
    """x with GELU(x) = y on the branch named by m (App. E.1 eq. 1): m=1 -> x in [x*, inf),
    m=0 -> x in (-inf, x*].  Plain bisection in float64, 200 halvings.

    y at or below the minimum value returns x*.  Entries outside a branch's range are
    clamped to the end of the bracket (the caller treats those cases separately)."""
    y = np.asarray(y, dtype=np.float64)
    m = np.asarray(m, dtype=bool)
    xs = GELU_XSTAR[kind]
    # right branch: x - GELU(x) = x Phi(-x) <= |y*| < 1 for x > 0, and x in [x*, 0] for y < 0
    # (SiLU: x - SiLU(x) = x sigma(-x) <= |y*| < 1 likewise).  Left branch: GELU(-64) and
    # SiLU(-128) lie below the smallest binary32 magnitude.
    finite_y = np.where(np.isfinite(y), y, 0.0)
    lo = np.where(m, xs, -128.0 if kind == "silu" else -64.0)
    hi = np.where(m, np.maximum(finite_y, 0.0) + 1.0, xs)
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        g = gelu_value(mid, kind)
        # right branch increasing, left branch decreasing in x
        go_up = np.where(m, g < y, g > y)
        lo = np.where(go_up, mid, lo)
        hi = np.where(go_up, hi, mid)
    x = 0.5 * (lo + hi)
    return np.where(y <= GELU_YSTAR[kind], xs, x)


def gelu_bwd(dy, y, m, kind: str, dt: str) -> np.ndarray:
    """dx = dy * (GELU' o GELU*^-1)(y, m)  (App. E.1 eq. 2), from the stored output only.

    Readings where the paper is silent:
      y <= y* (stored y rounded below the true minimum)      -> d = 0
      left branch with y >= 0 (underflow, or not from a fwd) -> d = 0
      y = +inf                                               -> d = 1
      NaN propagates.
    dx is stored in dt.
    """
    dy = np.asarray(dy, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    m = np.asarray(m, dtype=bool)
    x = gelu_inverse(y, m, kind)
    d = gelu_derivative(x, kind)
    d = np.where(y <= GELU_YSTAR[kind], 0.0, d)
    d = np.where(~m & (y >= 0.0), 0.0, d)
    d = np.where(m & np.isposinf(y), 1.0, d)
    d = np.where(np.isnan(y), np.nan, d)
    return round_to_dtype(dy * d, dt)


def gelu_bwd_from_input(dy, x, kind: str) -> np.ndarray:
    """Validation twin: the standard input-based gradient dy * GELU'(x), float64."""
    return np.asarray(dy, dtype=np.float64) * gelu_derivative(x, kind)


# --------------------------------------------------------------------------------------
# In-place LayerNorm  (Sec. 3.2; App. D.2, D.3)
# --------------------------------------------------------------------------------------
def layernorm_fwd(x, gamma, beta, eps: float, dt: str):
    """App. D.2: mu_i, biased sigma_i^2, xhat = (x-mu)/sqrt(sigma^2+eps), y = gamma xhat + beta.

    Returns (y in dt, rstd float32-valued, mean float32-valued); rstd = 1/sqrt(sigma^2+eps)
    is the per-row side information kept for backward."""
    x = np.asarray(x, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    M = x.shape[-1]
    mu = x.sum(axis=-1, keepdims=True) / M
    var = ((x - mu) ** 2).sum(axis=-1, keepdims=True) / M
    rstd = 1.0 / np.sqrt(var + float(eps))
    xhat = (x - mu) * rstd
    y = gamma * xhat + beta
    return (round_to_dtype(y, dt),
            round_to_dtype(rstd[..., 0], "f32"),
            round_to_dtype(mu[..., 0], "f32"))


def layernorm_bwd(dy, y, gamma, beta, rstd, dt: str):
    """App. D.3, gradients from the OUTPUT: xhat = (y - beta)/gamma, then
      dgamma_j = sum_i dy_ij xhat_ij,  dbeta_j = sum_i dy_ij,
      dx_ij = rstd_i [ dy_ij gamma_j - xhat_ij (1/M) sum_k dy_ik gamma_k xhat_ik
                                     - (1/M) sum_k dy_ik gamma_k ].
    gamma_j = 0 makes xhat undefined: rejected.  Returns (dx in dt, dgamma f32-valued,
    dbeta f32-valued)."""
    dy = np.asarray(dy, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    rstd = np.asarray(rstd, dtype=np.float64)
    if np.any(gamma == 0.0):
        raise ValueError("in-place LayerNorm backward needs gamma_j != 0")
    M = y.shape[-1]
    xhat = (y - beta) / gamma
    g = dy * gamma
    c1 = (g * xhat).sum(axis=-1, keepdims=True)
    c2 = g.sum(axis=-1, keepdims=True)
    dx = rstd[..., None] * (g - xhat * (c1 / M) - c2 / M)
    lead = tuple(range(dy.ndim - 1))
    dgamma = (dy * xhat).sum(axis=lead)
    dbeta = dy.sum(axis=lead)
    return round_to_dtype(dx, dt), round_to_dtype(dgamma, "f32"), round_to_dtype(dbeta, "f32")


def layernorm_bwd_from_input(dy, x, gamma, eps: float):
    """Validation twin: the standard gradient with xhat taken from the INPUT, float64."""
    dy = np.asarray(dy, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    M = x.shape[-1]
    mu = x.sum(axis=-1, keepdims=True) / M
    var = ((x - mu) ** 2).sum(axis=-1, keepdims=True) / M
    rstd = 1.0 / np.sqrt(var + float(eps))
    xhat = (x - mu) * rstd
    g = dy * gamma
    c1 = (g * xhat).sum(axis=-1, keepdims=True)
    c2 = g.sum(axis=-1, keepdims=True)
    dx = rstd * (g - xhat * (c1 / M) - c2 / M)
    lead = tuple(range(dy.ndim - 1))
    return dx, (dy * xhat).sum(axis=lead), dy.sum(axis=lead)


# --------------------------------------------------------------------------------------
# counter-based RNG for the dropout mask (the paper is silent on the generator)
# Philox4x32-10 as published by Salmon, Moraes, Dror, Shaw (SC'11).
# --------------------------------------------------------------------------------------
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = np.uint64(0x9E3779B9)  # floor(2^32 / golden ratio)
_PHILOX_W1 = np.uint64(0xBB67AE85)  # floor(2^32 (sqrt(3) - 1))
_MASK32 = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox_round(c0, c1, c2, c3, k0, k1):
    """One Philox4x32 round on uint64 arrays holding 32-bit values."""
    p0 = _PHILOX_M0 * c0  # full 64-bit products of 32-bit operands
    p1 = _PHILOX_M1 * c2
    hi0, lo0 = p0 >> _SH32, p0 & _MASK32
    hi1, lo1 = p1 >> _SH32, p1 & _MASK32
    return hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0


def philox4x32_10(counter, key):
    """counter: 4 arrays (or scalars) of 32-bit words, key: 2 words.  Ten rounds, the key
    advanced by the Weyl constants before every round but the first.  Returns four uint64
    arrays holding 32-bit words."""
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) & _MASK32 for c in counter)
    k0 = np.uint64(int(key[0]) & 0xFFFFFFFF)
    k1 = np.uint64(int(key[1]) & 0xFFFFFFFF)
    for r in range(10):
        if r:
            k0 = (k0 + _PHILOX_W0) & _MASK32
            k1 = (k1 + _PHILOX_W1) & _MASK32
        c0, c1, c2, c3 = philox_round(c0, c1, c2, c3, k0, k1)
    return c0, c1, c2, c3


def keep_threshold16(p) -> int:
    """T16: element kept iff its 16-bit draw r < T16; T16 = round-half-up((1-p) 2^16)
    with p taken as the binary32 value handed to the library."""
    pf = float(np.float32(p))
    t = math.floor((1.0 - pf) * 65536.0 + 0.5)
    return max(0, min(65536, t))


def dropout_keep(n: int, p, seed: int, offset: int, start: int = 0) -> np.ndarray:
    """Keep bit K_e for flat element indices e = start .. start+n-1  (Sec. 3.3: each entry
    zeroed with probability p, independently).

    Contract: group g = e >> 3 draws philox4x32_10(counter=(g_lo, g_hi, offset_lo,
    offset_hi), key=(seed_lo, seed_hi)); element e takes 16-bit lane
    (w[(e & 7) >> 1] >> 16 (e & 1)) & 0xFFFF and is kept iff that is < T16.  p == 0 keeps all.
    """
    if n == 0:
        return np.zeros(0, dtype=bool)
    if float(np.float32(p)) == 0.0:
        return np.ones(n, dtype=bool)
    e = np.arange(start, start + n, dtype=np.uint64)
    g = e >> np.uint64(3)
    g_first = int(g[0])
    gs = np.arange(g_first, int(g[-1]) + 1, dtype=np.uint64)
    w = philox4x32_10(
        (gs & _MASK32, gs >> _SH32,
         np.uint64(offset & 0xFFFFFFFF), np.uint64((offset >> 32) & 0xFFFFFFFF)),
        (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF),
    )
    words = np.stack([np.broadcast_to(x, gs.shape) for x in w], axis=1)  # [groups, 4]
    lanes = np.stack([words & np.uint64(0xFFFF), (words >> np.uint64(16)) & np.uint64(0xFFFF)],
                     axis=2).reshape(len(gs), 8)  # lane = 2*word + half
    flat = lanes.reshape(-1)
    first = start - (g_first << 3)
    r = flat[first:first + n]
    return r < np.uint64(keep_threshold16(p))


def pack_bits(bits) -> np.ndarray:
    """Bit e mod 32 of word e div 32 (flat row-major order); pad bits of the last word 0."""
    b = np.asarray(bits, dtype=bool).reshape(-1)
    n_words = (b.size + 31) // 32
    padded = np.zeros(n_words * 32, dtype=np.uint8)
    padded[: b.size] = b
    weights = (np.uint64(1) << np.arange(32, dtype=np.uint64))
    return (padded.reshape(n_words, 32).astype(np.uint64) * weights).sum(axis=1).astype(np.uint32)


def unpack_bits(words, n: int) -> np.ndarray:
    w = np.asarray(words, dtype=np.uint32).astype(np.uint64)
    bits = (w[:, None] >> np.arange(32, dtype=np.uint64)) & np.uint64(1)
    return bits.reshape(-1)[:n].astype(bool)


# --------------------------------------------------------------------------------------
# attention softmax -> dropout, keeping only P and the mask  (Sec. 3.3, 3.4; App. E.3, E.4)
# --------------------------------------------------------------------------------------
def attention_valid(B, A, Sq, Sk, key_len=None, causal=False) -> np.ndarray:
    """True where a score takes part in the softmax: key column j < key_len[b] and, when
    causal, j <= i + (Sk - Sq)."""
    j = np.arange(Sk)[None, None, None, :]
    i = np.arange(Sq)[None, None, :, None]
    valid = np.ones((B, A, Sq, Sk), dtype=bool)
    if key_len is not None:
        kl = np.asarray(key_len).reshape(B, 1, 1, 1)
        valid &= j < kl
    if causal:
        valid &= j <= i + (Sk - Sq)
    return valid


def attn_softmax_dropout_fwd(scores, key_len, causal, p, seed: int, offset: int, dt: str):
    """P = softmax over unmasked scores (masked entries 0; a fully masked row is all 0),
    stored in dt; K ~ Bernoulli(1-p) per element; Out = P K / (1-p) stored in dt.
    Returns (P, Out, K bool [B,A,Sq,Sk])."""
    s = np.asarray(scores, dtype=np.float64)
    B, A, Sq, Sk = s.shape
    valid = attention_valid(B, A, Sq, Sk, key_len, causal)
    neg = np.where(valid, s, -np.inf)
    mx = neg.max(axis=-1, keepdims=True) if Sk else np.zeros((B, A, Sq, 1))
    mx = np.where(np.isfinite(mx), mx, 0.0)
    ex = np.where(valid, np.exp(np.where(valid, s - mx, 0.0)), 0.0)
    den = ex.sum(axis=-1, keepdims=True)
    P = np.where(den > 0.0, ex / np.where(den > 0.0, den, 1.0), 0.0)
    P = round_to_dtype(P, dt)
    K = dropout_keep(s.size, p, seed, offset).reshape(s.shape)
    scale = float(np.float32(1.0) / (np.float32(1.0) - np.float32(p)))
    out = round_to_dtype(P * K * scale, dt)
    return P, out, K


def attn_softmax_dropout_bwd(dout, P, K, p, dt: str):
    """From (dOut, stored P, K): Out recomputed by the mask multiply (Sec. 3.3);
    dP = dOut K/(1-p); dS = P (dP - sum_k dP_k P_k) (softmax gradient from its output,
    Sec. 3.4).  Returns (dS in dt, Out_recomputed in dt)."""
    dout = np.asarray(dout, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    K = np.asarray(K, dtype=bool)
    scale = float(np.float32(1.0) / (np.float32(1.0) - np.float32(p)))
    out_re = round_to_dtype(P * K * scale, dt)
    dP = dout * K * scale
    c = (dP * P).sum(axis=-1, keepdims=True)
    dS = P * (dP - c)
    return round_to_dtype(dS, dt), out_re


# --------------------------------------------------------------------------------------
# activation-memory model per token and encoder layer  (Sec. 2.1; App. H, Fig. 10)
# --------------------------------------------------------------------------------------
def activation_bytes_baseline(H: int, A: int, S: int, e: int) -> int:
    """Bytes the unmodified encoder layer keeps per token for backward: sixteen H-sized
    float maps (layer input, Q, K, V, context, both LayerNorm inputs, first LayerNorm's
    output, the 4H GELU input and the 4H GELU output), two H-sized byte dropout masks, three
    [A,S] float maps (softmax input, softmax output, dropout output) and one [A,S] byte
    mask."""
    return 16 * H * e + 2 * H + 3 * A * S * e + A * S


def activation_bytes_saved_paper(H: int, A: int, S: int, e: int) -> dict:
    """Per-optimisation savings with the paper's 8-bit masks (App. H)."""
    return {
        "gelu": 4 * H * e - 4 * H,      # drop the 4H input, add a 4H byte mask
        "layernorm": 2 * H * e,         # drop both LayerNorm inputs
        "dropout": A * S * e,           # drop the dropout output (mask kept anyway)
        "softmax": A * S * e,           # drop the softmax input
    }


def activation_bytes_saved_bitmask(H: int, A: int, S: int, e: int) -> dict:
    """Same with 1-bit masks and rstd-only LayerNorm statistics (4 bytes less per row and
    LayerNorm than mean + rstd)."""
    return {
        "gelu": 4 * H * e - (4 * H) // 8,
        "layernorm": 2 * (H * e + 4),
        "dropout": A * S * e + (A * S - (A * S) // 8),  # byte mask -> bit mask as well
        "softmax": A * S * e,
    }
