"""fp64 CPU oracle of one GPT transformer block shard: forward and backward.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file;
only tests, the smoke check and the benchmark's CPU-baseline leg call it.  It
shares no code with the HIP kernels.

What it is the oracle of.  The paper's method (retain a subset S_i of a layer's
operator outputs, regenerate the rest before backward; Sec. 4.2 "Problem
definition", Eq. 3-4) is defined to be transparent: a recomputed tensor stands
in for the discarded one (Sec. 2.2), so whatever the retain/recompute policy,
the values of every activation and gradient are those of the plain store-all
forward and backward.  The oracle is therefore that plain definition written
out, with no policy machinery in the numeric path.  The paper defers the block
itself to the GPT architecture with Megatron-style tensor parallelism (Sec. 2.1
and the tensor-parallel figure there: an attention block and an MLP block, each
followed by an all-reduce); the block below is the textbook pre-LayerNorm GPT
block restricted to one tensor-parallel rank's heads and FFN columns, with the
all-reduce an identity.  Conventions the paper is silent on (epsilon, tanh
GeLU, the Philox element map, layouts) are listed next to each function.

Everything is float64; inputs arrive already rounded to the storage type and
are only promoted.  Matrix products use numpy's matmul as a library primitive;
there is no blocking, fusion or reordering beyond the textbook formulas.

Operator outputs ("activations") are numbered as in the 13-operator
decomposition of the layer:
  A0 X, A1 Y1, A2 QKV, A3 S, A4 P, A5 Pd, A6 C, A7 O, A8 X2, A9 Y2, A10 U,
  A11 G, A12 V2, A13 OUT.
"""
from __future__ import annotations

import math
from typing import Dict, Tuple

import numpy as np

ACT_NAMES = ("X", "Y1", "QKV", "S", "P", "Pd", "C", "O", "X2", "Y2", "U", "G",
             "V2", "OUT")

# --------------------------------------------------------------------------
# Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
# as 1, 2, 3", SC'11).  Pure integer arithmetic, so masks are exact.
# --------------------------------------------------------------------------
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = np.uint64(0x9E3779B9)
_PHILOX_W1 = np.uint64(0xBB67AE85)
_LO32 = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten rounds of Philox-4x32.  All arguments are 32-bit values (scalars or
    arrays, broadcast together); returns four uint64 arrays holding 32-bit words."""
    c0, c1, c2, c3, k0, k1 = (np.asarray(v, dtype=np.uint64) & _LO32
                              for v in (c0, c1, c2, c3, k0, k1))
    for _ in range(10):
        prod0 = _PHILOX_M0 * c0          # 32x32 -> 64 bit, exact in uint64
        prod1 = _PHILOX_M1 * c2
        hi0, lo0 = prod0 >> _SH32, prod0 & _LO32
        hi1, lo1 = prod1 >> _SH32, prod1 & _LO32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
        k0 = (k0 + _PHILOX_W0) & _LO32
        k1 = (k1 + _PHILOX_W1) & _LO32
    return c0, c1, c2, c3


def dropout_threshold(p: float) -> int:
    """16-bit drop threshold: an element is kept iff its 16 random bits are
    >= floor(p * 65536), p taken at float32 precision as the library receives it."""
    return int(math.floor(float(np.float32(p)) * 65536.0))


def dropout_keep(seed: int, step: int, layer_id: int, site: int,
                 idx: np.ndarray, p: float) -> np.ndarray:
    """Keep-mask (bool) for flat element indices `idx` (uint64) of one dropout
    site.  Convention: one Philox call serves 8 consecutive elements, 16 bits
    each.  key = (seed lo, seed hi); counter = (n lo, n hi, stream lo, stream
    hi) with n = idx // 8 and stream = step * 2^32 + layer_id * 4 + site;
    element idx uses bits [16*(l&1), +16) of output word l >> 1, l = idx % 8."""
    idx = np.asarray(idx, dtype=np.uint64)
    n = idx >> np.uint64(3)
    lane = idx & np.uint64(7)
    stream = (int(step) << 32) | (int(layer_id) << 2) | int(site)
    w = philox4x32_10(n & _LO32, n >> _SH32, stream & 0xFFFFFFFF, stream >> 32,
                      seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    word_sel = lane >> np.uint64(1)
    word = np.where(word_sel == 0, w[0],
                    np.where(word_sel == 1, w[1],
                             np.where(word_sel == 2, w[2], w[3])))
    u16 = (word >> (np.uint64(16) * (lane & np.uint64(1)))) & np.uint64(0xFFFF)
    return u16 >= np.uint64(dropout_threshold(p))


def dropout_keep_range(seed: int, step: int, layer_id: int, site: int,
                       first: int, count: int, p: float) -> np.ndarray:
    """dropout_keep for the contiguous indices first .. first+count-1, with the
    generator evaluated once per group of 8 elements instead of once per
    element (same values; first and count must be multiples of 8)."""
    if first % 8 or count % 8:
        return dropout_keep(seed, step, layer_id, site,
                            np.arange(first, first + count, dtype=np.uint64), p)
    n = np.arange(first // 8, (first + count) // 8, dtype=np.uint64)
    stream = (int(step) << 32) | (int(layer_id) << 2) | int(site)
    w = philox4x32_10(n & _LO32, n >> _SH32, stream & 0xFFFFFFFF, stream >> 32,
                      seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    fields = np.empty((n.size, 8), dtype=np.uint64)
    for k in range(4):
        fields[:, 2 * k] = w[k] & np.uint64(0xFFFF)
        fields[:, 2 * k + 1] = w[k] >> np.uint64(16)
    return (fields >= np.uint64(dropout_threshold(p))).reshape(-1)


def hidden_mask(cfg, step: int, site: int) -> np.ndarray:
    """Mask of a hidden-dropout site (1: after the attention projection, 2:
    after FC2), shape [T, h].  Element index t*h + j: the same on every
    tensor-parallel rank, as it must be for a tensor that follows an all-reduce."""
    T, h = cfg.micro_batch * cfg.seq, cfg.hidden
    return dropout_keep_range(cfg.seed, step, cfg.layer_id, site, 0, T * h,
                              cfg.dropout_p).reshape(T, h)


def attention_mask_slice(cfg, step: int, bi: int, hd: int) -> np.ndarray:
    """Mask of the attention-dropout site (0) for batch element bi and local
    head hd, shape [s, s].  Element index ((bi*A + g)*s + i)*s + j with A the
    global head count and g = tp_rank*a + hd the global head, so a shard's mask
    is the matching slice of the unsharded layer's mask."""
    s, a = cfg.seq, cfg.local_heads
    A = a * cfg.tp_size
    g = cfg.tp_rank * a + hd
    return dropout_keep_range(cfg.seed, step, cfg.layer_id, 0, (bi * A + g) * s * s,
                              s * s, cfg.dropout_p).reshape(s, s)


# --------------------------------------------------------------------------
# Elementary operators
# --------------------------------------------------------------------------
def layernorm_fwd(x, gamma, beta, eps):
    """Per-row LayerNorm with biased variance; returns (y, mean, rstd)."""
    mu = x.mean(axis=1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return gamma * xhat + beta, mu[:, 0], rstd[:, 0]


def layernorm_bwd(dy, x, mu, rstd, gamma):
    """Returns (dx, dgamma, dbeta) for y = gamma * xhat + beta."""
    xhat = (x - mu[:, None]) * rstd[:, None]
    g = dy * gamma
    dx = rstd[:, None] * (g - g.mean(axis=1, keepdims=True)
                          - xhat * (g * xhat).mean(axis=1, keepdims=True))
    return dx, (dy * xhat).sum(axis=0), dy.sum(axis=0)


_KAPPA = math.sqrt(2.0 / math.pi)
_GELU_C = 0.044715


def gelu(u):
    """tanh-form GeLU (the GPT-2 form)."""
    return 0.5 * u * (1.0 + np.tanh(_KAPPA * (u + _GELU_C * u ** 3)))


def gelu_grad(u):
    th = np.tanh(_KAPPA * (u + _GELU_C * u ** 3))
    return 0.5 * (1.0 + th) + 0.5 * u * (1.0 - th * th) * _KAPPA * (1.0 + 3.0 * _GELU_C * u * u)


def softmax_rows(z, causal: bool):
    """Row softmax of a square score slice; with causal masking entry (i, j) is
    excluded exactly (probability 0) for j > i."""
    s = z.shape[0]
    if causal:
        allowed = np.tril(np.ones((s, s), dtype=bool))
        z = np.where(allowed, z, -np.inf)
    m = z.max(axis=1, keepdims=True)
    e = np.exp(z - m)
    return e / e.sum(axis=1, keepdims=True)


def _f64(params: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {k: np.asarray(v, dtype=np.float64) for k, v in params.items()}


# --------------------------------------------------------------------------
# The layer
# --------------------------------------------------------------------------
def layer_forward(cfg, params, X, step: int = 0) -> Dict[str, np.ndarray]:
    """Forward of the block, operators 1..13 in order.  Returns every named
    activation, both LayerNorm statistics and the three keep-masks.

    Layouts: tokens are batch-major (t = bi*s + i); QKV columns are ordered
    [q|k|v][head][dd]; weights are [out, in]; S, P, Pd are [b, a, s, s].
    """
    w = _f64(params)
    X = np.asarray(X, dtype=np.float64)
    b, s, a, d = cfg.micro_batch, cfg.seq, cfg.local_heads, cfg.head_dim
    p_w, T = a * d, b * s
    c = 1.0 / (1.0 - float(np.float32(cfg.dropout_p)))
    causal = bool(cfg.causal)
    out: Dict[str, np.ndarray] = {"X": X}

    # OP1: LayerNorm 1
    Y1, mu1, r1 = layernorm_fwd(X, w["g1"], w["be1"], cfg.ln_eps)
    # OP2: QKV projection (column-parallel: this rank's heads)
    QKV = Y1 @ w["wqkv"].T + w["bqkv"]
    # OP3..OP6 per (batch element, head)
    S = np.zeros((b, a, s, s))
    P = np.zeros((b, a, s, s))
    Pd = np.zeros((b, a, s, s))
    keep0 = np.zeros((b, a, s, s), dtype=bool)
    C = np.zeros((T, p_w))
    for bi in range(b):
        rows = slice(bi * s, (bi + 1) * s)
        for hd in range(a):
            q = QKV[rows, 0 * p_w + hd * d:0 * p_w + (hd + 1) * d]
            k = QKV[rows, 1 * p_w + hd * d:1 * p_w + (hd + 1) * d]
            v = QKV[rows, 2 * p_w + hd * d:2 * p_w + (hd + 1) * d]
            S[bi, hd] = q @ k.T                                   # OP3 (unscaled)
            P[bi, hd] = softmax_rows(S[bi, hd] / math.sqrt(d), causal)   # OP4
            keep0[bi, hd] = attention_mask_slice(cfg, step, bi, hd)
            Pd[bi, hd] = keep0[bi, hd] * P[bi, hd] * c           # OP5
            C[rows, hd * d:(hd + 1) * d] = Pd[bi, hd] @ v        # OP6
    # OP7: attention output projection (row-parallel; the all-reduce that
    # follows is an identity for a lone rank, and the bias is added after it)
    O = C @ w["wo"].T
    # OP8: bias + dropout + residual
    keep1 = hidden_mask(cfg, step, 1)
    X2 = X + keep1 * (O + w["bo"]) * c
    # OP9: LayerNorm 2
    Y2, mu2, r2 = layernorm_fwd(X2, w["g2"], w["be2"], cfg.ln_eps)
    # OP10: FC1 (column-parallel), OP11: GeLU, OP12: FC2 (row-parallel)
    U = Y2 @ w["w1"].T + w["b1"]
    G = gelu(U)
    V2 = G @ w["w2"].T
    # OP13: bias + dropout + residual
    keep2 = hidden_mask(cfg, step, 2)
    OUT = X2 + keep2 * (V2 + w["b2"]) * c

    out.update(Y1=Y1, QKV=QKV, S=S, P=P, Pd=Pd, C=C, O=O, X2=X2, Y2=Y2, U=U,
               G=G, V2=V2, OUT=OUT, mu1=mu1, rstd1=r1, mu2=mu2, rstd2=r2,
               keep0=keep0, keep1=keep1, keep2=keep2)
    return out


def layer_backward(cfg, params, acts, dOUT, taps=None) -> Dict[str, np.ndarray]:
    """Backward of the block given the forward's activations and dL/dOUT.
    Returns dX and the gradient of every parameter (same names as params).
    If `taps` is a dict it also receives the gradients with respect to the
    named activations as they are formed on the way down (dV2, dU, dY2, dX2,
    dO, dC, dS, dQKV, dY1); nothing else changes."""
    w = _f64(params)
    dOUT = np.asarray(dOUT, dtype=np.float64)
    b, s, a, d = cfg.micro_batch, cfg.seq, cfg.local_heads, cfg.head_dim
    p_w = a * d
    c = 1.0 / (1.0 - float(np.float32(cfg.dropout_p)))
    g: Dict[str, np.ndarray] = {}

    # B13: OUT = X2 + keep2 * (V2 + b2) * c
    dV2 = acts["keep2"] * dOUT * c
    g["b2"] = dV2.sum(axis=0)
    dX2 = dOUT.copy()
    # B12: V2 = G W2^T
    dG = dV2 @ w["w2"]
    g["w2"] = dV2.T @ acts["G"]
    # B11: G = gelu(U)
    dU = dG * gelu_grad(acts["U"])
    g["b1"] = dU.sum(axis=0)
    # B10: U = Y2 W1^T + b1
    dY2 = dU @ w["w1"]
    g["w1"] = dU.T @ acts["Y2"]
    # B9: LayerNorm 2
    dx, g["g2"], g["be2"] = layernorm_bwd(dY2, acts["X2"], acts["mu2"], acts["rstd2"], w["g2"])
    dX2 = dX2 + dx
    # B8: X2 = X + keep1 * (O + bo) * c
    dO = acts["keep1"] * dX2 * c
    g["bo"] = dO.sum(axis=0)
    dX = dX2.copy()
    # B7: O = C Wo^T
    dC = dO @ w["wo"]
    g["wo"] = dO.T @ acts["C"]
    # B6..B3 per (batch element, head)
    QKV = acts["QKV"]
    dQKV = np.zeros_like(QKV)
    for bi in range(b):
        rows = slice(bi * s, (bi + 1) * s)
        for hd in range(a):
            cq = slice(0 * p_w + hd * d, 0 * p_w + (hd + 1) * d)
            ck = slice(1 * p_w + hd * d, 1 * p_w + (hd + 1) * d)
            cv = slice(2 * p_w + hd * d, 2 * p_w + (hd + 1) * d)
            q, k, v = QKV[rows, cq], QKV[rows, ck], QKV[rows, cv]
            dc = dC[rows, hd * d:(hd + 1) * d]
            P, Pd = acts["P"][bi, hd], acts["Pd"][bi, hd]
            dPd = dc @ v.T                                   # B6
            dQKV[rows, cv] = Pd.T @ dc
            dP = acts["keep0"][bi, hd] * dPd * c             # B5
            # B4: P is exactly 0 above the diagonal, hence so are dZ and dS
            dZ = P * (dP - (dP * P).sum(axis=1, keepdims=True))
            dS = dZ / math.sqrt(d)
            dQKV[rows, cq] = dS @ k                          # B3
            dQKV[rows, ck] = dS.T @ q
            if taps is not None:
                taps.setdefault("dS", np.zeros((b, a, s, s)))[bi, hd] = dS
    # B2: QKV = Y1 Wqkv^T + bqkv
    dY1 = dQKV @ w["wqkv"]
    g["wqkv"] = dQKV.T @ acts["Y1"]
    g["bqkv"] = dQKV.sum(axis=0)
    # B1: LayerNorm 1
    dx, g["g1"], g["be1"] = layernorm_bwd(dY1, acts["X"], acts["mu1"], acts["rstd1"], w["g1"])
    g["dX"] = dX + dx
    if taps is not None:
        taps.update(dV2=dV2, dU=dU, dY2=dY2, dX2=dX2, dO=dO, dC=dC, dQKV=dQKV, dY1=dY1)
    return g


def layer_forward_backward(cfg, params, X, dOUT, step: int = 0
                           ) -> Tuple[Dict[str, np.ndarray], Dict[str, np.ndarray]]:
    acts = layer_forward(cfg, params, X, step)
    return acts, layer_backward(cfg, params, acts, dOUT)
