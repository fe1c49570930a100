"""Pins for the fp64 oracle: everything here checks oracle/ against something
other than itself (published known answers, closed forms, invariants, library
routines differentiated by autograd, brute-force finite differences)."""
import math
import os

import numpy as np
import pytest
import torch

import lynx_synth as synth
from oracle import lynx_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_cfg(**kw):
    base = dict(dtype=synth.F32, hidden=8, local_heads=2, head_dim=4, local_ffn=16,
                seq=4, micro_batch=1, dropout_p=0.25, seed=7, layer_id=3)
    base.update(kw)
    return synth.LayerConfig(**base)


def f64_inputs(cfg, random_ln=True, scale_w=0.3):
    """Un-rounded fp64 inputs with O(1) weights so every path carries signal."""
    rng = np.random.default_rng(1234)
    params = {k: rng.standard_normal(shp) * scale_w for k, shp in synth.param_shapes(cfg).items()}
    params["g1"] = 1.0 + 0.2 * rng.standard_normal(cfg.hidden)
    params["g2"] = 1.0 + 0.2 * rng.standard_normal(cfg.hidden)
    X = rng.standard_normal((cfg.tokens, cfg.hidden))
    dOUT = rng.standard_normal((cfg.tokens, cfg.hidden))
    return params, X, dOUT


# ---------------------------------------------------------------- Philox
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = orc.philox4x32_10(*v[:6])
        assert [int(o) for o in out] == v[6:]


def test_philox_vectorised_equals_scalar_bigint():
    # brute force with Python integers (no fixed-width wrap-around to get wrong)
    def scalar(c, k):
        c, k = list(c), list(k)
        for _ in range(10):
            p0, p1 = 0xD2511F53 * c[0], 0xCD9E8D57 * c[2]
            c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
            k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
        return c
    rng = np.random.default_rng(0)
    ctr = rng.integers(0, 2 ** 32, size=(64, 4), dtype=np.uint64)
    key = rng.integers(0, 2 ** 32, size=(64, 2), dtype=np.uint64)
    out = orc.philox4x32_10(ctr[:, 0], ctr[:, 1], ctr[:, 2], ctr[:, 3], key[:, 0], key[:, 1])
    for r in range(64):
        assert [int(o[r]) for o in out] == scalar([int(x) for x in ctr[r]], [int(x) for x in key[r]])


def test_dropout_mask_uses_every_16bit_field_once():
    # eight consecutive elements are the eight 16-bit fields of one Philox call
    seed, step, layer, site = 0x1234567899, 5, 9, 2
    idx = np.arange(8, dtype=np.uint64) + np.uint64(8 * 77)
    stream = (step << 32) | (layer << 2) | site
    w = orc.philox4x32_10(77, 0, stream & 0xFFFFFFFF, stream >> 32,
                          seed & 0xFFFFFFFF, seed >> 32)
    fields = []
    for word in w:
        fields += [int(word) & 0xFFFF, int(word) >> 16]
    for p in (0.1, 0.5, 0.9):
        thr = int(math.floor(float(np.float32(p)) * 65536))
        keep = orc.dropout_keep(seed, step, layer, site, idx, p)
        assert list(keep) == [f >= thr for f in fields]


def test_dropout_range_form_equals_per_element_form():
    for first, count in ((0, 64), (8 * 12345, 256), (2 ** 33 + 16, 40), (3, 21)):
        idx = np.arange(first, first + count, dtype=np.uint64)
        assert np.array_equal(orc.dropout_keep_range(11, 2, 5, 1, first, count, 0.3),
                              orc.dropout_keep(11, 2, 5, 1, idx, 0.3))


def test_dropout_mask_statistics_and_determinism():
    cfg = tiny_cfg(hidden=512, seq=64, micro_batch=4, dropout_p=0.1)
    m1 = orc.hidden_mask(cfg, 0, 1)
    n = m1.size
    assert abs(m1.mean() - (1 - 6553 / 65536)) < 4 * math.sqrt(0.09 / n)
    assert np.array_equal(m1, orc.hidden_mask(cfg, 0, 1))
    for other in (orc.hidden_mask(cfg, 0, 2), orc.hidden_mask(cfg, 1, 1),
                  orc.hidden_mask(cfg.with_(layer_id=4), 0, 1),
                  orc.hidden_mask(cfg.with_(seed=8), 0, 1)):
        agree = (other == m1).mean()
        assert abs(agree - (0.9 ** 2 + 0.1 ** 2)) < 0.01      # independent masks
    assert orc.hidden_mask(cfg.with_(dropout_p=0.0), 0, 1).all()


def test_attention_mask_of_shard_is_slice_of_unsharded_mask():
    full = tiny_cfg(local_heads=4, tp_size=1, seq=8, micro_batch=2)
    for rank in range(2):
        shard = full.with_(local_heads=2, tp_size=2, tp_rank=rank)
        for bi in range(2):
            for hd in range(2):
                assert np.array_equal(orc.attention_mask_slice(shard, 3, bi, hd),
                                      orc.attention_mask_slice(full, 3, bi, rank * 2 + hd))


# ------------------------------------------------------------ LayerNorm
def test_layernorm_forward_invariants():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 64)) * 3 + 1.5
    eps = 1e-5
    y, mu, r = orc.layernorm_fwd(x, np.ones(64), np.zeros(64), eps)
    var = x.var(axis=1)
    assert np.allclose(y.mean(axis=1), 0, atol=1e-14)
    assert np.allclose((y ** 2).mean(axis=1), var / (var + eps), rtol=1e-12)
    assert np.allclose(mu, x.mean(axis=1)) and np.allclose(r, 1 / np.sqrt(var + eps))
    y2, _, _ = orc.layernorm_fwd(x + 10.0, np.ones(64), np.zeros(64), eps)
    assert np.allclose(y, y2, atol=1e-12)
    beta = rng.standard_normal(64)
    yc, _, _ = orc.layernorm_fwd(np.full((2, 64), 3.25), rng.standard_normal(64), beta, eps)
    assert np.allclose(yc, beta)
    # library routine
    g, b = rng.standard_normal(64), rng.standard_normal(64)
    yt = torch.nn.functional.layer_norm(torch.from_numpy(x), (64,), torch.from_numpy(g),
                                        torch.from_numpy(b), eps).numpy()
    assert np.allclose(orc.layernorm_fwd(x, g, b, eps)[0], yt, atol=1e-13)


def test_layernorm_backward_invariants():
    rng = np.random.default_rng(1)
    x, dy, g = rng.standard_normal((6, 32)), rng.standard_normal((6, 32)), rng.standard_normal(32)
    # with eps = 0 the gradient is exactly orthogonal to 1 and to xhat
    _, mu, r = orc.layernorm_fwd(x, g, np.zeros(32), 0.0)
    dx, dg, db = orc.layernorm_bwd(dy, x, mu, r, g)
    xhat = (x - mu[:, None]) * r[:, None]
    assert np.allclose(dx.sum(axis=1), 0, atol=1e-13)
    assert np.allclose((dx * xhat).sum(axis=1), 0, atol=1e-13)
    assert np.allclose(db, dy.sum(axis=0))


# -------------------------------------------------------------- softmax
def test_softmax_invariants():
    rng = np.random.default_rng(2)
    z = rng.standard_normal((16, 16)) * 4
    P = orc.softmax_rows(z, True)
    assert np.allclose(P.sum(axis=1), 1, atol=1e-14) and (P >= 0).all()
    assert (np.triu(P, 1) == 0).all()
    assert P[0, 0] == 1.0
    assert np.allclose(P, orc.softmax_rows(z + 123.0, True), atol=1e-13)
    zt = torch.from_numpy(z).masked_fill(~torch.tril(torch.ones(16, 16, dtype=torch.bool)), -math.inf)
    assert np.allclose(P, torch.softmax(zt, dim=1).numpy(), atol=1e-15)
    assert np.allclose(orc.softmax_rows(z, False), torch.softmax(torch.from_numpy(z), 1).numpy(), atol=1e-15)


# ----------------------------------------------------------------- GeLU
def test_gelu_identities():
    u = np.linspace(-6, 6, 241)
    assert orc.gelu(np.zeros(1))[0] == 0.0
    assert orc.gelu_grad(np.zeros(1))[0] == 0.5
    assert np.allclose(orc.gelu(u) - orc.gelu(-u), u, atol=1e-15)
    assert np.allclose(orc.gelu(np.array([20.0, 35.0])), [20.0, 35.0])
    assert np.allclose(orc.gelu(u), torch.nn.functional.gelu(torch.from_numpy(u), approximate="tanh").numpy(), atol=1e-15)
    hstep = 1e-6
    fd = (orc.gelu(u + hstep) - orc.gelu(u - hstep)) / (2 * hstep)
    assert np.allclose(orc.gelu_grad(u), fd, atol=1e-8)


# ---------------------------------------------------------- whole layer
def test_zero_output_projections_make_layer_identity():
    cfg = tiny_cfg(seq=8, micro_batch=2)
    params, X, dOUT = f64_inputs(cfg)
    for k in ("wo", "bo", "w2", "b2"):
        params[k] = np.zeros_like(params[k])
    acts, g = orc.layer_forward_backward(cfg, params, X, dOUT, step=2)
    assert np.array_equal(acts["OUT"], X)
    assert np.allclose(g["dX"], dOUT, atol=1e-15)


def test_single_position_attention_returns_v():
    cfg = tiny_cfg(seq=1, micro_batch=3, dropout_p=0.0)
    params, X, _ = f64_inputs(cfg)
    acts = orc.layer_forward(cfg, params, X)
    p = cfg.proj
    assert (acts["P"] == 1.0).all()
    assert np.allclose(acts["C"], acts["QKV"][:, 2 * p:], atol=1e-15)


def test_zero_query_gives_running_mean_of_v():
    cfg = tiny_cfg(seq=8, micro_batch=2, dropout_p=0.0)
    params, X, _ = f64_inputs(cfg)
    p = cfg.proj
    params["wqkv"][:p] = 0
    params["bqkv"][:p] = 0
    acts = orc.layer_forward(cfg, params, X)
    s = cfg.seq
    for i in range(s):
        assert np.allclose(acts["P"][:, :, i, :i + 1], 1.0 / (i + 1), atol=1e-15)
    v = acts["QKV"][:, 2 * p:].reshape(cfg.micro_batch, s, p)
    run_mean = np.cumsum(v, axis=1) / np.arange(1, s + 1)[None, :, None]
    assert np.allclose(acts["C"].reshape(cfg.micro_batch, s, p), run_mean, atol=1e-14)


def test_dropout_scaling_and_mask_application():
    cfg = tiny_cfg(seq=8, micro_batch=2, dropout_p=0.25)
    params, X, _ = f64_inputs(cfg)
    acts = orc.layer_forward(cfg, params, X, step=1)
    c = 1 / (1 - 0.25)
    assert np.allclose(acts["Pd"], np.where(acts["keep0"], acts["P"] * c, 0.0))
    assert np.allclose(acts["X2"] - X, np.where(acts["keep1"], (acts["O"] + params["bo"]) * c, 0.0))
    assert np.allclose(acts["OUT"] - acts["X2"], np.where(acts["keep2"], (acts["V2"] + params["b2"]) * c, 0.0))
    assert not acts["keep1"].all() and acts["keep1"].any()


def test_softmax_backward_row_dot_is_dc_dot_c():
    """The identity the GPU's one-pass dS kernel rests on: the row term of the softmax
    backward, sum_j dP_ij P_ij with dP = keep c dPd and dPd = dC V^T, equals
    sum_j dPd_ij Pd_ij = dC_i . (Pd V)_i = dC_i . C_i, for any dC.  Checked on the oracle's own
    forward tensors (its backward forms the sum over j as written in the definition)."""
    cfg = tiny_cfg(seq=12, micro_batch=2, dropout_p=0.25)
    params, X, _ = f64_inputs(cfg)
    acts = orc.layer_forward(cfg, params, X, step=2)
    b, s, a, d = cfg.micro_batch, cfg.seq, cfg.local_heads, cfg.head_dim
    p = a * d
    c = 1 / (1 - 0.25)
    rng = np.random.default_rng(3)
    dC = rng.standard_normal((b * s, p))
    for bi in range(b):
        rows = slice(bi * s, (bi + 1) * s)
        for hd in range(a):
            v = acts["QKV"][rows, 2 * p + hd * d:2 * p + (hd + 1) * d]
            dc = dC[rows, hd * d:(hd + 1) * d]
            dP = acts["keep0"][bi, hd] * (dc @ v.T) * c
            by_definition = (dP * acts["P"][bi, hd]).sum(axis=1)
            from_context = (dc * acts["C"][rows, hd * d:(hd + 1) * d]).sum(axis=1)
            assert np.allclose(by_definition, from_context, rtol=1e-12, atol=1e-13)
    assert not acts["keep0"].all()      # the masks do drop something


def _torch_block(cfg, params, X, masks):
    """The same block from library primitives, differentiated by autograd."""
    F = torch.nn.functional
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in params.items()}
    x = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    b, s, a, d, h = cfg.micro_batch, cfg.seq, cfg.local_heads, cfg.head_dim, cfg.hidden
    p = a * d
    c = 1.0 / (1.0 - float(np.float32(cfg.dropout_p)))
    k0, k1, k2 = (torch.tensor(m, dtype=torch.float64) for m in masks)
    y1 = F.layer_norm(x, (h,), t["g1"], t["be1"], cfg.ln_eps)
    qkv = F.linear(y1, t["wqkv"], t["bqkv"]).view(b, s, 3, a, d)
    q, k, v = (qkv[:, :, i].permute(0, 2, 1, 3) for i in range(3))      # [b,a,s,d]
    sc = torch.matmul(q, k.transpose(-1, -2)) / math.sqrt(d)
    if cfg.causal:
        sc = sc.masked_fill(~torch.tril(torch.ones(s, s, dtype=torch.bool)), -math.inf)
    pd = torch.softmax(sc, dim=-1) * k0 * c
    ctx = torch.matmul(pd, v).permute(0, 2, 1, 3).reshape(b * s, p)
    x2 = x + k1 * F.linear(ctx, t["wo"], t["bo"]) * c
    y2 = F.layer_norm(x2, (h,), t["g2"], t["be2"], cfg.ln_eps)
    g = F.gelu(F.linear(y2, t["w1"], t["b1"]), approximate="tanh")
    out = x2 + k2 * F.linear(g, t["w2"], t["b2"]) * c
    return out, x, t


@pytest.mark.parametrize("causal", [1, 0])
def test_layer_against_library_autograd(causal):
    cfg = tiny_cfg(hidden=32, local_heads=3, head_dim=8, local_ffn=40, seq=16, micro_batch=2,
                   dropout_p=0.1, causal=causal, tp_size=2, tp_rank=1)
    params, X, dOUT = f64_inputs(cfg)
    acts, g = orc.layer_forward_backward(cfg, params, X, dOUT, step=4)
    out, x, t = _torch_block(cfg, params, X, (acts["keep0"], acts["keep1"], acts["keep2"]))
    assert np.allclose(acts["OUT"], out.detach().numpy(), rtol=1e-12, atol=1e-12)
    out.backward(torch.tensor(dOUT))
    assert np.allclose(g["dX"], x.grad.numpy(), rtol=1e-10, atol=1e-12)
    for k in synth.PARAM_NAMES:
        assert np.allclose(g[k], t[k].grad.numpy(), rtol=1e-10, atol=1e-12), k


def test_layer_against_library_autograd_at_c1_shape():
    cfg = synth.CONFIGS["C1"]
    params = synth.make_params(cfg, random_ln=True)
    X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
    acts, g = orc.layer_forward_backward(cfg, params, X, dOUT)
    out, x, t = _torch_block(cfg, params, X, (acts["keep0"], acts["keep1"], acts["keep2"]))
    assert np.allclose(acts["OUT"], out.detach().numpy(), rtol=1e-11, atol=1e-11)
    out.backward(torch.tensor(dOUT, dtype=torch.float64))
    assert np.allclose(g["dX"], x.grad.numpy(), rtol=1e-9, atol=1e-11)
    for k in synth.PARAM_NAMES:
        assert np.allclose(g[k], t[k].grad.numpy(), rtol=1e-9, atol=1e-11), k


def test_gradients_by_central_finite_differences():
    """Brute force: perturb every input and parameter element of a tiny layer
    (masks are a pure function of indices, so they stay fixed)."""
    cfg = tiny_cfg()
    params, X, dOUT = f64_inputs(cfg)
    _, g = orc.layer_forward_backward(cfg, params, X, dOUT, step=1)

    def loss(pr, x):
        return float((orc.layer_forward(cfg, pr, x, step=1)["OUT"] * dOUT).sum())

    hstep = 1e-6
    worst = 0.0
    targets = [("dX", None)] + [(k, k) for k in synth.PARAM_NAMES]
    for gname, pname in targets:
        base = X if pname is None else params[pname]
        fd = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = base[i]
            base[i] = old + hstep
            lp = loss(params, X)
            base[i] = old - hstep
            lm = loss(params, X)
            base[i] = old
            fd[i] = (lp - lm) / (2 * hstep)
        err = np.abs(fd - g[gname]).max() / max(np.abs(g[gname]).max(), 1e-30)
        worst = max(worst, err)
        assert err < 1e-6, (gname, err)
    assert worst < 1e-6
