"""Dropout decisions inside the kernels that apply them, against the oracle's
keep-masks, element by element.

lynx_dropout_mask (tests/test_gpu_parity.py) checks the generator through a dump
kernel.  The kernels of the layer each form the Philox counter from their own
index arithmetic: the softmax + dropout forward, the stand-alone attention
dropout, the bias + dropout + residual epilogue of the matrix-core products
(with its column offset on edge strips), its stand-alone form, the dropout
backward with the bias gradient, the LayerNorm backward that also undoes the
dropout below it, and the score-gradient kernel.  Every one of those operators
is an exact function of tensors the library hands out (activations, tapped
gradients) and of the keep-mask: out = f(in, keep) with one or two fp32
operations and one rounding.  So the test replays f on the GPU's own inputs
with the ORACLE's mask and demands the GPU's output bit for bit; the zero
patterns (kept <=> nonzero, both directions) are asserted on top.  For dS,
which sits behind a matrix product, the GPU's decision is read off each element
(is it nearer to the kept or to the dropped candidate?) wherever the two
candidates are far apart, and compared with the oracle's bit."""
import numpy as np
import pytest
import torch

import lynx_synth as synth
from oracle import lynx_oracle as orc
from oracle import policy_model as pm
from harness import GpuLayer
from test_gpu_parity import SMALL

pytestmark = pytest.mark.gpu

STEP = 5


def scale32(cfg):
    """1 / (1 - p) as the library forms it: fp32 throughout."""
    return float(np.float32(1.0) / (np.float32(1.0) - np.float32(cfg.dropout_p)))


def storage(t, cfg):
    return t.to(torch.bfloat16) if cfg.dtype == synth.BF16 else t


def keep_hidden(cfg, site):
    return torch.from_numpy(orc.hidden_mask(cfg, STEP, site)).cuda()


def keep_attn(cfg, slices):
    return {z: torch.from_numpy(orc.attention_mask_slice(cfg, STEP, z[0], z[1])).cuda() for z in slices}


def replay_dropout(x, keep, c):
    """keep ? x * c : 0 in fp32."""
    return torch.where(keep, x.float() * c, torch.zeros((), device=x.device))


def check_forward(cfg, layer, slices, params_dev):
    """Pd from P, X2 from (X, O), OUT from (X2, V2): bit for bit under the oracle's masks."""
    c = scale32(cfg)
    T, h, s, a = cfg.tokens, cfg.hidden, cfg.seq, cfg.local_heads
    P = layer.activation_raw(4).view(cfg.micro_batch, a, s, s)
    Pd = layer.activation_raw(5).view(cfg.micro_batch, a, s, s)
    lower = torch.ones(s, s, dtype=torch.bool, device="cuda").tril()
    for (bi, hd), keep in keep_attn(cfg, slices).items():
        want = storage(replay_dropout(P[bi, hd], keep, c), cfg)
        assert torch.equal(Pd[bi, hd][lower], want[lower]), ("Pd", bi, hd)
        # zero pattern, both directions
        assert torch.equal((Pd[bi, hd] != 0) & lower, keep & (P[bi, hd] != 0) & lower), ("Pd pattern", bi, hd)
    del P, Pd
    for site, res_id, prod_id, out_id, bias in ((1, 0, 7, 8, "bo"), (2, 8, 12, 13, "b2")):
        keep = keep_hidden(cfg, site)
        res = layer.activation_raw(res_id).view(T, h).float()
        prod = layer.activation_raw(prod_id).view(T, h).float()
        out = layer.activation_raw(out_id).view(T, h)
        a_ = replay_dropout(prod + params_dev[bias].float(), keep, c)
        want = storage(res + a_, cfg)
        assert torch.equal(out, want), ("bias+dropout+residual", site)
        # zero pattern: the residual stream changes only where the mask keeps, and everywhere
        # it keeps unless the addend is zero or too small to change the stored value
        changed = out.float() != res
        assert not (changed & ~keep).any(), ("changed where dropped", site)
        assert torch.equal(changed, keep & (want.float() != res)), ("pattern", site)
        assert (changed.sum().item() > 0.8 * keep.sum().item()), site
        del keep, res, prod, out, a_, want, changed


def check_backward(cfg, layer, slices, acts_before):
    """dV2 from dOUT, dO from dX2 (bit for bit); dS: the decision read off every element."""
    c = scale32(cfg)
    T, h, s, a, d, b = cfg.tokens, cfg.hidden, cfg.seq, cfg.local_heads, cfg.head_dim, cfg.micro_batch
    p_w = a * d
    taps = layer.taps
    keep2, keep1 = keep_hidden(cfg, 2), keep_hidden(cfg, 1)
    dout = layer.dout.view(T, h)
    want = storage(replay_dropout(dout, keep2, c), cfg)
    assert torch.equal(taps["dV2"].view(T, h), want), "dV2"
    assert torch.equal(taps["dV2"].view(T, h) != 0, keep2 & (dout != 0)), "dV2 pattern"
    dx2 = taps["dX2"].view(T, h)
    want = storage(replay_dropout(dx2, keep1, c), cfg)
    assert torch.equal(taps["dO"].view(T, h), want), "dO"
    assert torch.equal(taps["dO"].view(T, h) != 0, keep1 & (dx2 != 0)), "dO pattern"
    del keep1, keep2, want
    # dS = scale P (keep c round(dPd) - dot), dPd = dC V^T, dot = sum_dd dC C
    eps = 2.0 ** -8 if cfg.dtype == synth.BF16 else 2.0 ** -20
    sc = 1.0 / np.sqrt(d)
    dS = taps["dS"].view(b, a, s, s)
    dC = taps["dC"].view(T, p_w).float()
    P, C, QKV = acts_before["P"].view(b, a, s, s), acts_before["C"].view(T, p_w).float(), acts_before["QKV"].view(T, 3 * p_w).float()
    lower = torch.ones(s, s, dtype=torch.bool, device="cuda").tril()
    decided_total = 0
    lower_total = 0
    for (bi, hd), keep in keep_attn(cfg, slices).items():
        rows = slice(bi * s, (bi + 1) * s)
        dc = dC[rows, hd * d:(hd + 1) * d]
        v = QKV[rows, 2 * p_w + hd * d:2 * p_w + (hd + 1) * d]
        dpd = storage(dc.double() @ v.double().T, cfg).float() if cfg.dtype == synth.BF16 else (dc.double() @ v.double().T).float()
        dot = (dc * C[rows, hd * d:(hd + 1) * d]).sum(dim=1, keepdim=True)
        pr = P[bi, hd].float()
        kept = sc * pr * (c * dpd - dot)
        dropped = sc * pr * (-dot)
        got = dS[bi, hd].float()
        gap = (kept - dropped).abs()
        noise = eps * (torch.maximum(kept.abs(), dropped.abs()) + sc * pr * dot.abs()) + 1e-30
        decidable = lower & (gap > 32 * noise)
        gpu_keep = (got - kept).abs() < (got - dropped).abs()
        assert torch.equal(gpu_keep[decidable], keep[decidable]), ("dS decision", bi, hd)
        decided_total += int(decidable.sum())
        lower_total += int(lower.sum())
    assert decided_total > 0.5 * lower_total, (decided_total, lower_total)


def all_slices(cfg):
    return [(bi, hd) for bi in range(cfg.micro_batch) for hd in range(cfg.local_heads)]


@pytest.mark.parametrize("name", [n for n in SMALL if SMALL[n].dropout_p > 0])
def test_masks_inside_forward_and_backward_kernels(name):
    cfg = SMALL[name]
    params = synth.make_params(cfg, random_ln=True)
    X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
    layer = GpuLayer(cfg, params)
    slices = all_slices(cfg)[:8]
    layer.forward(X, pm.STORE_ALL, step=STEP)
    torch.cuda.synchronize()
    check_forward(cfg, layer, slices, layer.params)
    before = {"P": layer.activation_raw(4), "C": layer.activation_raw(6), "QKV": layer.activation_raw(2)}
    layer.tap_gradients(["dV2", "dX2", "dO", "dC", "dS"])
    layer.backward(dOUT)
    torch.cuda.synchronize()
    check_backward(cfg, layer, slices, before)
    layer.close()


@pytest.mark.parametrize("name", ["tiles_bf16", "edge_bf16", "ragged_bf16", "ragged_f32", "C1"])
def test_masks_inside_the_standalone_dropout_kernels(name):
    """Regeneration in pieces runs the stand-alone forms: Pd from a resident P (operator 5
    alone), X2 from a resident O (operator 8 alone), OUT is always the fused or forward form."""
    cfg = SMALL[name]
    params = synth.make_params(cfg, random_ln=True)
    X = synth.make_x(cfg)
    from paper_2406_08756_amd import binding as B
    retain = pm.FULL_RECOMPUTE | (1 << 4) | (1 << 7) | (1 << 12)   # keep P, O and V2; drop Pd, X2
    phases = [(1 << 1) | (1 << 2), 1 << 5, 1 << 8, 0]
    layer = GpuLayer(cfg, params, workspace_bytes=B.lynx_workspace_bytes_for_schedule(cfg, retain, phases))
    layer.forward(X, retain, step=STEP)
    layer.recompute(phases[0])
    layer.recompute(phases[1])                   # attn_dropout_fwd from the resident P
    layer.recompute(phases[2])                   # bias_dropout_add from the resident O
    torch.cuda.synchronize()
    live = B.lynx_layer_live_mask(layer.handle)
    assert (live >> 5) & 1 and (live >> 8) & 1 and (live >> 4) & 1 and (live >> 7) & 1
    check_forward(cfg, layer, all_slices(cfg)[:8], layer.params)
    layer.close()


def test_masks_inside_kernels_at_the_benchmark_shape():
    """C4 in the launch configuration bench.py times: whole [T, h] tensors for the hidden
    sites, sampled (batch element, head) slices for the attention site."""
    cfg = synth.CONFIGS["C4"]
    params = synth.make_params(cfg)
    X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
    layer = GpuLayer(cfg, params)
    slices = [(0, 0), (3, 2), (7, 4), (5, 1)]
    layer.forward(X, pm.STORE_ALL, step=STEP)
    torch.cuda.synchronize()
    check_forward(cfg, layer, slices, layer.params)
    before = {"P": layer.activation_raw(4), "C": layer.activation_raw(6), "QKV": layer.activation_raw(2)}
    layer.tap_gradients(["dV2", "dX2", "dO", "dC", "dS"])
    layer.backward(dOUT)
    torch.cuda.synchronize()
    check_backward(cfg, layer, slices, before)
    layer.close()
