"""GPU parity at the full workload shapes (C2..C5), in the launch configuration
bench.py times: sampled entries of every tensor against values the fp64 oracle
computed on the same seeded inputs (tests/golden/full_size_*.npz, written by
tests/golden/make_full_size_samples.py, which calls only the oracle).  Bound for
one layer: |gpu - ref| <= 2e-2 * max|ref| per tensor (bf16 storage).  Also:
results are bit-identical across retain policies at full size.

In the six-layer slice every layer boundary tensor (OUT going up, dX coming
down) is stored in bf16, so the independent rounding errors of successive
layers add in quadrature: a gradient that has come down through k layer
backward passes is held to 2e-2 * sqrt(k), the per-layer bar for k = 1.  The
forward outputs OUT are held to the plain 2e-2 at every depth."""
import os

import numpy as np
import pytest
import torch

import lynx_synth as synth
from oracle import policy_model as pm
from harness import ACT_NAMES, GpuLayer

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
TOL = 2e-2
POLICY = {"C2": pm.FULL_RECOMPUTE, "C3": pm.ELEMENTWISE_ONLY, "C4": pm.FULL_RECOMPUTE}


def load(name):
    path = os.path.join(GOLDEN, "full_size_%s.npz" % name)
    if not os.path.exists(path):
        pytest.skip("golden samples for %s not generated" % name)
    return np.load(path)


def check(gold, key, flat_gpu, tol=TOL):
    idx = torch.from_numpy(gold[key + ".idx"]).cuda()
    got = flat_gpu.reshape(-1)[idx].float().cpu().numpy().astype(np.float64)
    err = np.abs(got - gold[key + ".val"]).max() / max(float(gold[key + ".max"]), 1e-30)
    assert err <= tol, (key, err, tol)
    return err


@pytest.mark.parametrize("name", ["C4", "C3", "C2"])
def test_single_layer_full_size(name):
    gold = load(name)
    cfg = synth.CONFIGS[name]
    params = synth.make_params(cfg)
    X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
    from paper_2406_08756_amd import binding as B
    policies = [POLICY[name]] if name != "C2" else [pm.ATTENTION_ONLY, pm.FULL_RECOMPUTE]
    # the workspace size is exact per policy (buffers are placed differently under each)
    need = max(B.lynx_workspace_bytes(cfg, m) for m in [pm.STORE_ALL] + policies)
    layer = GpuLayer(cfg, params, workspace_bytes=need)
    # every activation, from a store-all forward
    layer.forward(X, pm.STORE_ALL)
    torch.cuda.synchronize()
    for i in range(1, 14):
        raw = layer.activation_raw(i)
        check(gold, "act." + ACT_NAMES[i], raw)
        del raw
    layer.backward(dOUT)
    torch.cuda.synchronize()
    ref_dx = layer.dx.clone()
    ref_grads = {k: v.clone() for k, v in layer.grads.items()}
    check(gold, "grad.dX", layer.dx)
    for k, v in layer.grads.items():
        check(gold, "grad." + k, v)
    # the timed configuration: policy forward, regeneration, backward -- same bits
    for mask in policies:
        layer.dx.zero_()
        for v in layer.grads.values():
            v.zero_()
        layer.forward(layer.x, mask)
        layer.recompute(B.LYNX_SEG_ALL_MISSING)
        layer.backward(layer.dout)
        torch.cuda.synchronize()
        assert torch.equal(layer.dx, ref_dx), hex(mask)
        for k, v in layer.grads.items():
            assert torch.equal(v, ref_grads[k]), (hex(mask), k)
    layer.close()


def test_six_layer_slice_full_size():
    gold = load("C5")
    base = synth.CONFIGS["C5"]
    L = synth.C5_LAYERS
    masks = synth.c5_retain_masks()
    layers = []
    for l in range(L):
        cfg = base.with_(layer_id=l)
        layers.append(GpuLayer(cfg, synth.make_params(cfg), retain_mask_for_size=masks[l]))
    x = synth.make_x(base)
    for l in range(L):
        layers[l].forward(x if l == 0 else layers[l - 1].out, masks[l])
    torch.cuda.synchronize()
    for l in range(L):
        check(gold, "L%d.act.OUT" % l, layers[l].out)
    g = synth.make_dout(base)
    for l in reversed(range(L)):
        layers[l].backward(g if l == L - 1 else layers[l + 1].dx)
    torch.cuda.synchronize()
    for l in range(L):
        tol = TOL * np.sqrt(L - l)  # backward passes between the injected dOUT and this layer's gradients
        check(gold, "L%d.grad.dX" % l, layers[l].dx, tol)
        for k, v in layers[l].grads.items():
            check(gold, "L%d.grad.%s" % (l, k), v, tol)
    for lay in layers:
        lay.close()
