"""lynx_layer_create_static: the layer in the library's built-in workspace block gives the
bits of the layer in a caller-allocated workspace, on two layers in a row in the same block,
the second smaller than the first (so it runs over what the first left behind)."""
import numpy as np
import pytest
import torch

import lynx_synth as synth
from oracle import lynx_oracle as orc
from oracle import policy_model as pm
from harness import GpuLayer, rel_err
from test_gpu_parity import SMALL

pytestmark = pytest.mark.gpu


def run(cfg, params, X, dOUT, mask, static_workspace):
    layer = GpuLayer(cfg, params, static_workspace=static_workspace)
    layer.forward(X, mask, step=4)
    layer.recompute(layer.B.LYNX_SEG_ALL_MISSING)
    layer.backward(dOUT)
    torch.cuda.synchronize()
    res = (layer.out.clone(), layer.dx.clone(), {k: v.clone() for k, v in layer.grads.items()})
    layer.close()
    return res


def test_layers_in_the_built_in_workspace_match_the_allocated_one():
    for name, mask in (("tiles_bf16", pm.STORE_ALL), ("pair128_bf16", pm.FULL_RECOMPUTE)):
        cfg = SMALL[name]
        params = synth.make_params(cfg, random_ln=True)
        X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
        ref_out, ref_dx, ref_grads = run(cfg, params, X, dOUT, mask, False)
        out, dx, grads = run(cfg, params, X, dOUT, mask, True)
        assert torch.equal(out, ref_out), name
        assert torch.equal(dx, ref_dx), name
        for k, v in grads.items():
            assert torch.equal(v, ref_grads[k]), (name, k)
        # and both are the oracle's numbers
        acts, g = orc.layer_forward_backward(cfg, params, X, dOUT, step=4)
        assert rel_err(out.float().cpu().numpy().astype(np.float64), acts["OUT"]) <= 2e-2
        assert rel_err(dx.float().cpu().numpy().astype(np.float64), g["dX"]) <= 2e-2
        for k, v in grads.items():
            assert rel_err(v.float().cpu().numpy().astype(np.float64), g[k]) <= 2e-2, (name, k)


def test_built_in_workspace_limits():
    from paper_2406_08756_amd import binding as B
    with pytest.raises(B.LynxError) as e:                      # 1.8 GB at the least: beyond the block
        B.lynx_layer_create_static(synth.CONFIGS["C4"])
    assert e.value.status == B.LYNX_ERR_OOM
    first = B.lynx_layer_create_static(SMALL["tiles_bf16"])
    with pytest.raises(B.LynxError) as e:                      # one layer at a time per GPU
        B.lynx_layer_create_static(SMALL["pair128_bf16"])
    assert e.value.status == B.LYNX_ERR_STATE
    B.lynx_layer_destroy(first)
    again = B.lynx_layer_create_static(SMALL["pair128_bf16"])
    B.lynx_layer_destroy(again)
    with pytest.raises(B.LynxError) as e:                      # 122 MB at the least
        B.lynx_layer_create_static(SMALL["edge_bf16"])
    assert e.value.status == B.LYNX_ERR_OOM
