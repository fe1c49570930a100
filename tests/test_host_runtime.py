"""Host logic of the library (no GPU): the C ABI loads and exports every symbol
the header declares, and in dry-run mode its bookkeeping agrees call by call
with the reference model written from the paper's constraints (resident bytes
= sum S_i M_i, Eq. 8; dependency rule, Eq. 4; exactly-once = no-op when
resident, Eq. 3) and reports the documented errors before launching anything."""
import ctypes
import os
import re

import numpy as np
import pytest

import lynx_synth as synth
from oracle import policy_model as pm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
B = pytest.importorskip("paper_2406_08756_amd.binding")

FAKE_WS = 0x7000_0000_0000
FAKE = {n: 0x6000_0000_0000 + 4096 * i for i, n in enumerate(B.PARAM_FIELDS)}
FX, FOUT, FDOUT, FDX = 0x5000_0000_0000, 0x5100_0000_0000, 0x5200_0000_0000, 0x5300_0000_0000


def dry_layer(cfg, ws_bytes=None):
    if ws_bytes is None:
        ws_bytes = B.lynx_workspace_bytes(cfg, B.LYNX_RETAIN_STORE_ALL)
    h = B.lynx_layer_create(cfg, FAKE_WS, ws_bytes)
    B.lynx_layer_set_dry_run(h, True)
    B.lynx_layer_set_params(h, FAKE)
    return h


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "lynx.h")).read()
    declared = set(re.findall(r"\b(lynx_[a-z_]+)\s*\(", header))
    assert declared, "no declarations found"
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTED)


def test_status_strings():
    for s in range(7):
        assert B.lynx_status_string(s) not in ("", "unknown status")


def test_activation_bytes_match_model():
    for cfg in synth.CONFIGS.values():
        M = pm.activation_bytes(cfg)
        assert [B.lynx_activation_bytes(cfg, i) for i in range(14)] == M


@pytest.mark.parametrize("name", ["C1", "C4", "C4+fused"])
def test_bookkeeping_matches_model_for_many_masks(name):
    cfg = synth.CONFIGS[name.split("+")[0]]
    rng = np.random.default_rng(5)
    masks = [pm.STORE_ALL, pm.FULL_RECOMPUTE, pm.ATTENTION_ONLY, pm.ELEMENTWISE_ONLY, 0]
    masks += [int(m) for m in rng.integers(0, 1 << 14, size=40)]
    if name.endswith("+fused"):
        # attention without the seq x seq tensors wherever the mask drops S, P and Pd
        cfg = cfg.with_(flags=1)
        masks += [int(m) & ~0x38 for m in rng.integers(0, 1 << 14, size=20)]
        assert sum(pm.fused_attention(cfg, m) for m in masks) >= 20
    # explicit segments in arbitrary order can fragment the workspace beyond the
    # exact size of the canonical sequence, so this test is generous
    h = dry_layer(cfg, ws_bytes=2 * B.lynx_workspace_bytes(cfg, B.LYNX_RETAIN_STORE_ALL))
    for mask in masks:
        model = pm.LayerBookkeeping(cfg)
        model.forward(mask)
        B.lynx_layer_forward(h, FX, FOUT, mask, 0)
        assert B.lynx_layer_live_mask(h) == model.live_mask()
        assert B.lynx_layer_live_bytes(h) == model.live_bytes()
        # split the regeneration into two explicit segments, then backward
        ops = pm.missing_closure(set(model.live), model.fused)
        half = len(ops) // 2
        for seg in (ops[:half], ops[half:]):
            m = sum(1 << i for i in seg)
            model.recompute(m)
            B.lynx_recompute(h, m)
            assert B.lynx_layer_live_mask(h) == model.live_mask()
            assert B.lynx_layer_live_bytes(h) == model.live_bytes()
        B.lynx_layer_backward(h, FDOUT, FDX, FAKE)
        model.backward()
        assert B.lynx_layer_live_mask(h) == 0 and B.lynx_layer_live_bytes(h) == 0
    B.lynx_layer_destroy(h)


def test_dependency_errors_change_nothing():
    h = dry_layer(synth.CONFIGS["C1"])
    B.lynx_layer_forward(h, FX, FOUT, B.LYNX_RETAIN_FULL_RECOMPUTE, 0)
    before = B.lynx_layer_live_mask(h)
    for seg in (1 << 2, 1 << 4, (1 << 1) | (1 << 3), 1 << 9, 1 << 6):
        with pytest.raises(B.LynxError) as e:
            B.lynx_recompute(h, seg)
        assert e.value.status == B.LYNX_ERR_DEPENDENCY
        assert B.lynx_layer_live_mask(h) == before
    B.lynx_recompute(h, (1 << 1) | (1 << 2))
    B.lynx_recompute(h, 1 << 2)          # resident already: no-op
    assert B.lynx_layer_live_mask(h) == before | 0b110
    B.lynx_layer_destroy(h)


def test_state_errors():
    h = dry_layer(synth.CONFIGS["C1"])
    for call in (lambda: B.lynx_recompute(h, 2), lambda: B.lynx_layer_backward(h, FDOUT, FDX, FAKE)):
        with pytest.raises(B.LynxError) as e:
            call()
        assert e.value.status == B.LYNX_ERR_STATE
    B.lynx_layer_forward(h, FX, FOUT, 1, 0)
    with pytest.raises(B.LynxError) as e:
        B.lynx_layer_forward(h, FX, FOUT, 1, 0)
    assert e.value.status == B.LYNX_ERR_STATE
    B.lynx_layer_reset(h)
    B.lynx_layer_forward(h, FX, FOUT, 1, 0)
    B.lynx_layer_destroy(h)
    h2 = B.lynx_layer_create(synth.CONFIGS["C1"], FAKE_WS, 1 << 20)
    with pytest.raises(B.LynxError) as e:       # parameters never set
        B.lynx_layer_forward(h2, FX, FOUT, 1, 0)
    assert e.value.status == B.LYNX_ERR_STATE
    B.lynx_layer_destroy(h2)


def test_workspace_too_small_is_oom_and_harmless():
    cfg = synth.CONFIGS["C1"]
    need_full = B.lynx_workspace_bytes(cfg, B.LYNX_RETAIN_FULL_RECOMPUTE)
    need_all = B.lynx_workspace_bytes(cfg, B.LYNX_RETAIN_STORE_ALL)
    assert 0 < need_full < need_all
    # forward with store-all does not fit a workspace sized for its retained set only
    retained = sum(pm.activation_bytes(cfg)[1:13])
    h = dry_layer(cfg, ws_bytes=retained // 2)
    with pytest.raises(B.LynxError) as e:
        B.lynx_layer_forward(h, FX, FOUT, B.LYNX_RETAIN_STORE_ALL, 0)
    assert e.value.status == B.LYNX_ERR_OOM
    assert B.lynx_layer_live_mask(h) == 0 and B.lynx_layer_live_bytes(h) == 0
    B.lynx_layer_destroy(h)
    # exact size works end to end and the high-water mark equals the prediction
    for mask, need in ((B.LYNX_RETAIN_FULL_RECOMPUTE, need_full), (B.LYNX_RETAIN_STORE_ALL, need_all)):
        h = dry_layer(cfg, ws_bytes=need)
        B.lynx_layer_forward(h, FX, FOUT, mask, 0)
        B.lynx_layer_backward(h, FDOUT, FDX, FAKE)
        assert B.lynx_layer_peak_bytes(h) == need
        B.lynx_layer_destroy(h)


def test_discarding_lowers_forward_high_water_mark():
    cfg = synth.CONFIGS["C4"]
    peaks = {}
    for mask in (B.LYNX_RETAIN_STORE_ALL, B.LYNX_RETAIN_ATTENTION_ONLY, B.LYNX_RETAIN_FULL_RECOMPUTE):
        h = dry_layer(cfg)
        B.lynx_layer_forward(h, FX, FOUT, mask, 0)
        peaks[mask] = B.lynx_layer_peak_bytes(h)
        B.lynx_layer_destroy(h)
    assert peaks[B.LYNX_RETAIN_FULL_RECOMPUTE] < peaks[B.LYNX_RETAIN_ATTENTION_ONLY] < peaks[B.LYNX_RETAIN_STORE_ALL]


def test_bad_arguments():
    cfg = synth.CONFIGS["C1"]
    bad = [cfg.with_(hidden=250), cfg.with_(seq=12), cfg.with_(dropout_p=1.0), cfg.with_(tp_rank=1),
           cfg.with_(causal=0), cfg.with_(micro_batch=0), cfg.with_(hidden=16384)]
    for c in bad:
        with pytest.raises(B.LynxError) as e:
            B.lynx_layer_create(c, FAKE_WS, 1 << 20)
        assert e.value.status == B.LYNX_ERR_SHAPE
        assert B.lynx_workspace_bytes(c, 1) == 0
    with pytest.raises(B.LynxError) as e:
        B.lynx_layer_create(cfg, FAKE_WS + 8, 1 << 20)
    assert e.value.status == B.LYNX_ERR_INVALID_ARG
    h = dry_layer(cfg)
    with pytest.raises(B.LynxError) as e:
        B.lynx_layer_forward(h, FX + 4, FOUT, 1, 0)
    assert e.value.status == B.LYNX_ERR_INVALID_ARG
    with pytest.raises(B.LynxError) as e:
        B.lynx_layer_forward(h, FX, FOUT, 1 << 14, 0)
    assert e.value.status == B.LYNX_ERR_INVALID_ARG
    B.lynx_layer_destroy(h)


def test_bench_refuses_more_than_one_gpu():
    """The measurement script is for one GPU: any other count ends with a message, before
    anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""
