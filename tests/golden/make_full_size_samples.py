#!/usr/bin/env python3
"""Writes tests/golden/full_size_<cfg>.npz: sampled entries of every tensor of
the fp64 oracle's forward and backward at the full workload shapes (C2..C5),
on the seeded synthetic inputs.  Calls only oracle/ and the input generator;
the GPU parity test regenerates the same inputs and compares the same entries.

usage: python tests/golden/make_full_size_samples.py C2 C3 C4 C5
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import lynx_synth as synth                    # noqa: E402
from oracle import lynx_oracle as orc         # noqa: E402

N_SAMPLES = 1024
ACTS = ("Y1", "QKV", "S", "P", "Pd", "C", "O", "X2", "Y2", "U", "G", "V2", "OUT")


def sample_indices(rng, name, arr, cfg):
    """Flat indices into arr; for the seq x seq tensors only entries with j <= i."""
    if name in ("S", "P", "Pd"):
        b, a, s = cfg.micro_batch, cfg.local_heads, cfg.seq
        bi = rng.integers(0, b, N_SAMPLES)
        hd = rng.integers(0, a, N_SAMPLES)
        i = rng.integers(0, s, N_SAMPLES)
        j = (rng.random(N_SAMPLES) * (i + 1)).astype(np.int64)
        return ((bi * a + hd) * s + i) * s + j
    return rng.integers(0, arr.size, N_SAMPLES)


def record(out, rng, prefix, name, arr, cfg):
    idx = sample_indices(rng, name, arr, cfg)
    ref = arr
    if name in ("S", "P", "Pd"):
        scale = float(np.abs(np.tril(arr)).max())
    else:
        scale = float(np.abs(arr).max())
    out[prefix + name + ".idx"] = idx.astype(np.int64)
    out[prefix + name + ".val"] = ref.reshape(-1)[idx].astype(np.float64)
    out[prefix + name + ".max"] = np.float64(scale)


def one_layer(name):
    cfg = synth.CONFIGS[name]
    params = synth.make_params(cfg)
    X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
    acts, grads = orc.layer_forward_backward(cfg, params, X, dOUT, step=0)
    rng = np.random.default_rng(20240608)
    out = {}
    for a in ACTS:
        record(out, rng, "act.", a, acts[a], cfg)
    for k, v in grads.items():
        record(out, rng, "grad.", k, v, cfg)
    return out


def c5_slice():
    base = synth.CONFIGS["C5"]
    L = synth.C5_LAYERS
    cfgs = [base.with_(layer_id=l) for l in range(L)]
    params = [synth.make_params(c) for c in cfgs]
    x = synth.make_x(base).astype(np.float64)
    dout = synth.make_dout(base).astype(np.float64)
    rng = np.random.default_rng(20240608)
    out = {}
    acts = []
    for l in range(L):
        a = orc.layer_forward(cfgs[l], params[l], x, step=0)
        acts.append(a)
        x = a["OUT"]
        record(out, rng, "L%d.act." % l, "OUT", x, base)
    g = dout
    for l in reversed(range(L)):
        gr = orc.layer_backward(cfgs[l], params[l], acts[l], g)
        for k, v in gr.items():
            record(out, rng, "L%d.grad." % l, k, v, base)
        g = gr["dX"]
        acts[l] = None
    return out


if __name__ == "__main__":
    for name in sys.argv[1:]:
        out = c5_slice() if name == "C5" else one_layer(name)
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "full_size_%s.npz" % name)
        np.savez_compressed(path, **out)
        print("wrote", path, len(out) // 3, "tensors", flush=True)
