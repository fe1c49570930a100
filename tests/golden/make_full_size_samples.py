#!/usr/bin/env python3
"""Writes tests/golden/full_size_<name>.npz: sampled entries of every tensor of
the fp64 oracle's forward and backward at the full workload shapes, on the
seeded synthetic inputs.  Calls only oracle/ and the input generator; the GPU
parity tests regenerate the same inputs and compare the same entries.

Sampling is stratified so that no output tile of any kernel can be wrong
unnoticed: every 2-D tensor is cut into 128 x 128 blocks (the finest tile any
matrix-core kernel uses; 256-wide tiles, 128-wide edge strips and the two K
ranges of a cut weight gradient are unions of such blocks) and one entry at a
random position is taken from every block; the seq x seq tensors give one entry
with j <= i from every 128 x 128 block on or below the diagonal of every
(batch element, head) slice; vectors are taken whole; 1024 uniformly random
entries come on top.  Values are stored as float32 (6e-8 relative, far below
the 2e-2 bar they are compared at); `.max` is max|tensor| of the fp64 result.

usage: python tests/golden/make_full_size_samples.py C2 C3 C4 C5 C5L0 .. C5L5
  C2..C4  one layer: every activation, every gradient, every tapped gradient
  C5      the six-layer chain: OUT going up, gradients coming down
  C5L<l>  layer l of the slice on its own (layer_id = l, that layer's seeded
          parameters, the seeded X and dOUT): OUT and every gradient
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import lynx_synth as synth                    # noqa: E402
from oracle import lynx_oracle as orc         # noqa: E402

N_RANDOM = 1024
BLOCK = 128
ACTS = ("Y1", "QKV", "S", "P", "Pd", "C", "O", "X2", "Y2", "U", "G", "V2", "OUT")
TAPS = ("dV2", "dU", "dY2", "dX2", "dO", "dC", "dS", "dQKV", "dY1")
SQUARE = ("S", "P", "Pd", "dS")


def matrix_indices(rng, rows, cols):
    """One entry per BLOCK x BLOCK block (ragged last blocks included) + random ones."""
    r0 = np.arange(0, rows, BLOCK)
    c0 = np.arange(0, cols, BLOCK)
    R0, C0 = np.meshgrid(r0, c0, indexing="ij")
    R0, C0 = R0.reshape(-1), C0.reshape(-1)
    r = R0 + (rng.random(R0.size) * np.minimum(BLOCK, rows - R0)).astype(np.int64)
    c = C0 + (rng.random(C0.size) * np.minimum(BLOCK, cols - C0)).astype(np.int64)
    strat = r * cols + c
    return np.concatenate([strat, rng.integers(0, rows * cols, N_RANDOM)])


def square_indices(rng, cfg):
    """One entry with j <= i per block on or below the diagonal of every (bi, hd) slice."""
    b, a, s = cfg.micro_batch, cfg.local_heads, cfg.seq
    nb = (s + BLOCK - 1) // BLOCK
    tm, tn = np.tril_indices(nb)
    out = []
    for z in range(b * a):
        i = tm * BLOCK + (rng.random(tm.size) * np.minimum(BLOCK, s - tm * BLOCK)).astype(np.int64)
        hi = np.minimum(np.minimum(BLOCK, s - tn * BLOCK), i - tn * BLOCK + 1)  # columns allowed in the block
        j = tn * BLOCK + (rng.random(tn.size) * hi).astype(np.int64)
        out.append((z * s + i) * s + j)
    bi = rng.integers(0, b * a, N_RANDOM)
    i = rng.integers(0, s, N_RANDOM)
    j = (rng.random(N_RANDOM) * (i + 1)).astype(np.int64)
    out.append((bi * s + i) * s + j)
    return np.concatenate(out)


def record(out, rng, key, name, arr, cfg):
    if name in SQUARE:
        idx = square_indices(rng, cfg)
        scale = float(np.abs(np.tril(arr)).max())
    elif arr.ndim == 1:
        idx = np.arange(arr.size)
        scale = float(np.abs(arr).max())
    else:
        idx = matrix_indices(rng, arr.shape[0], arr.shape[1])
        scale = float(np.abs(arr).max())
    assert idx.max() < (1 << 31)
    out[key + ".idx"] = idx.astype(np.int32)
    out[key + ".val"] = arr.reshape(-1)[idx].astype(np.float32)
    out[key + ".max"] = np.float64(scale)


def one_layer(cfg, what_acts=ACTS, with_taps=True):
    params = synth.make_params(cfg)
    X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
    acts = orc.layer_forward(cfg, params, X, step=0)
    taps = {} if with_taps else None
    grads = orc.layer_backward(cfg, params, acts, dOUT, taps)
    rng = np.random.default_rng(20240608)
    out = {}
    for a in what_acts:
        record(out, rng, "act." + a, a, acts[a], cfg)
    for k, v in grads.items():
        record(out, rng, "grad." + k, k, v, cfg)
    if with_taps:
        for k in TAPS:
            record(out, rng, "tap." + k, k, taps[k], cfg)
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
        record(out, rng, "L%d.act.OUT" % l, "OUT", x, base)
    g = dout
    for l in reversed(range(L)):
        gr = orc.layer_backward(cfgs[l], params[l], acts[l], g)
        for k, v in gr.items():
            record(out, rng, "L%d.grad.%s" % (l, k), k, v, base)
        g = gr["dX"]
        acts[l] = None
    return out


if __name__ == "__main__":
    for name in sys.argv[1:]:
        if name == "C5":
            out = c5_slice()
        elif name.startswith("C5L"):
            out = one_layer(synth.CONFIGS["C5"].with_(layer_id=int(name[3:])), what_acts=("OUT",), with_taps=False)
        else:
            out = one_layer(synth.CONFIGS[name])
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "full_size_%s.npz" % name)
        np.savez_compressed(path, **out)
        print("wrote", path, len(out) // 3, "tensors", sum(v.size for k, v in out.items() if k.endswith(".idx")),
              "entries", flush=True)
