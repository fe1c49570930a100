"""GPU parity: the HIP path, driven through the C ABI, against the fp64 oracle
on the same seeded inputs.  Masks must match bit for bit; float tensors must
satisfy max|gpu - ref| / max|ref| <= 1e-4 (fp32 storage) or 2e-2 (bf16
storage) per tensor; regenerated activations must equal the forward's bits."""
import numpy as np
import pytest
import torch

import lynx_synth as synth
from oracle import lynx_oracle as orc
from oracle import policy_model as pm
from harness import ACT_NAMES, GpuLayer, rel_err

pytestmark = pytest.mark.gpu

TOL = {synth.F32: 1e-4, synth.BF16: 2e-2}

SMALL = {
    # ragged: no dimension is a multiple of a 64/128 tile
    "ragged_f32": synth.LayerConfig(synth.F32, 72, 3, 24, 136, 40, 3, tp_size=2, tp_rank=1,
                                    dropout_p=0.2, seed=11, layer_id=5),
    "ragged_bf16": synth.LayerConfig(synth.BF16, 264, 3, 40, 328, 136, 2, tp_size=4, tp_rank=2,
                                     dropout_p=0.1, seed=3, layer_id=1),
    # several tiles of every kernel, tile-aligned
    "tiles_bf16": synth.LayerConfig(synth.BF16, 512, 4, 128, 1024, 384, 2, tp_size=2, tp_rank=0,
                                    dropout_p=0.1, seed=0, layer_id=2),
    # multiples of 128 but not of 256: the smaller matrix-core tiles
    "tiles128_bf16": synth.LayerConfig(synth.BF16, 640, 3, 128, 1152, 128, 3, tp_size=2, tp_rank=1,
                                       dropout_p=0.1, seed=4, layer_id=7),
    # sequence of two 256-tiles: the large score tiles and multi-slab causal contractions
    "tiles256_bf16": synth.LayerConfig(synth.BF16, 256, 2, 128, 256, 512, 1, tp_size=1,
                                       dropout_p=0.1, seed=6, layer_id=3),
    # the longest rows the softmax kernels take in registers at half their limit, 32 row
    # blocks in the contraction-restricted attention products
    "long_seq_bf16": synth.LayerConfig(synth.BF16, 256, 1, 128, 256, 4096, 1, tp_size=1,
                                       dropout_p=0.1, seed=8, layer_id=4),
    # the widest rows the LayerNorm kernels accept (four vectors per thread), K = 8192 GEMMs
    "wide_bf16": synth.LayerConfig(synth.BF16, 8192, 1, 128, 128, 128, 1, tp_size=1,
                                   dropout_p=0.1, seed=12, layer_id=6),
    # many tokens, widths of 256 + 128: a column range of large tiles plus an edge strip of
    # narrow ones in one launch, with and without a fused epilogue
    "edge_bf16": synth.LayerConfig(synth.BF16, 384, 1, 128, 384, 128, 128, tp_size=1,
                                   dropout_p=0.1, seed=5, layer_id=9),
    # FFN width of 256 + 128 with whole 256-row token tiles: the paired backward launch with
    # 128-wide input-gradient tiles and the GeLU backward in their epilogue
    "pair128_bf16": synth.LayerConfig(synth.BF16, 256, 2, 128, 384, 256, 2, tp_size=1,
                                      dropout_p=0.1, seed=13, layer_id=8),
    # thousands of rows wider than 4096: the streaming LayerNorm forward (ragged last vector
    # group per thread); everything else tiny
    "ln_stream_bf16": synth.LayerConfig(synth.BF16, 4104, 1, 8, 8, 128, 32, tp_size=1,
                                        dropout_p=0.1, seed=14, layer_id=10),
    "C1": synth.CONFIGS["C1"],
    "nodrop_bf16": synth.LayerConfig(synth.BF16, 256, 2, 64, 512, 128, 1, dropout_p=0.0),
    "minimal_f32": synth.LayerConfig(synth.F32, 8, 1, 8, 8, 8, 1, dropout_p=0.5, seed=9),
}


def compare_forward(layer, acts, tol, names=None):
    worst = {}
    for i, name in enumerate(ACT_NAMES):
        if i == 0 or (names and name not in names):
            continue
        got = layer.activation(i)
        if got is None:
            continue
        ref = acts[name]
        if i in (3, 4, 5):
            got, ref = np.tril(got), np.tril(ref)
        worst[name] = rel_err(got, ref)
        assert worst[name] <= tol, (name, worst[name])
    return worst


@pytest.mark.parametrize("name", list(SMALL))
def test_dropout_masks_bit_exact(name):
    from paper_2406_08756_amd import binding as B
    cfg = SMALL[name]
    step = 3
    T, h, b, a, s = cfg.tokens, cfg.hidden, cfg.micro_batch, cfg.local_heads, cfg.seq
    for site in (1, 2):
        out = torch.zeros(T * h, dtype=torch.uint8, device="cuda")
        B.lynx_dropout_mask(cfg, step, site, out)
        ref = orc.hidden_mask(cfg, step, site).astype(np.uint8).reshape(-1)
        assert np.array_equal(out.cpu().numpy(), ref)
    out = torch.zeros(b * a * s * s, dtype=torch.uint8, device="cuda")
    B.lynx_dropout_mask(cfg, step, 0, out)
    got = out.cpu().numpy().reshape(b, a, s, s)
    for bi in range(b):
        for hd in range(a):
            assert np.array_equal(got[bi, hd], orc.attention_mask_slice(cfg, step, bi, hd).astype(np.uint8))


@pytest.mark.parametrize("name", list(SMALL))
def test_store_all_forward_and_backward_match_oracle(name):
    cfg = SMALL[name]
    tol = TOL[cfg.dtype]
    params = synth.make_params(cfg, random_ln=True)
    X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
    acts, grads = orc.layer_forward_backward(cfg, params, X, dOUT, step=1)
    layer = GpuLayer(cfg, params)
    layer.forward(X, pm.STORE_ALL, step=1)
    torch.cuda.synchronize()
    compare_forward(layer, acts, tol)
    for act, (mu_ref, r_ref) in ((1, (acts["mu1"], acts["rstd1"])), (9, (acts["mu2"], acts["rstd2"]))):
        mu, r = layer.stats(act)
        assert np.abs(mu - mu_ref).max() <= tol * max(1.0, np.abs(mu_ref).max())
        assert rel_err(r, r_ref) <= tol
    # the dropped entries are exactly the oracle's
    k1 = (layer.activation(8) - X) != 0
    assert not (k1 & ~acts["keep1"]).any()
    layer.backward(dOUT)
    got = layer.results()
    for k, ref in grads.items():
        assert rel_err(got[k], ref) <= tol, (k, rel_err(got[k], ref))
    layer.close()


@pytest.mark.parametrize("name", ["C1", "ragged_bf16", "tiles_bf16", "tiles128_bf16", "tiles256_bf16", "long_seq_bf16",
                                  "wide_bf16", "edge_bf16", "pair128_bf16", "ln_stream_bf16",
                                  "tiles_bf16+fused", "tiles128_bf16+fused", "tiles256_bf16+fused",
                                  "long_seq_bf16+fused", "edge_bf16+fused", "pair128_bf16+fused"])
def test_recompute_is_bit_identical_and_policy_does_not_change_results(name):
    """'+fused': the same layer with LYNX_FLAG_FUSED_ATTENTION: the store-all reference runs the
    unfused kernels (it keeps S, P, Pd), every mask that drops the three runs the kernels that
    never store them, and all results must still be the same bits."""
    cfg = SMALL[name.split("+")[0]]
    if name.endswith("+fused"):
        cfg = cfg.with_(flags=1)
    params = synth.make_params(cfg, random_ln=True)
    X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
    from paper_2406_08756_amd import binding as B
    rng = np.random.default_rng(17)
    masks = [pm.FULL_RECOMPUTE, pm.ATTENTION_ONLY, pm.ELEMENTWISE_ONLY, 1]
    masks += [int(m) | 1 for m in rng.integers(0, 1 << 14, size=12)]
    if cfg.flags & 1:
        masks += [int(m) & ~0x38 | 1 for m in rng.integers(0, 1 << 14, size=6)]   # more masks that run fused
        assert sum(pm.fused_attention(cfg, m) for m in masks) >= 8
    # every run starts from an empty workspace, so the exact size per mask applies to each
    layer = GpuLayer(cfg, params, workspace_bytes=max(B.lynx_workspace_bytes(cfg, m) for m in [pm.STORE_ALL] + masks))

    def lower(i, t):
        if i in (3, 4, 5):
            s = cfg.seq
            return torch.tril(t.view(-1, s, s)).reshape(-1)
        return t

    layer.forward(X, pm.STORE_ALL, step=2)
    torch.cuda.synchronize()
    ref_acts = {i: lower(i, layer.activation_raw(i)) for i in range(1, 14)}
    ref_stats = {i: layer.stats(i) for i in (1, 9)}
    layer.backward(dOUT)
    torch.cuda.synchronize()
    ref_out = layer.out.clone()
    ref_dx = layer.dx.clone()
    ref_grads = {k: v.clone() for k, v in layer.grads.items()}

    for n, mask in enumerate(masks):
        layer.out.zero_(); layer.dx.zero_()
        for v in layer.grads.values():
            v.zero_()
        layer.forward(X, mask, step=2)
        torch.cuda.synchronize()
        assert torch.equal(layer.out, ref_out), hex(mask)
        if n % 2 == 0:
            # explicit regeneration: every activation backward reads is back, bit for bit
            layer.recompute(B.LYNX_SEG_ALL_MISSING)
            torch.cuda.synchronize()
            live = B.lynx_layer_live_mask(layer.handle)
            fused = pm.fused_attention(cfg, mask)
            if fused:
                assert not live & 0x38, hex(mask)     # S, P, Pd never exist under such a policy
            for i in pm.backward_needs(fused):
                assert (live >> i) & 1
                if i == 0:
                    continue
                assert torch.equal(lower(i, layer.activation_raw(i)), ref_acts[i]), (hex(mask), i)
            for i in (1, 9):
                mu, r = layer.stats(i)
                assert np.array_equal(mu, ref_stats[i][0]) and np.array_equal(r, ref_stats[i][1])
        layer.backward(dOUT)
        torch.cuda.synchronize()
        assert torch.equal(layer.dx, ref_dx), hex(mask)
        for k, v in layer.grads.items():
            assert torch.equal(v, ref_grads[k]), (hex(mask), k)
    layer.close()


def test_explicit_segments_in_phases_then_backward():
    """Regeneration split over several calls (the paper's phases 1-4) followed
    by backward's on-demand remainder gives the same bits as one shot."""
    cfg = SMALL["tiles_bf16"]
    params = synth.make_params(cfg, random_ln=True)
    X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
    from paper_2406_08756_amd import binding as B
    phases = [(1 << 1) | (1 << 2), (1 << 3) | (1 << 4), 1 << 5, (1 << 6) | (1 << 7) | (1 << 8)]
    need = max(B.lynx_workspace_bytes(cfg, pm.STORE_ALL),
               B.lynx_workspace_bytes_for_schedule(cfg, pm.FULL_RECOMPUTE, phases))
    layer = GpuLayer(cfg, params, workspace_bytes=need)
    layer.forward(X, pm.STORE_ALL)
    layer.backward(dOUT)
    torch.cuda.synchronize()
    ref_dx = layer.dx.clone()
    ref_grads = {k: v.clone() for k, v in layer.grads.items()}
    layer.forward(X, pm.FULL_RECOMPUTE)
    with pytest.raises(B.LynxError) as e:
        layer.recompute(1 << 6)
    assert e.value.status == B.LYNX_ERR_DEPENDENCY
    layer.recompute(phases[0])                      # "phase 1"
    layer.recompute(phases[1])                      # "phase 2": P alone, S dropped again
    assert not (B.lynx_layer_live_mask(layer.handle) >> 3) & 1
    layer.recompute(phases[2])                      # "phase 3": Pd from the resident P
    layer.recompute(phases[3])                      # "phase 4"
    assert B.lynx_layer_peak_bytes(layer.handle) <= need
    layer.backward(dOUT)                            # phase 5: the rest on demand
    torch.cuda.synchronize()
    assert torch.equal(layer.dx, ref_dx)
    for k, v in layer.grads.items():
        assert torch.equal(v, ref_grads[k]), k
    layer.close()


def test_solved_policies_run_through_the_layer():
    """Policies from lynx_policy_solve (Sec. 4.2): the retain mask drives the forward,
    phase masks 1-4 are handed to lynx_recompute in order, phase 5 is left to backward;
    every segment's inputs are there when it runs, the resident bytes after forward are
    sum_i S_i M_i, and the gradients are the store-all bits."""
    cfg = SMALL["tiles_bf16"]
    params = synth.make_params(cfg, random_ln=True)
    X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
    from paper_2406_08756_amd import binding as B
    M = pm.activation_bytes(cfg)
    cost = [1.0, 6.0, 1.5, 1.2, 0.0, 1.5, 2.0, 1.0, 1.0, 8.0, 0.5, 8.0, 1.0]
    policies = []
    for frac, ctime in [(0.0, [0, 0, 0, 0]), (0.0, [0, 0, 4.0, 9.0]), (0.3, [2.0, 2.0, 3.0, 3.0]),
                        (0.6, [0, 0, 2.0, 2.0]), (0.15, [8.0, 0, 0, 8.0]), (0.5, [3.0, 3.0, 0, 0]),
                        (1.0, [0, 0, 0, 0])]:
        budget = M[13] + frac * sum(M[1:13])
        prob = B.lynx_policy_layer_problem(cfg, cost, ctime=ctime, m_budget=budget + 1.0)
        pol = B.lynx_policy_solve(prob)
        assert pol is not None
        policies.append(pol)
    # the workspace each schedule needs, exactly (Eq. cons15-17 count the same things)
    need = [B.lynx_workspace_bytes_for_schedule(cfg, q["retain_mask"], q["phase_mask"][:4]) for q in policies]
    assert all(n > 0 for n in need)
    layer = GpuLayer(cfg, params, workspace_bytes=max(need + [B.lynx_workspace_bytes(cfg, pm.STORE_ALL)]))
    layer.forward(X, pm.STORE_ALL)
    layer.backward(dOUT)
    torch.cuda.synchronize()
    ref_dx = layer.dx.clone()
    ref_grads = {k: v.clone() for k, v in layer.grads.items()}
    seen = set()
    for pol in policies:
        seen.add((pol["retain_mask"], tuple(pol["phase_mask"])))
        layer.dx.zero_()
        for v in layer.grads.values():
            v.zero_()
        layer.forward(X, pol["retain_mask"])
        kept = sum(M[i] for i in range(1, 13) if (pol["retain_mask"] >> i) & 1)
        assert B.lynx_layer_live_bytes(layer.handle) == kept
        for t in range(4):
            if pol["phase_mask"][t]:
                layer.recompute(pol["phase_mask"][t])
        layer.backward(dOUT)
        torch.cuda.synchronize()
        assert torch.equal(layer.dx, ref_dx), pol
        for k, v in layer.grads.items():
            assert torch.equal(v, ref_grads[k]), (pol, k)
    assert len(seen) >= 4   # the instances really exercise different schedules
    layer.close()


def test_zero_output_projections_make_layer_identity_on_gpu():
    cfg = SMALL["tiles_bf16"]
    params = synth.make_params(cfg)
    for k in ("wo", "bo", "w2", "b2"):
        params[k] = np.zeros_like(params[k])
    X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
    layer = GpuLayer(cfg, params)
    layer.forward(X, pm.FULL_RECOMPUTE)
    layer.backward(dOUT)
    got = layer.results()
    assert np.array_equal(layer.out.float().cpu().numpy(), X)
    assert np.array_equal(got["dX"], dOUT.astype(np.float64))
    layer.close()


@pytest.mark.parametrize("name", ["tiles_bf16", "C4"])
def test_regeneration_on_a_side_stream_under_the_comm_standin_keeps_the_bits(name):
    """The paper's mechanism at one-GPU fidelity (Sec. 4, phases 1-4; Eq. cons13): the
    regeneration segments run on a side stream while a stand-in for the tensor-parallel
    all-reduce (a bounded-width copy) occupies the main stream; backward then waits for the
    side stream.  Nothing about the results may change: same activations, same gradients
    as the single-stream run."""
    from paper_2406_08756_amd import binding as B
    cfg = SMALL[name] if name in SMALL else synth.CONFIGS[name]
    params = synth.make_params(cfg, random_ln=True)
    X, dOUT = synth.make_x(cfg), synth.make_dout(cfg)
    phases = [(1 << 1) | (1 << 2) | (1 << 3) | (1 << 4) | (1 << 5), (1 << 6) | (1 << 7) | (1 << 8), 1 << 9,
              (1 << 10) | (1 << 11)]
    need = max(B.lynx_workspace_bytes(cfg, pm.FULL_RECOMPUTE),
               B.lynx_workspace_bytes_for_schedule(cfg, pm.FULL_RECOMPUTE, phases))
    layer = GpuLayer(cfg, params, workspace_bytes=need)
    main = torch.cuda.current_stream()
    layer.forward(X, pm.FULL_RECOMPUTE, step=7)
    layer.backward(dOUT)
    torch.cuda.synchronize()
    ref_dx = layer.dx.clone()
    ref_grads = {k: v.clone() for k, v in layer.grads.items()}

    side = torch.cuda.Stream()                      # default priority
    src = torch.randn(cfg.tokens, cfg.hidden, device="cuda").to(layer.tdtype)
    dst = torch.empty_like(src)
    for rep in range(3):
        layer.dx.zero_()
        for v in layer.grads.values():
            v.zero_()
        B.lynx_layer_forward(layer.handle, layer.x, layer.out, pm.FULL_RECOMPUTE, 7, main)
        fork = torch.cuda.Event()
        fork.record(main)
        side.wait_event(fork)
        for seg in phases:
            # one stand-in per communication window on the main stream, its segment beside it
            B.lynx_comm_standin(dst, src, src.numel() * src.element_size(), 32, main)
            B.lynx_recompute(layer.handle, seg, side)
        join = torch.cuda.Event()
        join.record(side)
        main.wait_event(join)
        B.lynx_layer_backward(layer.handle, layer.dout, layer.dx, layer.grads, main)
        torch.cuda.synchronize()
        assert torch.equal(dst, src)
        assert torch.equal(layer.dx, ref_dx), rep
        for k, v in layer.grads.items():
            assert torch.equal(v, ref_grads[k]), (rep, k)
    layer.close()


def test_two_handles_from_two_host_threads_are_independent():
    """Distinct handles share nothing: two layers of different shapes, each driven by its own
    host thread on its own stream (forward under full recomputation, regeneration, backward,
    several times over), end with the bits of the same calls made one after the other."""
    import threading
    from paper_2406_08756_amd import binding as B
    names = ["tiles_bf16", "edge_bf16"]
    layers, refs = [], []
    for name in names:
        cfg = SMALL[name]
        layer = GpuLayer(cfg, synth.make_params(cfg, random_ln=True))
        layer.forward(synth.make_x(cfg), pm.FULL_RECOMPUTE, step=3)
        layer.backward(synth.make_dout(cfg))
        torch.cuda.synchronize()
        refs.append((layer.out.clone(), layer.dx.clone(), {k: v.clone() for k, v in layer.grads.items()}))
        layers.append(layer)
    errors = []

    def drive(layer, ref):
        try:
            st = torch.cuda.Stream()
            st.wait_stream(torch.cuda.default_stream())
            for rep in range(4):
                B.lynx_layer_forward(layer.handle, layer.x, layer.out, pm.FULL_RECOMPUTE, 3, st)
                B.lynx_recompute(layer.handle, B.LYNX_SEG_ALL_MISSING, st)
                B.lynx_layer_backward(layer.handle, layer.dout, layer.dx, layer.grads, st)
                st.synchronize()
                if not (torch.equal(layer.out, ref[0]) and torch.equal(layer.dx, ref[1])
                        and all(torch.equal(v, ref[2][k]) for k, v in layer.grads.items())):
                    errors.append(rep)
        except Exception as exc:   # surfaced by the assert below
            errors.append(repr(exc))

    threads = [threading.Thread(target=drive, args=(l, r)) for l, r in zip(layers, refs)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    for layer in layers:
        layer.close()
    assert errors == []


def test_comm_standin_copies_and_checks_arguments():
    from paper_2406_08756_amd import binding as B
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    B.lynx_comm_standin(dst, src, src.numel() * 4, 7)          # 7 workgroups, ragged share per workgroup
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    dst.zero_()
    B.lynx_comm_standin(dst, src, 48, 1)                       # three vectors
    torch.cuda.synchronize()
    assert torch.equal(dst[:12], src[:12]) and int(dst[12:].abs().sum()) == 0
    for bad in [dict(nbytes=40, workgroups=1), dict(nbytes=64, workgroups=0), dict(nbytes=64, workgroups=5000)]:
        with pytest.raises(B.LynxError) as e:
            B.lynx_comm_standin(dst, src, bad["nbytes"], bad["workgroups"])
        assert e.value.status == B.LYNX_ERR_INVALID_ARG
    with pytest.raises(B.LynxError):
        B.lynx_comm_standin(dst.data_ptr() + 4, src, 64, 1)    # misaligned
