"""Single-layer recomputation policy (Sec. 4.2, Lynx-HEU): the brute-force
reference is pinned to hand-worked instances and to the invariants the
formulation implies; the library's exact solver (lynx_policy_solve) is then
compared with it on random small instances and checked on the 13-operator
layer.  Host only."""
import random

import pytest

from oracle import policy_bruteforce as bf


def chain(n, cost, nbytes, **kw):
    p = dict(n=n, cost=list(cost), bytes=list(nbytes),
             parents=[()] + [(i,) for i in range(1, n)], comm=set(), needed=set(range(1, n + 1)),
             ctime=[0.0] * 4, m_budget=1e18, m_static=0.0, n_layer=1, n_batch=1, last_stage=False)
    p.update(kw)
    return p


# ---- the reference against values worked out by hand ---------------------------
def test_everything_fits_means_store_all():
    val, S, phase = bf.brute_force(chain(3, (1, 2, 3), (10, 10, 10)))
    assert val == 0.0


def test_only_the_checkpoint_fits_and_nothing_overlaps():
    # budget holds OP_3 alone; no communication time: OP_1, OP_2 on the critical path: 1 + 2
    val, S, phase = bf.brute_force(chain(3, (1, 2, 3), (10, 10, 10), m_budget=10))
    assert val == 3.0 and S == [0, 0, 1] and phase == [5, 5, 0]


def test_backward_windows_hide_what_fits():
    # CTime_3 = 1.5 hides OP_1 (cost 1); OP_2 (cost 2) must come no earlier: phase 4 holds it
    p = chain(3, (1, 2, 3), (10, 10, 10), m_budget=10, ctime=[0, 0, 1.5, 2.0])
    val, S, phase = bf.brute_force(p)
    assert val == 0.0 and phase == [3, 4, 0]
    # with CTime_4 too short OP_2 stays on the critical path
    p["ctime"] = [0, 0, 1.5, 1.9]
    assert bf.brute_force(p)[0] == 2.0
    # a window cannot be used out of order: OP_2 alone fits phase 3, but OP_1 must not come
    # later than it and the two together (3) overflow the window; phase 4 (1.0) is too short
    # for OP_2, so the best is OP_1 hidden and OP_2 on the critical path
    p["ctime"] = [0, 0, 2.0, 1.0]
    val, S, phase = bf.brute_force(p)
    assert val == 2.0 and phase[0] in (3, 4) and phase[1] == 5


def test_forward_windows_cost_memory():
    # regenerating in phase 1 keeps the tensor through the forward: Eq. (cons17)
    p = chain(2, (1, 5), (10, 10), m_budget=10, ctime=[1.0, 0, 0, 0])
    assert bf.brute_force(p)[0] == 1.0          # 10 (S_2) + 10 (phase-1 copy of OP_1) > budget
    p["m_budget"] = 20
    assert bf.brute_force(p)[0] == 0.0          # now either keep OP_1 or regenerate it in phase 1
    p["last_stage"] = True
    p["m_budget"] = 10
    assert bf.brute_force(p)[0] == 1.0          # the last stage has no forward windows at all


def test_communication_operators_stay_on_the_critical_path():
    p = chain(3, (1, 2, 3), (10, 10, 10), m_budget=10, ctime=[0, 0, 10, 10], comm={2})
    val, S, phase = bf.brute_force(p)
    assert val == 2.0 and phase[1] == 5 and phase[0] in (3, 4)


def test_unneeded_operators_are_never_regenerated():
    # only OP_2 is read by backward; its input OP_1 is a stepping stone; OP_3 is the checkpoint
    p = chain(3, (1, 2, 3), (10, 10, 10), m_budget=10, needed={2})
    assert bf.brute_force(p)[0] == 3.0
    p["needed"] = {1}
    assert bf.brute_force(p)[0] == 1.0
    p["needed"] = set()
    assert bf.brute_force(p)[0] == 0.0


def test_layers_and_batches_multiply_the_resident_bytes():
    p = chain(2, (4, 1), (10, 10), m_budget=79, n_layer=2, n_batch=2)   # store-all needs 2*2*20 = 80
    assert bf.brute_force(p)[0] == 4.0
    p["m_budget"] = 80
    assert bf.brute_force(p)[0] == 0.0


def random_problem(rng, n):
    parents = [()]
    for i in range(2, n + 1):
        k = rng.choice((1, 1, 2))
        parents.append(tuple(sorted(rng.sample(range(1, i), min(k, i - 1)))))
    nbytes = [rng.choice((1, 2, 4, 8)) * 10.0 for _ in range(n)]
    p = dict(n=n, cost=[rng.choice((0.5, 1, 2, 3, 5)) for _ in range(n)], bytes=nbytes, parents=parents,
             comm=set(rng.sample(range(1, n + 1), rng.choice((0, 0, 1)))),
             needed=set(i for i in range(1, n + 1) if rng.random() < 0.7),
             ctime=[rng.choice((0, 1, 2.5, 4)) for _ in range(4)],
             m_static=rng.choice((0.0, 15.0)), n_layer=rng.choice((1, 2)), n_batch=rng.choice((1, 3)),
             last_stage=rng.random() < 0.25)
    full = p["m_static"] + p["n_layer"] * p["n_batch"] * sum(nbytes)
    least = p["m_static"] + p["n_layer"] * p["n_batch"] * nbytes[-1]
    p["m_budget"] = least + rng.random() * (full - least) * 1.1
    return p


def test_reference_is_monotone_in_budget_and_windows():
    rng = random.Random(7)
    for _ in range(25):
        p = random_problem(rng, 5)
        base = bf.brute_force(p)[0]
        q = dict(p, m_budget=p["m_budget"] * 1.5)
        assert bf.brute_force(q)[0] <= base + 1e-12
        q = dict(p, ctime=[c + 1.0 for c in p["ctime"]])
        assert bf.brute_force(q)[0] <= base + 1e-12
        q = dict(p, m_budget=1e18)
        assert bf.brute_force(q)[0] == 0.0


# ---- the library's solver against the reference ---------------------------------
B = pytest.importorskip("paper_2406_08756_amd.binding")
needs_solver = pytest.mark.skipif(not hasattr(B, "lynx_policy_solve"), reason="library without the policy solver")


def solve(p):
    return B.lynx_policy_solve(p)


@needs_solver
def test_solver_matches_reference_on_random_instances():
    rng = random.Random(11)
    for trial in range(120):
        p = random_problem(rng, rng.choice((3, 4, 5, 6)))
        ref = bf.brute_force(p)
        got = solve(p)
        assert got is not None and ref is not None, trial
        S = [(got["retain_mask"] >> (i + 1)) & 1 for i in range(p["n"])]
        phase = [0] * p["n"]
        for t in range(1, 6):
            for i in range(p["n"]):
                if (got["phase_mask"][t - 1] >> (i + 1)) & 1:
                    assert phase[i] == 0
                    phase[i] = t
        assert bf.feasible(p, S, phase), (trial, p, got)
        assert abs(bf.objective(p, S, phase) - got["critical_cost"]) < 1e-9
        assert abs(got["critical_cost"] - ref[0]) < 1e-9, (trial, p, got, ref)
        assert abs(got["peak_bytes"] - bf.peak_bytes(p, S, phase)) < 1e-6


@needs_solver
def test_solver_reports_infeasible():
    p = chain(3, (1, 2, 3), (10, 10, 10), m_budget=5)       # not even the checkpoint fits
    assert bf.brute_force(p) is None
    assert solve(p) is None


@needs_solver
def test_solver_on_the_gpt_layer():
    import lynx_synth as synth
    from oracle import policy_model as pm
    cfg = synth.CONFIGS["C4"]
    cost = [0.0] + [0.076, 0.37, 0.087, 0.098, 0.0, 0.084, 0.135, 0.09, 0.073, 0.417, 0.032, 0.38, 0.085]
    p = B.lynx_policy_layer_problem(cfg, cost[1:], ctime=[0.27] * 4, m_budget=1e18, m_static=0.0,
                                    n_layer=1, n_batch=1, last_stage=False)
    # the library's own dependency table and sizes are the bookkeeping model's
    assert [tuple(sorted(q)) for q in p["parents"]] == [tuple(sorted(j for j in pm.PARENTS[i] if j > 0))
                                                        for i in range(1, 14)]
    assert p["needed"] == set(i for i in pm.BACKWARD_NEEDS if i > 0)
    M = pm.activation_bytes(cfg)
    assert p["bytes"] == [float(M[i]) for i in range(1, 14)]
    got = solve(p)
    assert got["critical_cost"] == 0.0 and got["retain_mask"] & 1
    # the caller's checkpoint alone: everything backward reads must come back somewhere
    least = float(M[13])
    p["m_budget"] = least
    p["ctime"] = [0.0] * 4
    got = solve(p)
    assert got["retain_mask"] == pm.FULL_RECOMPUTE
    closure = pm.missing_closure({0, 13})
    assert got["phase_mask"][4] == sum(1 << i for i in closure)
    assert abs(got["critical_cost"] - sum(cost[i] for i in closure)) < 1e-12
    # the backward windows take over what they can hold, in dependency order
    p["ctime"] = [0.0, 0.0, 0.5, 0.5]
    mid = solve(p)
    assert 0.0 < mid["critical_cost"] < got["critical_cost"]
    # a budget in between keeps the expensive operators' outputs first
    p["m_budget"] = least + sum(p["bytes"]) * 0.5
    half = solve(p)
    assert half["critical_cost"] <= mid["critical_cost"]
    assert half["peak_bytes"] <= p["m_budget"]
