"""Recomputation-aware model partitioning (Sec. 5): the greedy search written
out in oracle/policy_bruteforce.py is pinned to hand-worked instances (one of
them has the shape of the section's two-stage, four-layer illustration) and to
the bounds the method implies; the library's lynx_partition_solve is then
compared with it on random instances.  Host only."""
import random

import pytest

from oracle import policy_bruteforce as bf
from test_policy_solver import chain, random_problem


# ---- the reference against values worked out by hand -----------------------------
def two_op_layer():
    # OP_1 costs 4 to regenerate, OP_2 is the layer output (always resident); 10 bytes each
    return chain(2, (4, 1), (10, 10))


def test_enough_memory_keeps_equal_shares():
    # stage 0 holds 2 micro-batches of 2 layers of 20 bytes = 80: store-all fits both stages,
    # both take 2 * (1 + 2) = 6, nothing to move
    layers, times = bf.greedy_partition(two_op_layer(), 4, 2, 1.0, 2.0, 0.0, 80.0)
    assert layers == [2, 2] and times == [6.0, 6.0]


def test_memory_bound_first_stage_gives_a_layer_away():
    # budget 60: stage 0 with two layers (2 in flight) cannot keep OP_1 (80 > 60), so it
    # regenerates it on the critical path: 2 * (3 + 4) = 14; stage 1 (1 in flight): 40, time 6.
    # One layer moved: stage 0 = 1 layer, 40 bytes, store-all, time 3; stage 1 = 3 layers,
    # 60 bytes, store-all, time 9.  9 < 14: adopted.  Moving it back gives 14 again: stop.
    layers, times = bf.greedy_partition(two_op_layer(), 4, 2, 1.0, 2.0, 0.0, 60.0)
    assert layers == [1, 3] and times == [3.0, 9.0]
    assert bf.best_partition_exhaustive(two_op_layer(), 4, 2, 1.0, 2.0, 0.0, 60.0) == (9.0, [1, 3])


def test_remainder_goes_to_the_first_stages_and_static_memory_counts():
    # 5 layers over 2 stages start as [3, 2]; with ample memory stage 0 is slowest (9 vs 6),
    # the move gives [2, 3] whose slowest stage is 9 again: not shorter, so [3, 2] stays
    layers, times = bf.greedy_partition(two_op_layer(), 5, 2, 1.0, 2.0, 0.0, 1e9)
    assert layers == [3, 2] and times == [9.0, 6.0]
    # static bytes per layer eat the budget: 3 layers * (25 + 2 * 20) = 195 > 190 forces
    # regeneration on stage 0 (3 * 7 = 21), so a layer moves: [2, 3], stage 1 3 * (25 + 20) = 135
    layers, times = bf.greedy_partition(two_op_layer(), 5, 2, 1.0, 2.0, 25.0, 190.0)
    assert layers == [2, 3] and times == [6.0, 9.0]


def test_invalid_initial_scheme_is_reported():
    # not even the layer outputs fit: 2 layers * 2 in flight * 10 = 40 > 30
    assert bf.greedy_partition(two_op_layer(), 4, 2, 1.0, 2.0, 0.0, 30.0) is None


def random_partition_case(rng):
    p = random_problem(rng, rng.choice((3, 4)))
    n_stages = rng.choice((2, 3, 4))
    n_total = rng.randint(n_stages, n_stages + 6)
    static = rng.choice((0.0, 20.0))
    per_layer = sum(p["bytes"])
    # between "only outputs fit at the fullest stage" and "everything fits everywhere"
    share = -(-n_total // n_stages)
    least = share * (static + n_stages * p["bytes"][-1])
    full = share * (static + n_stages * per_layer)
    budget = least + rng.random() * (full - least) * 1.2
    return p, n_total, n_stages, rng.choice((0.5, 1.0, 2.0)), rng.choice((1.0, 3.0)), static, budget


def test_greedy_is_bounded_by_equal_shares_and_by_the_best_composition():
    rng = random.Random(5)
    seen_move = 0
    for _ in range(40):
        p, L, P, tf, tb, static, budget = random_partition_case(rng)
        got = bf.greedy_partition(p, L, P, tf, tb, static, budget)
        base, extra = divmod(L, P)
        equal = [base + (1 if s < extra else 0) for s in range(P)]
        t_equal = [bf.stage_time(p, n, s, P, tf, tb, static, budget) for s, n in enumerate(equal)]
        if any(t is None for t in t_equal):
            assert got is None
            continue
        layers, times = got
        assert sum(layers) == L and min(layers) >= 1
        assert max(times) <= max(t[0] for t in t_equal) + 1e-12
        best = bf.best_partition_exhaustive(p, L, P, tf, tb, static, budget)
        assert best[0] <= max(times) + 1e-12
        seen_move += layers != equal
    assert seen_move >= 3          # the cases do exercise step (4)


# ---- the library against the reference -------------------------------------------
B = pytest.importorskip("paper_2406_08756_amd.binding")


def test_library_partition_matches_reference_on_hand_worked_cases():
    layers, times, policies = B.lynx_partition_solve(two_op_layer(), 4, 2, 1.0, 2.0, 0.0, 60.0)
    assert layers == [1, 3] and times == [3.0, 9.0]
    assert all(q["critical_cost"] == 0.0 for q in policies)
    assert B.lynx_partition_solve(two_op_layer(), 4, 2, 1.0, 2.0, 0.0, 30.0) is None
    with pytest.raises(B.LynxError):
        B.lynx_partition_solve(two_op_layer(), 1, 2, 1.0, 2.0, 0.0, 60.0)      # fewer layers than stages


def test_library_partition_matches_reference_on_random_instances():
    rng = random.Random(9)
    for trial in range(60):
        p, L, P, tf, tb, static, budget = random_partition_case(rng)
        ref = bf.greedy_partition(p, L, P, tf, tb, static, budget)
        got = B.lynx_partition_solve(p, L, P, tf, tb, static, budget)
        if ref is None:
            assert got is None, trial
            continue
        assert got is not None, trial
        layers, times, policies = got
        assert layers == ref[0], (trial, layers, ref)
        assert all(abs(a - b) < 1e-9 for a, b in zip(times, ref[1])), trial
        for s, q in enumerate(policies):
            assert abs(layers[s] * (tf + tb + q["critical_cost"]) - times[s]) < 1e-9


def test_library_partition_on_the_gpt_layer():
    import lynx_synth as synth
    cfg = synth.CONFIGS["C4"]
    cost = [0.076, 0.37, 0.087, 0.098, 0.0, 0.084, 0.135, 0.09, 0.073, 0.417, 0.032, 0.38, 0.085]
    p = B.lynx_policy_layer_problem(cfg, cost, ctime=[0.27] * 4, m_budget=0.0, m_static=0.0,
                                    n_layer=1, n_batch=1, last_stage=False)
    act = sum(p["bytes"])
    # 40 layers on 4 stages, 1.9 ms forward + 3.2 ms backward per layer; a budget that holds
    # store-all for 10 layers at 2 micro-batches in flight but not at 4
    got = B.lynx_partition_solve(p, 40, 4, 1.9, 3.2, 0.0, 10 * 2.5 * act)
    assert got is not None
    layers, times, policies = got
    assert sum(layers) == 40
    assert layers[0] <= layers[-1]                       # early stages hold more in flight
    assert max(times) <= 10 * (1.9 + 3.2 + sum(cost[:11])) + 1e-9
    assert policies[-1]["critical_cost"] == 0.0          # the last stage keeps everything
