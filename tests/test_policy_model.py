"""Pins for the bookkeeping model against the paper's formulas: resident bytes
after forward equal sum_i S_i * M_i (memory constraint, Eq. 8), an operator may
be regenerated only when every operator it depends on is available (dependency
constraint, Eq. 4), and Full / Selective recomputation as described in Sec. 2.2."""
import itertools

import pytest

import lynx_synth as synth
from oracle import policy_model as pm


def test_activation_sizes_closed_form_c4():
    cfg = synth.CONFIGS["C4"]
    M = pm.activation_bytes(cfg)
    T, h = 16384, 5120
    assert M[0] == T * h * 2 == 167772160
    assert M[1] == T * h * 2 + 2 * T * 4
    assert M[2] == T * 1920 * 2
    assert M[3] == M[4] == M[5] == 8 * 5 * 2048 * 2048 * 2
    assert M[6] == T * 640 * 2 + 8 * 5 * 2048 * 2 * 4      # C and its attention row statistics
    assert M[10] == M[11] == T * 2560 * 2


@pytest.mark.parametrize("name", ["C1", "C4"])
def test_live_bytes_is_sum_of_retained_sizes(name):
    cfg = synth.CONFIGS[name]
    M = pm.activation_bytes(cfg)
    for mask in list(range(0, 1 << 14, 37)) + [pm.STORE_ALL, pm.FULL_RECOMPUTE, pm.ATTENTION_ONLY]:
        bk = pm.LayerBookkeeping(cfg)
        bk.forward(mask)
        assert bk.live_bytes() == sum(M[i] for i in range(1, 13) if (mask >> i) & 1)
        assert bk.live_mask() == (mask & 0x1FFE) | 1 | (1 << 13)


def test_full_recompute_regenerates_ops_1_to_11():
    bk = pm.LayerBookkeeping(synth.CONFIGS["C1"])
    bk.forward(pm.FULL_RECOMPUTE)
    assert bk.recompute(pm.SEG_ALL_MISSING) == list(range(1, 12))
    # stepping stones S and O are dropped again once P and X2 exist
    assert bk.live_mask() == sum(1 << i for i in (0, 1, 2, 4, 5, 6, 8, 9, 10, 11, 13))
    assert bk.backward() == []
    assert bk.live_bytes() == 0


def test_attention_only_regenerates_the_s2_tensors():
    bk = pm.LayerBookkeeping(synth.CONFIGS["C1"])
    bk.forward(pm.ATTENTION_ONLY)
    assert bk.recompute(pm.SEG_ALL_MISSING) == [3, 4, 5]


def test_store_all_needs_nothing():
    bk = pm.LayerBookkeeping(synth.CONFIGS["C1"])
    bk.forward(pm.STORE_ALL)
    assert bk.recompute(pm.SEG_ALL_MISSING) == []


def test_dependency_rule():
    bk = pm.LayerBookkeeping(synth.CONFIGS["C1"])
    bk.forward(pm.FULL_RECOMPUTE)
    with pytest.raises(pm.DependencyError):
        bk.recompute(1 << 2)                 # QKV needs Y1
    assert bk.live_mask() == pm.FULL_RECOMPUTE      # nothing changed
    assert bk.recompute((1 << 1) | (1 << 2)) == [1, 2]
    with pytest.raises(pm.DependencyError):
        bk.recompute(1 << 4)                 # P needs S
    assert bk.recompute((1 << 3) | (1 << 4)) == [3, 4]
    assert not (bk.live_mask() >> 3) & 1     # S released after P exists
    assert bk.recompute(1 << 2) == []        # already resident: no-op
    with pytest.raises(pm.DependencyError):
        bk.recompute(1 << 9)                 # Y2 needs X2


def test_split_phases_equal_one_shot():
    for mask in range(0, 1 << 14, 131):
        one = pm.LayerBookkeeping(synth.CONFIGS["C1"])
        one.forward(mask)
        ops = one.recompute(pm.SEG_ALL_MISSING)
        two = pm.LayerBookkeeping(synth.CONFIGS["C1"])
        two.forward(mask)
        half = len(ops) // 2
        two.recompute(sum(1 << i for i in ops[:half]))
        two.recompute(sum(1 << i for i in ops[half:]))
        needed = sum(1 << i for i in pm.BACKWARD_NEEDS)
        assert one.live_mask() & needed == needed
        assert two.live_mask() & needed == needed


def test_state_errors():
    bk = pm.LayerBookkeeping(synth.CONFIGS["C1"])
    with pytest.raises(pm.StateError):
        bk.backward()
    with pytest.raises(pm.StateError):
        bk.recompute(2)
    bk.forward(1)
    with pytest.raises(pm.StateError):
        bk.forward(1)
