"""Reference model of the retain/recompute bookkeeping (no numerics).

TEST INFRASTRUCTURE ONLY; shares no code with the library's host runtime.

Follows Sec. 4.2 of the paper: a layer is a chain of operators OP_1..OP_n; the
Boolean S_i says whether OP_i's output stays resident after the forward pass;
a discarded output is regenerated exactly once (Eq. 3) in one of the phases,
and an operator may run in a phase only if each operator it depends on has been
regenerated in that or an earlier phase or is stored (Eq. 4, read as "for every
dependency edge j -> i"); memory held after forward is sum_i S_i * M_i (Eq. 8).
Phases 1-4 are explicit recompute calls with a segment (set of operators);
phase 5 is the on-demand regeneration at the start of backward.

Activation A_i is OP_i's output (A0 = the layer input, always retained as the
checkpoint; A13 = the layer output, owned by the caller).
"""
from __future__ import annotations

from typing import Dict, List, Set

N_OPS = 13
# activation ids each operator reads
PARENTS: Dict[int, tuple] = {
    1: (0,), 2: (1,), 3: (2,), 4: (3,), 5: (4,), 6: (5, 2), 7: (6,),
    8: (0, 7), 9: (8,), 10: (9,), 11: (10,), 12: (11,), 13: (8, 12),
}
# activations the backward pass reads (S, O are stepping stones; V2, OUT never)
BACKWARD_NEEDS = (0, 1, 2, 4, 5, 6, 8, 9, 10, 11)

STORE_ALL = 0x3FFF
FULL_RECOMPUTE = 0x0001 | (1 << 13)
ATTENTION_ONLY = STORE_ALL & ~((1 << 3) | (1 << 4) | (1 << 5))
ELEMENTWISE_ONLY = STORE_ALL & ~((1 << 4) | (1 << 5) | (1 << 11))
SEG_ALL_MISSING = 0xFFFFFFFF


class DependencyError(Exception):
    pass


class StateError(Exception):
    pass


def activation_bytes(cfg) -> List[int]:
    """M_i in bytes for A0..A13.  LayerNorm outputs carry their two fp32
    per-token statistics; the s^2 tensors are stored densely as [b, a, s, s]."""
    e = 2 if cfg.dtype == 1 else 4
    T, h, f = cfg.micro_batch * cfg.seq, cfg.hidden, cfg.local_ffn
    p = cfg.local_heads * cfg.head_dim
    ss = cfg.micro_batch * cfg.local_heads * cfg.seq * cfg.seq
    th, stats = T * h * e, 2 * T * 4
    # C carries two fp32 attention row statistics per (batch element, head, row)
    attn_stats = cfg.micro_batch * cfg.local_heads * cfg.seq * 2 * 4
    return [th, th + stats, T * 3 * p * e, ss * e, ss * e, ss * e, T * p * e + attn_stats,
            th, th, th + stats, T * f * e, T * f * e, th, th]


def fused_attention(cfg, retain_mask: int) -> bool:
    """Whether the layer runs its attention without the seq x seq tensors: the
    configuration asks for it (flags bit 0), the policy keeps none of S, P, Pd (the tensors Selective Recomputation singles
    out, Sec. 2.2) and the shape is one those kernels are built for (bf16,
    head dimension 128, sequence a multiple of 128).  Then operators 3-5 never
    run, operator 6 reads QKV alone, and backward reads C (with its row
    statistics) instead of P and Pd."""
    return (bool(getattr(cfg, "flags", 0) & 1) and not (retain_mask & 0x38) and cfg.dtype == 1
            and cfg.head_dim == 128 and cfg.seq % 128 == 0 and cfg.seq >= 128)


def parents_of(i: int, fused: bool) -> tuple:
    return (2,) if (fused and i == 6) else PARENTS[i]


def backward_needs(fused: bool) -> tuple:
    return tuple(i for i in BACKWARD_NEEDS if not (fused and i in (4, 5)))


def missing_closure(live: Set[int], fused: bool = False) -> List[int]:
    """Operators that must run, in index order, so that backward finds every
    activation it reads: the needed-but-absent ones plus, transitively, their
    absent parents."""
    todo: Set[int] = set()
    stack = [i for i in backward_needs(fused) if i not in live]
    while stack:
        i = stack.pop()
        if i in todo:
            continue
        todo.add(i)
        stack.extend(j for j in parents_of(i, fused) if j not in live and j not in todo)
    return sorted(todo)


class LayerBookkeeping:
    """Which activations are resident, call by call."""

    def __init__(self, cfg):
        self.cfg = cfg
        self.M = activation_bytes(cfg)
        self.live: Set[int] = set()
        self.retain: Set[int] = set()
        self.state = "idle"
        self.fused = False

    def forward(self, retain_mask: int):
        if self.state != "idle":
            raise StateError("forward twice without backward")
        self.retain = {i for i in range(1, 13) if (retain_mask >> i) & 1} | {0, 13}
        self.live = set(self.retain)
        self.state = "forwarded"
        self.fused = fused_attention(self.cfg, retain_mask)

    def _release_stepping_stones(self):
        # a regenerated activation that backward never reads and whose
        # consumers are all resident is dropped again at once
        for i in (3, 7, 12):
            if i in self.live and i not in self.retain:
                consumers = [op for op, ps in PARENTS.items() if i in ps]
                if all(op in self.live for op in consumers):
                    self.live.discard(i)

    def recompute(self, segment_mask: int) -> List[int]:
        """Returns the operators actually run."""
        if self.state != "forwarded":
            raise StateError("recompute before forward")
        if segment_mask == SEG_ALL_MISSING:
            ops = missing_closure(self.live, self.fused)
        else:
            ops = [i for i in range(1, N_OPS + 1) if (segment_mask >> i) & 1]
        if self.fused:
            ops = [i for i in ops if i not in (3, 4, 5)]   # those operators do not exist in this mode
        # validate before changing anything
        live = set(self.live)
        for i in ops:
            if i in live:
                continue
            for j in parents_of(i, self.fused):
                if j not in live:
                    raise DependencyError(f"OP{i} needs A{j}")
            live.add(i)
        ran = []
        for i in ops:
            if i in self.live:
                continue
            self.live.add(i)
            ran.append(i)
            self._release_stepping_stones()
        return ran

    def backward(self) -> List[int]:
        if self.state != "forwarded":
            raise StateError("backward before forward")
        ran = self.recompute(SEG_ALL_MISSING)
        self.live = set()
        self.state = "idle"
        return ran

    def live_mask(self) -> int:
        m = 0
        for i in self.live:
            m |= 1 << i
        return m

    def live_bytes(self) -> int:
        """Library-resident bytes: A0 and A13 belong to the caller."""
        return sum(self.M[i] for i in self.live if 1 <= i <= 12)
