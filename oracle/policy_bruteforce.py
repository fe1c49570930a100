"""Brute-force reference for the single-layer recomputation policy (Lynx-HEU).

Test infrastructure only: the product solver (csrc/policy.cpp, C ABI
lynx_policy_solve) is checked against this on small instances; nothing in the
product imports it.

The problem is the one of Sec. 4.2 ("Problem definition" to "Memory
constraints"): a layer of n operators OP_1..OP_n; Boolean S_i = "the output of
OP_i stays resident"; a discarded output is regenerated in exactly one of five
phases, R_{t,i} = 1: phases 1, 2 overlap the two forward communications,
phases 3, 4 the two backward ones, phase 5 is the critical path.

  objective   Eq. (objective2):  minimise  sum_i (1 - S_i) R_{5,i} C_i
  once        Eq. (cons11):      every regenerated operator runs in one phase
  dependency  Eq. (cons12):      OP_i may run in phase t only if every input
                                 OP_j is resident or was regenerated in a phase <= t
  overlap     Eq. (cons13):      sum_i (1 - S_i) R_{t,i} C_i <= CTime_t, t = 1..4
  comm        Eq. (cons14):      communication operators only in phase 5
  memory      Eq. (cons15-17):   M_static + N_layer N_batch sum_i S_i M_i
                                 + N_layer sum_i (1 - S_i)(R_{1,i} + R_{2,i}) M_i <= M_budget
  checkpoint  S_n = 1 (the layer output is the next layer's input)
  last stage  ("Optimizations"): phases 1 and 2 do not exist and the third
                                 memory term is dropped

Reading where the text leaves a gap: Eq. (cons11) sums to one for every i, also
for operators whose output is resident (where R is meaningless) and for
operators nothing downstream ever reads.  Here an operator is regenerated only
if something requires it: `needed` lists the operators whose outputs the
backward pass reads; a discarded operator in `needed` must be regenerated, and
a regenerated operator requires its discarded inputs to be regenerated no
later.  With needed = all operators this is the paper's model as printed.

A problem is a dict: n, cost[n], bytes[n], parents[n] (tuples of 1-based
operator indices, all < i; inputs that are the layer input are simply omitted),
comm (set of 1-based indices), needed (set), ctime[4], m_budget, m_static,
n_layer, n_batch, last_stage.  A policy is (S, phase): S[i] in {0, 1},
phase[i] in {0 (not regenerated), 1..5}, both indexed 0..n-1 for OP_1..OP_n.
"""
import itertools


def objective(problem, S, phase):
    """Eq. (objective2): regeneration time left on the critical path."""
    return sum(problem["cost"][i] for i in range(problem["n"]) if not S[i] and phase[i] == 5)


def peak_bytes(problem, S, phase):
    """Left side of Eq. (cons15) with Eq. (cons16) and Eq. (cons17)."""
    n = problem["n"]
    m_fwd = problem["n_layer"] * problem["n_batch"] * sum(problem["bytes"][i] for i in range(n) if S[i])
    m_comm = 0.0
    if not problem["last_stage"]:
        m_comm = problem["n_layer"] * sum(problem["bytes"][i] for i in range(n)
                                          if not S[i] and phase[i] in (1, 2))
    return problem["m_static"] + m_fwd + m_comm


def feasible(problem, S, phase):
    n = problem["n"]
    if not S[n - 1]:
        return False                                        # S_n = 1
    for i in range(n):
        if S[i] and phase[i] != 0:
            return False                                    # a resident output is not regenerated
        if not S[i] and (i + 1) in problem["needed"] and phase[i] == 0:
            return False                                    # backward would miss it
        if phase[i] != 0:
            if problem["last_stage"] and phase[i] in (1, 2):
                return False
            if (i + 1) in problem["comm"] and phase[i] != 5:
                return False                                # Eq. (cons14)
            for j in problem["parents"][i]:                 # Eq. (cons12)
                if not S[j - 1] and not (1 <= phase[j - 1] <= phase[i]):
                    return False
    for t in (1, 2, 3, 4):                                  # Eq. (cons13)
        if sum(problem["cost"][i] for i in range(n) if phase[i] == t) > problem["ctime"][t - 1] + 1e-12:
            return False
    return peak_bytes(problem, S, phase) <= problem["m_budget"] + 1e-9   # Eq. (cons15)


def brute_force(problem):
    """Every (S, phase) pair; returns (best objective, S, phase) or None when
    nothing is feasible.  Exponential: for n <= 7 only."""
    n = problem["n"]
    best = None
    for S in itertools.product((0, 1), repeat=n):
        if not S[n - 1]:
            continue
        free = [i for i in range(n) if not S[i]]
        for choice in itertools.product(range(6), repeat=len(free)):
            phase = [0] * n
            for i, t in zip(free, choice):
                phase[i] = t
            if not feasible(problem, S, phase):
                continue
            val = objective(problem, S, phase)
            if best is None or val < best[0] - 1e-12:
                best = (val, list(S), phase)
    return best


# ---- recomputation-aware model partitioning (Sec. 5) --------------------------------
# The greedy search of the section's "Key idea", steps (1)-(5), transcribed with the
# brute-force policy search above as the Recomputation Policy Generator.  The section
# gives no formula for the Training Cost Model; the reading used (here and in the
# library) is: a stage's time per micro-batch is its number of layers times
# (forward time + backward time + regeneration time left on the critical path), all per
# layer; stage s of P holds N_batch = P - s forward passes before its first backward
# (one-forward-one-backward schedule) and the last stage uses the last-stage variant of
# the policy program; M_static of a stage is static_per_layer times its layers.  Step (1),
# "approximately the same number of layers": floor(L / P) each, the remainder one each to
# the first stages.  Ties for slowest / fastest go to the lowest stage index.
def stage_time(layer_problem, n_layers, stage, n_stages, t_fwd, t_bwd, static_per_layer, m_budget):
    """(time per micro-batch, policy) of one stage, or None when no policy fits."""
    if n_layers == 0:
        return 0.0, None
    p = dict(layer_problem, n_layer=n_layers, n_batch=n_stages - stage, last_stage=(stage == n_stages - 1),
             m_static=static_per_layer * n_layers, m_budget=m_budget)
    best = brute_force(p)
    if best is None:
        return None
    return n_layers * (t_fwd + t_bwd + best[0]), best


def greedy_partition(layer_problem, n_total_layers, n_stages, t_fwd, t_bwd, static_per_layer, m_budget):
    """Returns (layers per stage, stage times) or None when the initial scheme is invalid."""
    base, extra = divmod(n_total_layers, n_stages)
    layers = [base + (1 if s < extra else 0) for s in range(n_stages)]              # step (1)

    def evaluate(scheme):                                                           # steps (2), (3)
        times = []
        for s, n in enumerate(scheme):
            r = stage_time(layer_problem, n, s, n_stages, t_fwd, t_bwd, static_per_layer, m_budget)
            if r is None:
                return None
            times.append(r[0])
        return times

    times = evaluate(layers)
    if times is None:
        return None
    while True:
        slow = max(range(n_stages), key=lambda s: (times[s], -s))
        fast = min(range(n_stages), key=lambda s: (times[s], s))
        if slow == fast or layers[slow] <= 1:
            break
        trial = list(layers)                                                        # step (4)
        trial[slow] -= 1
        trial[fast] += 1
        t2 = evaluate(trial)
        if t2 is None or max(t2) >= max(times) - 1e-12:
            break
        layers, times = trial, t2
    return layers, times


def best_partition_exhaustive(layer_problem, n_total_layers, n_stages, t_fwd, t_bwd, static_per_layer, m_budget):
    """Minimum over every composition of the layers into non-empty stages of the slowest
    stage's time: what the greedy search can at best reach."""
    best = None

    def rec(prefix, left):
        nonlocal best
        s = len(prefix)
        if s == n_stages - 1:
            scheme = prefix + [left]
            if left < 1:
                return
            worst = 0.0
            for st, n in enumerate(scheme):
                r = stage_time(layer_problem, n, st, n_stages, t_fwd, t_bwd, static_per_layer, m_budget)
                if r is None:
                    return
                worst = max(worst, r[0])
            if best is None or worst < best[0] - 1e-12:
                best = (worst, scheme)
            return
        for n in range(1, left - (n_stages - s - 1) + 1):
            rec(prefix + [n], left - n)

    rec([], n_total_layers)
    return best
