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
