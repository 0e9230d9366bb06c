"""Expected time of checkpointed training under soft errors (arXiv 1903.01042, "Speedup in
Computation Time": Theorem 2 and the Markov-chain lemma of its appendix).

TEST INFRASTRUCTURE ONLY, like the rest of oracle/: used by tests and by the benchmark's
strategy-comparison leg to put the paper's model next to measured times.

The model.  Between two checkpoints (period I_0 iterations) the state is the number of iterations
completed since the checkpoint.  In every iteration one of three things happens:
    no error                        probability p_0: one step forward, time tau_f
    errors the strategy corrects    probability p_1: one step forward, time tau_b
    errors it cannot correct        probability p_2 = 1 - p_0 - p_1: back to state 0, time tau_b
(replication is the same chain with p_1 = 0: it detects but never corrects).  The expected time
of M iterations is  M / I_0 * (tau_cpt + E[T_{I_0}])  with T_k the time to reach state k from 0.

Reading of a point where the paper is at odds with itself.  The appendix derives the recursion
    E[T_{k+1}] = (E[T_k] + c) / (p_0 + p_1),     c = tau_f p_0 + tau_b (1 - p_0),
which with E[T_0] = 0 gives  E[T_k] = c * sum_{i=1..k} (p_0 + p_1)^-i.  Its base case then sets
E[T_1] = c (dropping the division that its own line above it has), and the lemma and Theorem 2
are printed as  c * sum_{i=0..k-1} (p_0 + p_1)^-i  -- smaller by the factor (p_0 + p_1).  The
chain is the definition; `expected_time_to_reach` solves it (hitting times of the chain, a linear
system solved by substitution) and agrees with the recursion, `printed_closed_form` is the formula as printed.  Both are
reported wherever the model is quoted.  Pins (tests/test_strategy_model.py): I_0 = 1 worked by
hand (a geometric number of attempts), the recursion, a Monte-Carlo walk of the chain.
"""
import numpy as np


def cost_per_attempt(p0, tau_f, tau_b):
    return tau_f * p0 + tau_b * (1.0 - p0)


def expected_time_to_reach(k, p0, p1, tau_f, tau_b):
    """E[T_k]: expected time from state 0 to state k, from the chain itself.  With h_s the expected
    time from state s to k:  h_s = c + (p0 + p1) h_{s+1} + p2 h_0,  h_k = 0  (c: expected cost of one
    iteration).  Solved by substitution from the far end: h_s = a_s + b_s h_0, so h_0 = a_0 / (1 - b_0).
    Where reaching k is so unlikely that 1 - b_0 vanishes in double precision the answer is infinite
    for every practical purpose, and inf is returned."""
    q, p2 = p0 + p1, 1.0 - p0 - p1
    c = cost_per_attempt(p0, tau_f, tau_b)
    a = b = 0.0
    for _ in range(k):
        a = c + q * a
        b = q * b + p2
    return a / (1.0 - b) if 1.0 - b > 1e-9 else float("inf")


def printed_closed_form(k, p0, p1, tau_f, tau_b):
    """The lemma as printed:  c * ((p0+p1)^-k - 1) / ((p0+p1)^-1 - 1)."""
    q = p0 + p1
    c = cost_per_attempt(p0, tau_f, tau_b)
    if q >= 1.0:
        return c * k
    return c * (q ** -k - 1.0) / (1.0 / q - 1.0)


def expected_total_time(M, I0, p0, p1, tau_f, tau_b, tau_cpt, printed=False):
    """M iterations with a checkpoint every I0:  M / I0 * (tau_cpt + E[T_{I0}])."""
    t = printed_closed_form(I0, p0, p1, tau_f, tau_b) if printed else expected_time_to_reach(I0, p0, p1, tau_f, tau_b)
    return M / I0 * (tau_cpt + t)


def best_period(M, p0, p1, tau_f, tau_b, tau_cpt, periods, printed=False):
    """(I0, expected time) minimising the expected total time over the given periods."""
    times = [expected_total_time(M, I0, p0, p1, tau_f, tau_b, tau_cpt, printed) for I0 in periods]
    j = int(np.argmin(times))
    return periods[j], times[j]


def replication_over_codenet(M, p0, p1, tau_f, tau_b, tau_cpt, periods, printed=False):
    """Theorem 2: ratio of the expected times, each strategy at its own best checkpoint period."""
    _, rep = best_period(M, p0, 0.0, tau_f, tau_b, tau_cpt, periods, printed)
    _, cod = best_period(M, p0, p1, tau_f, tau_b, tau_cpt, periods, printed)
    return rep / cod


def walk(k, p0, p1, tau_f, tau_b, rng):
    """One random walk of the chain from state 0 to state k; returns the time it took."""
    t, s = 0.0, 0
    while s < k:
        u = rng.random()
        if u < p0:
            t += tau_f
            s += 1
        elif u < p0 + p1:
            t += tau_b
            s += 1
        else:
            t += tau_b
            s = 0
    return t


def node_failure_probabilities(p, uses, t=1):
    """Independent node failures, each of `uses` node uses of an iteration failing with probability p
    (the paper counts 3 P^ L of them): p_0 = (1-p)^uses, and the paper's lower bound on p_1 for
    t = 1, a single failure: uses * p * (1-p)^(uses-1)."""
    p0 = (1.0 - p) ** uses
    p1 = uses * p * (1.0 - p) ** (uses - 1) if t >= 1 else 0.0
    return p0, p1
