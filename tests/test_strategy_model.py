"""Pins of the expected-time model (Theorem 2 and the Markov-chain lemma of its appendix)."""
import numpy as np
import pytest

from oracle import strategy_model as S


def test_one_iteration_between_checkpoints_worked_by_hand():
    """I_0 = 1: every attempt costs tau_f with probability p_0 and tau_b otherwise, and succeeds with
    probability q = p_0 + p_1; the number of attempts is geometric with mean 1 / q, so by Wald's
    identity E[T_1] = (tau_f p_0 + tau_b (1 - p_0)) / q.  Numbers: p_0 = 1/2, p_1 = 1/4, tau_f = 1,
    tau_b = 9: c = 1/2 + 9/2 = 5, E[T_1] = 5 / (3/4) = 20/3.  The lemma as printed gives c = 5: the
    paper's base case drops the division by q that its own recursion has."""
    assert abs(S.expected_time_to_reach(1, 0.5, 0.25, 1.0, 9.0) - 20.0 / 3.0) < 1e-12
    assert abs(S.printed_closed_form(1, 0.5, 0.25, 1.0, 9.0) - 5.0) < 1e-12
    # two states by hand as well: h_1 = c + (1/4) h_0, h_0 = c + (3/4) h_1 + (1/4) h_0
    #   => h_0 (3/4) = c + (3/4) c + (3/16) h_0  => h_0 = (7/4) c / (9/16) = 140/9
    assert abs(S.expected_time_to_reach(2, 0.5, 0.25, 1.0, 9.0) - 140.0 / 9.0) < 1e-12


@pytest.mark.parametrize("p0,p1", [(0.9, 0.08), (0.5, 0.3), (0.7, 0.0), (0.2, 0.1)])
def test_chain_solution_obeys_the_recursion_of_the_appendix(p0, p1):
    """E[T_{k+1}] = (E[T_k] + c) / (p_0 + p_1), E[T_0] = 0; the printed closed form is the same sum
    shifted by one power, i.e. smaller by the factor p_0 + p_1."""
    tau_f, tau_b = 1.0, 25.0
    c = S.cost_per_attempt(p0, tau_f, tau_b)
    prev = 0.0
    for k in range(1, 12):
        cur = S.expected_time_to_reach(k, p0, p1, tau_f, tau_b)
        assert abs(cur - (prev + c) / (p0 + p1)) < 1e-9 * cur
        assert abs(S.printed_closed_form(k, p0, p1, tau_f, tau_b) - (p0 + p1) * cur) < 1e-9 * cur
        prev = cur


def test_a_random_walk_of_the_chain_takes_the_expected_time():
    rng = np.random.default_rng(5)
    p0, p1, tau_f, tau_b, k = 0.8, 0.12, 1.0, 30.0, 6
    mean = np.mean([S.walk(k, p0, p1, tau_f, tau_b, rng) for _ in range(40000)])
    want = S.expected_time_to_reach(k, p0, p1, tau_f, tau_b)
    assert abs(mean - want) < 0.02 * want
    assert abs(mean - S.printed_closed_form(k, p0, p1, tau_f, tau_b)) > 0.05 * want


def test_no_errors_and_the_ratio_of_theorem_2():
    """Without errors M iterations cost M tau_f plus the checkpoints; the ratio replication / CodeNet
    is 1 when nothing is correctable (p_1 = 0), above 1 for the theoretical plot's setting (Poisson
    errors, t = 1, tau_cpt = tau_b = 1000, tau_f = 1) and grows with p_1 at fixed p_0."""
    assert abs(S.expected_total_time(100, 10, 1.0, 0.0, 2.0, 50.0, 7.0) - (100 * 2.0 + 10 * 7.0)) < 1e-9
    periods = list(range(1, 400))
    assert abs(S.replication_over_codenet(1000, 0.7, 0.0, 1.0, 1000.0, 1000.0, periods) - 1.0) < 1e-12
    ratios = []
    for lam in (0.1, 0.5, 1.0, 2.0):
        p0, p1 = np.exp(-lam), lam * np.exp(-lam)
        ratios.append(S.replication_over_codenet(1000, p0, p1, 1.0, 1000.0, 1000.0, periods))
    assert all(r > 1.5 for r in ratios)
    ratios = [S.replication_over_codenet(1000, 0.5, p1, 1.0, 1000.0, 1000.0, periods) for p1 in (0.0, 0.1, 0.3, 0.45)]
    assert ratios[0] == 1.0 and all(b > a for a, b in zip(ratios, ratios[1:])) and ratios[-1] > 2.5
    p0, p1 = S.node_failure_probabilities(3e-4, 3 * 38 * 3)
    assert abs(p0 - (1 - 3e-4) ** 342) < 1e-15 and 0.09 < p1 < 0.1
