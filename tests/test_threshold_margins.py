"""Where the thresholds tau_detect / tau_resid of every workload sit (no GPU).

The paper tests "syndrome = 0" exactly; in floating point that is a threshold (this build's
reading, parity unpinned by the paper).  A threshold is defensible when the quantities it
separates are far apart.  For both codes of each workload this file measures, with the oracle,
    floor      the relative syndrome of a fault-free product computed in the precision of the
               workload's arithmetic (bf16-rounded factors, or float32 products), and the relative
               residual of the true support in that precision,
    smallest   the smallest relative syndrome that a fault of the workload's law can give, and
               the smallest relative residual that any wrong support can give,
prints them, and asserts  5 x floor <= tau <= smallest / 5  -- the margin that the GPU parity
tests then demand of every single decision (harness.MARGIN).

The wrong-support residuals follow from the geometry of H alone.  With dense noise e_i on the
blocks of a support I, the syndrome at a position is H_I e(pos) and the least-squares residual
against another support J, over many positions with independent e of per-block variance v_i, is
    resid^2 / ||syndrome||^2 = tr(Q_J S) / tr(S),   S = H_I diag(v) H_I^T,  Q_J = I - H_J pinv(H_J).
For one erroneous block this is sin of the angle between the columns h_i and h_j, whatever v is.
"""
import itertools

import numpy as np
import pytest

from oracle import codenet_oracle as O
from paper_1903_01042_amd import workloads as WL

MARGIN = 5.0


def to_bf16(x):
    """Round float32 values to bf16 (round to nearest even), returned as float64."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def block_rms_of_clean_output(P):
    """Systematic output blocks have the rms of the data (taken as 1); parity block k is
    sum_i P[i,k] block_i of independent blocks."""
    return np.concatenate([np.ones(P.shape[0]), np.sqrt(np.sum(P * P, axis=0))])


def smallest_fault_syndrome(P, lo):
    """Smallest max_k ||syn_k|| / ref_k over single faulty blocks whose every element has the
    smallest magnitude lo x rms of the law (noise independent of the data)."""
    H = O.parity_check(P)
    rms = block_rms_of_clean_output(P)
    worst = np.inf
    for i in range(H.shape[1]):
        e2 = (lo * rms[i]) ** 2
        ratios = [abs(H[k, i]) * np.sqrt(e2) / np.sqrt(np.sum(H[k] ** 2 * rms ** 2) + H[k, i] ** 2 * e2)
                  for k in range(H.shape[0])]
        worst = min(worst, max(ratios))
    return worst


def wrong_support_residual(P, I, J, var):
    H = O.parity_check(P)
    HI, HJ = H[:, I], H[:, J]
    S = HI @ np.diag(var[list(I)]) @ HI.T
    Q = np.eye(H.shape[0]) - HJ @ np.linalg.pinv(HJ)
    return float(np.sqrt(max(np.trace(Q @ S), 0.0) / np.trace(S)))


def smallest_wrong_support_residual(P, var):
    """Over every true support I of 1 .. t+1 blocks and every support J != I of at most
    min(|I|, t) blocks that the search would try: the smallest relative residual.  (For |I| = t+1
    these are the residuals that must be rejected to report UNCORRECTABLE.)"""
    H = O.parity_check(P)
    r, L = H.shape
    t = r // 2
    worst, where = np.inf, None
    for ki in range(1, min(t + 1, L) + 1):
        for I in itertools.combinations(range(L), ki):
            for kj in range(1, min(ki, t) + 1):
                for J in itertools.combinations(range(L), kj):
                    if J == I:
                        continue
                    res = wrong_support_residual(P, I, J, var)
                    if res < worst:
                        worst, where = res, (I, J)
    return worst, where


def floors(P, B, b, dtype, seed):
    """Relative syndrome of a fault-free codeword and relative residual of the true support of one
    faulty block, with the product computed in the workload's arithmetic: K = 8 B terms per output."""
    a, r = P.shape
    g = np.random.default_rng(seed)
    K = 8 * B
    W = (g.standard_normal((a * B, K)) / np.sqrt(K)).astype(np.float32)
    X = g.standard_normal((K, b)).astype(np.float32)
    Wt = O.encode_vector(W.astype(np.float64), P, B).astype(np.float32)          # coded rows, float32 master
    if dtype == "bf16":
        out = to_bf16(Wt) @ to_bf16(X)
    else:
        out = (Wt @ X).astype(np.float64)                                        # float32 accumulation
    clean = O.detect_decode(out, P, B, 0.0, 0.0)
    floor_syn = float(np.max(clean["syn_rel"]))
    floor_res = 0.0
    if r >= 2:
        rms = np.sqrt(np.mean(out[:B] ** 2))
        for i in (0, a - 1, a, a + r - 1):
            bad = out.copy()
            bad[i * B:(i + 1) * B] += rms * g.uniform(1.0, 10.0, (B, b)) * g.choice([-1.0, 1.0], (B, b))
            res = O.detect_decode(bad, P, B, 0.0, 1.0)
            assert res["located"] == [i]
            floor_res = max(floor_res, res["resid_rel"])
    return floor_syn, floor_res


CASES = [(name, axis) for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5") for axis in (0, 1)]


@pytest.mark.parametrize("name,axis", CASES)
def test_thresholds_sit_between_the_rounding_floor_and_the_smallest_signal(name, axis):
    wl = WL.WORKLOADS[name]
    P = wl.generators(0)[axis]
    r = P.shape[1]
    floor_syn, floor_res = floors(P, 32, 48, wl.dtype, seed=77 + axis)
    sig_syn = smallest_fault_syndrome(P, lo=1.0)
    print("\n%s %s code (a=%d, r=%d, %s): clean syndrome floor %.2e  <  tau_detect %.1e  <  smallest fault %.2e"
          % (name, "row" if axis == 0 else "column", P.shape[0], r, wl.dtype, floor_syn, wl.tau_detect, sig_syn))
    assert MARGIN * floor_syn <= wl.tau_detect, "tau_detect is within 5x of the rounding floor"
    assert wl.tau_detect * MARGIN <= sig_syn, "a fault of the smallest magnitude is within 5x of tau_detect"
    if r >= 2:
        var = block_rms_of_clean_output(P) ** 2
        wrong, where = smallest_wrong_support_residual(P, var)
        print("   true-support residual floor %.2e  <  tau_resid %.1e  <  smallest wrong-support residual %.3f %s"
              % (floor_res, wl.tau_resid, wrong, where))
        assert MARGIN * floor_res <= wl.tau_resid, "tau_resid is within 5x of the residual of the true support"
        assert wl.tau_resid * MARGIN <= wrong, "a wrong support comes within 5x of tau_resid"


def test_one_block_residual_is_the_sine_of_the_angle_between_columns():
    """The closed form used above, against the oracle's own search: one erroneous block i, support
    {j} forced by leaving only j as candidate -- residual / ||syndrome|| = sin(angle(h_i, h_j))."""
    P = WL.vandermonde_like(8, 2)
    H = O.parity_check(P)
    g = np.random.default_rng(3)
    B, b = 5, 4
    for i, j in ((0, 1), (3, 9), (8, 2)):
        e = g.standard_normal((B * b,))
        syn = np.outer(H[:, i], e)
        E, *_ = np.linalg.lstsq(H[:, [j]], syn, rcond=None)
        direct = np.linalg.norm(H[:, [j]] @ E - syn) / np.linalg.norm(syn)
        hi, hj = H[:, i], H[:, j]
        sine = np.sqrt(1.0 - (hi @ hj) ** 2 / ((hi @ hi) * (hj @ hj)))
        assert abs(direct - sine) < 1e-12
        assert abs(wrong_support_residual(P, (i,), (j,), np.ones(10)) - sine) < 1e-12


@pytest.mark.parametrize("a,r,seed", [(3, 4, 8), (3, 4, 21), (3, 4, 5), (3, 4, 6), (4, 4, 8), (4, 4, 9)])
def test_the_four_parity_generators_of_the_gpu_tests_keep_wrong_supports_away(a, r, seed):
    """The t = 2 campaigns on the GPU use Gaussian generators with these seeds at float32
    thresholds (tau_resid = 2e-3) and demand the 5x margin of every decision."""
    P = WL.gaussian_generator(a, r, seed)
    var = block_rms_of_clean_output(P) ** 2
    wrong, where = smallest_wrong_support_residual(P, var)
    floor_syn, floor_res = floors(P, 16, 24, "f32", seed=5)
    print("\nGaussian (a=%d, r=%d, seed %d): floors %.1e / %.1e, smallest wrong-support residual %.3f %s"
          % (a, r, seed, floor_syn, floor_res, wrong, where))
    assert 2e-3 * MARGIN <= wrong
    assert MARGIN * floor_syn <= 1e-3 and MARGIN * floor_res <= 2e-3
