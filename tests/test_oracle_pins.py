"""Pins of the float64 oracle against what the paper prints and what the
mathematics fixes (no GPU).  Each test names the passage it relies on."""
import itertools

import numpy as np
import pytest

from oracle import codenet_oracle as O
from paper_1903_01042_amd import workloads as WL

rng = np.random.default_rng(12345)


def _example(ex):
    G_r, G_c = np.array(ex["G_r"]), np.array(ex["G_c"])
    return G_r, G_c, G_r[:, 2:], G_c[:, 2:]


# ----------------------------------------------------------- code construction
def test_generators_match_worked_example(worked_example):
    """Section on pre-processing: G_r and G_c as printed; G = [I | P]."""
    G_r, G_c, P_r, P_c = _example(worked_example)
    assert np.array_equal(O.generator(P_r), G_r)
    assert np.array_equal(O.generator(P_c), G_c)
    pr, pc = WL.paper_example_generators()
    assert np.array_equal(pr, P_r) and np.array_equal(pc, P_c)


@pytest.mark.parametrize("a,r,kind", [(2, 2, "paper"), (4, 2, "spread"), (8, 2, "spread"),
                                      (16, 2, "spread"), (4, 4, "positive"), (3, 1, "gauss"),
                                      (5, 3, "positive"), (4, 1, "gauss")])
def test_parity_check_annihilates_and_spark(a, r, kind, worked_example):
    """Appendix, proof of Lemma 2: H G^T = 0, H full rank, Spark(H) = r + 1
    (= 2t + 1 for r = 2t); systematic MDS: any a columns of G independent."""
    if kind == "paper":
        P = _example(worked_example)[2]
    elif kind == "gauss":
        P = WL.gaussian_generator(a, r, seed=3)
    else:
        P = WL.vandermonde_like(a, r, nodes=kind)
    G, H = O.generator(P), O.parity_check(P)
    assert G.shape == (a, a + r) and H.shape == (r, a + r)
    assert np.array_equal(G[:, :a], np.eye(a))
    assert np.max(np.abs(H @ G.T)) < 1e-12
    assert np.linalg.matrix_rank(H) == r
    assert O.is_mds(P)
    if a + r <= 12:
        assert O.spark(H) == r + 1


def test_non_mds_generator_is_rejected():
    P = np.array([[1.0, 2.0], [1.0, 2.0], [1.0, 3.0]])     # rows 0 and 1 give a zero minor
    assert not O.is_mds(P)
    assert O.spark(O.parity_check(P)) < 3


def test_node_count_of_the_experiment(worked_example):
    """Theorem 1 with t1+t3 = t2+t3 = t: P^ = P + 2(m+n)t; 5x4 grid, t=1 -> 38 nodes."""
    m, n = (int(v) for v in worked_example["ec2_grid"])
    t = int(worked_example["ec2_t"][0])
    nodes = WL.active_nodes(WL.PHASE_WEIGHT, m, n, 2 * t, 2 * t)
    assert len(nodes) == int(worked_example["ec2_nodes"][0]) == m * n + 2 * (m + n) * t
    assert len(WL.active_nodes(WL.PHASE_FWD, m, n, 2 * t, 2 * t)) == (m + 2 * t) * n
    assert len(WL.active_nodes(WL.PHASE_BWD, m, n, 2 * t, 2 * t)) == m * (n + 2 * t)


# --------------------------------------------------------------------- encoding
def test_encode_worked_example_blocks(worked_example):
    """Pre-processing example: W~_{2,j} = W_{0,j}+W_{1,j}, W~_{3,j} = W_{0,j}-W_{1,j},
    W~_{i,2} = W_{i,0}+W_{i,1}, W~_{i,3} = W_{i,0}+2W_{i,1}; systematic blocks unchanged."""
    ex = worked_example
    _, _, P_r, P_c = _example(ex)
    Br, Bc = 3, 5
    W = rng.standard_normal((2 * Br, 2 * Bc))
    Wt = O.encode(W, P_r, P_c)
    blk = lambda M, i, j: M[i * Br:(i + 1) * Br, j * Bc:(j + 1) * Bc]
    for i in range(2):
        for j in range(2):
            assert np.array_equal(blk(Wt, i, j), blk(W, i, j))
    for row in (2, 3):
        c = ex["parity_row_%d" % row]
        for j in range(2):
            assert np.allclose(blk(Wt, row, j), c[0] * blk(W, 0, j) + c[1] * blk(W, 1, j), atol=1e-14)
    for col in (2, 3):
        c = ex["parity_col_%d" % col]
        for i in range(2):
            assert np.allclose(blk(Wt, i, col), c[0] * blk(W, i, 0) + c[1] * blk(W, i, 1), atol=1e-14)
    assert np.all(O.encode(W, P_r, P_c, store_corner=False)[2 * Br:, 2 * Bc:] == 0)


@pytest.mark.parametrize("N_out,N_in,m,n,r_r,r_c,Br,Bc", [
    (6, 8, 2, 2, 2, 2, None, None), (10, 9, 4, 3, 1, 2, None, None),
    (10, 9, 4, 3, 2, 4, 4, 4), (5, 7, 3, 2, 2, 0, 3, 4)])
def test_encode_is_the_kronecker_form_elementwise(N_out, N_in, m, n, r_r, r_c, Br, Bc):
    """Claim 1: W~ = (G_r^T (x) I) W (G_c (x) I), evaluated two other ways: with
    explicit Kronecker matrices and element by element with plain loops."""
    P_r = WL.vandermonde_like(m, r_r, "positive")
    P_c = WL.gaussian_generator(n, r_c, seed=5) if r_c else np.zeros((n, 0))
    W = rng.standard_normal((N_out, N_in))
    Wt = O.encode(W, P_r, P_c, Br, Bc)
    Br = Br or O.block_size(N_out, m)
    Bc = Bc or O.block_size(N_in, n)
    # zero padded W, by hand
    B0r, B0c = -(-N_out // m), -(-N_in // n)
    Wp = np.zeros((m * Br, n * Bc))
    for g in range(N_out):
        for h in range(N_in):
            Wp[(g // B0r) * Br + g % B0r, (h // B0c) * Bc + h % B0c] = W[g, h]
    G_r = np.hstack([np.eye(m), P_r])
    G_c = np.hstack([np.eye(n), P_c])
    kron = np.kron(G_r.T, np.eye(Br)) @ Wp @ np.kron(G_c, np.eye(Bc))
    assert np.allclose(Wt, kron, atol=1e-13)
    loops = np.zeros_like(Wt)
    for i in range(m + r_r):
        for j in range(n + r_c):
            for rho in range(Br):
                for kap in range(Bc):
                    acc = 0.0
                    for i2 in range(m):
                        for j2 in range(n):
                            acc += G_r[i2, i] * G_c[j2, j] * Wp[i2 * Br + rho, j2 * Bc + kap]
                    loops[i * Br + rho, j * Bc + kap] = acc
    assert np.allclose(Wt, loops, atol=1e-13)


# ------------------------------------------------------------- coded products
def test_forward_codeword_of_worked_example(worked_example):
    """Feedforward example: outputs are [s_0; s_1; s_0+s_1; s_0-s_1]."""
    ex = worked_example
    _, _, P_r, P_c = _example(ex)
    Br, Bc, b = 4, 3, 2
    W = rng.standard_normal((2 * Br, 2 * Bc))
    X = rng.standard_normal((2 * Bc, b))
    lay = O.CodedLayer(W, P_r, P_c)
    St = lay.forward(X)
    S = W @ X
    s = [S[:Br], S[Br:]]
    assert np.allclose(St[:2 * Br], S, atol=1e-13)
    for row in (2, 3):
        c = ex["fwd_codeword_%d" % row]
        assert np.allclose(St[row * Br:(row + 1) * Br], c[0] * s[0] + c[1] * s[1], atol=1e-13)


@pytest.mark.parametrize("N_out,N_in,m,n,r,b", [(12, 8, 3, 2, 2, 3), (10, 9, 4, 3, 1, 1),
                                                (16, 16, 4, 4, 4, 2)])
def test_products_without_errors_are_the_textbook_products(N_out, N_in, m, n, r, b):
    """Lemma 2, first display of the proof: the outputs are the codeword
    (G^T (x) I) s; with no errors the decoded result is exactly W x (and W^T delta);
    the syndrome is zero (third display after Lemma 2's proof of part 2)."""
    P_r = WL.vandermonde_like(m, r, "positive")
    P_c = WL.gaussian_generator(n, r, seed=9)
    W = rng.standard_normal((N_out, N_in))
    X = rng.standard_normal((N_in, b))
    D = rng.standard_normal((N_out, b))
    lay = O.CodedLayer(W, P_r, P_c)
    St = lay.forward(X)
    Ct = lay.backward(D)
    S, C = W @ X, W.T @ D
    Sp = O.pad_blocks(S, m)
    Cp = O.pad_blocks(C, n)
    assert np.allclose(St, np.kron(np.hstack([np.eye(m), P_r]).T, np.eye(lay.Br)) @ Sp, atol=1e-12)
    assert np.allclose(Ct, np.kron(np.hstack([np.eye(n), P_c]).T, np.eye(lay.Bc)) @ Cp, atol=1e-12)
    for phase, out, ref in ((O.PHASE_FWD, St, S), (O.PHASE_BWD, Ct, C)):
        res = lay.detect_decode(phase, out)
        assert res["verdict"] == O.CLEAN and res["located"] == []
        assert np.max(res["syn_rel"]) < 1e-12
        assert np.allclose(res["decoded"], ref, atol=1e-12)


def test_vector_encodings_of_worked_example(worked_example):
    """Step 4 of both stages: x~_2 = x_0+x_1, x~_3 = x_0+2x_1; d~_2 = d_0+d_1, d~_3 = d_0-d_1."""
    ex = worked_example
    _, _, P_r, P_c = _example(ex)
    B, b = 3, 2
    x = rng.standard_normal((2 * B, b))
    d = rng.standard_normal((2 * B, b))
    xt = O.encode_vector(x, P_c, B)
    dt = O.encode_vector(d, P_r, B)
    assert np.array_equal(xt[:2 * B], x) and np.array_equal(dt[:2 * B], d)
    for k in (2, 3):
        cx, cd = ex["x_parity_%d" % k], ex["delta_parity_%d" % k]
        assert np.allclose(xt[k * B:(k + 1) * B], cx[0] * x[:B] + cx[1] * x[B:], atol=1e-14)
        assert np.allclose(dt[k * B:(k + 1) * B], cd[0] * d[:B] + cd[1] * d[B:], atol=1e-14)


# ------------------------------------------------------------ detect / decode
def test_subset_checks_of_worked_example(worked_example):
    """Feedforward example with s_1 erroneous: of the four 3-subsets only
    {s_0, s~_2, s~_3} is consistent (2 s_0 = s~_2 + s~_3), and s_1 = s~_2 - s_0."""
    ex = worked_example
    _, _, P_r, P_c = _example(ex)
    B, b = 4, 2
    W = rng.standard_normal((2 * B, 2 * B))
    X = rng.standard_normal((2 * B, b))
    lay = O.CodedLayer(W, P_r, P_c, tau_detect=1e-9, tau_resid=1e-9)
    St = lay.forward(X)
    e1 = rng.standard_normal((B, b))
    bad = St.copy()
    bad[B:2 * B] += e1
    out = [bad[i * B:(i + 1) * B] for i in range(4)]
    G = np.array(ex["G_r"])
    passing = []
    for sub in itertools.combinations(range(4), 3):
        # a 3-subset of a (4,2) code is consistent iff its blocks lie in the row space of G[:, sub]
        A = G[:, sub].T                                  # 3 x 2
        Y = np.stack([out[i].reshape(-1) for i in sub])  # 3 x (B b)
        sol, *_ = np.linalg.lstsq(A, Y, rcond=None)
        if np.max(np.abs(A @ sol - Y)) < 1e-10:
            passing.append(list(sub))
    assert passing == [[int(v) for v in ex["passing_subset_s1_error"]]]
    chk = ex["passing_check"]
    assert np.max(np.abs(sum(c * o for c, o in zip(chk, out)))) < 1e-12
    dec = ex["decode_s1"]
    s1 = sum(c * o for c, o in zip(dec, out))
    assert np.allclose(s1, (W @ X)[B:], atol=1e-12)
    res = lay.detect_decode(O.PHASE_FWD, bad)
    assert res["verdict"] == O.CORRECTED and res["located"] == [1]
    assert np.allclose(res["decoded"], W @ X, atol=1e-11)


def test_syndrome_is_H_times_error():
    """Appendix: (H (x) I) out = (H (x) I) e for out = codeword + e."""
    m, r, B, b = 4, 2, 3, 2
    P = WL.vandermonde_like(m, r)
    s = rng.standard_normal((m * B, b))
    cw = O.encode_vector(s, P, B)
    e = np.zeros_like(cw)
    e[2 * B:3 * B] = rng.standard_normal((B, b))
    e[5 * B:6 * B] = rng.standard_normal((B, b))
    H = np.hstack([P.T, -np.eye(r)])
    assert np.allclose(O.syndromes(cw + e, P, B), np.kron(H, np.eye(B)) @ e, atol=1e-12)
    assert np.max(np.abs(O.syndromes(cw, P, B))) < 1e-12


@pytest.mark.parametrize("m,r", [(2, 2), (4, 2), (6, 2), (3, 4), (4, 4)])
def test_every_error_pattern_within_capability_is_located(m, r):
    """Lemma 2 (1): any t or fewer erroneous blocks are located and corrected,
    for every support, by exhaustive enumeration."""
    t, L, B, b = r // 2, m + r, 3, 2
    P = WL.vandermonde_like(m, r, "spread" if r <= 2 else "positive")
    s = rng.standard_normal((m * B, b))
    cw = O.encode_vector(s, P, B)
    for k in range(1, t + 1):
        for A in itertools.combinations(range(L), k):
            bad = cw.copy()
            for i in A:
                bad[i * B:(i + 1) * B] += rng.uniform(1, 10, (B, b)) * rng.choice([-1, 1], (B, b))
            res = O.detect_decode(bad, P, B, 1e-9, 1e-7)
            assert res["verdict"] == O.CORRECTED, (A, res["resid_rel"])
            assert res["located"] == list(A)
            assert np.allclose(res["out"], cw, atol=1e-8)


@pytest.mark.parametrize("m,r", [(2, 2), (4, 2), (3, 4)])
def test_more_errors_than_capability_are_detected_not_miscorrected(m, r):
    """Lemma 2 (2) and the remark after the decoding algorithm: with t+1..r
    erroneous blocks of continuous noise the check never passes and no sparse
    solution is accepted."""
    t, L, B, b = r // 2, m + r, 3, 2
    P = WL.vandermonde_like(m, r, "spread" if r <= 2 else "positive")
    s = rng.standard_normal((m * B, b))
    cw = O.encode_vector(s, P, B)
    for k in range(t + 1, r + 1):
        for A in itertools.combinations(range(L), k):
            bad = cw.copy()
            for i in A:
                bad[i * B:(i + 1) * B] += rng.uniform(1, 10, (B, b)) * rng.choice([-1, 1], (B, b))
            res = O.detect_decode(bad, P, B, 1e-9, 1e-7)
            assert res["verdict"] == O.UNCORRECTABLE, (A, res)
            assert res["located"] == []
            assert np.array_equal(res["out"], bad)


def test_relative_syndrome_of_a_hand_computed_case():
    """H = [2 3 | -1]; blocks (3,0), (0,4), parity (1,1): syndrome (5,11),
    ref^2 = 4*9 + 9*16 + 1*2 = 182, so the ratio is sqrt(146/182)."""
    P = np.array([[2.0], [3.0]])
    out = np.array([[3.0, 0.0], [0.0, 4.0], [1.0, 1.0]])        # B = 1, b = 2
    res = O.detect_decode(out, P, 1, 1e-3, 1e-2)
    assert res["verdict"] == O.UNCORRECTABLE
    assert abs(res["syn_rel"][0] - np.sqrt(146.0 / 182.0)) < 1e-14
    assert np.allclose(O.syndromes(out, P, 1), [[5.0, 11.0]])


def test_relative_residual_of_hand_computed_cases():
    """Decoding algorithm of the appendix, least-squares reading.  H = [1 1 -1 0; 1 2 0 -1] (the
    worked example's column code): columns h0 = (1,1), h1 = (1,2), h2 = (-1,0), h3 = (0,-1).

    Two erroneous blocks, one position: out = (1, 1, 0, 0) gives the syndrome s = (2, 3), |s|^2 = 13.
    Residual^2 of the one-block support {i} is |s|^2 - (h_i . s)^2 / |h_i|^2:
      {0}: 13 - 25/2 = 1/2     {1}: 13 - 64/5 = 1/5     {2}: 13 - 4 = 9     {3}: 13 - 9 = 4
    so the best support is {1} with relative residual sqrt((1/5)/13) = sqrt(1/65), its error estimate
    is (h1 . s)/|h1|^2 = 8/5, and the repaired block is 1 - 8/5 = -3/5.  Beyond the threshold the same
    number is reported with the verdict UNCORRECTABLE and the output untouched.

    Two positions (B = 2): block 0 = (1, 0), block 1 = (1, 1) give s(0) = (2, 3), s(1) = (1, 2) = h1.
    {1}: 1/5 + 0 of 13 + 5 = 18, relative residual sqrt(1/90); {0}: 1/2 + (5 - 9/2) = 1 of 18.
    One erroneous block, out = (0, 2, 0, 0): s = 2 h1, residual exactly 0."""
    P = np.array([[1.0, 1.0], [1.0, 2.0]])
    out = np.array([[1.0], [1.0], [0.0], [0.0]])
    res = O.detect_decode(out, P, 1, 1e-3, 0.2)
    assert res["verdict"] == O.CORRECTED and res["located"] == [1]
    assert abs(res["resid_rel"] - np.sqrt(1.0 / 65.0)) < 1e-15
    assert np.allclose(res["out"].ravel(), [1.0, -0.6, 0.0, 0.0], atol=1e-15)
    res = O.detect_decode(out, P, 1, 1e-3, 0.12)          # sqrt(1/65) = 0.12403...: just above the threshold
    assert res["verdict"] == O.UNCORRECTABLE and res["located"] == []
    assert abs(res["resid_rel"] - np.sqrt(1.0 / 65.0)) < 1e-15
    assert np.array_equal(res["out"], out)
    out2 = np.array([[1.0], [0.0], [1.0], [1.0], [0.0], [0.0], [0.0], [0.0]])
    res = O.detect_decode(out2, P, 2, 1e-3, 0.2)
    assert res["verdict"] == O.CORRECTED and res["located"] == [1]
    assert abs(res["resid_rel"] - np.sqrt(1.0 / 90.0)) < 1e-15
    assert np.allclose(res["out"].ravel(), [1.0, 0.0, -0.6, 0.0, 0, 0, 0, 0], atol=1e-15)
    res = O.detect_decode(np.array([[0.0], [2.0], [0.0], [0.0]]), P, 1, 1e-3, 1e-9)
    assert res["verdict"] == O.CORRECTED and res["located"] == [1] and res["resid_rel"] == 0.0
    assert np.array_equal(res["out"], np.zeros((4, 1)))


def test_equal_residuals_go_to_the_first_support_in_lexicographic_order():
    """This build's tie rule (the paper's true support is unique, so it needs none).
    H = [1 1 -1 0; 1 -1 0 -1]: h0 = (1,1), h1 = (1,-1), h2 = (-1,0), h3 = (0,-1), three positions.
    Syndromes (1,0), (1,0), (1,1) (written into the parity blocks): |s|^2 sums to 4;
      {0}: 1/2 + 1/2 + 0 = 1     {2}: 0 + 0 + 1 = 1     {1}: 1/2 + 1/2 + 2 = 3     {3}: 1 + 1 + 1 = 3
    -- {0} and {2} tie at relative residual 1/2 and {0} is taken.  A change of 1e-9 in the last
    syndrome towards h2 hands the decision to {2}: it is the residual that decides, the order only
    breaks the tie.  Mirrored syndromes (0,1), (0,1), (1,-1) tie {1} and {3}: {1} is taken; syndromes
    (1,0), (0,1) tie all four supports at 1/sqrt(2): {0} is taken."""
    P = np.array([[1.0, 1.0], [1.0, -1.0]])

    def coded(s0, s1):           # out with zero systematic blocks: syndrome_k = -parity block k
        B = len(s0)
        out = np.zeros((4 * B, 1))
        out[2 * B:3 * B, 0] = -np.asarray(s0, dtype=np.float64)
        out[3 * B:4 * B, 0] = -np.asarray(s1, dtype=np.float64)
        return out

    res = O.detect_decode(coded([1, 1, 1], [0, 0, 1]), P, 3, 1e-3, 0.6)
    assert res["verdict"] == O.CORRECTED and res["located"] == [0] and res["resid_rel"] == 0.5
    res = O.detect_decode(coded([1, 1, 1], [0, 0, 1 - 1e-9]), P, 3, 1e-3, 0.6)
    assert res["located"] == [2] and res["resid_rel"] < 0.5
    res = O.detect_decode(coded([1, 1, 1], [0, 0, 1 + 1e-9]), P, 3, 1e-3, 0.6)
    assert res["located"] == [0] and res["resid_rel"] < 0.5
    res = O.detect_decode(coded([0, 0, 1], [1, 1, -1]), P, 3, 1e-3, 0.6)
    assert res["verdict"] == O.CORRECTED and res["located"] == [1] and res["resid_rel"] == 0.5
    res = O.detect_decode(coded([1, 0], [0, 1]), P, 2, 1e-3, 0.8)
    assert res["verdict"] == O.CORRECTED and res["located"] == [0]
    assert abs(res["resid_rel"] - np.sqrt(0.5)) < 1e-15


def test_single_parity_block_only_detects():
    """r = 1 gives t = 0 (Theorem 1 needs 2t parity blocks to correct t): an
    error is detected, nothing is located."""
    m, B, b = 3, 4, 2
    P = WL.gaussian_generator(m, 1, seed=0)
    cw = O.encode_vector(rng.standard_normal((m * B, b)), P, B)
    assert O.detect_decode(cw, P, B, 1e-9, 1e-7)["verdict"] == O.CLEAN
    for i in range(m + 1):
        bad = cw.copy()
        bad[i * B:(i + 1) * B] += 1.0
        res = O.detect_decode(bad, P, B, 1e-9, 1e-7)
        assert res["verdict"] == O.UNCORRECTABLE and res["located"] == []


def test_several_faulty_nodes_in_one_grid_row_are_one_error():
    """Proof of Theorem 1: more than one erroneous node in a row still counts as
    one erroneous row."""
    W = rng.standard_normal((8, 8))
    P_r, P_c = WL.vandermonde_like(4, 2), WL.vandermonde_like(4, 2)
    lay = O.CodedLayer(W, P_r, P_c, tau_detect=1e-9, tau_resid=1e-7)
    X = rng.standard_normal((8, 3))
    St = lay.forward(X)
    faults = [WL.make_fault(O.PHASE_FWD, 2, j, step=0) for j in (0, 1, 3)]
    res = lay.detect_decode(O.PHASE_FWD, lay.inject(faults, St))
    assert res["verdict"] == O.CORRECTED and res["located"] == [2]
    assert np.allclose(res["decoded"], W @ X, atol=1e-9)
    faults.append(WL.make_fault(O.PHASE_FWD, 4, 1, step=0))        # a second row -> beyond t = 1
    res = lay.detect_decode(O.PHASE_FWD, lay.inject(faults, St))
    assert res["verdict"] == O.UNCORRECTABLE


# ------------------------------------------------------------------- update
def test_update_of_worked_example_node(worked_example):
    """Update example: node (0,3) after its own update holds
    (W_00 + eta d_0 x_0^T) + 2 (W_01 + eta d_0 x_1^T)."""
    ex = worked_example
    _, _, P_r, P_c = _example(ex)
    Br, Bc, eta = 3, 2, 0.37
    W = rng.standard_normal((2 * Br, 2 * Bc))
    x = rng.standard_normal((2 * Bc, 1))
    d = rng.standard_normal((2 * Br, 1))
    lay = O.CodedLayer(W, P_r, P_c)
    lay.forward(x)
    lay.backward(d)
    lay.update(eta)
    c = ex["update_node_0_3"]
    up = lambda i, j: W[i * Br:(i + 1) * Br, j * Bc:(j + 1) * Bc] + eta * d[i * Br:(i + 1) * Br] @ x[j * Bc:(j + 1) * Bc].T
    assert np.allclose(lay.Wt[0:Br, 3 * Bc:4 * Bc], c[0] * up(0, 0) + c[1] * up(0, 1), atol=1e-13)
    assert np.allclose(lay.weights(), W + eta * d @ x.T, atol=1e-13)


@pytest.mark.parametrize("N_out,N_in,m,n,r,b,T", [(12, 8, 3, 2, 2, 3, 7), (10, 9, 4, 3, 1, 2, 5),
                                                  (8, 8, 2, 2, 4, 1, 9)])
def test_T_coded_updates_equal_encoding_of_T_plain_updates(N_out, N_in, m, n, r, b, T):
    """Check-sum invariance (start of the section on the strategy; update stage):
    W~ after T coded updates = encode(W after T plain updates), corner included."""
    P_r = WL.gaussian_generator(m, r, seed=1)
    P_c = WL.vandermonde_like(n, r, "positive")
    W = rng.standard_normal((N_out, N_in))
    lay = O.CodedLayer(W, P_r, P_c)
    Wplain = W.copy()
    for step in range(T):
        X = rng.standard_normal((N_in, b))
        D = rng.standard_normal((N_out, b))
        lay.forward(X)
        lay.backward(D)
        lay.update(0.05)
        Wplain = Wplain + 0.05 * D @ X.T          # O3 summed over the batch
    ref = O.encode(Wplain, P_r, P_c)
    assert np.max(np.abs(lay.Wt - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))
    assert np.allclose(lay.weights(), Wplain, atol=1e-12)


def test_regeneration_of_worked_example(worked_example):
    """Regeneration example: W_{1,0} = W~_{2,0} - W_{0,0}; the oracle rebuilds a
    whole corrupted block-row from the other rows."""
    ex = worked_example
    _, _, P_r, P_c = _example(ex)
    B = 3
    W = rng.standard_normal((2 * B, 2 * B))
    Wt = O.encode(W, P_r, P_c)
    c = ex["regenerate_W10"]
    assert np.allclose(W[B:, :B], c[0] * Wt[:B, :B] + c[1] * Wt[2 * B:3 * B, :B], atol=1e-13)
    bad = Wt.copy()
    bad[B:2 * B] += rng.standard_normal((B, 4 * B))
    assert np.allclose(O.regenerate_block_row(bad, 1, P_r, 2, B), Wt, atol=1e-12)


@pytest.mark.parametrize("axis", [0, 1])
@pytest.mark.parametrize("r", [1, 2, 4])
def test_regeneration_restores_any_r_blocks_of_a_codeword(axis, r):
    """Every block-column (block-row) of the coded matrix is a codeword of an
    (a + r, a) MDS code, so up to r erased blocks of a line are determined by
    the rest: regenerating any set of at most r corrupted block-rows (columns)
    must give back the encoded matrix, whatever was stored in them."""
    m, n, B = 4, 3, 5
    P_r, P_c = WL.gaussian_generator(m, r, seed=41), WL.gaussian_generator(n, r, seed=42)
    W = rng.standard_normal((m * B, n * B))
    Wt = O.encode(W, P_r, P_c)
    P, L = (P_r, m + r) if axis == 0 else (P_c, n + r)
    for k in range(1, r + 1):
        for bad in itertools.combinations(range(L), k):
            hit = Wt.copy()
            for i in bad:
                if axis == 0:
                    hit[i * B:(i + 1) * B] = rng.standard_normal((B, Wt.shape[1])) * 10
                else:
                    hit[:, i * B:(i + 1) * B] = rng.standard_normal((Wt.shape[0], B)) * 10
            assert np.allclose(O.regenerate_blocks(hit, bad, P, B, axis), Wt, atol=1e-9), (axis, bad)


def test_any_choice_of_good_blocks_regenerates_the_same_line():
    """Regeneration passage: "any" a blocks of the line that are known to be correct may be accessed
    (MDS).  Every choice of a = 4 of the good blocks rebuilds two lost blocks of a consistent line
    identically; once one of the accessed blocks carries an error of its own, the choice shows."""
    a, r, B, cols = 4, 4, 3, 5
    P = WL.vandermonde_like(a, r, "positive")
    line = O.encode_vector(rng.standard_normal((a * B, cols)), P, B)          # 8 blocks of B x cols
    lost = line.copy()
    lost[1 * B:2 * B] = 99.0
    lost[6 * B:7 * B] = -99.0
    good = [0, 2, 3, 4, 5, 7]
    for src in itertools.combinations(good, a):
        assert np.allclose(O.regenerate_blocks(lost, [1, 6], P, B, 0, sources=src), line, atol=1e-9)
    assert np.allclose(O.regenerate_blocks(lost, [1, 6], P, B), line, atol=1e-9)
    hit = lost.copy()
    hit[4 * B:5 * B] += 1.0                       # block 4 passes for good but is not
    with_it = O.regenerate_blocks(hit, [1, 6], P, B, 0, sources=(0, 2, 3, 4))
    without = O.regenerate_blocks(hit, [1, 6], P, B, 0, sources=(0, 2, 3, 5))
    assert np.allclose(without[1 * B:2 * B], line[1 * B:2 * B], atol=1e-9)
    assert not np.allclose(with_it[1 * B:2 * B], line[1 * B:2 * B], atol=1e-3)


def test_regeneration_of_a_parity_block_is_reencoding():
    """Special case with a textbook form: a lost parity block-row q is the
    encoding of the systematic ones, sum_i P[i][q] W~_i."""
    m, n, r, B = 3, 3, 2, 4
    P_r, P_c = WL.vandermonde_like(m, r), WL.vandermonde_like(n, r)
    Wt = O.encode(rng.standard_normal((m * B, n * B)), P_r, P_c)
    hit = Wt.copy()
    hit[(m + 1) * B:(m + 2) * B] = 0.0
    want = sum(P_r[i, 1] * Wt[i * B:(i + 1) * B] for i in range(m))
    got = O.regenerate_blocks(hit, [m + 1], P_r, B, 0)
    assert np.allclose(got[(m + 1) * B:(m + 2) * B], want, atol=1e-12)
    assert np.allclose(got, Wt, atol=1e-12)


def test_layer_regeneration_after_a_weight_fault_gives_clean_products():
    """Oracle layer: a weight fault at node (i, j) makes block-row i of every
    later forward product erroneous; after regenerating the located row the
    stored matrix is the clean code again."""
    N, m, r, b = 12, 3, 2, 4
    P = WL.vandermonde_like(m, r)
    lay = O.CodedLayer(rng.standard_normal((N, N)), P, P)
    clean = lay.Wt.copy()
    lay.inject([WL.make_fault(WL.PHASE_WEIGHT, 1, 2, 7)])
    assert not np.allclose(lay.Wt, clean)
    res = lay.detect_decode(O.PHASE_FWD, lay.forward(rng.standard_normal((N, b))))
    assert res["verdict"] == O.CORRECTED and list(res["located"]) == [1]
    lay.regenerate(O.PHASE_FWD, res["located"])
    assert np.allclose(lay.Wt, clean, atol=1e-10)
    assert lay.detect_decode(O.PHASE_FWD, lay.forward(rng.standard_normal((N, b))))["verdict"] == O.CLEAN


def test_relu_steps_are_the_function_and_its_derivative():
    """C1 / C2 for f = ReLU: g(f(u)) = f'(u), checked against a central difference away from 0."""
    u = rng.standard_normal(1000)
    u = u[np.abs(u) > 1e-3]
    x = O.relu(u)
    assert np.array_equal(x, np.where(u > 0, u, 0.0))
    h = 1e-6
    fprime = (O.relu(u + h) - O.relu(u - h)) / (2 * h)
    c = rng.standard_normal(u.shape)
    assert np.allclose(O.relu_backward(c, x), c * fprime, atol=1e-9)


# ------------------------------------------------------------------ geometry
def test_results_do_not_depend_on_block_pitch():
    N_out, N_in, m, n, r, b = 10, 9, 4, 3, 2, 3
    P_r, P_c = WL.vandermonde_like(m, r), WL.vandermonde_like(n, r)
    W = rng.standard_normal((N_out, N_in))
    X = rng.standard_normal((N_in, b))
    D = rng.standard_normal((N_out, b))
    a = O.CodedLayer(W, P_r, P_c, tau_detect=1e-9, tau_resid=1e-7)
    c = O.CodedLayer(W, P_r, P_c, Br=8, Bc=4, tau_detect=1e-9, tau_resid=1e-7)
    fw = [WL.make_fault(O.PHASE_FWD, 3, 1, step=2)]
    bw = [WL.make_fault(O.PHASE_BWD, 1, 4, step=2)]
    for lay in (a, c):
        lay.res_f = lay.detect_decode(O.PHASE_FWD, lay.inject(fw, lay.forward(X)))
        lay.res_b = lay.detect_decode(O.PHASE_BWD, lay.inject(bw, lay.backward(D)))
        lay.update(0.1)
        lay.inject([WL.make_fault(O.PHASE_WEIGHT, 0, 2, step=3)])
    assert a.res_f["located"] == c.res_f["located"] == [3]
    assert a.res_b["located"] == c.res_b["located"] == [4]
    assert np.allclose(a.res_f["decoded"], c.res_f["decoded"], atol=1e-10)
    assert np.allclose(a.res_b["decoded"], c.res_b["decoded"], atol=1e-10)
    assert np.allclose(a.res_f["syn_rel"], c.res_f["syn_rel"], rtol=1e-9)
    assert np.allclose(a.weights(), c.weights(), atol=1e-12)
    # last systematic block-row of N_out = 10, m = 4 has one real row (10 = 3+3+3+1)
    assert [O.logical_rows_of_block(i, N_out, m) for i in range(m + r)] == [3, 3, 3, 1, 3, 3]


# ----------------------------------------------------------------- injection
def test_counter_hash_matches_published_splitmix64_outputs():
    """First outputs of SplitMix64 from state 0 and from state 1234567 (values
    printed with the reference implementation of the generator)."""
    assert O._mix64(0) == 0xE220A8397B1DCDAF
    state, outs = 1234567, []
    for _ in range(2):
        outs.append(O._mix64(state))
        state = (state + 0x9E3779B97F4A7C15) & ((1 << 64) - 1)
    assert outs == [6457827717110365317, 3203168211198807973]
    arr = O._mix64(np.array([0, 1234567], dtype=np.uint64))
    assert [int(v) for v in arr] == [0xE220A8397B1DCDAF, 6457827717110365317]


def test_fault_key_is_this_builds_own_specification():
    """Parity unpinned: the paper only asks for independent continuous noise per erroneous element
    (Error Model 2); how (seed, step, phase, bi, bj) select a noise stream is this build's choice
    and nothing in the paper can confirm it.  The specification, stated here once: three chained
    applications of the SplitMix64 output function (pinned above), the node packed as
    phase * 2^40 + bi * 2^20 + bj.  What a noise stream selector must do is checked: the same
    tuple gives the same key, and tuples that differ in any one coordinate give different keys
    (no two of 3 x 3 x 3 x 41 x 41 tuples collide), so no two faults of a run share their noise."""
    assert O.fault_key(5000, 3, 1, 2, 7) == O.fault_key(5000, 3, 1, 2, 7)
    assert O.fault_key(5000, 3, 1, 2, 7) == O._mix64(O._mix64(O._mix64(5000) ^ 3) ^ ((1 << 40) | (2 << 20) | 7))
    keys = {O.fault_key(seed, step, phase, bi, bj)
            for seed in (0, 5000, 5007) for step in (0, 1, 199) for phase in (0, 1, 2)
            for bi in range(41) for bj in range(41)}
    assert len(keys) == 3 * 3 * 3 * 41 * 41
    # consecutive elements of two different faults do not overlap either: the streams are key + idx
    a, b = O.fault_key(5000, 0, 0, 0, 0), O.fault_key(5000, 0, 0, 0, 1)
    assert abs(a - b) > 1 << 32


def test_fault_draws_are_deterministic_and_well_distributed():
    hit, u, s = O.fault_draws(5000, 3, O.PHASE_FWD, 2, 1, 200000)
    hit2, u2, s2 = O.fault_draws(5000, 3, O.PHASE_FWD, 2, 1, 200000)
    assert np.array_equal(u, u2) and np.array_equal(s, s2) and np.array_equal(hit, hit2)
    _, u3, _ = O.fault_draws(5000, 4, O.PHASE_FWD, 2, 1, 1000)
    assert not np.array_equal(u[:1000], u3)
    assert u.min() >= 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 5e-3 and abs(u.var() - 1 / 12) < 2e-3
    assert abs(s.mean()) < 1e-2 and set(np.unique(s)) == {-1.0, 1.0}
    assert abs((hit < np.uint64(int(0.005 * 2 ** 32))).mean() - 0.005) < 1e-3
    # every u is a multiple of 2^-24
    assert np.array_equal(u * 2 ** 24, np.round(u * 2 ** 24))


def test_output_fault_law():
    """Error Model 2: additive noise on every element of the erroneous block;
    dense law = sign * U[lo, hi) * rms(clean block)."""
    m, B, b = 3, 4, 5
    out = rng.standard_normal(((m + 2) * B, b))
    f = WL.make_fault(O.PHASE_FWD, 1, 2, step=7, lo=1.0, hi=10.0)
    bad = O.inject_output(out, [f], m * B, m, B, O.PHASE_FWD)
    diff = bad - out
    blk = out[B:2 * B]
    rms = np.sqrt(np.mean(blk ** 2))
    assert np.all(diff[:B] == 0) and np.all(diff[2 * B:] == 0)
    mag = np.abs(diff[B:2 * B]) / rms
    assert mag.min() >= 1.0 - 1e-12 and mag.max() < 10.0
    signs = np.sign(diff[B:2 * B]).reshape(-1)
    assert 3 <= np.count_nonzero(signs > 0) <= signs.size - 3      # both signs occur
    # two faults on the same block both use the clean rms
    f2 = WL.make_fault(O.PHASE_FWD, 1, 0, step=7)
    both = O.inject_output(out, [f, f2], m * B, m, B, O.PHASE_FWD)
    only2 = O.inject_output(out, [f2], m * B, m, B, O.PHASE_FWD)
    assert np.allclose(both - out, (bad - out) + (only2 - out), atol=1e-12)


def test_weight_fault_laws():
    N_out, N_in, m, n, r = 8, 12, 2, 3, 2
    P_r, P_c = WL.vandermonde_like(m, r), WL.vandermonde_like(n, r)
    Wt = O.encode(rng.standard_normal((N_out, N_in)), P_r, P_c)
    f = WL.make_fault(O.PHASE_WEIGHT, 1, 4, step=1)
    bad = O.inject_weight(Wt, [f], N_out, N_in, m, n, 4, 4)
    d = bad - Wt
    assert np.count_nonzero(d) == 16 and np.all(d[4:8, 16:20] != 0)
    big = O.encode(rng.standard_normal((400, 400)), P_r[:2], P_c[:2])
    fs = WL.make_fault(O.PHASE_WEIGHT, 0, 1, step=1, lo=-5.0, hi=5.0, mode=O.MODE_SPARSE_ABS, density=0.005)
    d = O.inject_weight(big, [fs], 400, 400, 2, 2, 200, 200) - big
    nz = np.count_nonzero(d)
    assert np.count_nonzero(d[:200, 200:400]) == nz and 100 < nz < 320       # 0.005 * 40000 = 200
    assert np.abs(d).max() < 5.0


# ------------------------------------------------- verification steps (Error Model 2)
def _coded_output(a, r, B, b, seed):
    P = WL.vandermonde_like(a, r, nodes="spread")
    g = np.random.default_rng(seed)
    base = g.standard_normal((a * B, b))
    return P, O.encode_vector(base, P, B)


@pytest.mark.parametrize("n_err,verdict", [(0, O.CLEAN), (1, O.CORRECTED), (2, O.UNCORRECTABLE)])
def test_verification_with_agreement_is_the_plain_check(n_err, verdict):
    """Decentralized implementation, "Errors in Error-Detection" / "Errors in decoding" under
    Error Model 2: if all evaluators agree the algorithm moves forward -- same verdict, same
    located nodes and same repaired output as the check without verification."""
    a, r, B, b = 4, 2, 6, 3
    P, out = _coded_output(a, r, B, b, 5)
    for i in range(n_err):
        out[(1 + 2 * i) * B:(2 + 2 * i) * B] += rng.standard_normal((B, b))
    plain = O.detect_decode(out, P, B, 1e-9, 1e-6)
    ver = O.verified_detect_decode(out, P, B, 1e-9, 1e-6, evaluators=5)
    assert plain["verdict"] == verdict == ver["verdict"]
    assert plain["located"] == ver["located"]
    assert np.array_equal(plain["out"], ver["out"])


@pytest.mark.parametrize("n_err", [0, 1, 2])
@pytest.mark.parametrize("who", [0, 1, 3])
def test_any_disagreement_stops_the_step_and_leaves_the_output(n_err, who):
    """The same passages: a difference in one evaluator's consistency checks (step 1) or in its
    list of erroneous nodes (step 2) is a disagreement, whatever the state of the product and
    whichever evaluator it is; nothing is corrected then (the network is restored instead)."""
    a, r, B, b = 4, 2, 6, 3
    P, out = _coded_output(a, r, B, b, 6)
    for i in range(n_err):
        out[(2 * i) * B:(1 + 2 * i) * B] += rng.standard_normal((B, b))
    for kw in (dict(check_faults=[(who, 1, 0.25)]), dict(list_faults=[(who,)])):
        ver = O.verified_detect_decode(out, P, B, 1e-9, 1e-6, evaluators=4, **kw)
        assert ver["verdict"] == O.DISAGREE and ver["located"] == []
        assert np.array_equal(ver["out"], out)


def test_the_same_error_in_every_evaluator_is_not_a_disagreement():
    """Comparing evaluations only finds errors that differ between evaluators: identical
    corruption of every evaluation passes step 1 (the lists, taken from the output itself in
    this model, agree as well)."""
    a, r, B, b = 3, 2, 4, 2
    P, out = _coded_output(a, r, B, b, 7)
    ver = O.verified_detect_decode(out, P, B, 1e-9, 1e-6, evaluators=3,
                                   check_faults=[(v, 0, 0.5) for v in range(3)])
    assert ver["verdict"] == O.CLEAN
