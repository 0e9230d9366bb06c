"""Plain float64 oracle of the CodeNet coded layer step (arXiv 1903.01042).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the
benchmark's CPU-baseline leg; never by the product path.  It shares no code
with the HIP library.

Everything is written in the paper's orientation: activations are column
blocks, X is (N_in x b), S is (N_out x b), Delta is (N_out x b), C is
(N_in x b); a batch of b columns is b independent codewords that share one
error support (the paper has b = 1).  Blocks are addressed as in Section
"Some Notations": W is an m x n grid of blocks W_{i,j}; the coded grid has
m + r_r block-rows and n + r_c block-columns.

Block geometry.  A dimension of N entries split in `parts` "equal parts" uses
blocks of B0 = ceil(N / parts) entries, the last ones zero padded (the paper
assumes divisibility; zero padding is this build's reading).  A caller may
ask for a larger block pitch B >= B0 (extra zero rows at the end of every
block); every result below is independent of that pitch, which a test checks.

Pins (tests/test_oracle_*.py): the paper's worked example for m = n = 2, t = 1
(values printed in the sections on pre-processing, feedforward, backpropagation,
update and regeneration), H G^T = 0, brute-force MDS / spark enumeration,
element-wise triple-loop evaluation of the Kronecker encoding, decoded output
equal to the textbook product, T coded updates equal to encode(T plain
updates), exhaustive enumeration of error supports on tiny grids, and for the
verification steps of Error Model 2: agreement reproduces the plain check, any
planted difference in any evaluator gives DISAGREE with the output untouched;
the relative residual of detect_decode against hand-computed cases (one and two
erroneous blocks, one and two positions) and its tie rule on exact ties.
Parity unpinned by the paper (fixed by this build's readings, documented in
the design notes): the relative thresholds tau_detect / tau_resid, the noise
law of the fault injector, the packing of (seed, step, phase, bi, bj) into the
key of its counter hash (fault_key; the hash itself is pinned to the published
SplitMix64 outputs), zero padding.
"""
import itertools

import numpy as np

CLEAN, CORRECTED, UNCORRECTABLE, DISAGREE = 0, 1, 2, 3
PHASE_FWD, PHASE_BWD, PHASE_WEIGHT = 0, 1, 2
MODE_DENSE_REL, MODE_SPARSE_ABS = 0, 1


# --------------------------------------------------------------------------
# Code construction (Section "Some Notations": systematic (b, a) MDS generator;
# Appendix "Error Detection and Correction Mechanism": annihilating matrix H)
# --------------------------------------------------------------------------
def _parity_part(P):
    """P as an a x r float64 matrix (r may be 0: no parity blocks)."""
    P = np.asarray(P, dtype=np.float64)
    a = P.shape[0]
    return P.reshape(a, -1) if P.size else np.zeros((a, 0))


def generator(P):
    """G = [I | P], the a x (a + r) generator of a systematic code."""
    P = _parity_part(P)
    return np.hstack([np.eye(P.shape[0]), P])


def parity_check(P):
    """H = [P^T | -I], r x (a + r), full rank, H G^T = 0.

    Any full-rank annihilator is allowed by the paper; with this one the k-th
    syndrome is "parity recomputed from the systematic blocks minus the parity
    that was actually produced".
    """
    P = _parity_part(P)
    return np.hstack([P.T, -np.eye(P.shape[1])])


def is_mds(P, tol=1e-9):
    """Definition check: any a of the a + r columns of G are independent."""
    G = generator(P)
    a, L = G.shape
    for cols in itertools.combinations(range(L), a):
        if abs(np.linalg.det(G[:, cols])) <= tol:
            return False
    return True


def spark(H, tol=1e-9):
    """Smallest number of linearly dependent columns of H (brute force)."""
    r, L = H.shape
    for k in range(1, L + 1):
        for cols in itertools.combinations(range(L), k):
            if np.linalg.matrix_rank(H[:, cols], tol=tol) < k:
                return k
    return L + 1


# --------------------------------------------------------------------------
# Block geometry helpers
# --------------------------------------------------------------------------
def block_size(N, parts):
    return -(-N // parts)


def logical_index(N, parts, B=None):
    """Position of logical entry g in the block-padded dimension of pitch B."""
    B0 = block_size(N, parts)
    B = B0 if B is None else B
    assert B >= B0
    g = np.arange(N)
    return (g // B0) * B + (g % B0)


def pad_blocks(V, parts, B=None):
    """Zero pad the rows of V (N x anything) into `parts` blocks of pitch B."""
    V = np.asarray(V, dtype=np.float64)
    N = V.shape[0]
    B0 = block_size(N, parts)
    B = B0 if B is None else B
    out = np.zeros((parts * B,) + V.shape[1:], dtype=np.float64)
    out[logical_index(N, parts, B)] = V
    return out


def unpad_blocks(Vp, N, parts, B=None):
    return np.asarray(Vp)[logical_index(N, parts, B)]


def logical_rows_of_block(i, N, parts):
    """How many entries of block i are real (not zero padding).

    Systematic block i < parts holds entries [i*B0, (i+1)*B0) of the N logical
    ones; a parity block (i >= parts) is a combination of full blocks and has
    B0 real entries.
    """
    B0 = block_size(N, parts)
    if i >= parts:
        return B0
    return int(min(B0, max(0, N - i * B0)))


# --------------------------------------------------------------------------
# Pre-processing: one-time encoding (Claim 1; Appendix, overview of the coding
# technique):  W~ = (G_r^T (x) I) W (G_c (x) I)
# --------------------------------------------------------------------------
def encode(W, P_r, P_c, Br=None, Bc=None, store_corner=True):
    W = np.asarray(W, dtype=np.float64)
    N_out, N_in = W.shape
    m, n = np.shape(P_r)[0], np.shape(P_c)[0]
    Br = block_size(N_out, m) if Br is None else Br
    Bc = block_size(N_in, n) if Bc is None else Bc
    Wp = pad_blocks(pad_blocks(W, m, Br).T, n, Bc).T          # (m Br) x (n Bc)
    G_r, G_c = generator(P_r), generator(P_c)
    # The Kronecker factors act on whole blocks: coded block (i, j) is
    # sum_{i', j'} G_r[i', i] G_c[j', j] W_{i', j'}.
    blocks = Wp.reshape(m, Br, n, Bc)
    Wt = np.einsum("ai,bj,apbq->ipjq", G_r, G_c, blocks, optimize=True)
    Wt = np.ascontiguousarray(Wt).reshape(G_r.shape[1] * Br, G_c.shape[1] * Bc)
    if not store_corner:
        Wt[m * Br:, n * Bc:] = 0.0     # the paper keeps no node there ("x")
    return Wt


def encode_vector(Vp, P, B):
    """Additional encoding step (Step 4 of the feedforward / backpropagation
    stage): [v; v~] = (G^T (x) I_B) v for a block-padded column block v."""
    G = generator(P)
    a, L = G.shape
    b = Vp.shape[1]
    return (G.T @ Vp.reshape(a, B * b)).reshape(L * B, b)


# --------------------------------------------------------------------------
# Coded products.  Each active node multiplies its own block; partial results
# are summed along the grid row (O1) or grid column (O2).
# --------------------------------------------------------------------------
def forward(Wt, Xp, m, n, r_r, Br, Bc):
    """O1 on active nodes (i < m + r_r, j < n):  s~_i = sum_j W~_{i,j} x_j."""
    b = Xp.shape[1]
    out = np.zeros(((m + r_r) * Br, b))
    for i in range(m + r_r):
        for j in range(n):
            node = Wt[i * Br:(i + 1) * Br, j * Bc:(j + 1) * Bc]
            out[i * Br:(i + 1) * Br] += node @ Xp[j * Bc:(j + 1) * Bc]
    return out


def backward(Wt, Dp, m, n, r_c, Br, Bc):
    """O2 on active nodes (i < m, j < n + r_c):  c~_j^T = sum_i d_i^T W~_{i,j}."""
    b = Dp.shape[1]
    out = np.zeros(((n + r_c) * Bc, b))
    for j in range(n + r_c):
        for i in range(m):
            node = Wt[i * Br:(i + 1) * Br, j * Bc:(j + 1) * Bc]
            out[j * Bc:(j + 1) * Bc] += node.T @ Dp[i * Br:(i + 1) * Br]
    return out


# --------------------------------------------------------------------------
# Detection, location, decoding (General Error-Detection Method; Lemma 2 and
# the Decoding Algorithm of the appendix)
# --------------------------------------------------------------------------
def syndromes(out, P, B):
    """out^ = (H (x) I_B) out, returned as r blocks stacked: (r B) x b."""
    H = parity_check(P)
    r, L = H.shape
    b = out.shape[1]
    return (H @ np.asarray(out).reshape(L, B * b)).reshape(r * B, b)


def detect_decode(out, P, B, tau_detect, tau_resid):
    """Check one coded output (L = a + r blocks of B x b) and repair it.

    Returns dict(verdict, located, out, syn_rel, resid_rel).

    1. out^ = (H (x) I) out.  The paper's test "out^ = 0" is relaxed for
       floating point to  max_k ||out^_k||_F / ref_k <= tau_detect  with
       ref_k = sqrt(sum_i H[k,i]^2 ||out_i||_F^2)  (0/0 read as 0).
    2. Otherwise look for e with at most t = floor(r/2) non-zero blocks and
       (H (x) I) e = out^: supports are tried by increasing cardinality; for
       one cardinality every support A is solved in the least-squares sense
       (the same r x |A| system for all B*b positions) and the one with the
       smallest relative residual wins (first in lexicographic order on a
       tie); it is accepted if that residual is <= tau_resid.  For <= t true
       errors the support with zero residual is unique (Spark(H) = 2t + 1).
    3. Accepted: out_i -= e_i on the support, CORRECTED.  Else UNCORRECTABLE
       (the paper then reverts to the last checkpoint) and out is untouched.
    """
    out = np.array(out, dtype=np.float64)
    H = parity_check(P)
    r, L = H.shape
    t = r // 2
    b = out.shape[1]
    blocks = np.stack([out[i * B:(i + 1) * B].reshape(-1) for i in range(L)])   # L x (B b)
    syn = H @ blocks                                                   # r x (B b)
    blk_sq = np.sum(blocks * blocks, axis=1)
    ref = np.sqrt((H * H) @ blk_sq)
    syn_norm = np.sqrt(np.sum(syn * syn, axis=1))
    syn_rel = np.where(ref > 0, syn_norm / np.where(ref > 0, ref, 1.0), 0.0)
    res = dict(verdict=CLEAN, located=[], out=out, syn_rel=syn_rel, resid_rel=0.0)
    if r == 0 or np.max(syn_rel) <= tau_detect:
        return res
    syn_tot = np.sqrt(np.sum(syn * syn))
    for k in range(1, t + 1):
        best = None
        for A in itertools.combinations(range(L), k):
            HA = H[:, A]
            E, *_ = np.linalg.lstsq(HA, syn, rcond=None)              # k x (B b)
            resid = np.sqrt(np.sum((HA @ E - syn) ** 2)) / syn_tot
            if best is None or resid < best[0]:
                best = (resid, A, E)
        if best is not None and best[0] <= tau_resid:
            resid, A, E = best
            for idx, i in enumerate(A):
                out[i * B:(i + 1) * B] -= E[idx].reshape(B, b)
            res.update(verdict=CORRECTED, located=list(A), out=out, resid_rel=resid)
            return res
        if best is not None:
            res["resid_rel"] = best[0]
    res["verdict"] = UNCORRECTABLE
    return res


# --------------------------------------------------------------------------
# Verification steps of Error Model 2 (decentralized implementation:
# "Errors in Error-Detection" and "Errors in decoding")
# --------------------------------------------------------------------------
def verified_detect_decode(out, P, B, tau_detect, tau_resid, evaluators=2,
                           check_faults=(), list_faults=()):
    """The check of one coded output when the checking itself is error-prone.

    Every one of `evaluators` evaluators works out the r consistency checks
    (H (x) I) out and the list of erroneous nodes for itself.
    Verification step 1: the evaluations of the checks are exchanged and
    compared; verification step 2: the lists of erroneous nodes (with the
    verdict they come with) are exchanged and compared.  The comparisons are
    exact and are themselves taken to be error-free.  Any disagreement gives
    the verdict DISAGREE and leaves `out` untouched (the paper then restores
    the network from the last checkpoint); full agreement gives exactly what
    detect_decode gives.

    Planted errors, for tests of the two steps:
      check_faults: (evaluator, k, scale) -- that evaluator's check k becomes
                    (1 + scale) * check + scale;
      list_faults:  (evaluator,) -- that evaluator's first erroneous node is
                    replaced by the next block (a CORRECTED verdict), or its
                    verdict flips between CLEAN and UNCORRECTABLE.
    """
    out = np.array(out, dtype=np.float64)
    H = parity_check(P)
    r, L = H.shape
    b = out.shape[1]
    blocks = np.stack([out[i * B:(i + 1) * B].reshape(-1) for i in range(L)])
    disagree = dict(verdict=DISAGREE, located=[], out=out.copy(),
                    syn_rel=np.zeros(r), resid_rel=0.0)
    # step 1: every evaluator's evaluation of the r checks
    evaluations = []
    for v in range(evaluators):
        syn = H @ blocks
        for who, k, scale in check_faults:
            if who == v:
                syn[k] = (1.0 + scale) * syn[k] + scale
        evaluations.append(syn)
    for syn in evaluations[1:]:
        if not np.array_equal(syn, evaluations[0]):
            return disagree
    # step 2: every evaluator's verdict and list of erroneous nodes
    lists = []
    result = None
    for v in range(evaluators):
        res = detect_decode(out, P, B, tau_detect, tau_resid)
        verdict, located = res["verdict"], list(res["located"])
        for (who,) in list_faults:
            if who == v:
                if verdict == CORRECTED:
                    located[0] = (located[0] + 1) % L
                else:
                    verdict = UNCORRECTABLE if verdict == CLEAN else CLEAN
        lists.append((verdict, tuple(located)))
        if v == 0:
            result = res
    for entry in lists[1:]:
        if entry != lists[0]:
            return disagree
    return result


# --------------------------------------------------------------------------
# Coded update (O3 with the three block rules; the corner is one more block
# updated by the same rule when it is stored)
# --------------------------------------------------------------------------
def update(Wt, Dt, Xt, eta, m, n, Br, Bc, store_corner=True):
    """W~_{i,j} += eta * d~_i x~_j^T on every stored block."""
    Wn = Wt + eta * (Dt @ Xt.T)
    if not store_corner:
        Wn[m * Br:, n * Bc:] = 0.0
    return Wn


def regenerate_blocks(Wt, bad, P, B, axis=0, sources=None):
    """Regeneration: rebuild every stored block of the block-rows (axis 0) or
    block-columns (axis 1) listed in `bad` from other blocks of the same grid
    column (row).  The paper accesses "any" a blocks of the line that are known
    to be correct (a = number of systematic blocks; any a of them determine the
    line, MDS).  `sources` names the blocks that are accessed; by default all
    good ones are, solved in the least-squares sense, which is the same thing
    whenever the accessed blocks are consistent.  (They are not when a block
    that passes for good carries an undetected error of its own: the rebuilt
    block then depends on which blocks were accessed, and the error shows at
    the next product that uses it.)"""
    if axis == 1:
        return regenerate_blocks(Wt.T, bad, P, B, 0, sources).T
    G = generator(P)                         # a x L
    L = G.shape[1]
    bad = sorted(set(int(i) for i in bad))
    good = [i for i in range(L) if i not in bad] if sources is None else [int(i) for i in sources]
    assert not set(good) & set(bad) and len(good) >= G.shape[0]
    Wn = Wt.copy()
    cols = Wt.shape[1]
    stack = np.stack([Wt[i * B:(i + 1) * B].reshape(-1) for i in good])     # |good| x (B cols)
    sys, *_ = np.linalg.lstsq(G[:, good].T, stack, rcond=None)              # a x (B cols)
    for i in bad:
        Wn[i * B:(i + 1) * B] = (G[:, i] @ sys).reshape(B, cols)
    return Wn


def regenerate_block_row(Wt, i_bad, P_r, m, Br):
    """One block-row, as in the paper's worked example."""
    return regenerate_blocks(Wt, [i_bad], P_r, Br, 0)


# --------------------------------------------------------------------------
# Elementwise primary steps (C1: x^{l+1} = f(s^l); C2: delta^{l-1} = g(x^l) (.) c^l,
# with g chosen such that g(f(u)) = f'(u)), for f = ReLU
# --------------------------------------------------------------------------
def relu(s):
    return np.maximum(s, 0.0)


def relu_backward(c, x):
    """g(x) (.) c with g(x) = 1[x > 0]: for x = relu(u), g(x) = relu'(u)."""
    return np.where(x > 0, c, 0.0)


# --------------------------------------------------------------------------
# Soft-error injection (Error Model 2: additive, every element of the
# erroneous block drawn independently from a continuous law; the experiment's
# sparse additive law is mode 1)
# --------------------------------------------------------------------------
_M64 = (1 << 64) - 1


def _mix64(x):
    """SplitMix64 output function (Steele, Lea, Flood 2014): add the golden
    gamma, two xor-shift-multiply rounds, a final xor-shift.  Works on a Python
    int or on a numpy uint64 array (arithmetic modulo 2^64)."""
    if isinstance(x, np.ndarray):
        with np.errstate(over="ignore"):
            z = x + np.uint64(0x9E3779B97F4A7C15)
            z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
            z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
            return z ^ (z >> np.uint64(31))
    z = (x + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def fault_key(seed, step, phase, bi, bj):
    k = _mix64(seed & _M64)
    k = _mix64(k ^ (step & _M64))
    return _mix64(k ^ ((phase << 40) | (bi << 20) | bj))


def fault_draws(seed, step, phase, bi, bj, count):
    """Per-element draws: (hit32, u01, sign).  Element idx uses the 64-bit word
    z = mix(key + idx): bits 0..31 -> hit32, bits 32..55 -> u01 = k / 2^24,
    bit 63 -> sign (+1 if clear)."""
    key = fault_key(seed, step, phase, bi, bj)
    with np.errstate(over="ignore"):
        z = _mix64(np.uint64(key) + np.arange(count, dtype=np.uint64))
    hit = z & np.uint64(0xFFFFFFFF)
    u01 = ((z >> np.uint64(32)) & np.uint64(0xFFFFFF)).astype(np.float64) / float(1 << 24)
    sgn = np.where((z >> np.uint64(63)) != 0, -1.0, 1.0)
    return hit, u01, sgn


def fault_values(fault, count, rms):
    """Additive noise for `count` payload elements of one fault.

    mode 0 (dense, relative): sign * (lo + (hi - lo) u01) * rms on every element.
    mode 1 (sparse, absolute): lo + (hi - lo) u01 where hit32 < floor(density 2^32).
    """
    hit, u01, sgn = fault_draws(fault["seed"], fault["step"], fault["phase"],
                                fault["bi"], fault["bj"], count)
    mag = fault["lo"] + (fault["hi"] - fault["lo"]) * u01
    if fault.get("mode", MODE_DENSE_REL) == MODE_DENSE_REL:
        return sgn * mag * rms
    thresh = int(np.floor(fault["density"] * float(1 << 32)))
    return np.where(hit < np.uint64(thresh), mag, 0.0)


def inject_output(out, faults, N, parts, B, phase):
    """Faults of one product.  A fault at node (bi, bj) lands in the summed
    output of its grid row (forward: block-row bi) or grid column (backward:
    block-column bj); the other coordinate only seeds the noise.  rms is taken
    over the logical payload of the still clean target block; element index is
    rho * b + beta over the logical rows rho of the block."""
    out = np.array(out, dtype=np.float64)
    clean = out.copy()
    b = out.shape[1]
    for f in faults:
        assert f["phase"] == phase
        tgt = f["bi"] if phase == PHASE_FWD else f["bj"]
        rows = logical_rows_of_block(tgt, N, parts)
        if rows == 0:
            continue
        payload = clean[tgt * B: tgt * B + rows]
        rms = float(np.sqrt(np.mean(payload * payload)))
        vals = fault_values(f, rows * b, rms).reshape(rows, b)
        out[tgt * B: tgt * B + rows] += vals
    return out


def inject_weight(Wt, faults, N_out, N_in, m, n, Br, Bc):
    """Update-stage faults: the stored block W~_{bi,bj} is corrupted.  Element
    index is rho * Bc0 + kappa over the logical payload (Bc0 = unpadded block
    width)."""
    Wt = np.array(Wt, dtype=np.float64)
    clean = Wt.copy()
    Bc0 = block_size(N_in, n)
    for f in faults:
        assert f["phase"] == PHASE_WEIGHT
        bi, bj = f["bi"], f["bj"]
        rows = logical_rows_of_block(bi, N_out, m)
        cols = logical_rows_of_block(bj, N_in, n)
        if rows == 0 or cols == 0:
            continue
        payload = clean[bi * Br: bi * Br + rows, bj * Bc: bj * Bc + cols]
        rms = float(np.sqrt(np.mean(payload * payload)))
        idx = (np.arange(rows)[:, None] * Bc0 + np.arange(cols)[None, :]).reshape(-1)
        vals_full = fault_values(f, rows * Bc0, rms)
        Wt[bi * Br: bi * Br + rows, bj * Bc: bj * Bc + cols] += vals_full[idx].reshape(rows, cols)
    return Wt


# --------------------------------------------------------------------------
# One coded layer (state + the step's calls in the paper's order)
# --------------------------------------------------------------------------
class CodedLayer:
    """One layer's coded state, driven in the order of the decentralized
    algorithm: forward product -> check -> (vector encoding) ... backward
    product -> check -> (vector encoding) ... update."""

    def __init__(self, W, P_r, P_c, Br=None, Bc=None, tau_detect=1e-3,
                 tau_resid=2e-3, store_corner=True):
        W = np.asarray(W, dtype=np.float64)
        self.N_out, self.N_in = W.shape
        self.P_r = _parity_part(P_r)
        self.P_c = _parity_part(P_c)
        self.m, self.r_r = self.P_r.shape
        self.n, self.r_c = self.P_c.shape
        self.Br = block_size(self.N_out, self.m) if Br is None else Br
        self.Bc = block_size(self.N_in, self.n) if Bc is None else Bc
        self.tau_detect, self.tau_resid = tau_detect, tau_resid
        self.store_corner = store_corner
        self.Wt = encode(W, self.P_r, self.P_c, self.Br, self.Bc, store_corner)
        self.Xt = None
        self.Dt = None

    # forward product; caches [x; x~] for the update
    def forward(self, X):
        Xp = pad_blocks(X, self.n, self.Bc)
        self.Xt = encode_vector(Xp, self.P_c, self.Bc)
        return forward(self.Wt, Xp, self.m, self.n, self.r_r, self.Br, self.Bc)

    def backward(self, D):
        Dp = pad_blocks(D, self.m, self.Br)
        self.Dt = encode_vector(Dp, self.P_r, self.Br)
        return backward(self.Wt, Dp, self.m, self.n, self.r_c, self.Br, self.Bc)

    def inject(self, faults, coded_out=None):
        if not faults:
            return coded_out
        phase = faults[0]["phase"]
        if phase == PHASE_FWD:
            return inject_output(coded_out, faults, self.N_out, self.m, self.Br, phase)
        if phase == PHASE_BWD:
            return inject_output(coded_out, faults, self.N_in, self.n, self.Bc, phase)
        self.Wt = inject_weight(self.Wt, faults, self.N_out, self.N_in,
                                self.m, self.n, self.Br, self.Bc)
        return None

    def detect_decode(self, phase, coded_out):
        if phase == PHASE_FWD:
            res = detect_decode(coded_out, self.P_r, self.Br, self.tau_detect, self.tau_resid)
            res["decoded"] = unpad_blocks(res["out"][: self.m * self.Br], self.N_out, self.m, self.Br)
        else:
            res = detect_decode(coded_out, self.P_c, self.Bc, self.tau_detect, self.tau_resid)
            res["decoded"] = unpad_blocks(res["out"][: self.n * self.Bc], self.N_in, self.n, self.Bc)
        return res

    def verified_detect_decode(self, phase, coded_out, evaluators=2, check_faults=(), list_faults=()):
        P, B, N, a = ((self.P_r, self.Br, self.N_out, self.m) if phase == PHASE_FWD
                      else (self.P_c, self.Bc, self.N_in, self.n))
        res = verified_detect_decode(coded_out, P, B, self.tau_detect, self.tau_resid,
                                     evaluators, check_faults, list_faults)
        res["decoded"] = unpad_blocks(res["out"][: a * B], N, a, B)
        return res

    def regenerate(self, phase, located, sources=None):
        """Rebuild the stored blocks at the nodes located in `phase`'s product:
        block-rows for the forward product, block-columns for the backward one
        (sources: the blocks of each line that are accessed, see regenerate_blocks)."""
        if len(located) == 0:
            return
        if phase == PHASE_FWD:
            self.Wt = regenerate_blocks(self.Wt, located, self.P_r, self.Br, 0, sources)
        else:
            self.Wt = regenerate_blocks(self.Wt, located, self.P_c, self.Bc, 1, sources)

    def update(self, eta):
        self.Wt = update(self.Wt, self.Dt, self.Xt, eta, self.m, self.n,
                         self.Br, self.Bc, self.store_corner)

    def weights(self):
        sys = self.Wt[: self.m * self.Br, : self.n * self.Bc]
        return unpad_blocks(unpad_blocks(sys, self.N_out, self.m, self.Br).T,
                            self.N_in, self.n, self.Bc).T
