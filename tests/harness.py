"""Drives the HIP library and the float64 oracle side by side on the same seeded
inputs and compares them.  Test infrastructure only."""
import numpy as np

from oracle import codenet_oracle as O
from paper_1903_01042_amd import workloads as WL

# Bounds on values.  TOL is the whole-tensor relative Frobenius error that the task states.  A
# whole-tensor norm alone is blind to a wrong row or a stale tile whose error drowns in the rest,
# so every comparison also holds each block (node output block, stored block W~_{i,j}) to its own
# relative Frobenius bound, and every element to a multiple of its block's rms.  Set from what the
# GPU tests measure (largest values over all tests, printed at the end of every run):
#   BLOCK_TOL  f32: largest block error measured 4.2e-6 (fp32 accumulation of up to 16384
#              products, ~ sqrt(K) 2^-24); bound 2e-5.  bf16: both factors rounded to 8 significant
#              bits give 2.2e-3 .. 3.4e-3 per block, 4.2e-3 at the most (small, ragged blocks);
#              bound 6.6e-3 = 3 x the typical and 1.6 x the largest value.
#   ELEM_C     largest element error measured: 2.2e-2 of the block's rms in bf16, 3.7e-5 in f32
#              (the variance of an element's error follows the products that went into it, so
#              the tail is heavier than a normal law's); bound 6 x BLOCK_TOL x rms: 4.0e-2 / 1.2e-4.
# A block that the check has corrected, or that was regenerated, carries the rounding noise of the
# blocks it was rebuilt from: its two bounds are scaled by that amplification (computed from the
# code's coefficients where it applies, see corrected_amp / regenerated_amp).
TOL = {"f32": 1e-4, "bf16": 2e-2}          # relative Frobenius error on values
BLOCK_TOL = {"f32": 2e-5, "bf16": 6.6e-3}
ELEM_C = 6.0
MARGIN = 5.0                               # every threshold decision must clear its tau by this factor


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a))


def to_np(t):
    return t.detach().cpu().numpy().astype(np.float64)


SMALL = 64       # a block of fewer nonzero entries has no stable rms of its own


def block_errors(got, ref, row_edges, col_edges=None):
    """Per block: (relative Frobenius error, largest |difference| / rms of the reference block's
    nonzero entries, number of nonzero entries).  Blocks are the rectangles between consecutive row
    (and column) edges; a block whose reference is all zero, or has fewer than SMALL nonzero
    entries, is measured against the rms of the whole reference if that is larger."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if col_edges is None:
        col_edges = [0, ref.shape[1]]
    nz_all = np.count_nonzero(ref)
    rms_all = np.sqrt(np.sum(ref * ref) / nz_all) if nz_all else 1.0
    nr, nc = len(row_edges) - 1, len(col_edges) - 1
    fro, elem, count = np.zeros((nr, nc)), np.zeros((nr, nc)), np.ones((nr, nc))
    for i in range(nr):
        for j in range(nc):
            g = got[row_edges[i]:row_edges[i + 1], col_edges[j]:col_edges[j + 1]]
            r = ref[row_edges[i]:row_edges[i + 1], col_edges[j]:col_edges[j + 1]]
            if r.size == 0:
                continue
            d = g - r
            ss, nz = np.sum(r * r), np.count_nonzero(r)
            count[i, j] = max(nz, 1)
            if nz == 0:
                fro[i, j] = np.sqrt(np.sum(d * d) / d.size) / rms_all
                elem[i, j] = np.max(np.abs(d)) / rms_all
            else:
                rms = np.sqrt(ss / nz)
                if nz < SMALL:
                    rms = max(rms, rms_all)
                fro[i, j] = np.sqrt(np.sum(d * d) / nz) / rms
                elem[i, j] = np.max(np.abs(d)) / rms
    return fro, elem, count


def pitch_edges(nblocks, B):
    return [i * B for i in range(nblocks + 1)]


def logical_edges(N, parts):
    B0 = -(-N // parts)
    return [min(i * B0, N) for i in range(parts + 1)]


def corrected_amp(P, located, blk_rms):
    """Noise amplification of the blocks that the check has corrected.  With out = true + noise +
    error, the estimate of the error on the support A is pinv(H_A) H out, so the repaired block i
    carries sum over j outside A of (pinv(H_A) H)[i, j] noise_j in place of its own noise."""
    H = O.parity_check(P)
    A = list(located)
    M = np.linalg.pinv(H[:, A]) @ H
    rest = [j for j in range(H.shape[1]) if j not in A]
    amp = {}
    for row, i in enumerate(A):
        own = blk_rms[i] if blk_rms[i] > 0 else 1.0
        amp[i] = 1.0 + float(np.sqrt(np.sum((M[row, rest] * blk_rms[rest]) ** 2))) / own
    return amp


def library_sources(P, bad):
    """The a blocks of a line that the library accesses to regenerate the blocks `bad` (the paper
    leaves the choice open: any a good ones): the good systematic blocks and, for ks lost
    systematic ones, the first ks good parity blocks."""
    a, r = np.shape(P)[0], (np.shape(P)[1] if np.ndim(P) == 2 else 0)
    bad = sorted(set(bad))
    ks = sum(1 for i in bad if i < a)
    return [i for i in range(a) if i not in bad] + [a + q for q in range(r) if a + q not in bad][:ks]


def regenerated_amp(P, bad, blk_rms):
    """The same for regenerated blocks: block i is the combination sum_j c_j block_j of the source
    blocks S that are accessed, G[:, S] c = G[:, i]."""
    G = O.generator(P)
    bad = sorted(set(bad))
    S = library_sources(P, bad)
    amp = {}
    for i in bad:
        c = np.linalg.solve(G[:, S], G[:, i])
        own = blk_rms[i] if blk_rms[i] > 0 else 1.0
        amp[i] = 1.0 + float(np.sqrt(np.sum((c * blk_rms[S]) ** 2))) / own
    return amp


class Stats:
    """Largest errors seen, per kind of comparison (printed by the tests that set the bounds)."""
    worst = {}

    @classmethod
    def note(cls, what, dtype, whole, blk, elem):
        w = cls.worst.setdefault((what, dtype), [0.0, 0.0, 0.0])
        w[0], w[1], w[2] = max(w[0], whole), max(w[1], blk), max(w[2], elem)

    @classmethod
    def lines(cls):
        return ["%-28s %-4s whole %.2e  block %.2e  element/rms %.2e" % (k[0], k[1], v[0], v[1], v[2])
                for k, v in sorted(cls.worst.items())]


def assert_close(got, ref, dtype, what, row_edges, col_edges=None, row_amp=None, col_amp=None, tol=None,
                 blk_tol=None, elem_scale=1.0):
    """The three bounds on one tensor.  row_amp / col_amp: {block index: factor} for the block-rows
    (block-columns) whose bounds are scaled (corrected or regenerated blocks).  elem_scale widens the
    per-element bound only (an elementwise multiplier applied after the product scales each
    element's error by its own factor, the block's rms by the factors' rms)."""
    tol = TOL[dtype] if tol is None else tol
    blk_tol = BLOCK_TOL[dtype] if blk_tol is None else blk_tol
    whole = rel_fro(got, ref)
    assert whole <= tol, "%s differs: rel %.3e" % (what, whole)
    fro, elem, count = block_errors(got, ref, row_edges, col_edges)
    # the relative error of a block of n entries scatters by about 1 / sqrt(2 n) around its mean:
    # small blocks get that allowance (four standard deviations), large ones are unaffected
    scale = 1.0 + 4.0 / np.sqrt(2.0 * count)
    for i, f in (row_amp or {}).items():
        scale[i, :] *= f
    for j, f in (col_amp or {}).items():
        scale[:, j] *= f
    bad = np.argwhere(fro > blk_tol * scale)
    assert bad.size == 0, "%s: block %s differs: rel %.3e (bound %.3e)" % (
        what, tuple(bad[0]), fro[tuple(bad[0])], blk_tol * scale[tuple(bad[0])])
    bad = np.argwhere(elem > ELEM_C * blk_tol * scale * elem_scale)
    assert bad.size == 0, "%s: an element of block %s is off by %.3e rms (bound %.3e)" % (
        what, tuple(bad[0]), elem[tuple(bad[0])], ELEM_C * blk_tol * scale[tuple(bad[0])] * elem_scale)
    Stats.note(what, dtype, whole, float(np.max(fro / scale)), float(np.max(elem / scale)) / elem_scale)
    return whole


class Pair:
    """One layer on the GPU and in the oracle."""

    def __init__(self, W, P_r, P_c, dtype="f32", max_batch=16, tau_detect=1e-3, tau_resid=2e-3):
        import torch
        from paper_1903_01042_amd import binding as B
        self.B = B
        self.dtype = dtype
        self.tol = TOL[dtype]
        self.tau_detect, self.tau_resid = tau_detect, tau_resid
        self.dev = torch.device("cuda:0")
        Wd = torch.from_numpy(np.ascontiguousarray(W, dtype=np.float32)).to(self.dev)
        self.gpu = B.CodedLayer(Wd, P_r, P_c, dtype=B.BF16_F32ACC if dtype == "bf16" else B.F32,
                                max_batch=max_batch, tau_detect=tau_detect, tau_resid=tau_resid)
        self.ora = O.CodedLayer(np.asarray(W, dtype=np.float32), P_r, P_c, Br=self.gpu.B_r, Bc=self.gpu.B_c,
                                tau_detect=tau_detect, tau_resid=tau_resid)
        self.report = self.gpu.new_report()
        self.log = []
        # block-rows / block-columns of the stored matrix that were regenerated in the bf16 mode: after
        # updates with bf16 operands the stored parity follows the systematic part only to bf16
        # accuracy, and a rebuilt line keeps the (amplified) difference for the rest of the run
        self.w_row_amp, self.w_col_amp = {}, {}
        self.blk_scale = 1.0        # widens the per-block and per-element bounds (independent trajectories)

    def dev_tensor(self, a):
        import torch
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.dev)

    def check_weights(self, tol=None, blk_tol=None, row_amp=None, col_amp=None):
        """The stored coded matrix against the oracle's: whole tensor, every stored block W~_{i,j},
        every element.  tol: one number for the whole-tensor and the per-block bound (set-up checks
        that ask for more than the product's tolerance)."""
        ora = self.ora
        return assert_close(to_np(self.gpu.export_coded()), ora.Wt, self.dtype, "coded weights",
                            pitch_edges(ora.m + ora.r_r, ora.Br), pitch_edges(ora.n + ora.r_c, ora.Bc),
                            row_amp=self.w_row_amp if row_amp is None else row_amp,
                            col_amp=self.w_col_amp if col_amp is None else col_amp,
                            tol=tol, blk_tol=blk_tol if blk_tol else (tol if tol else BLOCK_TOL[self.dtype] * self.blk_scale))

    def _cmp(self, got, ref, what, row_edges, **kw):
        return assert_close(got, ref, self.dtype, what, row_edges, blk_tol=BLOCK_TOL[self.dtype] * self.blk_scale, **kw)

    def _weight_amp(self, phase):
        """Bound scaling of a product's output blocks that stems from regenerated lines of the stored
        matrix (bf16 mode, see w_row_amp): output block i of the forward product sums the blocks
        W~_{i,j} x_j over the base columns j, the backward one W~_{i,j}^T delta_i over the base rows i;
        a term's noise is scaled by its block's factor."""
        o = self.ora
        f = lambda d, k: d.get(k, 1.0)
        amp = {}
        if phase == self.B.FWD:
            for i in range(o.m + o.r_r):
                v = np.sqrt(np.mean([(f(self.w_row_amp, i) * f(self.w_col_amp, j)) ** 2 for j in range(o.n)]))
                if v > 1.0:
                    amp[i] = float(v)
        else:
            for j in range(o.n + o.r_c):
                v = np.sqrt(np.mean([(f(self.w_row_amp, i) * f(self.w_col_amp, j)) ** 2 for i in range(o.m)]))
                if v > 1.0:
                    amp[j] = float(v)
        return amp

    def _code(self, phase):
        """(P, number of blocks, block pitch, logical length, systematic blocks) of the phase's codeword."""
        o = self.ora
        if phase == self.B.FWD:
            return o.P_r, o.m + o.r_r, o.Br, o.N_out, o.m
        return o.P_c, o.n + o.r_c, o.Bc, o.N_in, o.n

    def product(self, phase, V, faults=(), check_margins=True, epilogue=0, aux=None, verified=False,
                check_fault=None, V_ora=None, aux_ora=None):
        """One coded product + injection + check on both sides; V is batch-major [b][N].
        V_ora / aux_ora: the oracle's own input and auxiliary array where it follows a trajectory of
        its own (multi-layer runs in which each side feeds on its own activations).
        epilogue / aux (batch-major numpy): the elementwise step fused into the GPU's check.
        verified: the check with the verification steps of Error Model 2; check_fault =
        dict(target=CHECK_EVALUATION | CHECK_LIST, who, seed, hi) plants an error in the checking."""
        B = self.B
        Vd = self.dev_tensor(V)
        Vo = np.asarray(V, dtype=np.float32).T.astype(np.float64) if V_ora is None else np.asarray(V_ora, dtype=np.float64).T
        if phase == B.FWD:
            out_g = self.gpu.forward(Vd)
            out_o = self.ora.forward(Vo)
        else:
            out_g = self.gpu.backward(Vd)
            out_o = self.ora.backward(Vo)
        P, L, Bp, N, a = self._code(phase)
        edges = pitch_edges(L, Bp)
        wamp = self._weight_amp(phase)
        self._cmp(to_np(out_g).T, out_o, "coded product", edges, row_amp=wamp)
        faults = list(faults)
        if faults:
            self.gpu.inject(faults, out_g)
            out_o = self.ora.inject(faults, out_o)
            self._cmp(to_np(out_g).T, out_o, "injected output", edges, row_amp=wamp)
        if check_fault is not None:
            self.gpu.inject([dict(phase=B.CHECK, bi=check_fault["target"], bj=check_fault["who"],
                                  seed=check_fault.get("seed", 0), step=0, lo=0.0, hi=check_fault["hi"])])
        dec_g = self.gpu.detect_decode(phase, out_g, report=self.report, epilogue=epilogue,
                                       aux=None if aux is None else self.dev_tensor(aux), verified=verified)
        rep = self.gpu.read_report(self.report)
        if verified:
            kw = {}
            if check_fault is not None and check_fault["target"] == B.CHECK_EVALUATION:
                kw = dict(check_faults=[(check_fault["who"] % 2, 0, check_fault["hi"])])
            elif check_fault is not None:
                kw = dict(evaluators=check_fault["who"] + 2, list_faults=[(check_fault["who"],)])
            res = self.ora.verified_detect_decode(phase, out_o, **kw)
        else:
            res = self.ora.detect_decode(phase, out_o)
        if epilogue == B.EPI_RELU:
            res["decoded"] = O.relu(res["decoded"])
        elif epilogue == B.EPI_MASK_POS:
            res["decoded"] = O.relu_backward(res["decoded"], np.asarray(aux if aux_ora is None else aux_ora, dtype=np.float64).T)
        elif epilogue == B.EPI_MUL:
            res["decoded"] = res["decoded"] * np.asarray(aux if aux_ora is None else aux_ora, dtype=np.float64).T
        self.log.append((phase, [(f["bi"], f["bj"]) for f in faults], rep["verdict"], rep["located"]))
        assert rep["verdict"] == res["verdict"], (rep, res["verdict"], res["located"], res["syn_rel"], res["resid_rel"])
        assert rep["located"] == res["located"], (rep, res["located"])
        if rep["verdict"] == B.DISAGREE:
            if check_fault["target"] == B.CHECK_EVALUATION:   # found before anything was corrected
                self._cmp(to_np(out_g).T, res["out"], "output before a disagreement", edges, row_amp=wamp)
            return dec_g, rep, res
        if check_margins and (self.ora.r_r if phase == B.FWD else self.ora.r_c) > 0:
            # check_margins: True = the factor MARGIN; a number = that factor (seeded random grids and
            # generators, whose geometry is not chosen for separation, are held to a smaller one)
            self._margins(rep, res, self.ora.r_r if phase == B.FWD else self.ora.r_c,
                          MARGIN if check_margins is True else float(check_margins))
        if rep["verdict"] != B.UNCORRECTABLE:
            # repaired blocks carry the rounding noise of the blocks they were rebuilt from
            # (scale of a repaired block: its rms after the repair -- a block produced from a corrupted
            # stored block is large before it)
            fixed_rms = np.sqrt(np.mean(res["out"].reshape(L, -1) ** 2, axis=1))
            noise_rms = fixed_rms * np.array([wamp.get(i, 1.0) for i in range(L)])
            amp = dict(wamp)
            if res["located"]:
                for i, f in corrected_amp(P, res["located"], noise_rms).items():
                    amp[i] = f * wamp.get(i, 1.0)
            mul = np.asarray(aux if aux_ora is None else aux_ora, dtype=np.float64) if epilogue == B.EPI_MUL else None
            self._cmp(to_np(dec_g).T, res["decoded"], "decoded output", logical_edges(N, a),
                      row_amp={i: f for i, f in amp.items() if i < a},
                      elem_scale=1.0 if mul is None else max(1.0, float(np.max(np.abs(mul)) / np.sqrt(np.mean(mul ** 2)))))
            self._cmp(to_np(out_g).T, res["out"], "corrected coded output", edges, row_amp=amp)
        else:
            self._cmp(to_np(out_g).T, res["out"], "output left as it was", edges, row_amp=wamp)
        return dec_g, rep, res

    def _margins(self, rep, res, r, MARGIN):
        """Both sides' thresholded quantities must sit a factor MARGIN away from the
        thresholds, so that float32/bf16 rounding cannot flip a decision silently."""
        for side, syn, resid in (("gpu", max(rep["syn_rel"]), rep["resid_rel"]),
                                 ("oracle", float(np.max(res["syn_rel"])), res["resid_rel"])):
            if res["verdict"] == O.CLEAN:
                assert syn * MARGIN <= self.tau_detect, (side, "clean but close to tau_detect", syn)
            else:
                assert syn >= MARGIN * self.tau_detect, (side, "detected but close to tau_detect", syn)
            if res["verdict"] == O.CORRECTED:
                assert resid * MARGIN <= self.tau_resid, (side, "accepted but close to tau_resid", resid)
            elif res["verdict"] == O.UNCORRECTABLE and r >= 2:
                assert resid >= MARGIN * self.tau_resid, (side, "rejected but close to tau_resid", resid)

    def update(self, eta):
        self.gpu.update(eta)
        self.ora.update(eta)

    def regenerate(self, phase, res):
        """GPU: from the device-side report of the last product of `phase`; oracle: from its located set.
        Returns the bound scaling of the rebuilt lines for check_weights: dict(row_amp=...) after a
        forward check, dict(col_amp=...) after a backward one (empty when nothing was rebuilt)."""
        self.gpu.regenerate(phase, self.report)
        if res["verdict"] != O.CORRECTED:
            return {}
        o = self.ora
        rows = phase == self.B.FWD
        P, L, Bp = (o.P_r, o.m + o.r_r, o.Br) if rows else (o.P_c, o.n + o.r_c, o.Bc)
        # the oracle accesses the same a good blocks as the library: where one of them carries an
        # undetected error of its own (a second stored block hit in the same grid column), the
        # rebuilt block depends on the choice, and both sides must make the same one
        self.ora.regenerate(phase, res["located"], sources=library_sources(P, res["located"]))
        lines = (o.Wt if rows else o.Wt.T).reshape(L, -1)
        amp = regenerated_amp(P, res["located"], np.sqrt(np.mean(lines ** 2, axis=1)))
        if self.dtype == "bf16":
            keep = self.w_row_amp if rows else self.w_col_amp
            for i, f in amp.items():
                keep[i] = max(keep.get(i, 1.0), f)
        return {"row_amp" if rows else "col_amp": amp}

    def inject_weights(self, faults):
        if faults:
            self.gpu.inject(list(faults))
            self.ora.inject(list(faults))

    def close(self):
        self.gpu.destroy()


# ---------------------------------------------------------------------------------
# Multi-layer driver (feedforward l = 1..L, backpropagation l = L..1, update), the
# per-iteration schedule of the decentralized algorithm, on both sides.  Activation
# f = ReLU, g(x) = 1[x > 0]; loss head: mean softmax cross-entropy, delta^L = (Y - p) / b
# (delta is minus the gradient, so the update adds eta * delta x^T).  An UNCORRECTABLE
# product is recomputed once without replaying the fault (transient output errors).
# ---------------------------------------------------------------------------------
class MlpPair:
    EPI_RELU, EPI_MASK_POS = 1, 2

    def __init__(self, wl, max_layers=None, roll_forward=False, independent=False):
        """roll_forward: the stored blocks of every located node are regenerated after a CORRECTED
        check, and the workload's update-stage (weight) faults are planted after every update.
        independent: the oracle follows its own trajectory in float64 (its own activations, loss head
        and backpropagated errors from the first input on) instead of being handed the GPU's
        activations before every product; the two sides then differ by the accumulated float32
        rounding of the whole run, so the per-block and per-element bounds are five times wider.
        One decision is shared: where an activation is within 1e-5 rms of the ReLU kink, the oracle's
        mask g(x) takes the GPU's side (a sign decided by rounding is taken in one precision)."""
        self.wl = wl
        self.roll_forward = roll_forward
        self.independent = independent
        self.regenerated = 0
        self.restored = 0
        self.snapped = 0
        self.ckpt = {}
        widths = wl.widths if max_layers is None else wl.widths[: max_layers + 1]
        self.layers = []
        for l in range(len(widths) - 1):
            P_r, P_c = wl.generators(l)
            W = WL.layer_weights(widths[l + 1], widths[l], l)
            self.layers.append(Pair(W, P_r, P_c, wl.dtype, wl.batch, wl.tau_detect, wl.tau_resid))
            if independent:
                self.layers[-1].blk_scale = 5.0
        self.widths = widths
        self.counts = {0: 0, 1: 0, 2: 0}

    def _product(self, l, phase, V, faults, epilogue=0, aux=None, V_ora=None, aux_ora=None):
        pair = self.layers[l]
        kw = dict(epilogue=epilogue, aux=aux, V_ora=V_ora, aux_ora=aux_ora)
        dec, rep, res = pair.product(phase, V, faults, **kw)
        self.counts[rep["verdict"]] += 1
        if rep["verdict"] == O.UNCORRECTABLE:
            dec, rep, res = pair.product(phase, V, (), **kw)   # roll back = recompute the product
            if rep["verdict"] == O.UNCORRECTABLE and self.roll_forward and l in self.ckpt:
                # more persistent (weight) faults than the code corrects: the paper restores the last
                # checkpoint -- here the layer as it was after its last update, encoded afresh
                pair = self.restore(l)
                dec, rep, res = pair.product(phase, V, (), **kw)
            if not self.roll_forward:
                assert rep["verdict"] == O.CLEAN
            else:        # a single persistent fault may still be there: it is located now
                assert rep["verdict"] != O.UNCORRECTABLE
        if self.roll_forward and rep["verdict"] == O.CORRECTED:
            pair.regenerate(phase, res)
            self.regenerated += 1
        return to_np(dec).astype(np.float32), res["decoded"].T

    @staticmethod
    def _head(logits, labels):
        """Mean softmax cross-entropy: loss and delta^L = (Y - p) / b."""
        b = logits.shape[0]
        p = np.exp(logits - logits.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        Y = np.zeros_like(p)
        Y[np.arange(b), labels] = 1.0
        return float(-np.mean(np.log(p[np.arange(b), labels] + 1e-30))), (Y - p) / b

    def step(self, step, labels=None):
        wl, L = self.wl, len(self.layers)
        b = wl.batch
        ind = self.independent
        X = wl.inputs(step)[:, : self.widths[0]]
        xs_g, xs_o = [X], [X.astype(np.float64)]
        for l in range(L):
            # the activation is fused into the check on the GPU side (all layers but the last)
            s_g, s_o = self._product(l, WL.PHASE_FWD, xs_g[-1], wl.product_faults(WL.PHASE_FWD, step, l),
                                     epilogue=self.EPI_RELU if l < L - 1 else 0, V_ora=xs_o[-1] if ind else None)
            if l < L - 1:
                assert (s_g >= 0).all()
            xs_g.append(s_g)
            # unless the oracle runs on its own, both sides continue from the GPU activations
            # and the comparison is per product
            xs_o.append(s_o if ind else s_g.astype(np.float64))
        if labels is None:
            labels = np.random.default_rng(WL.SEED_DELTAS + step).integers(0, xs_g[-1].shape[1], size=b)
        loss, delta = self._head(xs_g[-1].astype(np.float64), labels)
        delta = delta.astype(np.float32)
        self.loss_ora, delta_o = self._head(xs_o[-1], labels) if ind else (loss, delta.astype(np.float64))
        for l in range(L - 1, -1, -1):
            # delta^{l-1} = g(x^l) (.) c^l, fused into the check of the backward product
            aux_o = None
            if ind and l > 0:
                near = np.abs(xs_o[l]) < 1e-5 * np.sqrt(np.mean(xs_o[l] ** 2))
                flip = near & ((xs_o[l] > 0) != (xs_g[l] > 0))
                self.snapped += int(flip.sum())
                aux_o = np.where(flip, xs_g[l].astype(np.float64), xs_o[l])
            c_g, c_o = self._product(l, WL.PHASE_BWD, delta, wl.product_faults(WL.PHASE_BWD, step, l),
                                     epilogue=self.EPI_MASK_POS if l > 0 else 0, aux=xs_g[l] if l > 0 else None,
                                     V_ora=delta_o if ind else None, aux_ora=aux_o)
            if l > 0:
                delta = c_g.astype(np.float32)
                delta_o = c_o if ind else delta.astype(np.float64)
        for l in range(L):
            self.layers[l].update(wl.eta)
        if self.roll_forward and wl.weight_faults:
            for l in range(L):       # errors of the update stage: seen by the next step's products
                self.ckpt[l] = self.layers[l].ora.weights().copy()      # checkpoint: the state the update should leave
                self.layers[l].inject_weights(wl.update_faults(step, l))
        return loss

    def restore(self, l):
        """Both sides of layer l re-created from the checkpointed weights."""
        old = self.layers[l]
        P_r, P_c = self.wl.generators(l)
        old.close()
        self.layers[l] = Pair(self.ckpt[l], P_r, P_c, self.wl.dtype, self.wl.batch, self.wl.tau_detect, self.wl.tau_resid)
        self.layers[l].blk_scale = old.blk_scale
        self.restored += 1
        return self.layers[l]

    def close(self):
        for p in self.layers:
            p.close()
