"""GPU parity: the HIP path, called through the C ABI, against the float64 oracle
on the same seeded inputs.  Located block sets and verdicts must be identical;
values within 1e-4 (f32) / 2e-2 (bf16 inputs) relative Frobenius error."""
import itertools
import sys

import numpy as np
import pytest

from paper_1903_01042_amd import workloads as WL
from harness import TOL, MlpPair, Pair, rel_fro, to_np

pytestmark = pytest.mark.gpu

FWD, BWD, WEIGHT = WL.PHASE_FWD, WL.PHASE_BWD, WL.PHASE_WEIGHT
CLEAN, CORRECTED, UNCORRECTABLE = 0, 1, 2


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def layer_step(pair, wl, step, layer=0, n_out=None, n_in=None):
    """forward -> inject -> check, backward -> inject -> check, update (-> weight faults)."""
    b = wl.batch
    X = WL.normal((b, n_in), WL.SEED_INPUTS + step) if wl.input_law == "normal" else \
        WL.uniform01((b, n_in), WL.SEED_INPUTS + step)
    D = WL.normal((b, n_out), WL.SEED_DELTAS + step)
    _, rf, _ = pair.product(FWD, X, wl.product_faults(FWD, step, layer))
    _, rb, _ = pair.product(BWD, D, wl.product_faults(BWD, step, layer))
    pair.update(wl.eta)
    return rf, rb


# ------------------------------------------------------------------ worked example
def test_paper_example_grid_every_single_block_error():
    """m = n = 2, t = 1 with the paper's generators on a 256 x 256 layer: every
    single erroneous block-row / block-column is located and corrected."""
    P_r, P_c = WL.paper_example_generators()
    W = WL.layer_weights(256, 256)
    pair = Pair(W, P_r, P_c, "f32", max_batch=16)
    pair.check_weights(1e-6)
    X, D = WL.normal((16, 256), 1), WL.normal((16, 256), 2)
    for bi in range(4):
        say("paper grid fwd fault row", bi)
        _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, bi, 1, step=bi)])
        assert rep["verdict"] == CORRECTED and rep["located"] == [bi]
    for bj in range(4):
        say("paper grid bwd fault col", bj)
        _, rep, _ = pair.product(BWD, D, [WL.make_fault(BWD, 0, bj, step=bj)])
        assert rep["verdict"] == CORRECTED and rep["located"] == [bj]
    _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, 0, 0, 9), WL.make_fault(FWD, 3, 1, 9)])
    assert rep["verdict"] == UNCORRECTABLE
    _, rep, _ = pair.product(FWD, X)
    assert rep["verdict"] == CLEAN
    pair.product(BWD, D)
    pair.update(0.01)
    pair.check_weights()
    assert rel_fro(to_np(pair.gpu.export_weights()), pair.ora.weights()) < 1e-5
    pair.close()


def test_hand_computed_residuals_and_ties_on_the_gpu():
    """The check fed with outputs written by hand (the cases worked out in the oracle's pins): the
    relative residual of the best support as a number -- sqrt(1/65) with two erroneous blocks at
    one position, accepted or rejected around it, sqrt(1/90) at two positions -- and exact ties,
    which go to the first support in lexicographic order on both sides."""
    import torch
    from oracle import codenet_oracle as O
    from paper_1903_01042_amd import binding as B
    P_r, P_c = WL.paper_example_generators()         # H_r columns (1,1), (1,-1), (-1,0), (0,-1); H_c columns (1,1), (1,2), ...
    dev = torch.device("cuda:0")

    def run(n_out, n_in, phase, blocks, tau_resid, want_verdict, want_located, want_resid, want_blocks):
        lay = B.CodedLayer(torch.zeros((n_out, n_in), device=dev), P_r, P_c, max_batch=1, tau_detect=1e-3,
                           tau_resid=tau_resid)
        Bp = lay.B_r if phase == FWD else lay.B_c
        out = np.zeros((1, 4 * Bp), dtype=np.float32)
        for i, vals in enumerate(blocks):
            out[0, i * Bp: i * Bp + len(vals)] = vals
        out_d = torch.from_numpy(out).to(dev)
        rep = lay.new_report()
        dec = lay.detect_decode(phase, out_d, report=rep)
        got = lay.read_report(rep)
        res = O.detect_decode(out.astype(np.float64).T, P_r if phase == FWD else P_c, Bp, 1e-3, tau_resid)
        say("hand case", blocks, "->", got["verdict"], got["located"], got["resid_rel"])
        assert got["verdict"] == res["verdict"] == want_verdict
        assert got["located"] == res["located"] == want_located
        assert abs(got["resid_rel"] - want_resid) <= 2e-6 and abs(res["resid_rel"] - want_resid) <= 1e-12
        fixed = to_np(out_d)[0]
        for i, vals in enumerate(want_blocks):
            assert np.allclose(fixed[i * Bp: i * Bp + len(vals)], vals, atol=1e-6), (i, fixed)
            assert np.allclose(res["out"][i * Bp: i * Bp + len(vals), 0], vals, atol=1e-12)
        n_dec = n_out if phase == FWD else n_in
        assert np.allclose(to_np(dec)[0], np.concatenate(want_blocks[:2])[:n_dec], atol=1e-6)
        lay.destroy()

    s65, s90 = np.sqrt(1.0 / 65.0), np.sqrt(1.0 / 90.0)
    run(2, 2, BWD, [[1], [1], [0], [0]], 0.2, CORRECTED, [1], s65, [[1], [-0.6], [0], [0]])
    run(2, 2, BWD, [[1], [1], [0], [0]], 0.12, UNCORRECTABLE, [], s65, [[1], [1], [0], [0]])
    run(2, 4, BWD, [[1, 0], [1, 1], [0, 0], [0, 0]], 0.2, CORRECTED, [1], s90, [[1, 0], [-0.6, 0], [0, 0], [0, 0]])
    run(2, 2, BWD, [[0], [2], [0], [0]], 1e-6, CORRECTED, [1], 0.0, [[0], [0], [0], [0]])
    # ties: supports {0} and {2}, then {1} and {3}, then all four
    run(6, 2, FWD, [[0, 0, 0], [0, 0, 0], [-1, -1, -1], [0, 0, -1]], 0.6, CORRECTED, [0], 0.5,
        [[-0.5, -0.5, -1.0], [0, 0, 0], [-1, -1, -1], [0, 0, -1]])
    run(6, 2, FWD, [[0, 0, 0], [0, 0, 0], [0, 0, -1], [-1, -1, 1]], 0.6, CORRECTED, [1], 0.5,
        [[0, 0, 0], [0.5, 0.5, -1.0], [0, 0, -1], [-1, -1, 1]])
    run(4, 2, FWD, [[0, 0], [0, 0], [-1, 0], [0, -1]], 0.8, CORRECTED, [0], np.sqrt(0.5),
        [[-0.5, -0.5], [0, 0], [-1, 0], [0, -1]])


# ------------------------------------------------------------------- cfg1, full size
def test_cfg1_full():
    wl = WL.WORKLOADS["cfg1"]
    P_r, P_c = wl.generators()
    pair = Pair(WL.layer_weights(256, 256), P_r, P_c, "f32", wl.batch, wl.tau_detect, wl.tau_resid)
    seen = set()
    for step in range(wl.steps):
        say("cfg1 step", step)
        rf, rb = layer_step(pair, wl, step, n_out=256, n_in=256)
        seen.update([rf["verdict"], rb["verdict"]])
        pair.check_weights()
    # one parity block only detects: every corrupted product is flagged, none located
    assert seen == {CLEAN, UNCORRECTABLE}
    pair.close()


# ------------------------------------------------------------------- cfg2, full size
def test_cfg2_mlp_full_size():
    """784-1024-1024-10 MLP, 4x4 grid + 1 parity row/col per layer (detect only),
    ReLU, softmax-CE on random labels, Bernoulli(0.05) faults per node and product, all 100 steps
    of the workload: every product of every step against the oracle (which is handed the GPU's
    activations before each product), weights of all layers every 25 steps."""
    wl = WL.WORKLOADS["cfg2"]
    mlp = MlpPair(wl)
    losses = []
    for step in range(wl.steps):
        say("cfg2 step", step)
        losses.append(mlp.step(step))
        if (step + 1) % 25 == 0:
            for l, pair in enumerate(mlp.layers):
                say("cfg2 layer", l, "after", step + 1, "steps: coded weights rel err", pair.check_weights())
    say("cfg2 verdict counts", mlp.counts, "loss", losses[0], "->", losses[-1])
    assert mlp.counts[2] > 0 and mlp.counts[1] == 0        # r = 1: faults are detected, never located
    assert all(np.isfinite(losses))
    mlp.close()


def test_cfg2_mlp_against_an_oracle_on_its_own_trajectory():
    """The same 100 steps with the oracle never seeing a GPU value after the first input: it runs
    feedforward, loss head, backpropagation and update on its own activations in float64, and every
    product, every decoded activation, every backpropagated error and the weights of all layers
    are compared along the way (bounds five times the per-product ones: the difference is the
    float32 rounding accumulated over the run)."""
    wl = WL.WORKLOADS["cfg2"]
    mlp = MlpPair(wl, independent=True)
    for step in range(wl.steps):
        say("cfg2 independent step", step)
        loss = mlp.step(step)
        assert abs(loss - mlp.loss_ora) <= 1e-4 * max(1.0, abs(mlp.loss_ora)), (step, loss, mlp.loss_ora)
        if (step + 1) % 25 == 0:
            for l, pair in enumerate(mlp.layers):
                say("cfg2 independent layer", l, "after", step + 1, "steps: coded weights rel err", pair.check_weights())
    say("cfg2 independent: verdict counts", mlp.counts, "mask decisions taken from the GPU", mlp.snapped,
        "loss gpu", loss, "oracle", mlp.loss_ora)
    assert mlp.snapped <= 64
    mlp.close()


def test_cfg4_style_mlp_rolls_forward_through_update_stage_faults():
    """A width-scaled copy of cfg4 (all 8 layers, 8 x 8 grid + 2 parity rows / columns per layer, ReLU,
    the workload's 20 steps) with its three kinds of faults -- forward outputs, backward outputs and stored blocks after the
    update: every located node is regenerated and training goes on; where more stored blocks are hit
    than the code corrects, the layer is restored from its checkpoint (the state after its last update)
    as the paper prescribes; every product of every step as the oracle's, weights at the end."""
    import dataclasses
    wl = dataclasses.replace(WL.WORKLOADS["cfg4"].scaled(32, batch=48), fault_p=0.003)
    L = len(wl.widths) - 1
    assert L == 8
    mlp = MlpPair(wl, roll_forward=True)
    planted = 0
    for step in range(wl.steps):
        say("cfg4-style step", step)
        mlp.step(step)
        planted += sum(len(wl.update_faults(step, l)) for l in range(L))
    for l, pair in enumerate(mlp.layers):
        say("cfg4-style layer", l, "coded weights rel err", pair.check_weights())
    say("cfg4-style verdict counts", mlp.counts, "regenerations", mlp.regenerated, "restores", mlp.restored,
        "weight faults planted", planted)
    assert planted > 0 and mlp.regenerated > 0 and mlp.counts[1] > 0 and mlp.restored >= 1
    mlp.close()


# ------------------------------------------------- full-size single layers, one step
@pytest.mark.parametrize("name", ["cfg3", "cfg4", "cfg5"])
def test_full_size_layer_step(name):
    """One layer-step at the benchmark size (for cfg4: one of its eight equal layers),
    every output element compared with the oracle."""
    wl = WL.WORKLOADS[name]
    n_in, n_out = wl.widths[0], wl.widths[1]
    P_r, P_c = wl.generators()
    say(name, "full size: encoding", n_out, n_in)
    pair = Pair(WL.layer_weights(n_out, n_in), P_r, P_c, wl.dtype, wl.batch, wl.tau_detect, wl.tau_resid)
    pair.check_weights(1e-6)
    m, n = wl.grid
    X, D = wl.inputs(0), wl.deltas(0)
    say(name, "forward with one fault")
    _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, m, 1, 0)])
    assert rep["verdict"] == CORRECTED and rep["located"] == [m]
    say(name, "backward with two faulty block-columns")
    _, rep, _ = pair.product(BWD, D, [WL.make_fault(BWD, 0, 2, 0), WL.make_fault(BWD, 1, n + 1, 0)])
    assert rep["verdict"] == UNCORRECTABLE
    say(name, "backward clean")
    _, rep, _ = pair.product(BWD, D)
    assert rep["verdict"] == CLEAN
    say(name, "update")
    pair.update(wl.eta)
    pair.check_weights()
    say(name, "weight faults on block-row 1, located by the next forward product, regenerated")
    coded, coded_gpu = pair.ora.Wt.copy(), to_np(pair.gpu.export_coded())
    pair.inject_weights([WL.make_fault(WEIGHT, 1, j, 1) for j in range(n)])
    _, rep, res = pair.product(FWD, wl.inputs(1))
    assert rep["verdict"] == CORRECTED and rep["located"] == [1]
    pair.regenerate(FWD, res)
    assert rel_fro(pair.ora.Wt, coded) <= 1e-9
    # after an update with bf16 operands the stored parity blocks follow the systematic ones only to
    # bf16 accuracy of the increment, so the rebuilt row matches the lost one to that accuracy
    pair.check_weights()
    assert rel_fro(to_np(pair.gpu.export_coded()), coded_gpu) <= (1e-5 if wl.dtype == "f32" else pair.tol)
    _, rep, _ = pair.product(FWD, wl.inputs(2))
    assert rep["verdict"] == CLEAN
    pair.close()


@pytest.mark.parametrize("name,steps,drift_every,probe_every", [("cfg3", 50, 25, 10), ("cfg5", 200, 50, 50)])
def test_full_size_multi_step_invariants(name, steps, drift_every, probe_every):
    """Many steps at the benchmark size under the workload's own fault law, as bench.py drives them
    (the oracle cannot follow every step at this size; a width-scaled copy is followed step by step
    elsewhere).  What must hold at any size: (i) the number of faulty blocks planted decides the
    verdict (none: CLEAN; at most t: CORRECTED with exactly those blocks located; more:
    UNCORRECTABLE, output untouched); (ii) an accepted output checks CLEAN when checked again;
    (iii) every `drift_every` steps the stored matrix is still a codeword: it equals the oracle's
    encoding of its own systematic part; (iv) at the end the systematic part equals the plain
    float64 update W + eta sum_s Delta_s X_s^T (cfg3; the product of the method, O-upd); (v) every
    `probe_every` steps both coded products pass a float64 Freivalds probe against the stored
    matrix of that step: out^T z = W~ (V^T z) for a random z over the batch (library-independent
    float64 arithmetic in torch)."""
    import torch
    from oracle import codenet_oracle as O
    from paper_1903_01042_amd import binding as B
    wl = WL.WORKLOADS[name]
    n_in, n_out = wl.widths[0], wl.widths[1]
    m, n = wl.grid
    t = wl.r // 2
    P_r, P_c = wl.generators()
    W0 = WL.layer_weights(n_out, n_in)
    dev = torch.device("cuda:0")
    lay = B.CodedLayer(torch.from_numpy(W0).to(dev), P_r, P_c, dtype=B.BF16_F32ACC if wl.dtype == "bf16" else B.F32,
                       max_batch=wl.batch, tau_detect=wl.tau_detect, tau_resid=wl.tau_resid)
    tol = TOL[wl.dtype]
    rep, rep2 = lay.new_report(), lay.new_report()
    ref = W0.astype(np.float64) if name == "cfg3" else None
    seen = set()

    def probe(phase, V, out, Wc64, step):
        z = torch.from_numpy(np.random.default_rng(9000 + step).standard_normal(wl.batch)).to(dev)
        lhs = out.double().T @ z
        if phase == FWD:
            rhs = Wc64[:, : n * lay.B_c] @ (V.double().T @ z)
        else:
            rhs = Wc64[: m * lay.B_r, :].T @ (V.double().T @ z)
        err = float(torch.linalg.norm(lhs - rhs) / torch.linalg.norm(rhs))
        assert err <= tol, (name, phase, step, err)
        return err

    def checked_product(phase, V, faults, Wc64=None, step=0):
        out = lay.forward(V) if phase == FWD else lay.backward(V)
        if Wc64 is not None:
            say(name, "Freivalds probe, phase", phase, "step", step, "%.2e" % probe(phase, V, out, Wc64, step))
        lay.inject(faults, out)
        before = out.clone()
        lay.detect_decode(phase, out, report=rep, want_decoded=False)
        got = lay.read_report(rep)
        hit = sorted({f["bi"] if phase == FWD else f["bj"] for f in faults})
        want = CLEAN if not hit else (CORRECTED if len(hit) <= t else UNCORRECTABLE)
        assert got["verdict"] == want, (phase, hit, got)
        seen.add(want)
        if want == CORRECTED:
            assert got["located"] == hit, (hit, got)
        if want == UNCORRECTABLE:
            assert got["located"] == [] and torch.equal(out, before)
        else:
            lay.detect_decode(phase, out, report=rep2, want_decoded=False)
            assert lay.read_report(rep2)["verdict"] == CLEAN
        return got

    for step in range(steps):
        say(name, "full size step", step)
        X, D = wl.inputs(step), wl.deltas(step)
        Xd, Dd = torch.from_numpy(X).to(dev), torch.from_numpy(D).to(dev)
        Wc64 = lay.export_coded().double() if step % probe_every == 0 else None
        checked_product(FWD, Xd, wl.product_faults(FWD, step), Wc64, step)
        checked_product(BWD, Dd, wl.product_faults(BWD, step), Wc64, step)
        del Wc64
        lay.update(wl.eta)
        if ref is not None:
            ref += wl.eta * (D.astype(np.float64).T @ X.astype(np.float64))
        if (step + 1) % drift_every == 0:
            Wc = to_np(lay.export_coded()).astype(np.float64)
            sys_part = Wc[: m * lay.B_r, : n * lay.B_c]
            again = O.encode(sys_part, P_r, P_c, lay.B_r, lay.B_c)
            drift = rel_fro(Wc, again)
            say(name, "drift after", step + 1, "steps: %.3e" % drift)
            assert drift <= tol, drift
            del Wc, again
    assert len(seen) >= 2, seen            # the fault law produces more than one kind of step
    if ref is not None:
        err = rel_fro(to_np(lay.export_weights()), ref)
        say(name, "weights after", steps, "steps against the plain float64 update: %.3e" % err)
        assert err <= tol, err
    lay.destroy()


def test_cfg4_full_size_mlp_invariants():
    """The 8-layer width-8192 MLP of cfg4 at its real size (8 x 8 grid + 2 per layer, batch 1024,
    float32), the workload's 20 training steps driven through the library alone: forward chain with the ReLU fused
    into the check, squared-error head, backward chain with g(x) (.) c fused into the check, update of
    every layer, faults in forward and backward outputs and one stored block hit after the first
    update.  Checked at this size: float64 Freivalds probes of every product of the first step, the
    verdict that the number of planted blocks dictates, the decoded activations as the elementwise
    step of the corrected systematic part (bit for bit), the hit block-row located by the next
    step's forward product and regenerated, and the stored code of two layers against the oracle's
    re-encoding at the end."""
    import dataclasses
    import torch
    from oracle import codenet_oracle as O
    from paper_1903_01042_amd import binding as B
    wl = dataclasses.replace(WL.WORKLOADS["cfg4"], fault_p=0.004)
    L = len(wl.widths) - 1
    N, b = wl.widths[0], wl.batch
    m, n = wl.grid
    t = wl.r // 2
    dev = torch.device("cuda:0")
    layers = []
    for l in range(L):
        say("cfg4 full size: encoding layer", l)
        P_r, P_c = wl.generators(l)
        layers.append(B.CodedLayer(torch.from_numpy(WL.layer_weights(N, N, l)).to(dev), P_r, P_c, dtype=B.F32,
                                   max_batch=b, tau_detect=wl.tau_detect, tau_resid=wl.tau_resid))
    rep = layers[0].new_report()
    tol = TOL["f32"]
    counts = {CLEAN: 0, CORRECTED: 0, UNCORRECTABLE: 0}

    def product(l, phase, V, faults, step, epilogue, aux, also_hit=()):
        lay = layers[l]
        out = lay.forward(V) if phase == FWD else lay.backward(V)
        if step == 0:
            Wc = lay.export_coded().double()
            z = torch.from_numpy(np.random.default_rng(9100 + 2 * l + phase).standard_normal(b)).to(dev)
            rhs = (Wc[:, : n * lay.B_c] @ (V.double().T @ z)) if phase == FWD else (Wc[: m * lay.B_r, :].T @ (V.double().T @ z))
            err = float(torch.linalg.norm(out.double().T @ z - rhs) / torch.linalg.norm(rhs))
            assert err <= tol, (l, phase, err)
            del Wc
        lay.inject(faults, out)
        dec = lay.detect_decode(phase, out, report=rep, epilogue=epilogue, aux=aux)
        got = lay.read_report(rep)
        hit = sorted({f["bi"] if phase == FWD else f["bj"] for f in faults} | set(also_hit))
        want = CLEAN if not hit else (CORRECTED if len(hit) <= t else UNCORRECTABLE)
        assert got["verdict"] == want and (want != CORRECTED or got["located"] == hit), (l, phase, hit, got)
        counts[want] += 1
        if want == UNCORRECTABLE:                 # transient faults: the product is computed again;
            out = lay.forward(V) if phase == FWD else lay.backward(V)       # a hit stored block is still there
            dec = lay.detect_decode(phase, out, report=rep, epilogue=epilogue, aux=aux)
            got = lay.read_report(rep)
            want = CORRECTED if also_hit else CLEAN
            assert got["verdict"] == want and (want != CORRECTED or got["located"] == sorted(also_hit)), got
        if want == CORRECTED:
            lay.regenerate(phase, rep)
        sys_part = out[:, :N]
        if epilogue == B.EPI_RELU:
            sys_part = torch.relu(sys_part)
        elif epilogue == B.EPI_MASK_POS:
            sys_part = torch.where(aux > 0, sys_part, torch.zeros_like(sys_part))
        assert torch.equal(dec, sys_part), (l, phase)
        return dec

    for step in range(wl.steps):
        acts = [torch.from_numpy(wl.inputs(step)).to(dev)]
        for l in range(L):
            say("cfg4 full size step", step, "forward layer", l)
            extra = (3,) if (step == 1 and l == 5) else ()       # the stored block hit after the first update
            acts.append(product(l, FWD, acts[-1], wl.product_faults(FWD, step, l), step,
                                B.EPI_RELU if l < L - 1 else B.EPI_NONE, None, extra))
        Y = torch.from_numpy(WL.normal((b, N), WL.SEED_DELTAS + step)).to(dev)
        delta = (Y - acts[-1]) / b                                  # squared-error head
        for l in range(L - 1, -1, -1):
            say("cfg4 full size step", step, "backward layer", l)
            c = product(l, BWD, delta, wl.product_faults(BWD, step, l), step,
                        B.EPI_MASK_POS if l > 0 else B.EPI_NONE, acts[l] if l > 0 else None)
            if l > 0:
                delta = c
        for lay in layers:
            lay.update(wl.eta)
        if step == 0:
            layers[5].inject([WL.make_fault(WEIGHT, 3, 2, 0)])
    say("cfg4 full size verdicts", counts)
    assert counts[CORRECTED] >= 1 and counts[CLEAN] >= 1
    for l in (0, 5):
        P_r, P_c = wl.generators(l)
        Wc = to_np(layers[l].export_coded()).astype(np.float64)
        drift = rel_fro(Wc, O.encode(Wc[: m * layers[l].B_r, : n * layers[l].B_c], P_r, P_c, layers[l].B_r, layers[l].B_c))
        say("cfg4 full size layer", l, "drift %.3e" % drift)
        assert drift <= tol
    for lay in layers:
        lay.destroy()


# ------------------------------------------------------------- ragged / odd shapes
@pytest.mark.parametrize("n_out,n_in,m,n,r,b,dtype", [
    (10, 1024, 4, 4, 1, 128, "f32"),      # cfg2's last layer: 10 outputs on 4 block-rows
    (100, 52, 3, 5, 2, 7, "f32"),         # nothing divides anything
    (300, 200, 5, 4, 2, 33, "bf16"),
    (300, 200, 5, 4, 2, 260, "bf16"),     # batch of 256 or more: the persistent update kernel on edge tiles
    (700, 452, 3, 7, 2, 512, "bf16"),     # the same with several tiles per side and 8 slabs
    (130, 70, 2, 2, 4, 5, "f32"),         # t = 2
    (64, 64, 2, 2, 0, 8, "f32"),          # uncoded baseline path (r = 0)
])
def test_ragged_shapes(n_out, n_in, m, n, r, b, dtype):
    say("ragged", n_out, n_in, m, n, r, b, dtype)
    P_r = WL.vandermonde_like(m, r) if r in (0, 2) else WL.gaussian_generator(m, r, 3)
    P_c = WL.vandermonde_like(n, r) if r in (0, 2) else WL.gaussian_generator(n, r, 4)
    tau = (1e-3, 2e-3) if dtype == "f32" else (2e-2, 2e-2)
    pair = Pair(WL.layer_weights(n_out, n_in), P_r, P_c, dtype, b, *tau)
    pair.check_weights(1e-6)
    X, D = WL.normal((b, n_in), 11), WL.normal((b, n_out), 12)
    pair.product(FWD, X)
    pair.product(BWD, D)
    pair.update(0.02)
    pair.check_weights()
    if r >= 2:
        _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, m - 1, 0, 1)])   # last, partly padded block-row
        assert rep["verdict"] == CORRECTED and rep["located"] == [m - 1]
        _, rep, _ = pair.product(BWD, D, [WL.make_fault(BWD, 0, n + r - 1, 1)])
        assert rep["verdict"] == CORRECTED and rep["located"] == [n + r - 1]
    if r >= 4:
        _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, 0, 0, 2), WL.make_fault(FWD, m + 1, 1, 2)])
        assert rep["verdict"] == CORRECTED and rep["located"] == [0, m + 1]
    if r == 1:
        _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, 1, 0, 1)])
        assert rep["verdict"] == UNCORRECTABLE and rep["located"] == []
    pair.product(FWD, X)
    pair.product(BWD, D)
    pair.update(0.02)
    pair.check_weights()
    assert rel_fro(to_np(pair.gpu.export_weights()), pair.ora.weights()) < pair.tol
    pair.close()


# ------------------------------------------------------------- both bf16 update kernels
@pytest.mark.parametrize("b", [64, 192, 255, 256, 257, 320, 512, 700])
def test_bf16_update_kernels_on_either_side_of_their_batch_boundary(b):
    """The coded update of the bf16 mode has two kernels: one tile per workgroup up to a batch of
    192, the persistent one from 193 on (batches are padded to 64: 255 and 256 contract over 256
    columns, four slabs of 64, the fewest that its pipeline takes; 257 and 320 over five).  The same
    layer through both, two steps each: 1180 x 612 coded entries, ragged against the 128 x 128 tiles
    of the persistent kernel in both directions."""
    say("update kernels, batch", b)
    n_out, n_in, m, n, r = 700, 452, 3, 7, 2
    pair = Pair(WL.layer_weights(n_out, n_in), WL.vandermonde_like(m, r), WL.vandermonde_like(n, r), "bf16", b,
                2e-2, 2e-2)
    for step in range(2):
        X, D = WL.normal((b, n_in), 21 + step), WL.normal((b, n_out), 31 + step)
        _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, 1, 0, step)])
        assert rep["verdict"] == CORRECTED and rep["located"] == [1]
        _, rep, _ = pair.product(BWD, D, [WL.make_fault(BWD, 0, n, step)])
        assert rep["verdict"] == CORRECTED and rep["located"] == [n]
        pair.update(0.02)
        pair.check_weights()
    pair.close()


def test_bf16_persistent_update_with_several_tiles_per_workgroup():
    """4120 x 4120 coded entries are 33 x 33 tiles of the persistent update kernel on 256 workgroups:
    every workgroup walks over four or five tiles, tiles inside the matrix and tiles that stick out of
    it in either direction following each other in both orders (the walk alternates its direction from
    one update to the next).  Batches of 200 (four slabs per tile, the fewest) and 448 (seven)."""
    for b in (200, 448):
        say("persistent update over several tiles per workgroup, batch", b)
        n = 3282
        pair = Pair(WL.layer_weights(n, n), WL.vandermonde_like(8, 2), WL.vandermonde_like(8, 2), "bf16", b, 2e-2, 2e-2)
        assert pair.gpu.coded_rows == pair.gpu.coded_cols == 4120
        for step in range(3):
            X, D = WL.normal((b, n), 51 + step), WL.normal((b, n), 61 + step)
            pair.product(FWD, X)
            pair.product(BWD, D)
            pair.update(0.02)
            pair.check_weights()
        pair.close()


# ------------------------------------------------------------- float32 update of a thin batch
@pytest.mark.parametrize("b", [1, 7, 64, 65, 130, 256, 257])
def test_f32_update_of_a_thin_batch(b):
    """Float32 layers of more than 1024 coded rows and columns update through a kernel of their own
    up to a batch of 256 (the matrix read and written straight from the accumulators, 64 batch rows
    per LDS stage: 65 and 130 leave a ragged second or third stage, odd batches a k-row without a
    partner); 257 goes through the general kernel.  1656 x 1820 coded entries: ragged against the
    128 x 128 tiles in both directions.  Two steps each, with one corrected fault per product."""
    say("f32 thin-batch update, batch", b)
    n_out, n_in, m, n, r = 1100, 1300, 4, 5, 2
    pair = Pair(WL.layer_weights(n_out, n_in), WL.vandermonde_like(m, r), WL.vandermonde_like(n, r), "f32", b,
                1e-3, 2e-3)
    assert pair.gpu.coded_rows == 1656 and pair.gpu.coded_cols == 1820
    for step in range(2):
        X, D = WL.normal((b, n_in), 71 + step), WL.normal((b, n_out), 81 + step)
        _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, 1, 0, step)])
        assert rep["verdict"] == CORRECTED and rep["located"] == [1]
        _, rep, _ = pair.product(BWD, D, [WL.make_fault(BWD, 0, n, step)])
        assert rep["verdict"] == CORRECTED and rep["located"] == [n]
        pair.update(0.02)
        pair.check_weights()
    pair.close()


def test_f32_thin_batch_update_on_more_tiles_than_fit_the_chip():
    """4120 x 4120 coded entries are 33 x 33 tiles of the thin-batch update kernel, more workgroups
    than are resident at a time, edge tiles among them.  Batch 33."""
    b, n = 33, 3282
    say("f32 thin-batch update, 1089 tiles")
    pair = Pair(WL.layer_weights(n, n), WL.vandermonde_like(8, 2), WL.vandermonde_like(8, 2), "f32", b, 1e-3, 2e-3)
    assert pair.gpu.coded_rows == pair.gpu.coded_cols == 4120
    for step in range(3):
        X, D = WL.normal((b, n), 91 + step), WL.normal((b, n), 95 + step)
        pair.product(FWD, X)
        pair.product(BWD, D)
        pair.update(0.02)
        pair.check_weights()
    pair.close()


# ------------------------------------------------------------- degenerate grids and sizes
@pytest.mark.parametrize("n_out,n_in,m,n,r,b,dtype", [
    (64, 48, 1, 1, 2, 4, "f32"),          # one systematic block per dimension: the code is a repetition-like [1 | P]
    (5, 6, 4, 4, 2, 2, "f32"),            # blocks of two entries: the last block-row is all padding, the third half
    (16, 16, 2, 2, 2, 1, "f32"),          # batch of one, as in the paper
    (260, 260, 2, 2, 2, 300, "bf16"),     # bf16 with a batch above 256 on a grid of two blocks
])
def test_degenerate_grids(n_out, n_in, m, n, r, b, dtype):
    say("degenerate", n_out, n_in, m, n, r, b, dtype)
    from paper_1903_01042_amd import binding as B
    P_r, P_c = WL.vandermonde_like(m, r), WL.vandermonde_like(n, r)
    tau = (1e-3, 2e-3) if dtype == "f32" else (2e-2, 2e-2)
    pair = Pair(WL.layer_weights(n_out, n_in), P_r, P_c, dtype, b, *tau)
    pair.check_weights(1e-6)
    X, D = WL.normal((b, n_in), 41), WL.normal((b, n_out), 42)
    _, rep, _ = pair.product(FWD, X)
    assert rep["verdict"] == CLEAN
    _, rep, _ = pair.product(BWD, D)
    assert rep["verdict"] == CLEAN
    pair.update(0.05)
    pair.check_weights()
    # a fault on the first block-row (always has real entries) is corrected; one on a block that is
    # all padding changes nothing
    _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, 0, 0, 1)])
    assert rep["verdict"] == CORRECTED and rep["located"] == [0]
    if (m - 1) * -(-n_out // m) >= n_out:       # the last block-row holds no real entry
        _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, m - 1, 0, 2)])
        assert rep["verdict"] == CLEAN
        with pytest.raises(B.CodenetError) as e:   # more block-rows than outputs is refused outright
            B.CodedLayer(pair.dev_tensor(np.zeros((m - 1, n_in))), P_r, P_c, max_batch=b)
        assert e.value.code == B.E_SHAPE
    _, rep, _ = pair.product(BWD, D, [WL.make_fault(BWD, 0, n + 1, 3)])
    assert rep["verdict"] == CORRECTED and rep["located"] == [n + 1]
    assert rel_fro(to_np(pair.gpu.export_weights()), pair.ora.weights()) < pair.tol
    # empty calls: no faults is a no-op, a batch of zero is refused
    pair.gpu.inject([], pair.gpu.forward(pair.dev_tensor(X)))
    lib, vp = B.load_library(), __import__("ctypes").c_void_p
    assert lib.codenet_forward(pair.gpu._h, vp(pair.dev_tensor(X).data_ptr()), 0, vp(0), None) in (B.E_BATCH, B.E_NULL)
    pair.close()


def test_different_parity_counts_for_rows_and_columns():
    """r_rows = 2 (t = 1 for the forward product), r_cols = 4 (t = 2 for the backward one): each
    product is held to its own capability."""
    m, n, b = 4, 3, 12
    P_r, P_c = WL.vandermonde_like(m, 2), WL.gaussian_generator(n, 4, 21)
    pair = Pair(WL.layer_weights(96, 90), P_r, P_c, "f32", b)
    X, D = WL.normal((b, 90), 51), WL.normal((b, 96), 52)
    _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, 2, 0, 0)])
    assert rep["verdict"] == CORRECTED and rep["located"] == [2]
    _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, 2, 0, 1), WL.make_fault(FWD, 4, 1, 1)])
    assert rep["verdict"] == UNCORRECTABLE
    _, rep, res = pair.product(BWD, D, [WL.make_fault(BWD, 0, 1, 2), WL.make_fault(BWD, 1, 5, 2)])
    assert rep["verdict"] == CORRECTED and rep["located"] == [1, 5]
    _, rep, _ = pair.product(BWD, D, [WL.make_fault(BWD, 0, j, 3) for j in (0, 2, 6)])
    assert rep["verdict"] == UNCORRECTABLE
    pair.update(0.03)
    pair.check_weights()
    # weight faults in two block-columns: located by the backward product, regenerated along the rows of blocks
    clean = pair.ora.Wt.copy()
    pair.inject_weights([WL.make_fault(WEIGHT, i, j, 4) for j in (0, 4) for i in range(m)])
    _, rep, res = pair.product(BWD, D)
    assert rep["verdict"] == CORRECTED and rep["located"] == [0, 4]
    pair.regenerate(BWD, res)
    assert rel_fro(pair.ora.Wt, clean) <= 1e-8
    pair.check_weights(1e-5)
    pair.close()


# ------------------------------------------------------------ exhaustive campaigns
@pytest.mark.parametrize("m,r,dtype", [(4, 2, "f32"), (8, 2, "bf16"), (3, 4, "f32")])
def test_every_error_pattern_on_a_small_grid(m, r, dtype):
    """All supports up to size r: within capability (<= t) located exactly and
    corrected, beyond it UNCORRECTABLE -- identical to the oracle every time."""
    t, L = r // 2, m + r
    P = WL.vandermonde_like(m, r) if r <= 2 else WL.gaussian_generator(m, r, 8)
    n_out = n_in = 64 * m
    tau = (1e-3, 2e-3) if dtype == "f32" else (2e-2, 2e-2)
    pair = Pair(WL.layer_weights(n_out, n_in), P, P, dtype, 24, *tau)
    X = WL.normal((24, n_in), 5)
    D = WL.normal((24, n_out), 6)
    count = 0
    for k in range(1, min(r, t + 1) + 1):
        for A in itertools.combinations(range(L), k):
            say("campaign", m, r, dtype, "support", A)
            faults = [WL.make_fault(FWD, i, (i + k) % m, step=count) for i in A]
            _, rep, _ = pair.product(FWD, X, faults)
            assert rep["verdict"] == (CORRECTED if k <= t else UNCORRECTABLE)
            assert rep["located"] == (list(A) if k <= t else [])
            if k == 1:
                faults = [WL.make_fault(BWD, (A[0] + 1) % m, A[0], step=count)]
                _, rep, _ = pair.product(BWD, D, faults)
                assert rep["verdict"] == CORRECTED and rep["located"] == list(A)
            count += 1
    pair.close()


def test_largest_parity_count_four_blocks_located_and_regenerated():
    """The limits of the interface: r = 8 parity blocks, t = 4.  Four erroneous block-rows
    (systematic and parity) are located and corrected, five are not; four block-rows hit by
    weight faults are located by the next product and regenerated in one call."""
    m, r, b = 12, 8, 8
    P = WL.gaussian_generator(m, r, 12)
    n_out = n_in = 16 * m
    pair = Pair(WL.layer_weights(n_out, n_in), P, P, "f32", b)
    X = WL.normal((b, n_in), 31)
    rows = [0, 5, 11, m + 3]
    _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, i, 1, 0) for i in rows])
    assert rep["verdict"] == CORRECTED and rep["located"] == rows
    _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, i, 1, 1) for i in rows + [7]])
    assert rep["verdict"] == UNCORRECTABLE and rep["located"] == []
    clean = pair.ora.Wt.copy()
    pair.inject_weights([WL.make_fault(WEIGHT, i, j, 2) for i in rows for j in range(m)])
    _, rep, res = pair.product(FWD, X)
    assert rep["verdict"] == CORRECTED and rep["located"] == rows
    pair.regenerate(FWD, res)
    assert rel_fro(pair.ora.Wt, clean) <= 1e-8
    assert rel_fro(to_np(pair.gpu.export_coded()), clean) <= 1e-4
    _, rep, _ = pair.product(FWD, X)
    assert rep["verdict"] == CLEAN
    pair.close()


def test_longest_codeword():
    """The longest codeword the interface takes, m + r = n + r = 40 blocks, in both dimensions (the
    kernels walk the blocks in chunks of 8 and 16: last chunk full, indices clamped at the end):
    clean products, one corrected block at either end of the codeword, two with t = 2, update."""
    m, n, b = 38, 36, 5
    P_r, P_c = WL.vandermonde_like(m, 2), WL.gaussian_generator(n, 4, 21)
    n_out, n_in = 4 * m, 8 * n - 3            # the last block-column is ragged
    pair = Pair(WL.layer_weights(n_out, n_in), P_r, P_c, "f32", b)
    assert pair.gpu.coded_rows == 40 * pair.gpu.B_r and pair.gpu.coded_cols == 40 * pair.gpu.B_c
    pair.check_weights(1e-6)
    X, D = WL.normal((b, n_in), 51), WL.normal((b, n_out), 52)
    for step, (rows, cols) in enumerate((((), ()), ((0,), (0, 39)), ((39,), (17, 35)), ((38,), (36,)))):
        _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, i, 0, step) for i in rows])
        assert rep["verdict"] == (CORRECTED if rows else CLEAN) and rep["located"] == list(rows)
        _, rep, _ = pair.product(BWD, D, [WL.make_fault(BWD, 0, j, step) for j in cols])
        assert rep["verdict"] == (CORRECTED if cols else CLEAN) and rep["located"] == list(cols)
        pair.update(0.05)
        pair.check_weights()
    _, rep, _ = pair.product(FWD, X, [WL.make_fault(FWD, 3, 0, 9), WL.make_fault(FWD, 30, 0, 9)])
    assert rep["verdict"] == UNCORRECTABLE
    pair.close()


@pytest.mark.parametrize("seed", [7, 2026])
def test_random_ragged_layers_agree_with_the_oracle(seed):
    """Seeded random layers -- grids up to 11 x 11, r in {1, 2, 4}, nothing dividing anything, batches
    from 1 to 260, both dtypes -- two steps each with up to t + 1 faulty blocks per product, plain and
    verified checks, regeneration after every forward check, update: verdicts, located sets, outputs
    and coded weights as the oracle's every time.  Grids and generators here are drawn, not chosen for
    the separation of their columns: every thresholded quantity is asked to clear its threshold by a
    factor 2 instead of the 5 that the workloads' own codes are held to."""
    g = np.random.default_rng(seed)
    for case in range(25):
        m, n = int(g.integers(1, 12)), int(g.integers(1, 12))
        r = int(g.choice([1, 2, 2, 2, 4]))
        n_out = max(int(m * g.integers(1, 40) + g.integers(0, m)), m)
        n_in = max(int(n * g.integers(1, 40) + g.integers(0, n)), n)
        b = int(g.choice([1, 3, 8, 17, 64, 130, 260]))
        dtype = "bf16" if g.random() < 0.4 else "f32"
        if r <= 2:
            P_r, P_c = WL.vandermonde_like(m, r), WL.vandermonde_like(n, r)
        else:
            P_r, P_c = WL.gaussian_generator(m, r, 100 + case), WL.gaussian_generator(n, r, 200 + case)
        tau = (1e-3, 2e-3) if dtype == "f32" else (2e-2, 2e-2)
        say("random layer", seed, case, n_out, n_in, m, n, r, b, dtype)
        pair = Pair(WL.layer_weights(n_out, n_in), P_r, P_c, dtype, b, *tau)
        X, D = WL.normal((b, n_in), 300 + case), WL.normal((b, n_out), 400 + case)
        t = r // 2
        for step in range(2):
            rows = sorted(g.choice(m + r, size=min(int(g.integers(0, t + 2)), m + r), replace=False).tolist())
            faults = [WL.make_fault(FWD, i, int(g.integers(0, n)), step) for i in rows]
            _, _, res = pair.product(FWD, X, faults, check_margins=2.0, verified=bool(g.integers(0, 2)))
            pair.regenerate(FWD, res)
            cols = sorted(g.choice(n + r, size=min(int(g.integers(0, t + 2)), n + r), replace=False).tolist())
            faults = [WL.make_fault(BWD, int(g.integers(0, m)), j, step) for j in cols]
            pair.product(BWD, D, faults, check_margins=2.0)
            pair.update(0.05)
            pair.check_weights()
        pair.close()


# --------------------------------------------------------- multi-step, scaled copies
@pytest.mark.parametrize("name,block", [("cfg3", 64), ("cfg5", 32), ("cfg4", 32)])
def test_multi_step_on_a_width_scaled_copy(name, block):
    """Same grid, parity count, dtype, thresholds, fault law and number of steps (50 / 200 / 20) as
    the full workload with blocks of `block`: the oracle follows every step; where the workload
    asks for a drift check (cfg5: every 50 steps) the stored matrix is also compared with the
    oracle's encoding of its own systematic part."""
    from oracle import codenet_oracle as O
    full = WL.WORKLOADS[name]
    wl = full.scaled(block, batch=min(full.batch, 96))
    assert wl.steps == full.steps
    P_r, P_c = wl.generators()
    n_in, n_out = wl.widths[0], wl.widths[1]
    m, n = wl.grid
    pair = Pair(WL.layer_weights(n_out, n_in), P_r, P_c, wl.dtype, wl.batch, wl.tau_detect, wl.tau_resid)
    verdicts = []
    for step in range(wl.steps):
        say(name, "scaled step", step)
        rf, rb = layer_step(pair, wl, step, n_out=n_out, n_in=n_in)
        verdicts += [rf["verdict"], rb["verdict"]]
        pair.check_weights()
        if wl.drift_every and (step + 1) % wl.drift_every == 0:
            Wc = to_np(pair.gpu.export_coded())
            again = O.encode(Wc[: m * pair.gpu.B_r, : n * pair.gpu.B_c], P_r, P_c, pair.gpu.B_r, pair.gpu.B_c)
            drift = rel_fro(Wc, again)
            say(name, "scaled copy: drift after", step + 1, "steps %.3e" % drift)
            assert drift <= pair.tol
    say(name, "verdicts", verdicts)
    assert len(set(verdicts)) >= 2
    pair.close()


def test_weight_fault_shows_up_in_the_next_products():
    """An update-stage error corrupts a stored block; it is seen at the next
    forward product (block-row bi) and, for a base-row block, at the next
    backward product (block-column bj)."""
    m = n = 4
    P = WL.vandermonde_like(m, 2)
    pair = Pair(WL.layer_weights(256, 256), P, P, "f32", 32)
    X, D = WL.normal((32, 256), 21), WL.normal((32, 256), 22)
    pair.product(FWD, X)
    pair.product(BWD, D)
    pair.update(0.01)
    pair.inject_weights([WL.make_fault(WEIGHT, 2, 1, step=0)])
    pair.check_weights()
    _, rep, _ = pair.product(FWD, X)
    assert rep["verdict"] == CORRECTED and rep["located"] == [2]
    _, rep, _ = pair.product(BWD, D)
    assert rep["verdict"] == CORRECTED and rep["located"] == [1]
    # the paper's sparse law on a parity-column block: only the backward product sees it
    pair.inject_weights([WL.make_fault(WEIGHT, 0, 5, step=1, lo=-5.0, hi=5.0, mode=WL.MODE_SPARSE_ABS, density=0.005)])
    pair.check_weights()
    # (no margin asked here: the sparse law's few small hits on a parity-column block are a fault that the
    # threshold margin was not designed around -- the verdict and located set must still be the oracle's)
    _, rep, _ = pair.product(BWD, D, check_margins=False)
    assert rep["verdict"] == UNCORRECTABLE        # columns 1 and 5 are now both erroneous, t = 1
    pair.close()


# ------------------------------------------------------------------ regeneration of located blocks
@pytest.mark.parametrize("N_out,N_in,m,n,r,b,dtype,bad", [
    (96, 80, 4, 4, 2, 8, "f32", [(FWD, [1])]),                 # a systematic block-row
    (96, 80, 4, 4, 2, 8, "f32", [(FWD, [5])]),                 # a parity block-row
    (96, 80, 4, 4, 2, 8, "f32", [(BWD, [2])]),                 # a systematic block-column
    (300, 200, 5, 4, 2, 33, "bf16", [(FWD, [0]), (BWD, [4])]),   # ragged, bf16 copy refreshed, both axes in turn
    (130, 70, 3, 3, 4, 5, "f32", [(FWD, [0, 2])]),             # two systematic block-rows (t = 2)
    (130, 70, 3, 3, 4, 5, "f32", [(BWD, [1, 5])]),             # a systematic and a parity block-column
    (1024, 1024, 8, 8, 2, 64, "bf16", [(FWD, [3]), (BWD, [9])]),   # several 64 x 64 tiles per block
])
def test_regeneration_restores_the_stored_code(N_out, N_in, m, n, r, b, dtype, bad):
    """Weight faults on several nodes of one block-row (column) persist: the next
    product locates that row (column), the regeneration rebuilds its stored blocks, and
    the stored matrix is the clean code again on both sides; the following products are
    clean.  A regeneration call after a CLEAN verdict changes nothing, bit for bit."""
    import torch
    P_r = WL.vandermonde_like(m, r) if r <= 2 else WL.gaussian_generator(m, r, seed=5)
    P_c = WL.vandermonde_like(n, r) if r <= 2 else WL.gaussian_generator(n, r, seed=6)
    tau = (2e-2, 2e-2) if dtype == "bf16" else (1e-3, 2e-3)
    pair = Pair(WL.layer_weights(N_out, N_in), P_r, P_c, dtype, b, *tau)
    clean = pair.ora.Wt.copy()
    step = 0
    for phase, lines in bad:
        # corrupt every stored block of the chosen block-rows (columns) that a product of this phase reads
        faults = []
        for line in lines:
            others = range(n) if phase == FWD else range(m)
            for o in others:
                bi, bj = (line, o) if phase == FWD else (o, line)
                faults.append(WL.make_fault(WL.PHASE_WEIGHT, bi, bj, step))
        pair.inject_weights(faults)
        pair.check_weights(1e-5)
        V = WL.normal((b, N_in if phase == FWD else N_out), seed=100 + step)
        _, rep, res = pair.product(phase, V)
        assert rep["verdict"] == CORRECTED and rep["located"] == sorted(lines), rep
        pair.regenerate(phase, res)
        assert rel_fro(pair.ora.Wt, clean) <= 1e-9
        err = pair.check_weights(1e-5)
        assert rel_fro(to_np(pair.gpu.export_coded()), clean) <= 1e-5
        # the copy that the bf16 products read was refreshed too: both products are clean again
        for ph in (FWD, BWD):
            V = WL.normal((b, N_in if ph == FWD else N_out), seed=200 + step + ph)
            _, rep, res = pair.product(ph, V)
            assert rep["verdict"] == CLEAN, rep
        before = pair.gpu.export_coded().clone()
        pair.regenerate(BWD, res)              # verdict CLEAN: nothing to do
        # a report whose located set does not fit the code is ignored as well
        from paper_1903_01042_amd import binding as B
        for located in ([m + n + 2 * r + 5], [0, 0], list(range(r // 2 + 1))):
            bogus = B.Report(verdict=CORRECTED, n_located=len(located))
            for q, i in enumerate(located[:4]):
                bogus.located[q] = i
            raw = torch.frombuffer(bytearray(bytes(bogus)), dtype=torch.uint8).cuda()
            pair.gpu.regenerate(FWD, raw)
        torch.cuda.synchronize()
        assert torch.equal(before, pair.gpu.export_coded())
        step += 1
    pair.close()


def test_device_time_stamps_bracket_a_call():
    """Two stamps around an update: a positive, plausible number of ticks of a clock whose
    rate the call reports; NULL destination is refused."""
    import torch
    from paper_1903_01042_amd import binding as B
    P = WL.vandermonde_like(4, 2)
    lay = B.CodedLayer(torch.zeros((512, 512), device="cuda"), P, P, max_batch=64)
    lay.forward(torch.zeros((64, 512), device="cuda"))
    lay.backward(torch.zeros((64, 512), device="cuda"))
    stamps = torch.zeros(2, dtype=torch.int64, device="cuda")
    rate = B.timestamp(stamps, 0)
    lay.update(0.1)
    B.timestamp(stamps, 1)
    torch.cuda.synchronize()
    a, b = (int(v) for v in stamps.cpu())
    assert rate >= 1 and a > 0
    assert 0 < (b - a) / rate < 5000.0, (a, b, rate)        # microseconds
    assert B.load_library().codenet_timestamp(None, None, None) == B.E_NULL
    lay.destroy()


# ------------------------------------------------------------------ elementwise step fused into the check
@pytest.mark.parametrize("n_out,n_in,m,n,r,b,dtype", [
    (512, 384, 4, 4, 2, 64, "f32"),       # aligned: float4 path
    (100, 52, 3, 5, 2, 7, "f32"),         # nothing divides anything: scalar path
    (300, 200, 5, 4, 2, 33, "bf16"),
])
def test_activation_fused_into_the_check(n_out, n_in, m, n, r, b, dtype):
    """ReLU on the decoded forward output, g(x) (.) c and a general multiplier on the decoded
    backward output, with and without a corrected fault; the coded buffer keeps the values
    before the elementwise step."""
    from paper_1903_01042_amd import binding as B
    P_r, P_c = WL.vandermonde_like(m, r), WL.vandermonde_like(n, r)
    tau = (1e-3, 2e-3) if dtype == "f32" else (2e-2, 2e-2)
    pair = Pair(WL.layer_weights(n_out, n_in), P_r, P_c, dtype, b, *tau)
    X, D = WL.normal((b, n_in), 21), WL.normal((b, n_out), 22)
    for faults_f, faults_b in (((), ()), ([WL.make_fault(FWD, 1, 0, 3)], [WL.make_fault(BWD, 0, n, 3)])):
        dec, rep, res = pair.product(FWD, X, faults_f, epilogue=B.EPI_RELU)
        assert rep["verdict"] == (CORRECTED if faults_f else CLEAN)
        got = to_np(dec)
        assert (got >= 0).all() and (got == 0).any() and (got > 0).any()
        dec, rep, _ = pair.product(BWD, D, faults_b, epilogue=B.EPI_MASK_POS, aux=X)
        assert rep["verdict"] == (CORRECTED if faults_b else CLEAN)
        assert (to_np(dec)[X <= 0] == 0).all()
        pair.product(BWD, D, faults_b, epilogue=B.EPI_MUL, aux=WL.normal((b, n_in), 23))
    lay = pair.gpu
    out = lay.forward(pair.dev_tensor(X))
    lib, vp = B.load_library(), __import__("ctypes").c_void_p
    dec = pair.dev_tensor(np.zeros((b, n_out)))
    args = (lay._h, B.FWD, vp(out.data_ptr()), b)
    assert lib.codenet_detect_decode_act(*args, vp(dec.data_ptr()), None, B.EPI_MUL, None, None) == B.E_NULL
    assert lib.codenet_detect_decode_act(*args, None, None, B.EPI_RELU, None, None) == B.E_NULL
    assert lib.codenet_detect_decode_act(*args, vp(dec.data_ptr()), None, 7, None, None) == B.E_DTYPE
    pair.close()


# ------------------------------------------- verification steps of Error Model 2
@pytest.mark.parametrize("n_out,n_in,m,n,r,b,dtype", [
    (256, 192, 4, 3, 2, 16, "f32"),       # 4 workgroups in the check
    (1024, 1024, 8, 8, 2, 128, "bf16"),   # 16 workgroups
    (320, 256, 4, 4, 4, 9, "f32"),        # t = 2 (generic decision); one workgroup of work, two evaluators
    (100, 52, 3, 5, 2, 7, "f32"),         # ragged blocks
])
def test_verified_check_agrees_or_reports_the_disagreement(n_out, n_in, m, n, r, b, dtype):
    """Without planted errors the verified check gives exactly the plain one (clean, corrected,
    uncorrectable; with a fused activation); an error planted in either evaluation of the checks or
    in any evaluator's list gives DISAGREE on both sides, and the next check is back to normal."""
    from paper_1903_01042_amd import binding as B
    if r <= 2:
        P_r, P_c = WL.vandermonde_like(m, r), WL.vandermonde_like(n, r)
    else:
        P_r, P_c = WL.gaussian_generator(m, r, 8), WL.gaussian_generator(n, r, 9)
    tau = (1e-3, 2e-3) if dtype == "f32" else (2e-2, 2e-2)
    pair = Pair(WL.layer_weights(n_out, n_in), P_r, P_c, dtype, b, *tau)
    X, D = WL.normal((b, n_in), 31), WL.normal((b, n_out), 32)
    t = r // 2
    one_f, one_b = [WL.make_fault(FWD, 1, 0, 5)], [WL.make_fault(BWD, 0, n, 5)]
    many_f = [WL.make_fault(FWD, i, 0, 6) for i in range(t + 1)]
    for faults_f, faults_b, want in (((), (), CLEAN), (one_f, one_b, CORRECTED), (many_f, (), UNCORRECTABLE)):
        _, rep, _ = pair.product(FWD, X, faults_f, verified=True, epilogue=B.EPI_RELU)
        assert rep["verdict"] == want
        if want != UNCORRECTABLE:
            _, rep, _ = pair.product(BWD, D, faults_b, verified=True)
            assert rep["verdict"] == want
    for faults_f in ((), one_f, many_f):
        for fault in (dict(target=B.CHECK_EVALUATION, who=0, seed=1, hi=0.5),
                      dict(target=B.CHECK_EVALUATION, who=1, seed=2, hi=1e-6),
                      dict(target=B.CHECK_LIST, who=0, hi=0.0),
                      dict(target=B.CHECK_LIST, who=3, hi=0.0)):
            _, rep, _ = pair.product(FWD, X, faults_f, verified=True, check_fault=fault)
            assert rep["verdict"] == B.DISAGREE and rep["n_located"] == 0, (faults_f, fault, rep)
            # the planted error is used up: the same product checks normally again
            _, rep, _ = pair.product(FWD, X, faults_f, verified=True)
            assert rep["verdict"] != B.DISAGREE
    # a pending CHECK fault waits for the next verified call; plain calls ignore it
    pair.gpu.inject([dict(phase=B.CHECK, bi=B.CHECK_LIST, bj=0, seed=0, step=0, lo=0.0, hi=0.0)])
    _, rep, _ = pair.product(FWD, X)
    assert rep["verdict"] == CLEAN
    out = pair.gpu.forward(pair.dev_tensor(X))
    pair.gpu.detect_decode(FWD, out, report=pair.report, verified=True)
    assert pair.gpu.read_report(pair.report)["verdict"] == B.DISAGREE
    lib, vp = B.load_library(), __import__("ctypes").c_void_p
    assert lib.codenet_detect_decode_verified(pair.gpu._h, B.FWD, vp(out.data_ptr()), b, None, None, 0, None,
                                              None) == B.E_NULL
    bad = B.pack_faults([dict(phase=B.CHECK, bi=2, bj=0, seed=0, step=0, lo=0.0, hi=0.0)])
    assert lib.codenet_inject(pair.gpu._h, bad, 1, None, 0, None) == B.E_FAULT
    two = B.pack_faults([dict(phase=B.CHECK, bi=0, bj=0, seed=0, step=0, lo=0.0, hi=0.1)] * 2)
    assert lib.codenet_inject(pair.gpu._h, two, 2, None, 0, None) == B.E_SHAPE
    pair.close()


# ------------------------------------------------------------------ checks evaluated in the product's epilogue
def test_checks_taken_in_the_product_epilogue():
    """bf16 layers whose row code fits the codeword-interleaved product kernel (at most ten blocks,
    four parity blocks) evaluate the consistency checks of the forward product in its epilogue; the
    check call then starts from those records.  Same verdicts, syndromes' effect and outputs as the
    stand-alone first pass (which is forced by checking a copy of the output in another buffer);
    records are dropped by injection and by a check; a buffer changed behind the library's back needs
    codenet_output_modified(); the decoded output may stay in place.  The backward product leaves no
    records: its check always reads the output."""
    import torch
    from paper_1903_01042_amd import binding as B
    for (n_out, n_in, m, n, r, b) in ((512, 384, 8, 6, 2, 96), (192, 320, 3, 5, 4, 70), (1024, 1024, 8, 8, 2, 200),
                                      (200, 150, 8, 6, 2, 130), (77, 90, 7, 3, 1, 64)):
        say("fused checks", n_out, n_in, m, n, r, b)
        P_r = WL.vandermonde_like(m, r) if r <= 2 else WL.gaussian_generator(m, r, 8)
        P_c = WL.vandermonde_like(n, r) if r <= 2 else WL.gaussian_generator(n, r, 9)
        pair = Pair(WL.layer_weights(n_out, n_in), P_r, P_c, "bf16", b, 2e-2, 2e-2)
        lay = pair.gpu
        X, D = WL.normal((b, n_in), 61), WL.normal((b, n_out), 62)
        # through the harness: clean products use the epilogue's records, faulty ones the stand-alone pass
        campaign = (((), ()), ([WL.make_fault(FWD, 1, 0, 3)], [WL.make_fault(BWD, 0, n, 3)]), ((), ()))
        for faults_f, faults_b in (campaign if r >= 2 else campaign[:1]):
            pair.product(FWD, X, faults_f, check_margins=True if r <= 2 else 2.0)
            pair.product(BWD, D, faults_b, check_margins=True if r <= 2 else 2.0)
            pair.update(0.02)
            pair.check_weights()
        rep_a, rep_b = lay.new_report(), lay.new_report()
        for phase, V in ((FWD, X), (BWD, D)):
            Vd = pair.dev_tensor(V)
            out = lay.forward(Vd) if phase == FWD else lay.backward(Vd)
            other = out.clone()                                   # another buffer: not the one the product wrote
            dec_b = lay.detect_decode(phase, other, report=rep_b)             # stand-alone first pass
            dec_a = lay.detect_decode(phase, out, report=rep_a)               # the epilogue's records
            ra, rb = lay.read_report(rep_a), lay.read_report(rep_b)
            assert ra["verdict"] == rb["verdict"] == CLEAN
            assert np.allclose(ra["syn_rel"], rb["syn_rel"], rtol=1e-4, atol=1e-9), (ra, rb)
            assert torch.equal(dec_a, dec_b)
            # a change behind the library's back: unseen until the library is told
            blk = lay.B_r if phase == FWD else lay.B_c
            out = lay.forward(Vd) if phase == FWD else lay.backward(Vd)
            out[:, blk:2 * blk] += 5.0 * out[:, blk:2 * blk].std()
            want = CORRECTED if r >= 2 else UNCORRECTABLE
            if phase == FWD:
                lay.detect_decode(phase, out, report=rep_a, want_decoded=False)
                assert lay.read_report(rep_a)["verdict"] == CLEAN             # stale records: documented hazard
            lay.detect_decode(phase, out, report=rep_a, want_decoded=False)   # the records are gone after one check
            got = lay.read_report(rep_a)
            assert got["verdict"] == want and (r < 2 or got["located"] == [1])
            out = lay.forward(Vd) if phase == FWD else lay.backward(Vd)
            out[:, blk:2 * blk] += 5.0 * out[:, blk:2 * blk].std()
            lay.output_modified(phase)
            lay.detect_decode(phase, out, report=rep_a, want_decoded=False)
            got = lay.read_report(rep_a)
            assert got["verdict"] == want and (r < 2 or got["located"] == [1])
            # decoded in place: nothing copied; with ReLU the systematic part is rectified where it is
            out = lay.forward(Vd) if phase == FWD else lay.backward(Vd)
            ref = out.clone()
            same = lay.detect_decode(phase, out, decoded=out, report=rep_a)
            assert same.data_ptr() == out.data_ptr() and torch.equal(out, ref)
            if phase == FWD:
                lay.detect_decode(phase, out, decoded=out, report=rep_a, epilogue=B.EPI_RELU)
                sys_cols = pair.ora.m * lay.B_r
                assert torch.equal(out[:, :sys_cols], torch.relu(ref[:, :sys_cols]))
                assert torch.equal(out[:, sys_cols:], ref[:, sys_cols:])
        pair.close()


def test_a_decoded_output_left_in_place_feeds_the_next_layer():
    """Two layers in a row, both arithmetic modes: the first layer's check leaves its decoded output in
    the coded buffer (with the activation applied where it is) and the second layer's forward product
    takes it from there as an input with a row pitch (codenet_forward_ld); on the way back the second
    layer's decoded backward output stays in place and feeds the first layer's backward product
    (codenet_backward_ld).  Bit for bit the results of the same chain through dense decoded copies."""
    import torch
    from paper_1903_01042_amd import binding as B
    for dtype, taus in ((B.F32, (1e-3, 2e-3)), (B.BF16_F32ACC, (2e-2, 2e-2))):
        say("in-place chain, dtype", dtype)
        n0, n1, n2, b = 320, 512, 256, 96
        dev = torch.device("cuda")
        P4, P8 = WL.vandermonde_like(4, 2), WL.vandermonde_like(8, 2)
        l1 = B.CodedLayer(torch.from_numpy(WL.layer_weights(n1, n0)).to(dev), P8, P4, dtype=dtype, max_batch=b,
                          tau_detect=taus[0], tau_resid=taus[1])
        l2 = B.CodedLayer(torch.from_numpy(WL.layer_weights(n2, n1, 1)).to(dev), P4, P8, dtype=dtype, max_batch=b,
                          tau_detect=taus[0], tau_resid=taus[1])
        assert l1.B_r * 8 == n1 and l2.B_c * 8 == n1          # no padding inside the blocks of the shared width
        X = torch.from_numpy(WL.normal((b, n0), 5)).to(dev)
        D = torch.from_numpy(WL.normal((b, n2), 6)).to(dev)
        rep = l1.new_report()
        # dense chain
        s1 = l1.forward(X)
        l1.inject([WL.make_fault(FWD, 2, 1, 0)], s1)
        x1 = l1.detect_decode(FWD, s1, report=rep, epilogue=B.EPI_RELU)
        s2 = l2.forward(x1)
        c2 = l2.backward(D)
        l2.inject([WL.make_fault(BWD, 1, 3, 0)], c2)
        d1 = l2.detect_decode(BWD, c2, report=rep)
        c1 = l1.backward(d1)
        # the same chain in place
        t1 = l1.forward(X)
        l1.inject([WL.make_fault(FWD, 2, 1, 0)], t1)
        l1.detect_decode(FWD, t1, decoded=t1, report=rep, epilogue=B.EPI_RELU)
        assert l1.read_report(rep)["verdict"] == CORRECTED
        t2 = l2.forward(t1[:, :n1])
        e2 = l2.backward(D)
        l2.inject([WL.make_fault(BWD, 1, 3, 0)], e2)
        l2.detect_decode(BWD, e2, decoded=e2, report=rep)
        assert l2.read_report(rep)["verdict"] == CORRECTED
        e1 = l1.backward(e2[:, :n1])
        assert torch.equal(t1[:, :n1], x1) and torch.equal(t2, s2) and torch.equal(e2[:, :n1], d1) and torch.equal(e1, c1)
        with pytest.raises(ValueError):
            l2.forward(t1[:, 1:n1 + 1].t())
        l1.destroy()
        l2.destroy()


# ------------------------------------------------------------------ API error paths
def test_api_errors_on_the_gpu():
    import torch
    from paper_1903_01042_amd import binding as B
    P = WL.vandermonde_like(2, 2)
    W = torch.zeros((64, 64), device="cuda")
    lay = B.CodedLayer(W, P, P, max_batch=8)
    with pytest.raises(B.CodenetError) as e:
        lay.update(0.1)
    assert e.value.code == B.E_ORDER
    with pytest.raises(B.CodenetError) as e:
        lay.forward(torch.zeros((9, 64), device="cuda"))
    assert e.value.code == B.E_BATCH
    S = lay.forward(torch.zeros((8, 64), device="cuda"))
    with pytest.raises(B.CodenetError) as e:
        lay.update(0.1)                      # forward only
    assert e.value.code == B.E_ORDER
    lay.backward(torch.zeros((4, 64), device="cuda"))
    with pytest.raises(B.CodenetError) as e:
        lay.update(0.1)                      # batches differ
    assert e.value.code == B.E_ORDER
    with pytest.raises(B.CodenetError) as e:
        lay.inject([WL.make_fault(FWD, 1, 2, 0)], S)      # column 2 is a parity column: inactive in forward
    assert e.value.code == B.E_FAULT
    with pytest.raises(B.CodenetError) as e:
        lay.inject([WL.make_fault(WEIGHT, 3, 3, 0)])      # corner holds no node
    assert e.value.code == B.E_FAULT
    with pytest.raises(B.CodenetError) as e:
        B.CodedLayer(W, np.array([[1.0, 2.0], [1.0, 2.0]]), P, max_batch=8)
    assert e.value.code == B.E_CODE
    torch.cuda.synchronize()
    lay.destroy()


# ------------------------------------------------------------------ hipGraph replay
def test_graph_replay_matches_eager_calls():
    """The calls only enqueue kernels, so a whole step can be captured in a hipGraph.
    Each replay (with unrelated eager work and synchronisations in between) must give
    exactly what the same calls give when launched one by one on a twin layer."""
    import torch
    from paper_1903_01042_amd import binding as B
    wl = WL.WORKLOADS["cfg3"].scaled(64, batch=96)
    n_in, n_out = wl.widths[0], wl.widths[1]
    P_r, P_c = wl.generators()
    dev = torch.device("cuda:0")
    W = torch.from_numpy(WL.layer_weights(n_out, n_in)).to(dev)
    mk = lambda: B.CodedLayer(W, P_r, P_c, dtype=B.BF16_F32ACC, max_batch=wl.batch,
                              tau_detect=wl.tau_detect, tau_resid=wl.tau_resid)
    eager, graphed = mk(), mk()
    X = torch.from_numpy(wl.inputs(0)).to(dev)
    D = torch.from_numpy(wl.deltas(0)).to(dev)
    fw = [WL.make_fault(FWD, 3, 1, 0)]
    bw = [WL.make_fault(BWD, 2, 9, 0)]

    def step(lay, bufs):
        S, C, dS, dC, r1, r2 = bufs
        lay.forward(X, S)
        lay.inject(fw, S)
        lay.detect_decode(B.FWD, S, decoded=dS, report=r1)
        lay.backward(D, C)
        lay.inject(bw, C)
        lay.detect_decode(B.BWD, C, decoded=dC, report=r2)
        lay.update(wl.eta)

    def bufs(lay):
        e = lambda *s: torch.empty(s, dtype=torch.float32, device=dev)
        return (e(wl.batch, lay.coded_rows), e(wl.batch, lay.coded_cols), e(wl.batch, n_out), e(wl.batch, n_in),
                lay.new_report(), lay.new_report())

    be, bg = bufs(eager), bufs(graphed)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(graphed, bg)                      # first use outside capture
    side.synchronize()
    step(eager, be)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step(graphed, bg)
    torch.cuda.synchronize()
    step(eager, be)                            # capture does not execute: the twin is now one step ahead
    for it in range(3):
        say("graph replay", it)
        g.replay()
        if it > 0:
            step(eager, be)
        junk = torch.randn(1 << 20, device=dev).sum()      # unrelated eager work between replays
        torch.cuda.synchronize()
        assert junk.isfinite()
        for a, b in zip(be[:4], bg[:4]):
            assert torch.equal(a, b)
        assert eager.read_report(be[4]) == graphed.read_report(bg[4])
        assert eager.read_report(be[5]) == graphed.read_report(bg[5])
        assert torch.equal(eager.export_coded(), graphed.export_coded())
    eager.destroy()
    graphed.destroy()
