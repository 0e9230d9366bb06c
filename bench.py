#!/usr/bin/env python3
"""Benchmark of the coded layer step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
coded forward product, fault injection, check + decode, coded backward product,
fault injection, check + decode, coded update.  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3]

Single-layer workloads (cfg1, cfg3, cfg5) time that layer's step.  The MLP workloads (cfg2:
784-1024-1024-10; cfg4: 8 layers of width 8192) time whole training iterations -- feedforward
through all layers with the activation fused into each check, loss head, backpropagation with
g(x) (.) c fused into each check, update of every layer -- and report layer-steps per second
(iterations x layers).  `--workload cfg4 --layers 1` is one layer of that network.
"""
import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
SAMPLED_STEPS = 8          # timed steps on which a kernel is bracketed (4 in runs of fewer than 64 steps)
PREWARM_SECONDS = 0.3      # untimed steps before the warm-up: the chip reaches its steady clocks


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="cfg3", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--layers", type=int, default=0, help="MLP workloads: only the first LAYERS layers (0 = all)")
    ap.add_argument("--cpu-steps", type=int, default=-1,
                    help="oracle layer-steps timed for cpu_baseline (0 = skip, -1 = sized to the workload)")
    ap.add_argument("--no-faults", action="store_true", help="run the coded path without injecting faults")
    ap.add_argument("--coded-only", action="store_true", help="skip the uncoded baseline and the CPU oracle (profiling runs)")
    ap.add_argument("--no-prewarm", action="store_true", help="skip the untimed steps that precede the warm-up")
    ap.add_argument("--strategies", action="store_true",
                    help="strategy comparison on the cfg2 network: CodeNet (t = 1), replication (two replicas, compare, "
                         "roll back) and uncoded (errors ignored), time to --steps iterations over a sweep of checkpoint "
                         "periods, next to the expected-time model of Theorem 2")
    ap.add_argument("--fault-p", type=float, default=0.002, help="--strategies: failure probability per node and product")
    ap.add_argument("--graph", action="store_true",
                    help="single-layer workloads: replay one hipGraph per step instead of launching every call from "
                         "Python (a kernel node of a graph takes about 3 us longer than the same kernel launched into "
                         "the stream; the step is not launch bound, so the default is the plain stream)")
    return ap.parse_args()


def sampled(steps, warmup, count=SAMPLED_STEPS, phase=0.5):
    """`count` step indices spread evenly over the timed region [warmup, warmup + steps)."""
    count = min(count, steps)
    return sorted({warmup + min(steps - 1, int((k + phase) * steps / count)) for k in range(count)})


class Runner:
    """Pre-marshalled calls of one single-layer workload (coded or uncoded)."""

    RING = 8

    def __init__(self, wl, coded, faults_on, total_steps, verified=False, in_place=False):
        import torch
        from paper_1903_01042_amd import binding as B
        from paper_1903_01042_amd import workloads as WL
        self.torch, self.B, self.wl, self.WL = torch, B, wl, WL
        self.lib = B.load_library()
        dev = torch.device("cuda:0")
        n_in, n_out = wl.widths[0], wl.widths[1]
        m, n = wl.grid
        self.b = wl.batch
        self.coded = coded
        self.verified = verified   # checks with the verification steps of Error Model 2
        self.in_place = in_place   # the decoded output stays in the coded buffer (no dense copy)
        W = torch.from_numpy(WL.layer_weights(n_out, n_in)).to(dev)
        if coded:
            P_r, P_c = wl.generators()
        else:
            P_r, P_c = np.zeros((m, 0)), np.zeros((n, 0))
        self.layer = B.CodedLayer(W, P_r, P_c, dtype=B.BF16_F32ACC if wl.dtype == "bf16" else B.F32,
                                  max_batch=wl.batch, tau_detect=wl.tau_detect, tau_resid=wl.tau_resid)
        L = self.layer
        self.X = [torch.from_numpy(wl.inputs(s)).to(dev) for s in range(self.RING)]
        self.D = [torch.from_numpy(wl.deltas(s)).to(dev) for s in range(self.RING)]
        self.St = torch.empty((self.b, L.coded_rows), dtype=torch.float32, device=dev)
        self.Ct = torch.empty((self.b, L.coded_cols), dtype=torch.float32, device=dev)
        self.S = torch.empty((self.b, n_out), dtype=torch.float32, device=dev)
        self.C = torch.empty((self.b, n_in), dtype=torch.float32, device=dev)
        self.reports = torch.zeros((total_steps + 1, 2, B.REPORT_BYTES), dtype=torch.uint8, device=dev)
        self.total_steps = total_steps
        self.faults = []
        for s in range(total_steps):
            ff = wl.product_faults(WL.PHASE_FWD, s) if (coded and faults_on) else []
            fb = wl.product_faults(WL.PHASE_BWD, s) if (coded and faults_on) else []
            self.faults.append(((B.pack_faults(ff), len(ff)), (B.pack_faults(fb), len(fb))))
        self.h = L._h
        vp = ctypes.c_void_p
        self.pX = [vp(t.data_ptr()) for t in self.X]
        self.pD = [vp(t.data_ptr()) for t in self.D]
        self.pSt, self.pCt, self.pS, self.pC = (vp(t.data_ptr()) for t in (self.St, self.Ct, self.S, self.C))
        self.eta = ctypes.c_float(wl.eta)
        self.flops = dict(fwd=2.0 * L.coded_rows * (n * L.B_c) * self.b,
                          bwd=2.0 * (m * L.B_r) * L.coded_cols * self.b,
                          upd=2.0 * L.coded_rows * L.coded_cols * self.b)
        self.weight_bytes = 4.0 * L.coded_rows * L.coded_cols

    def pre_update(self, s, stream, slot=None):
        """forward, faults, check, backward, faults, check of step s (everything but the update);
        the two reports go to row `slot` of self.reports (default: the step's own)."""
        lib, h, b = self.lib, self.h, self.b
        k = s % self.RING
        slot = s if slot is None else slot
        if self.verified:
            def check(phase, coded_out, decoded, report):
                return lib.codenet_detect_decode_verified(h, phase, coded_out, b, decoded, report, 0, None, stream)
        else:
            def check(phase, coded_out, decoded, report):
                return lib.codenet_detect_decode(h, phase, coded_out, b, decoded, report, stream)
        rc = lib.codenet_forward(h, self.pX[k], b, self.pSt, stream)
        if self.coded:
            (ff, nf), (fb, nb) = self.faults[s % self.total_steps]
            if nf:
                rc |= lib.codenet_inject(h, ff, nf, self.pSt, b, stream)
            rc |= check(0, self.pSt, self.pSt if self.in_place else self.pS, ctypes.c_void_p(self.reports[slot, 0].data_ptr()))
        rc |= lib.codenet_backward(h, self.pD[k], b, self.pCt, stream)
        if self.coded:
            if nb:
                rc |= lib.codenet_inject(h, fb, nb, self.pCt, b, stream)
            rc |= check(1, self.pCt, self.pCt if self.in_place else self.pC, ctypes.c_void_p(self.reports[slot, 1].data_ptr()))
        if rc:
            raise RuntimeError("a codenet call failed in step %d (rc=%d)" % (s, rc))

    STAMP_EVERY = 4     # graph replay: steps whose update kernel is bracketed by two device time stamps
    EVENT_EVERY = 20    # graph replay: steps (s % EVENT_EVERY == 10) whose update is launched on its own between two HIP events

    def update(self, s, stream):
        """Graph replay: the update of step s; on every STAMP_EVERY-th step between two device time stamps."""
        stamped = s % self.STAMP_EVERY == 0
        rc = 0
        if stamped:
            rc |= self.lib.codenet_timestamp(ctypes.c_void_p(self.stamps[s, 0].data_ptr()), stream,
                                             ctypes.byref(self.ticks_per_us))
        rc |= self.lib.codenet_update(self.h, self.eta, stream)
        if stamped:
            rc |= self.lib.codenet_timestamp(ctypes.c_void_p(self.stamps[s, 1].data_ptr()), stream, None)
        if rc:
            raise RuntimeError("codenet_update failed (rc=%d)" % rc)

    def split(self, s):
        """Graph replay: steps whose graph ends before the update: the update kernel is then launched
        directly, between two HIP events on the same stream (costs about 19 us of launch gaps on that step)."""
        return s % self.EVENT_EVERY == 10

    def capture(self, total_steps):
        """One hipGraph per step.  The library only enqueues kernels, so its calls can be captured
        as they are.  Host-recorded events cannot stamp a kernel inside a graph, and splitting the
        step into two launches with an event in between costs about 19 us of launch gaps per step:
        the update kernel is timed by device time stamps inside the graph instead."""
        torch = self.torch
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):          # first use outside capture (function attributes are set once)
            st = ctypes.c_void_p(side.cuda_stream)
            self.pre_update(0, st)
            self.update(0, st)
        side.synchronize()
        self.graphs = []
        for s in range(total_steps):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
                self.pre_update(s, st)
                if not self.split(s):
                    self.update(s, st)
            self.graphs.append(g)
        torch.cuda.synchronize()

    def prewarm(self, stream, seconds):
        """Untimed steps until `seconds` have passed (reports go to the spare row)."""
        torch = self.torch
        t0 = time.perf_counter()
        done = 0
        while time.perf_counter() - t0 < seconds:
            for _ in range(20):
                self.pre_update(done, stream, slot=self.total_steps)
                if self.lib.codenet_update(self.h, self.eta, stream):
                    raise RuntimeError("codenet_update failed")
                done += 1
            torch.cuda.synchronize()
        return done

    def run(self, steps, warmup, eager, prewarm_seconds=0.0):
        torch = self.torch
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        self.stamps = torch.zeros((steps + warmup, 2), dtype=torch.int64, device="cuda:0")
        self.product_stamps = torch.zeros((steps + warmup, 4), dtype=torch.int64, device="cuda:0")
        self.ticks_per_us = ctypes.c_int(0)
        if not eager:
            self.capture(steps + warmup)
        # plain stream: the update sits between two HIP events on SAMPLED_STEPS steps of the timed region, between
        # two device time stamps on as many others, and on a third set the products are stamped
        # (short runs: fewer of the other two kinds, every bracket costs the step a few microseconds)
        few = 2 if steps < 64 else SAMPLED_STEPS
        event_steps = set(sampled(steps, warmup, SAMPLED_STEPS if steps >= 64 else 4)) if eager else set()
        rest = [s for s in range(warmup, warmup + steps) if s not in event_steps] if eager else []
        product_steps = {rest[i] for i in sampled(len(rest), 0, 2 * few)} if rest else set()
        rest = [s for s in rest if s not in product_steps]
        stamp_steps = {rest[i] for i in sampled(len(rest), 0, few)} if rest else set()
        events = {}
        # every event that the timed region records exists and has been recorded once before it, and the
        # time stamp kernel has run once: first uses cost hundreds of microseconds, a tenth of a 20-step run
        pool = {s: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for s in event_steps}
        for a, b in pool.values():
            a.record()
            b.record()
        self.lib.codenet_profile_stamps(self.h, ctypes.c_void_p(self.product_stamps[0].data_ptr()))
        self.pre_update(0, stream, slot=self.total_steps)
        self.lib.codenet_profile_stamps(self.h, None)
        self.lib.codenet_timestamp(ctypes.c_void_p(self.stamps[0, 0].data_ptr()), stream, ctypes.byref(self.ticks_per_us))
        if self.lib.codenet_update(self.h, self.eta, stream):
            raise RuntimeError("codenet_update failed")
        torch.cuda.synchronize()
        self.product_stamps.zero_()
        self.stamps.zero_()

        def timed_update(s):
            ev = pool.get(s) or (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
            ev[0].record()
            rc = self.lib.codenet_update(self.h, self.eta, stream)
            ev[1].record()
            if rc:
                raise RuntimeError("codenet_update failed (rc=%d)" % rc)
            if s >= warmup:
                events[s] = ev

        def stamped_update(s):
            rc = self.lib.codenet_timestamp(ctypes.c_void_p(self.stamps[s, 0].data_ptr()), stream,
                                            ctypes.byref(self.ticks_per_us))
            rc |= self.lib.codenet_update(self.h, self.eta, stream)
            rc |= self.lib.codenet_timestamp(ctypes.c_void_p(self.stamps[s, 1].data_ptr()), stream, None)
            if rc:
                raise RuntimeError("codenet_update failed (rc=%d)" % rc)

        def one(s):
            if eager:
                if s in product_steps:
                    self.lib.codenet_profile_stamps(self.h, ctypes.c_void_p(self.product_stamps[s].data_ptr()))
                self.pre_update(s, stream)
                if s in product_steps:
                    self.lib.codenet_profile_stamps(self.h, None)
                if s in event_steps:
                    timed_update(s)
                elif s in stamp_steps:
                    stamped_update(s)       # a second clock on other steps: the GPU's own, read by two tiny kernels
                elif self.lib.codenet_update(self.h, self.eta, stream):
                    raise RuntimeError("codenet_update failed")
                return
            self.graphs[s].replay()
            if self.split(s):
                timed_update(s)

        # what a pair of event records reads with nothing between them (their own cost on this stream)
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
        for a, b in pairs:
            a.record()
            b.record()
        torch.cuda.synchronize()
        self.event_pair_ms = float(np.median([a.elapsed_time(b) for a, b in pairs]))
        # The untimed steps come last before the warm-up, with nothing but the warm-up's closing
        # synchronization between them and the timed region: the set-up above leaves the GPU idle for
        # milliseconds, and what runs right after an idle stretch runs at lower clocks.
        self.prewarm_steps = self.prewarm(stream, prewarm_seconds) if (eager and prewarm_seconds > 0) else 0
        for s in range(warmup):
            one(s)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            one(warmup + s)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        st = self.stamps[warmup:].cpu().numpy()
        st = st[(st[:, 0] != 0) & (st[:, 1] != 0)]
        tick = self.ticks_per_us.value or 100
        upd_ms = float(np.mean(st[:, 1] - st[:, 0])) / tick * 1e-3 if len(st) else None
        self.upd_ms_events = float(np.mean([a.elapsed_time(b) for a, b in events.values()])) if events else None
        self.upd_event_samples = len(events)
        ps = self.product_stamps[warmup:].cpu().numpy()
        ps = ps[ps[:, 0] != 0]
        self.product_ms = (float(np.mean(ps[:, 1] - ps[:, 0])) / tick * 1e-3, float(np.mean(ps[:, 3] - ps[:, 2])) / tick * 1e-3,
                           len(ps)) if len(ps) else None
        return (t1 - t0) * 1e3 / steps, upd_ms

    def update_by_events(self, reps=50):
        """The same update kernel launched `reps` times back to back between two HIP events."""
        torch = self.torch
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            self.lib.codenet_update(self.h, self.eta, stream)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            rc = self.lib.codenet_update(self.h, self.eta, stream)
        e1.record()
        torch.cuda.synchronize()
        if rc:
            raise RuntimeError("codenet_update failed (rc=%d)" % rc)
        return e0.elapsed_time(e1) / reps

    def time_regeneration(self, reps=10):
        """Weight faults on every stored block of block-row 1 that the forward product reads,
        one forward product that locates the row, then `reps` regenerations of it (each rebuilds
        the same row from the same good blocks) between two events."""
        torch, B, WL, L = self.torch, self.B, self.WL, self.layer
        if self.wl.r < 2:
            return None                   # r = 1 only detects: nothing is ever located
        n = self.wl.grid[1]
        L.inject([WL.make_fault(WL.PHASE_WEIGHT, 1, j, 10 ** 6) for j in range(n)])
        out = L.forward(self.X[0])
        rep = L.new_report()
        L.detect_decode(B.FWD, out, report=rep, want_decoded=False)
        got = L.read_report(rep)
        if got["verdict"] != B.CORRECTED or got["located"] != [1]:
            raise RuntimeError("regeneration set-up: the corrupted block-row was not located: %r" % (got,))
        L.regenerate(B.FWD, rep)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            L.regenerate(B.FWD, rep)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        L.detect_decode(B.FWD, L.forward(self.X[1]), report=rep, want_decoded=False)
        after = L.read_report(rep)["verdict"]
        m_sys = self.wl.grid[0]
        # reads the m good systematic block-rows, writes one block-row (+ its bf16 copy)
        row_bytes = 4.0 * L.B_r * L.coded_cols
        nbytes = row_bytes * (m_sys + 1) + (0.5 * row_bytes if self.wl.dtype == "bf16" else 0.0)
        return {"ms": ms, "algorithmic_bytes": nbytes, "GB/s": nbytes / (ms * 1e-3) / 1e9,
                "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "verdict_of_next_product": ["clean", "corrected", "uncorrectable"][after],
                "what": "one located block-row of the coded matrix rebuilt from the good systematic rows and a parity row"}

    def verdict_counts(self, lo, hi):
        return count_verdicts(self.B, self.reports[lo:hi].cpu().numpy().reshape(-1, self.B.REPORT_BYTES))


def count_verdicts(B, raw):
    counts = {"clean": 0, "corrected": 0, "uncorrectable": 0}
    for row in raw:
        v = B.Report.from_buffer_copy(row.tobytes()).verdict
        name = ["clean", "corrected", "uncorrectable", "disagree"][v]   # the last from verified checks only
        counts[name] = counts.get(name, 0) + 1
    return counts


class MlpRunner:
    """Whole training iterations of an MLP workload through the library: every activation, error and
    weight stays on the GPU; the loss head (a few elementwise kernels) is PyTorch's.

    Faults follow the workload's law.  The host knows which nodes it corrupts, hence whether a product
    is beyond what the code corrects (more than t erroneous blocks; any fault at all with one parity
    block): such a product is computed again right away, without its faults, as the step's roll-back
    (transient errors), so nothing corrupted propagates and no verdict has to be read back inside the
    timed loop.  The verdicts are read after the run and must be the ones the fault lists imply.
    Update-stage (weight) faults are planted after the update where the workload has them and the code
    can correct them (one block-row / block-column hit); every check is then followed by the
    regeneration call, which acts on the device-side report alone."""

    def __init__(self, wl, coded, faults_on, total_iters, n_layers):
        import torch
        from paper_1903_01042_amd import binding as B
        from paper_1903_01042_amd import workloads as WL
        self.torch, self.B, self.wl, self.WL = torch, B, wl, WL
        self.lib = B.load_library()
        dev = torch.device("cuda:0")
        self.widths = wl.widths[: n_layers + 1]
        self.Ln = n_layers
        self.b = b = wl.batch
        self.coded = coded
        self.faults_on = coded and faults_on
        self.t = wl.r // 2
        m, n = wl.grid
        self.layers = []
        for l in range(n_layers):
            W = torch.from_numpy(WL.layer_weights(self.widths[l + 1], self.widths[l], l)).to(dev)
            P_r, P_c = wl.generators(l) if coded else (np.zeros((m, 0)), np.zeros((n, 0)))
            self.layers.append(B.CodedLayer(W, P_r, P_c, dtype=B.F32, max_batch=b, tau_detect=wl.tau_detect,
                                            tau_resid=wl.tau_resid))
        f32 = dict(dtype=torch.float32, device=dev)
        self.X = [torch.from_numpy(wl.inputs(s)[:, : self.widths[0]].copy()).to(dev) for s in range(4)]
        self.act = [None] + [torch.empty((b, self.widths[l + 1]), **f32) for l in range(n_layers)]
        self.St = [torch.empty((b, lay.coded_rows), **f32) for lay in self.layers]
        self.Ct = [torch.empty((b, lay.coded_cols), **f32) for lay in self.layers]
        self.err = [torch.empty((b, self.widths[l]), **f32) for l in range(n_layers)] + [torch.empty((b, self.widths[-1]), **f32)]
        classes = self.widths[-1]
        if wl.name.startswith("cfg2"):
            labels = [np.random.default_rng(WL.SEED_DELTAS + s).integers(0, classes, size=b) for s in range(4)]
            self.Y = [torch.nn.functional.one_hot(torch.from_numpy(y), classes).to(**f32) for y in labels]
            self.head = "softmax cross-entropy on random labels"
        else:
            self.Y = [torch.from_numpy(WL.normal((b, classes), WL.SEED_DELTAS + s)).to(dev) for s in range(4)]
            self.head = "squared error against random targets"
        self.reports = torch.zeros((total_iters + 1, n_layers, 4, B.REPORT_BYTES), dtype=torch.uint8, device=dev)
        self.total_iters = total_iters
        self.eta = ctypes.c_float(wl.eta)
        self.expected = {"clean": 0, "corrected": 0, "uncorrectable": 0}
        self.plan = [self._plan(it) for it in range(total_iters)]
        self.flops = sum(2.0 * self.b * (lay.coded_rows * (n * lay.B_c) + (m * lay.B_r) * lay.coded_cols
                                         + lay.coded_rows * lay.coded_cols) for lay in self.layers)
        self.stamps = torch.zeros((total_iters + 1, 4), dtype=torch.int64, device=dev)
        self.ticks_per_us = ctypes.c_int(0)

    def _plan(self, it):
        """Marshalled fault lists of iteration `it`: per layer (fwd faults, redo?, bwd faults, redo?, weight faults)."""
        B, WL, wl = self.B, self.WL, self.wl
        rows = []
        for l in range(self.Ln):
            entry = []
            for phase in (WL.PHASE_FWD, WL.PHASE_BWD):
                ff = wl.product_faults(phase, it, l) if self.faults_on else []
                hit = {f["bi"] if phase == WL.PHASE_FWD else f["bj"] for f in ff}
                redo = len(hit) > self.t
                entry += [(B.pack_faults(ff), len(ff)), redo]
            wf = wl.update_faults(it, l) if self.faults_on else []
            lines_r, lines_c = {f["bi"] for f in wf}, {f["bj"] for f in wf}
            # plantable: the next forward product sees one erroneous block-row at most, the next backward one one block-column
            ok = len(wf) > 0 and len(lines_r) <= self.t and len(lines_c) <= self.t
            entry.append((B.pack_faults(wf), len(wf)) if ok else (None, 0))
            rows.append(entry)
        return rows

    def iteration(self, it, stream, slot=None, stamp=False):
        lib, B, b = self.lib, self.B, self.b
        L = self.Ln
        slot = it if slot is None else slot
        plan = self.plan[it % self.total_iters]
        vp = ctypes.c_void_p
        rc = 0
        regen = self.faults_on and self.wl.weight_faults
        x = self.X[it % 4]
        for l in range(L):
            lay = self.layers[l]
            (ff, nf), redo = plan[l][0], plan[l][1]
            epi = B.EPI_RELU if l < L - 1 else B.EPI_NONE
            pS, pA = vp(self.St[l].data_ptr()), vp(self.act[l + 1].data_ptr())
            if stamp and l == 0:
                rc |= lib.codenet_profile_stamps(lay._h, vp(self.stamps[slot].data_ptr()))
            rc |= lib.codenet_forward(lay._h, vp(x.data_ptr()), b, pS, stream)
            if self.coded:
                if nf:
                    rc |= lib.codenet_inject(lay._h, ff, nf, pS, b, stream)
                rc |= lib.codenet_detect_decode_act(lay._h, 0, pS, b, pA, vp(self.reports[slot, l, 0].data_ptr()), epi, None, stream)
                if redo:        # beyond the code's capability: the product again, without the transient faults
                    rc |= lib.codenet_forward(lay._h, vp(x.data_ptr()), b, pS, stream)
                    rc |= lib.codenet_detect_decode_act(lay._h, 0, pS, b, pA, vp(self.reports[slot, l, 1].data_ptr()), epi, None, stream)
                if regen:
                    rc |= lib.codenet_regenerate(lay._h, 0, vp(self.reports[slot, l, 1 if redo else 0].data_ptr()), stream)
            else:
                rc |= lib.codenet_detect_decode_act(lay._h, 0, pS, b, pA, None, epi, None, stream)
            x = self.act[l + 1]
        # loss head (PyTorch elementwise kernels): delta^L = -dLoss/ds^L
        if self.head.startswith("softmax"):
            self.torch.sub(self.Y[it % 4], self.torch.softmax(x, dim=1), out=self.err[L])
            self.err[L].mul_(1.0 / b)
        else:
            self.torch.sub(self.Y[it % 4], x, out=self.err[L])
            self.err[L].mul_(1.0 / b)
        d = self.err[L]
        for l in range(L - 1, -1, -1):
            lay = self.layers[l]
            (fb, nb), redo = plan[l][2], plan[l][3]
            epi = B.EPI_MASK_POS if l > 0 else B.EPI_NONE
            aux = vp(self.act[l].data_ptr()) if l > 0 else None
            pC, pE = vp(self.Ct[l].data_ptr()), vp(self.err[l].data_ptr())
            rc |= lib.codenet_backward(lay._h, vp(d.data_ptr()), b, pC, stream)
            if self.coded:
                if nb:
                    rc |= lib.codenet_inject(lay._h, fb, nb, pC, b, stream)
                rc |= lib.codenet_detect_decode_act(lay._h, 1, pC, b, pE, vp(self.reports[slot, l, 2].data_ptr()), epi, aux, stream)
                if redo:
                    rc |= lib.codenet_backward(lay._h, vp(d.data_ptr()), b, pC, stream)
                    rc |= lib.codenet_detect_decode_act(lay._h, 1, pC, b, pE, vp(self.reports[slot, l, 3].data_ptr()), epi, aux, stream)
                if regen:
                    rc |= lib.codenet_regenerate(lay._h, 1, vp(self.reports[slot, l, 3 if redo else 2].data_ptr()), stream)
            else:
                rc |= lib.codenet_detect_decode_act(lay._h, 1, pC, b, pE, None, epi, aux, stream)
            d = self.err[l]
        if stamp:
            rc |= lib.codenet_profile_stamps(self.layers[0]._h, None)
        for l in range(L):
            rc |= lib.codenet_update(self.layers[l]._h, self.eta, stream)
            wf, nw = plan[l][4]
            if nw:
                rc |= lib.codenet_inject(self.layers[l]._h, wf, nw, None, 0, stream)
        if rc:
            raise RuntimeError("a codenet call failed in iteration %d (rc=%d)" % (it, rc))

    def run(self, iters, warmup, prewarm_seconds=0.0):
        torch = self.torch
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        self.prewarm_iters = 0
        if prewarm_seconds > 0:
            t0 = time.perf_counter()
            while time.perf_counter() - t0 < prewarm_seconds:
                for _ in range(4):
                    self.iteration(self.prewarm_iters, stream, slot=self.total_iters)
                    self.prewarm_iters += 1
                torch.cuda.synchronize()
            # the pre-warm has trained the network a little and planted weight faults: harmless, its reports are dropped
        self.lib.codenet_timestamp(ctypes.c_void_p(self.stamps[self.total_iters].data_ptr()), stream, ctypes.byref(self.ticks_per_us))
        stamp_at = set(sampled(iters, warmup))
        for it in range(warmup):
            self.iteration(it, stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for it in range(warmup, warmup + iters):
            self.iteration(it, stream, stamp=it in stamp_at)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        st = self.stamps[warmup:warmup + iters].cpu().numpy()
        st = st[st[:, 0] != 0]
        tick = self.ticks_per_us.value or 100
        self.product_ms = (float(np.mean(st[:, 1] - st[:, 0])) / tick * 1e-3, float(np.mean(st[:, 3] - st[:, 2])) / tick * 1e-3,
                           len(st)) if len(st) else None
        return (t1 - t0) * 1e3 / iters

    def verdict_counts(self, lo, hi):
        """Counts over the reports that were written (a product's second slot only when it was computed again)."""
        raw = self.reports[lo:hi].cpu().numpy()
        rows = []
        for it in range(lo, hi):
            plan = self.plan[it % self.total_iters]
            for l in range(self.Ln):
                rows.append(raw[it - lo, l, 0])
                if plan[l][1]:
                    rows.append(raw[it - lo, l, 1])
                rows.append(raw[it - lo, l, 2])
                if plan[l][3]:
                    rows.append(raw[it - lo, l, 3])
        return count_verdicts(self.B, rows)

    def destroy(self):
        for lay in self.layers:
            lay.destroy()


class StrategyRun:
    """One strategy training the cfg2 network for M iterations under transient soft errors in the
    node outputs of both products (Bernoulli per node and product), with a checkpoint every I0
    iterations (the weights of all layers copied to host memory) and the paper's roll-back rule: an
    iteration whose errors the strategy cannot correct is thrown away and the network is restored
    from the last checkpoint (host copy -> device, encoded afresh), from where the iterations are
    repeated.  The verdicts of an iteration are read once, at its end.
      codenet      coded layers with 2 parity block-rows / columns (t = 1): corrects one erroneous
                   block per product and goes on (every check is followed by the regeneration call)
      replication  two uncoded replicas compute every product; outputs are compared on the device,
                   any difference means roll back (detection only)
      uncoded      one uncoded network, errors are neither detected nor corrected, no checkpoints"""

    def __init__(self, strategy, wl, p, period, iters, seed=0):
        import torch
        from paper_1903_01042_amd import binding as B
        from paper_1903_01042_amd import workloads as WL
        self.torch, self.B, self.WL, self.wl = torch, B, WL, wl
        self.lib = B.load_library()
        self.dev = torch.device("cuda:0")
        self.strategy, self.p, self.period, self.iters, self.seed = strategy, p, period, iters, seed
        self.Ln = len(wl.widths) - 1
        self.b = wl.batch
        m, n = wl.grid
        self.r = 2 if strategy == "codenet" else 0
        self.P = (WL.vandermonde_like(m, self.r), WL.vandermonde_like(n, self.r))
        self.replicas = 2 if strategy == "replication" else 1
        W0 = [WL.layer_weights(wl.widths[l + 1], wl.widths[l], l) for l in range(self.Ln)]
        self.ckpt = [torch.from_numpy(w) for w in W0]             # host copies
        self.nets = [[self._encode(self.ckpt[l]) for l in range(self.Ln)] for _ in range(self.replicas)]
        f32 = dict(dtype=torch.float32, device=self.dev)
        self.X = [torch.from_numpy(wl.inputs(s)).to(self.dev) for s in range(8)]
        classes = wl.widths[-1]
        self.Y = [torch.nn.functional.one_hot(torch.from_numpy(np.random.default_rng(WL.SEED_DELTAS + s).integers(0, classes, size=self.b)),
                                              classes).to(**f32) for s in range(8)]
        lay = self.nets[0]
        self.St = [[torch.empty((self.b, l.coded_rows), **f32) for l in net] for net in self.nets]
        self.Ct = [[torch.empty((self.b, l.coded_cols), **f32) for l in net] for net in self.nets]
        self.act = [None] + [torch.empty((self.b, wl.widths[l + 1]), **f32) for l in range(self.Ln)]
        self.err = [torch.empty((self.b, wl.widths[l]), **f32) for l in range(self.Ln + 1)]
        self.reports = torch.zeros((self.Ln, 2, B.REPORT_BYTES), dtype=torch.uint8, device=self.dev)
        self.mismatch = torch.zeros(1, dtype=torch.int32, device=self.dev)
        self.classes = {"clean": 0, "corrected": 0, "rolled_back": 0}
        self.t_iter = {"clean": [], "corrected": [], "rolled_back": []}
        self.t_ckpt = []

    def _encode(self, W_host):
        return self.B.CodedLayer(W_host.to(self.dev), self.P[0], self.P[1], dtype=self.B.F32, max_batch=self.b,
                                 tau_detect=self.wl.tau_detect, tau_resid=self.wl.tau_resid)

    def _faults(self, phase, attempt, layer, replica):
        WL = self.WL
        m, n = self.wl.grid
        ff = WL.bernoulli_faults(phase, m, n, self.r, self.r, self.p, attempt, layer, seed=WL.SEED_FAULTS + 17 * replica + 1000 * self.seed)
        return self.B.pack_faults(ff), len(ff)

    def _iteration(self, it, attempt, stream):
        """Iteration `it` of the training (inputs it % 8); `attempt` numbers every try, so that a repeated
        iteration draws new errors."""
        lib, B, b, L = self.lib, self.B, self.b, self.Ln
        vp = ctypes.c_void_p
        coded = self.strategy == "codenet"
        rc = 0
        self.mismatch.zero_()
        x = self.X[it % 8]
        for l in range(L):
            epi = B.EPI_RELU if l < L - 1 else B.EPI_NONE
            for k, net in enumerate(self.nets):
                lay, pS = net[l], vp(self.St[k][l].data_ptr())
                rc |= lib.codenet_forward(lay._h, vp(x.data_ptr()), b, pS, stream)
                ff, nf = self._faults(self.WL.PHASE_FWD, attempt, l, k)
                if nf:
                    rc |= lib.codenet_inject(lay._h, ff, nf, pS, b, stream)
            if self.replicas == 2:
                self.mismatch.add_((self.St[0][l] != self.St[1][l]).any().to(self.torch.int32))
            lay = self.nets[0][l]
            rep = vp(self.reports[l, 0].data_ptr()) if coded else None
            rc |= lib.codenet_detect_decode_act(lay._h, 0, vp(self.St[0][l].data_ptr()), b, vp(self.act[l + 1].data_ptr()), rep, epi, None, stream)
            if coded:
                rc |= lib.codenet_regenerate(lay._h, 0, rep, stream)
            x = self.act[l + 1]
        self.torch.sub(self.Y[it % 8], self.torch.softmax(x, dim=1), out=self.err[L])
        self.err[L].mul_(1.0 / b)
        d = self.err[L]
        for l in range(L - 1, -1, -1):
            epi = B.EPI_MASK_POS if l > 0 else B.EPI_NONE
            aux = vp(self.act[l].data_ptr()) if l > 0 else None
            for k, net in enumerate(self.nets):
                lay, pC = net[l], vp(self.Ct[k][l].data_ptr())
                rc |= lib.codenet_backward(lay._h, vp(d.data_ptr()), b, pC, stream)
                fb, nb = self._faults(self.WL.PHASE_BWD, attempt, l, k)
                if nb:
                    rc |= lib.codenet_inject(lay._h, fb, nb, pC, b, stream)
            if self.replicas == 2:
                self.mismatch.add_((self.Ct[0][l] != self.Ct[1][l]).any().to(self.torch.int32))
            lay = self.nets[0][l]
            rep = vp(self.reports[l, 1].data_ptr()) if coded else None
            rc |= lib.codenet_detect_decode_act(lay._h, 1, vp(self.Ct[0][l].data_ptr()), b, vp(self.err[l].data_ptr()), rep, epi, aux, stream)
            if coded:
                rc |= lib.codenet_regenerate(lay._h, 1, rep, stream)
            d = self.err[l]
        for net in self.nets:
            for lay in net:
                rc |= lib.codenet_update(lay._h, ctypes.c_float(self.wl.eta), stream)
        if rc:
            raise RuntimeError("a codenet call failed (rc=%d)" % rc)
        # the iteration's verdict, read once
        if coded:
            v = [self.B.Report.from_buffer_copy(row.tobytes()).verdict for row in self.reports.cpu().numpy().reshape(-1, B.REPORT_BYTES)]
            return "rolled_back" if B.UNCORRECTABLE in v else ("corrected" if B.CORRECTED in v else "clean")
        if self.replicas == 2:
            return "rolled_back" if int(self.mismatch.item()) else "clean"
        self.torch.cuda.synchronize()
        return "clean"

    def run(self):
        torch = self.torch
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        for w in range(3):                      # warm-up on the first input (state restored below)
            self._iteration(0, 10 ** 6 + w, stream)
        self._restore()
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        done, attempt, last_ckpt = 0, 0, 0
        self.finished = True
        while done < self.iters:
            if attempt >= 10 * self.iters:      # this period is hopeless at this error rate (the chain's expected time explodes)
                self.finished = False
                break
            t0 = time.perf_counter()
            kind = self._iteration(done, attempt, stream)
            attempt += 1
            if kind == "rolled_back" and self.strategy != "uncoded":
                self._restore()
                torch.cuda.synchronize()
                done = last_ckpt
            else:
                done += 1
            self.classes[kind] += 1
            self.t_iter[kind].append(time.perf_counter() - t0)
            if self.strategy != "uncoded" and done - last_ckpt == self.period and done < self.iters:
                t0 = time.perf_counter()
                self.ckpt = [lay.export_weights().cpu() for lay in self.nets[0]]
                last_ckpt = done
                self.t_ckpt.append(time.perf_counter() - t0)
        total = time.perf_counter() - t_start
        self.final = [lay.export_weights().cpu().numpy() for lay in self.nets[0]]
        for net in self.nets:
            for lay in net:
                lay.destroy()
        return total, attempt

    def _restore(self):
        for net in self.nets:
            for lay in net:
                lay.destroy()
        self.nets = [[self._encode(self.ckpt[l]) for l in range(self.Ln)] for _ in range(self.replicas)]


def main_strategies(args):
    """Time to M iterations of CodeNet, replication and uncoded over a sweep of checkpoint periods,
    next to the expected-time model (Theorem 2; the chain's own solution and the formula as printed)
    evaluated at the measured tau_f, tau_b, tau_cpt and at the class frequencies of the drawn errors."""
    from oracle import strategy_model as S
    from paper_1903_01042_amd import workloads as WL
    wl = WL.WORKLOADS["cfg2"]
    M, p = args.steps if args.steps != 1000 else 200, args.fault_p
    periods = [q for q in (5, 10, 20, 50, 100) if q <= M]
    out = {"metric": "time to M training iterations under soft errors", "unit": "s", "M": M, "fault_p_per_node_and_product": p,
           "network": list(wl.widths), "grid": "%dx%d" % wl.grid, "batch": wl.batch, "data": "synthetic",
           "strategies": {}}
    ref = StrategyRun("uncoded", wl, 0.0, M, M)
    t_ref, _ = ref.run()
    for name in ("codenet", "replication"):
        rows = []
        for I0 in periods:
            run = StrategyRun(name, wl, p, I0, M)
            total, attempts = run.run()
            n = sum(run.classes.values())
            med = lambda v: float(np.median(v)) if v else None
            tau_f, tau_b = med(run.t_iter["clean"]), med(run.t_iter["rolled_back"]) or med(run.t_iter["corrected"])
            tau_c = med(run.t_iter["corrected"])
            tau_cpt = med(run.t_ckpt) or 0.0
            p0, p1 = run.classes["clean"] / n, run.classes["corrected"] / n
            row = {"I0": I0, "seconds": total if run.finished else float("inf"), "finished": run.finished, "attempts": attempts, "classes": run.classes, "tau_f": tau_f, "tau_corrected": tau_c,
                   "tau_b": tau_b, "tau_cpt": tau_cpt, "p0": p0, "p1": p1,
                   # relative distance of every layer's final weights from those of a run without errors
                   "distance_from_fault_free_run": [float(np.linalg.norm(a - b) / np.linalg.norm(b))
                                                    for a, b in zip(run.final, ref.final)] if run.finished else None}
            if tau_f and tau_b:
                # the paper charges tau_b to a corrected iteration as well (its pessimistic assumption); measured
                # corrected iterations cost tau_corrected, so the model is given the mixture it assumes
                row["model_seconds_chain"] = S.expected_total_time(M, I0, p0, p1, tau_f, tau_b, tau_cpt)
                row["model_seconds_as_printed"] = S.expected_total_time(M, I0, p0, p1, tau_f, tau_b, tau_cpt, printed=True)
            rows.append(row)
        best = min(rows, key=lambda r: r["seconds"])
        out["strategies"][name] = {"sweep": rows, "best_I0": best["I0"], "best_seconds": best["seconds"]}
    unc = StrategyRun("uncoded", wl, p, M, M)
    t_unc, _ = unc.run()
    dist = [float(np.linalg.norm(a - b) / np.linalg.norm(b)) for a, b in zip(unc.final, ref.final)]
    out["strategies"]["uncoded"] = {"seconds": t_unc, "fault_free_seconds": t_ref,
                                    "relative_distance_of_final_weights_from_the_fault_free_run": dist}
    rep, cod = out["strategies"]["replication"], out["strategies"]["codenet"]
    out["replication_over_codenet_measured"] = rep["best_seconds"] / cod["best_seconds"]
    rb, cb = min(rep["sweep"], key=lambda r: r["seconds"]), min(cod["sweep"], key=lambda r: r["seconds"])
    if cb.get("model_seconds_chain") and rb.get("model_seconds_chain"):
        out["replication_over_codenet_model_chain"] = rb["model_seconds_chain"] / cb["model_seconds_chain"]
        out["replication_over_codenet_model_as_printed"] = rb["model_seconds_as_printed"] / cb["model_seconds_as_printed"]
    out["value"] = out["replication_over_codenet_measured"]
    out["note"] = ("one GPU: both replicas, and CodeNet's redundant blocks, run on the same device, so an error-free iteration "
                   "costs each strategy its own tau_f (the paper gives the redundancy extra nodes and one tau_f to both)")
    print(json.dumps(out))


def measured_traffic(workload_key):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size); None when no summary exists."""
    path = os.path.join(ROOT, "profiles", "%s_update_kernel_hbm_traffic.txt" % workload_key)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def host_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        return os.cpu_count() or 1


def cpu_baseline(wl, steps):
    """The float64 oracle as it stands, timed on the host for a few layer-steps of the first layer of
    the workload at full size (encoding excluded, as on the GPU; inputs and fault lists are drawn
    before the clock starts, as the GPU leg has them resident)."""
    from oracle import codenet_oracle as O
    from paper_1903_01042_amd import workloads as WL
    n_in, n_out = wl.widths[0], wl.widths[1]
    P_r, P_c = wl.generators()
    lay = O.CodedLayer(WL.layer_weights(n_out, n_in), P_r, P_c, tau_detect=wl.tau_detect, tau_resid=wl.tau_resid)
    work = []
    for s in range(steps):
        work.append((wl.inputs(s)[:, :n_in].T.astype(np.float64), WL.normal((wl.batch, n_out), WL.SEED_DELTAS + s).T.astype(np.float64),
                     wl.product_faults(WL.PHASE_FWD, s), wl.product_faults(WL.PHASE_BWD, s)))
    t0 = time.perf_counter()
    for X, D, ff, fb in work:
        out = lay.inject(ff, lay.forward(X))
        lay.detect_decode(O.PHASE_FWD, out)
        out = lay.inject(fb, lay.backward(D))
        lay.detect_decode(O.PHASE_BWD, out)
        lay.update(wl.eta)
    dt = time.perf_counter() - t0
    return {"value": steps / dt, "unit": "coded layer-steps/s", "cores": int(host_threads()), "kind": "oracle",
            "sample": "%d full-size layer-steps of layer 0 of %s (%d x %d, float64 numpy, encoding and input generation excluded)"
                      % (steps, wl.name, n_out, n_in)}


def product_roofline(wl, flops, product_ms, kernel):
    """The coded products against the MFMA peak of their arithmetic: flops of one product / its time on
    the GPU (device time stamps around the kernel: its duration plus one kernel boundary)."""
    if product_ms is None:
        return None
    fwd_ms, bwd_ms, n = product_ms
    peak = MFMA_PEAK_TFLOPS[wl.dtype]
    ach = 0.5 * (flops["fwd"] / (fwd_ms * 1e-3) + flops["bwd"] / (bwd_ms * 1e-3)) / 1e12
    return {"kernel": kernel, "bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak,
            "forward_ms": fwd_ms, "backward_ms": bwd_ms, "flops_forward": flops["fwd"], "flops_backward": flops["bwd"],
            "frac_forward": flops["fwd"] / (fwd_ms * 1e-3) / 1e12 / peak, "frac_backward": flops["bwd"] / (bwd_ms * 1e-3) / 1e12 / peak,
            "samples": n, "timed_by": "device time stamps (the GPU's 100 MHz clock) before and after the product kernel on %d "
                                      "steps of the timed region: the kernel plus one kernel boundary" % n}


def main_mlp(args, wl):
    import torch
    L_all = len(wl.widths) - 1
    L = args.layers if 0 < args.layers <= L_all else L_all
    total = args.steps + args.warmup
    pre = 0.0 if args.no_prewarm else PREWARM_SECONDS
    coded = MlpRunner(wl, True, not args.no_faults, total, L)
    ms_coded = coded.run(args.steps, args.warmup, pre)
    counts = coded.verdict_counts(args.warmup, total)
    lay0 = coded.layers[0]
    m, n = wl.grid
    flops0 = dict(fwd=2.0 * lay0.coded_rows * (n * lay0.B_c) * coded.b, bwd=2.0 * (m * lay0.B_r) * lay0.coded_cols * coded.b)
    out = {
        "metric": "coded layer-steps/s (fwd+bwd+detect/decode+update)",
        "value": 1e3 * L / ms_coded, "unit": "coded layer-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_coded / L,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "layers": L, "widths": list(coded.widths), "grid": "%dx%d+%d" % (m, n, wl.r),
                   "batch": wl.batch, "fault_law": "%s p=%g per node and product" % (wl.fault_law, wl.fault_p),
                   "step": "one training iteration of the whole MLP = %d layer-steps; `steps` counts iterations" % L,
                   "loss_head": coded.head, "launch": "every call launched into one stream",
                   "roll_back": "a product with more erroneous blocks than the code corrects is computed again inside the timed loop"},
        "ms_per_iteration": ms_coded,
        "tflops": coded.flops / (ms_coded * 1e-3) / 1e12,
        "mfma_frac_of_peak_whole_step": coded.flops / (ms_coded * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS[wl.dtype],
        "verdicts": counts,
        "prewarm_iterations": coded.prewarm_iters,
        "roofline": product_roofline(wl, flops0, coded.product_ms, "gemm_kernel (coded products of layer 0, float32 MFMA)"),
    }
    coded.destroy()
    if not args.coded_only:
        unc = MlpRunner(wl, False, False, total, L)
        ms_unc = unc.run(args.steps, args.warmup, pre)
        floor = coded.flops / unc.flops - 1.0
        unc.destroy()
        out.update({"uncoded_ms_per_step": ms_unc / L, "coding_overhead": ms_coded / ms_unc - 1.0,
                    "algorithmic_overhead_floor": floor, "excess_over_floor": (ms_coded / ms_unc) / (1.0 + floor) - 1.0})
        if not args.no_faults:
            clean = MlpRunner(wl, True, False, total, L)
            ms_clean = clean.run(args.steps, args.warmup, pre)
            clean.destroy()
            out.update({"ms_per_step_without_faults": ms_clean / L,
                        "coding_overhead_without_faults": ms_clean / ms_unc - 1.0,
                        "excess_over_floor_without_faults": (ms_clean / ms_unc) / (1.0 + floor) - 1.0})
        cpu_steps = args.cpu_steps if args.cpu_steps >= 0 else (40 if wl.widths[1] <= 2048 else 2)
        if cpu_steps > 0:
            out["cpu_baseline"] = cpu_baseline(wl, cpu_steps)
    print(json.dumps(out))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no cross-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1903_01042_amd import workloads as WL
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.strategies:
        return main_strategies(args)
    wl = WL.WORKLOADS[args.workload]
    if len(wl.widths) > 2 and args.layers != 1:
        return main_mlp(args, wl)
    total = args.steps + args.warmup
    pre = 0.0 if args.no_prewarm else PREWARM_SECONDS

    coded = Runner(wl, True, not args.no_faults, total)
    ms_coded, upd_ms = coded.run(args.steps, args.warmup, not args.graph, pre)
    counts = coded.verdict_counts(args.warmup, total)
    if args.coded_only:
        # a plain device-to-device copy of known size (the coded matrix) next to the kernels:
        # HBM byte counters of a profiling run are scaled by what they read for this copy
        for _ in range(3):
            coded.layer.export_coded()
        torch.cuda.synchronize()
        print(json.dumps({"ms_per_step": ms_coded, "update_kernel_ms": upd_ms if args.graph else coded.upd_ms_events,
                          "product_kernels_ms": coded.product_ms, "verdicts": counts, "workload": wl.name,
                          "calibration_copy_bytes": coded.weight_bytes}))
        return
    uncoded = Runner(wl, False, False, total)
    ms_uncoded, upd_ms_unc = uncoded.run(args.steps, args.warmup, not args.graph, pre)
    ms_clean = None
    if not args.no_faults:
        # the coded path without the injection kernels (scaffolding of the experiment, not of the method)
        clean = Runner(wl, True, False, total)
        ms_clean, _ = clean.run(args.steps, args.warmup, not args.graph, pre)
        clean.layer.destroy()
    # the coded step with the decoded outputs left in the coded buffers (a clean check writes nothing)
    inp = Runner(wl, True, not args.no_faults, total, in_place=True)
    ms_in_place, _ = inp.run(args.steps, args.warmup, not args.graph, pre)
    inp.layer.destroy()
    # the coded step with both verification steps of Error Model 2 in every check
    ver = Runner(wl, True, not args.no_faults, total, verified=True)
    ms_verified, _ = ver.run(args.steps, args.warmup, not args.graph, pre)
    counts_verified = ver.verdict_counts(args.warmup, total)
    ver.layer.destroy()

    L = coded.layer
    upd_events_ms = coded.update_by_events()
    flops_step = sum(coded.flops.values())
    m, n = wl.grid
    floor = sum(coded.flops.values()) / sum(uncoded.flops.values()) - 1.0
    # dominant kernel: the update, a read-modify-write of the whole fp32 coded matrix.
    # algorithmic bytes per launch: read + write W~ (2 * 4 B per element), the bf16 copy of W~ that
    # the two products read (bf16 mode: 2 B per element), both coded vectors once
    elem = 2.0 if wl.dtype == "bf16" else 4.0
    upd_bytes = 2.0 * coded.weight_bytes + elem * coded.b * (L.coded_rows + L.coded_cols)
    if wl.dtype == "bf16":
        upd_bytes += 0.5 * coded.weight_bytes
    # kernel duration: HIP events around the kernel, on its stream, on sampled steps of the timed region
    launch_ms = coded.upd_ms_events
    achieved = upd_bytes / (launch_ms * 1e-3) / 1e9
    out = {
        "metric": "coded layer-steps/s (fwd+bwd+detect/decode+update)",
        "value": 1e3 / ms_coded,
        "unit": "coded layer-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_coded,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "layer": "%dx%d" % (wl.widths[1], wl.widths[0]),
                   "grid": "%dx%d+%d" % (m, n, wl.r), "batch": wl.batch, "fault_law": wl.fault_law,
                   "launch": "hipGraph replay, one graph per step, one stream" if args.graph
                   else "every call launched into one stream"},
        "prewarm_steps": coded.prewarm_steps,
        "tflops": flops_step / (ms_coded * 1e-3) / 1e12,
        "mfma_frac_of_peak_whole_step": flops_step / (ms_coded * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS[wl.dtype],
        "uncoded_ms_per_step": ms_uncoded,
        "coding_overhead": ms_coded / ms_uncoded - 1.0,
        "ms_per_step_without_injection": ms_clean,
        "coding_overhead_without_injection": (ms_clean / ms_uncoded - 1.0) if ms_clean else None,
        "ms_per_step_verified_checks": ms_verified,
        "ms_per_step_decoded_in_place": ms_in_place,
        "verified_checks_agree": counts_verified == counts,
        "algorithmic_overhead_floor": floor,
        # what the checks, encodings and injection cost beyond the redundant rows themselves
        "excess_over_floor": (ms_coded / ms_uncoded) / (1.0 + floor) - 1.0,
        "excess_over_floor_without_injection": ((ms_clean / ms_uncoded) / (1.0 + floor) - 1.0) if ms_clean else None,
        "verdicts": counts,
        "update_kernel_ms_uncoded": upd_ms_unc if args.graph else uncoded.upd_ms_events,
        "roofline": {"kernel": "update3_kernel (W~ += eta [d;d~][x;x~]^T, fp32 RMW + bf16 copy)"
                     if wl.dtype == "bf16" else ("update_thin_kernel" if wl.batch <= 256 and min(L.coded_rows, L.coded_cols) >= 1024
                                                 else "gemm_kernel") + " (update, W~ += eta [d;d~][x;x~]^T, fp32 RMW)", "bound": "hbm",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(args.workload),
                     "avg_launch_ms": launch_ms,
                     "avg_launch_samples": coded.upd_event_samples,
                     "empty_event_pair_ms": coded.event_pair_ms,
                     "avg_launch_ms_by": ("HIP events around the kernel on every %d-th step of the timed region, "
                                          "where the step's graph ends before the update and the kernel is launched "
                                          "on its own" % Runner.EVENT_EVERY) if args.graph else
                     ("HIP events around the kernel, on its stream, on %d steps spread over the timed region"
                      % coded.upd_event_samples),
                     "in_graph_ms": upd_ms if args.graph else None,
                     "in_graph_ms_by": ("device time stamps before and after the kernel inside the graph of every "
                                        "%d-th step of the timed region" % Runner.STAMP_EVERY) if args.graph else None,
                     "device_stamp_ms": upd_ms,
                     "device_stamp_ms_by": "codenet_timestamp kernels (the GPU's 100 MHz wall clock) before and after the "
                                           "update on other steps of the timed region: the kernel plus one kernel boundary",
                     "back_to_back_ms_hip_events": upd_events_ms,
                     "algorithmic_bytes": upd_bytes,
                     "tflops": coded.flops["upd"] / (launch_ms * 1e-3) / 1e12},
        "roofline_products": product_roofline(
            wl, coded.flops, coded.product_ms,
            "product_kernel (coded forward and backward products, bf16 MFMA)" if wl.dtype == "bf16"
            else "gemm_kernel (coded forward and backward products, float32 MFMA)"),
    }
    out["regeneration"] = coded.time_regeneration()
    coded.layer.destroy()
    uncoded.layer.destroy()
    cpu_steps = args.cpu_steps if args.cpu_steps >= 0 else 40
    if cpu_steps > 0:
        out["cpu_baseline"] = cpu_baseline(wl, cpu_steps)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
