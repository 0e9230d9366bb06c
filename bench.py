#!/usr/bin/env python3
"""Benchmark of the coded layer step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
coded forward product, fault injection, check + decode, coded backward product,
fault injection, check + decode, coded update.  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3]
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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="cfg3", choices=["cfg1", "cfg3", "cfg4", "cfg5"],
                    help="cfg4: one layer (the first) of that 8-layer workload")
    ap.add_argument("--cpu-steps", type=int, default=40, help="oracle layer-steps timed for cpu_baseline (0 = skip)")
    ap.add_argument("--no-faults", action="store_true", help="run the coded path without injecting faults")
    ap.add_argument("--coded-only", action="store_true", help="skip the uncoded baseline and the CPU oracle (profiling runs)")
    ap.add_argument("--graph", action="store_true",
                    help="replay one hipGraph per step instead of launching every call from Python (a kernel node of a "
                         "graph takes about 3 us longer than the same kernel launched into the stream; the step is not "
                         "launch bound, so the default is the plain stream)")
    return ap.parse_args()


class Runner:
    """Pre-marshalled calls of one single-layer workload (coded or uncoded)."""

    RING = 8

    def __init__(self, wl, coded, faults_on, total_steps, verified=False):
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
        self.reports = torch.zeros((total_steps, 2, B.REPORT_BYTES), dtype=torch.uint8, device=dev)
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

    def pre_update(self, s, stream):
        """forward, faults, check, backward, faults, check of step s (everything but the update)."""
        lib, h, b = self.lib, self.h, self.b
        k = s % self.RING
        if self.verified:
            def check(phase, coded_out, decoded, report):
                return lib.codenet_detect_decode_verified(h, phase, coded_out, b, decoded, report, 0, None, stream)
        else:
            def check(phase, coded_out, decoded, report):
                return lib.codenet_detect_decode(h, phase, coded_out, b, decoded, report, stream)
        rc = lib.codenet_forward(h, self.pX[k], b, self.pSt, stream)
        if self.coded:
            (ff, nf), (fb, nb) = self.faults[s]
            if nf:
                rc |= lib.codenet_inject(h, ff, nf, self.pSt, b, stream)
            rc |= check(0, self.pSt, self.pS, ctypes.c_void_p(self.reports[s, 0].data_ptr()))
        rc |= lib.codenet_backward(h, self.pD[k], b, self.pCt, stream)
        if self.coded:
            if nb:
                rc |= lib.codenet_inject(h, fb, nb, self.pCt, b, stream)
            rc |= check(1, self.pCt, self.pC, ctypes.c_void_p(self.reports[s, 1].data_ptr()))
        if rc:
            raise RuntimeError("a codenet call failed in step %d (rc=%d)" % (s, rc))

    STAMP_EVERY = 4     # steps whose update kernel is bracketed by two device time stamps
    EVENT_EVERY = 20    # graph replay: steps (s % EVENT_EVERY == 10) whose update is launched on its own between two HIP events
    EAGER_EVENT_EVERY = 16  # plain stream: steps (s % EAGER_EVENT_EVERY == 2) whose update sits between two HIP events
                            # (a pair of records costs the stream several us: see roofline.empty_event_pair_ms)

    def update(self, s, stream):
        """The update of step s; on every STAMP_EVERY-th step between two device time stamps."""
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
        """Steps whose graph ends before the update: the update kernel is then launched directly,
        between two HIP events on the same stream (costs about 19 us of launch gaps on that step)."""
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

    def run(self, steps, warmup, eager):
        torch = self.torch
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        self.stamps = torch.zeros((steps + warmup, 2), dtype=torch.int64, device="cuda:0")
        self.ticks_per_us = ctypes.c_int(0)
        if not eager:
            self.capture(steps + warmup)

        events = {}

        def timed_update(s):
            ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
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
                self.pre_update(s, stream)
                if s % self.EAGER_EVENT_EVERY == 2:
                    timed_update(s)
                elif s % self.EAGER_EVENT_EVERY == 10:
                    stamped_update(s)       # a second clock on other steps: the GPU's own, read by two tiny kernels
                elif self.lib.codenet_update(self.h, self.eta, stream):
                    raise RuntimeError("codenet_update failed")
                return
            self.graphs[s].replay()
            if self.split(s):
                timed_update(s)

        for s in range(warmup):
            one(s)
        torch.cuda.synchronize()
        # what a pair of event records reads with nothing between them (their own cost on this stream)
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
        for a, b in pairs:
            a.record()
            b.record()
        torch.cuda.synchronize()
        self.event_pair_ms = float(np.median([a.elapsed_time(b) for a, b in pairs]))
        t0 = time.perf_counter()
        for s in range(steps):
            one(warmup + s)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        st = self.stamps[warmup:].cpu().numpy()
        st = st[st[:, 0] != 0]
        upd_ms = float(np.mean(st[:, 1] - st[:, 0])) / self.ticks_per_us.value * 1e-3 if len(st) else None
        self.upd_ms_events = float(np.mean([a.elapsed_time(b) for a, b in events.values()])) if events else None
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
        B = self.B
        raw = self.reports[lo:hi].cpu().numpy()
        counts = {"clean": 0, "corrected": 0, "uncorrectable": 0}
        for s in range(raw.shape[0]):
            for p in range(2):
                v = B.Report.from_buffer_copy(raw[s, p].tobytes()).verdict
                name = ["clean", "corrected", "uncorrectable", "disagree"][v]   # the last from verified checks only
                counts[name] = counts.get(name, 0) + 1
        return counts


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


def cpu_baseline(wl, steps):
    """The float64 oracle as it stands, timed on the host for a few layer-steps of
    the same workload (encoding excluded, as on the GPU)."""
    from oracle import codenet_oracle as O
    from paper_1903_01042_amd import workloads as WL
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    n_in, n_out = wl.widths[0], wl.widths[1]
    P_r, P_c = wl.generators()
    lay = O.CodedLayer(WL.layer_weights(n_out, n_in), P_r, P_c, tau_detect=wl.tau_detect, tau_resid=wl.tau_resid)
    t0 = time.perf_counter()
    for s in range(steps):
        X = wl.inputs(s).T.astype(np.float64)
        D = wl.deltas(s).T.astype(np.float64)
        out = lay.inject(wl.product_faults(WL.PHASE_FWD, s), lay.forward(X))
        lay.detect_decode(O.PHASE_FWD, out)
        out = lay.inject(wl.product_faults(WL.PHASE_BWD, s), lay.backward(D))
        lay.detect_decode(O.PHASE_BWD, out)
        lay.update(wl.eta)
    dt = time.perf_counter() - t0
    return {"value": steps / dt, "unit": "coded layer-steps/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d full-size layer-steps of %s (float64 numpy, encoding excluded)" % (steps, wl.name)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no cross-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1903_01042_amd import workloads as WL
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    wl = WL.WORKLOADS[args.workload]
    total = args.steps + args.warmup

    coded = Runner(wl, True, not args.no_faults, total)
    ms_coded, upd_ms = coded.run(args.steps, args.warmup, not args.graph)
    counts = coded.verdict_counts(args.warmup, total)
    if args.coded_only:
        # a plain device-to-device copy of known size (the coded matrix) next to the kernels:
        # HBM byte counters of a profiling run are scaled by what they read for this copy
        for _ in range(3):
            coded.layer.export_coded()
        torch.cuda.synchronize()
        print(json.dumps({"ms_per_step": ms_coded, "update_kernel_ms": upd_ms if args.graph else coded.upd_ms_events, "verdicts": counts, "workload": wl.name,
                          "calibration_copy_bytes": coded.weight_bytes}))
        return
    uncoded = Runner(wl, False, False, total)
    ms_uncoded, upd_ms_unc = uncoded.run(args.steps, args.warmup, not args.graph)
    ms_clean = None
    if not args.no_faults:
        # the coded path without the injection kernels (scaffolding of the experiment, not of the method)
        clean = Runner(wl, True, False, total)
        ms_clean, _ = clean.run(args.steps, args.warmup, not args.graph)
        clean.layer.destroy()
    # the coded step with both verification steps of Error Model 2 in every check
    ver = Runner(wl, True, not args.no_faults, total, verified=True)
    ms_verified, _ = ver.run(args.steps, args.warmup, not args.graph)
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
        "tflops": flops_step / (ms_coded * 1e-3) / 1e12,
        "mfma_frac_of_peak_whole_step": flops_step / (ms_coded * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS[wl.dtype],
        "uncoded_ms_per_step": ms_uncoded,
        "coding_overhead": ms_coded / ms_uncoded - 1.0,
        "ms_per_step_without_injection": ms_clean,
        "coding_overhead_without_injection": (ms_clean / ms_uncoded - 1.0) if ms_clean else None,
        "ms_per_step_verified_checks": ms_verified,
        "verified_checks_agree": counts_verified == counts,
        "algorithmic_overhead_floor": floor,
        # what the checks, encodings and injection cost beyond the redundant rows themselves
        "excess_over_floor": (ms_coded / ms_uncoded) / (1.0 + floor) - 1.0,
        "excess_over_floor_without_injection": ((ms_clean / ms_uncoded) / (1.0 + floor) - 1.0) if ms_clean else None,
        "verdicts": counts,
        "update_kernel_ms_uncoded": upd_ms_unc if args.graph else uncoded.upd_ms_events,
        "roofline": {"kernel": "update3_kernel (W~ += eta [d;d~][x;x~]^T, fp32 RMW + bf16 copy)"
                     if wl.dtype == "bf16" else "gemm_kernel (update, W~ += eta [d;d~][x;x~]^T)", "bound": "hbm",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(args.workload),
                     "avg_launch_ms": launch_ms,
                     "empty_event_pair_ms": coded.event_pair_ms,
                     "avg_launch_ms_by": ("HIP events around the kernel on every %d-th step of the timed region, "
                                          "where the step's graph ends before the update and the kernel is launched "
                                          "on its own" % Runner.EVENT_EVERY) if args.graph else
                     ("HIP events around the kernel, on its stream, on every %d-th step of the timed region"
                      % Runner.EAGER_EVENT_EVERY),
                     "in_graph_ms": upd_ms if args.graph else None,
                     "in_graph_ms_by": ("device time stamps before and after the kernel inside the graph of every "
                                        "%d-th step of the timed region" % Runner.STAMP_EVERY) if args.graph else None,
                     "device_stamp_ms": upd_ms,
                     "device_stamp_ms_by": "codenet_timestamp kernels (the GPU's 100 MHz wall clock) before and after the "
                                           "update on %s of the timed region: the kernel plus one kernel boundary"
                                           % ("every %d-th step" % (Runner.STAMP_EVERY if args.graph
                                                                     else Runner.EAGER_EVENT_EVERY)),
                     "back_to_back_ms_hip_events": upd_events_ms,
                     "algorithmic_bytes": upd_bytes,
                     "tflops": coded.flops["upd"] / (launch_ms * 1e-3) / 1e12},
    }
    out["regeneration"] = coded.time_regeneration()
    coded.layer.destroy()
    uncoded.layer.destroy()
    if args.cpu_steps > 0:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_steps)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
