"""Seeded synthetic inputs for the CodeNet coded layer step.

This module only draws inputs (weights, activations, generator coefficients,
fault lists) from seeded numpy generators.  It holds none of the method's
arithmetic and is the one module that both the HIP path's callers and the
test oracle's callers use, so that both sides see identical inputs.

The five workloads follow the benchmark configurations: layer shapes, node
grids, parity counts, batch sizes, value distributions and fault statistics.
They stand in for the paper's MNIST experiment (3-layer MLP, 784 inputs, 10
classes), whose data is not used here.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

PHASE_FWD, PHASE_BWD, PHASE_WEIGHT = 0, 1, 2
MODE_DENSE_REL, MODE_SPARSE_ABS = 0, 1

SEED_WEIGHTS, SEED_INPUTS, SEED_DELTAS, SEED_GENERATOR, SEED_FAULTS, SEED_NOISE = (
    1000, 2000, 3000, 0, 4000, 5000)


# ---------------------------------------------------------------- generators
def paper_example_generators():
    """Parity parts of the worked example's (4,2) codes: G_r = [I | P_r],
    G_c = [I | P_c] (Section on pre-processing, m = n = 2, t = 1)."""
    return (np.array([[1.0, 1.0], [1.0, -1.0]]), np.array([[1.0, 1.0], [1.0, 2.0]]))


def gaussian_generator(a, r, seed=SEED_GENERATOR, min_abs=0.25):
    """iid N(0,1) parity coefficients; draws with |g| < min_abs are redrawn so
    that no block is (nearly) invisible to a check."""
    rng = np.random.default_rng(seed)
    P = rng.standard_normal((a, r))
    while True:
        small = np.abs(P) < min_abs
        if not small.any():
            return P
        P[small] = rng.standard_normal(int(small.sum()))


def vandermonde_like(a, r, nodes="spread"):
    """P[i, k] = alpha_i ** k  (the worked example's P_c is this with alpha = (1, 2)).

    nodes="spread" (r <= 2): alpha_i = tan(theta_i) with the a angles spaced
    evenly inside (0, 90) and (90, 180) degrees, so that the a + 2 columns of
    H = [P^T | -I] point in well separated directions (the two parity columns
    sit at 0 and 90 degrees).  nodes="positive": alpha_i = 1 + i / a, distinct
    and positive, hence every minor of P is positive for any r.
    """
    if nodes == "spread" and r <= 2:
        q1 = (a + 1) // 2
        q2 = a - q1
        th = [90.0 * (q + 1) / (q1 + 1) for q in range(q1)]
        th += [90.0 + 90.0 * (q + 1) / (q2 + 1) for q in range(q2)]
        alpha = np.tan(np.deg2rad(np.array(th)))
    else:
        alpha = 1.0 + np.arange(a) / float(a)
    return np.stack([alpha ** k for k in range(r)], axis=1) if r > 0 else np.zeros((a, 0))


# -------------------------------------------------------------------- tensors
def normal(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


def uniform01(shape, seed):
    return np.random.default_rng(seed).random(shape, dtype=np.float64).astype(np.float32)


def layer_weights(n_out, n_in, layer=0):
    """W ~ N(0, 1 / n_in), float32."""
    return normal((n_out, n_in), SEED_WEIGHTS + layer, scale=1.0 / np.sqrt(n_in))


# --------------------------------------------------------------------- faults
def make_fault(phase, bi, bj, step, seed=SEED_NOISE, lo=1.0, hi=10.0,
               mode=MODE_DENSE_REL, density=0.0):
    return dict(phase=int(phase), bi=int(bi), bj=int(bj), step=int(step), seed=int(seed),
                lo=float(lo), hi=float(hi), mode=int(mode), density=float(density))


def active_nodes(phase, m, n, r_r, r_c):
    """Nodes that produce an output in a phase (forward: all block-rows, base
    columns; backward: base rows, all block-columns; update: every stored node
    outside the parity x parity corner)."""
    if phase == PHASE_FWD:
        return [(i, j) for i in range(m + r_r) for j in range(n)]
    if phase == PHASE_BWD:
        return [(i, j) for i in range(m) for j in range(n + r_c)]
    return [(i, j) for i in range(m + r_r) for j in range(n + r_c) if i < m or j < n]


def bernoulli_faults(phase, m, n, r_r, r_c, p, step, layer=0, seed=SEED_FAULTS, **kw):
    """Each active node fails independently with probability p in this product."""
    rng = np.random.default_rng([seed, step, layer, phase])
    nodes = active_nodes(phase, m, n, r_r, r_c)
    hits = rng.random(len(nodes)) < p
    return [make_fault(phase, i, j, step, seed=SEED_NOISE + 7 * layer, **kw)
            for (i, j), h in zip(nodes, hits) if h]


def exact_faults(phase, m, n, r_r, r_c, count, step, layer=0, seed=SEED_FAULTS, **kw):
    """Exactly `count` distinct active nodes fail in this product."""
    rng = np.random.default_rng([seed, step, layer, phase])
    nodes = active_nodes(phase, m, n, r_r, r_c)
    pick = rng.choice(len(nodes), size=count, replace=False)
    return [make_fault(phase, nodes[k][0], nodes[k][1], step, seed=SEED_NOISE + 7 * layer, **kw)
            for k in sorted(pick)]


def upto_faults(phase, m, n, r_r, r_c, max_count, step, layer=0, seed=SEED_FAULTS, **kw):
    """0..max_count failing nodes (uniform count) in this product."""
    rng = np.random.default_rng([seed + 1, step, layer, phase])
    count = int(rng.integers(0, max_count + 1))
    return exact_faults(phase, m, n, r_r, r_c, count, step, layer, seed, **kw)


# ------------------------------------------------------------------ workloads
@dataclass
class Workload:
    name: str
    widths: Tuple[int, ...]            # N_0, N_1, ..., N_L
    grid: Tuple[int, int]              # m, n
    r: int                             # parity block-rows = parity block-columns
    batch: int
    steps: int
    dtype: str                         # "f32" or "bf16"
    generator: str                     # "gaussian" | "vandermonde"
    input_law: str = "normal"          # "normal" | "uniform01"
    eta: float = 0.01
    fault_law: str = "none"            # "one" | "bernoulli" | "upto2"
    fault_p: float = 0.0
    weight_faults: bool = False
    tau_detect: float = 1e-3
    tau_resid: float = 2e-3
    drift_every: int = 0
    notes: str = ""

    def generators(self, layer=0):
        m, n = self.grid
        if self.r == 0:
            return np.zeros((m, 0)), np.zeros((n, 0))
        if self.generator == "gaussian":
            return (gaussian_generator(m, self.r, SEED_GENERATOR + 2 * layer),
                    gaussian_generator(n, self.r, SEED_GENERATOR + 2 * layer + 1))
        return vandermonde_like(m, self.r), vandermonde_like(n, self.r)

    def product_faults(self, phase, step, layer=0):
        m, n = self.grid
        if self.fault_law == "none" or self.r == 0:
            return []
        if self.fault_law == "one":
            # exactly one corrupted node-block output per step: the step's parity
            # decides which of the two products carries it
            if (step % 2 == 0) != (phase == PHASE_FWD):
                return []
            return exact_faults(phase, m, n, self.r, self.r, 1, step, layer)
        if self.fault_law == "upto2":
            return upto_faults(phase, m, n, self.r, self.r, 2, step, layer)
        return bernoulli_faults(phase, m, n, self.r, self.r, self.fault_p, step, layer)

    def update_faults(self, step, layer=0):
        m, n = self.grid
        if not self.weight_faults or self.r == 0:
            return []
        return bernoulli_faults(PHASE_WEIGHT, m, n, self.r, self.r, self.fault_p, step, layer)

    def inputs(self, step):
        shape = (self.batch, self.widths[0])
        if self.input_law == "uniform01":
            return uniform01(shape, SEED_INPUTS + step)
        return normal(shape, SEED_INPUTS + step)

    def deltas(self, step, layer=None):
        """Backpropagated error fed to a single-layer workload (no loss head)."""
        layer = len(self.widths) - 2 if layer is None else layer
        return normal((self.batch, self.widths[layer + 1]), SEED_DELTAS + step)

    def scaled(self, block, batch=None, steps=None):
        """Same grid, parity count and fault law with every width shrunk so that a
        block is `block` wide: the size the float64 oracle follows for many steps."""
        m, n = self.grid
        widths = tuple(min(w, block * (n if k == 0 else m)) for k, w in enumerate(self.widths))
        return Workload(**{**self.__dict__, "name": self.name + "-scaled", "widths": widths,
                           "batch": batch or self.batch, "steps": steps or self.steps})


WORKLOADS = {
    # one 256x256 layer, 2x2 grid + 1 parity row/col (detect-only: t = 0)
    "cfg1": Workload("cfg1-256-2x2+1", (256, 256), (2, 2), 1, 16, 10, "f32", "gaussian",
                     fault_law="one"),
    # 784-1024-1024-10 MLP, 4x4 grid + 1 parity row/col per layer
    "cfg2": Workload("cfg2-mlp784-4x4+1", (784, 1024, 1024, 10), (4, 4), 1, 128, 100, "f32",
                     "gaussian", input_law="uniform01", fault_law="bernoulli", fault_p=0.05),
    # one 4096x4096 layer, bf16 inputs / fp32 accumulate, 8x8 grid + 2 parity rows/cols
    "cfg3": Workload("cfg3-4096-8x8+2-bf16", (4096, 4096), (8, 8), 2, 512, 50, "bf16",
                     "vandermonde", fault_law="upto2", tau_detect=2e-2, tau_resid=2e-2),
    # 8-layer width-8192 MLP, 8x8 grid + 2 parity rows/cols, faults in fwd, bwd and update
    "cfg4": Workload("cfg4-mlp8192x8-8x8+2", (8192,) * 9, (8, 8), 2, 1024, 20, "f32",
                     "vandermonde", fault_law="bernoulli", fault_p=0.02, weight_faults=True),
    # update-heavy: one 16384x16384 layer, 16x16 grid + 2, batch 64, drift check every 50 steps
    "cfg5": Workload("cfg5-16384-16x16+2", (16384, 16384), (16, 16), 2, 64, 200, "f32",
                     "vandermonde", fault_law="bernoulli", fault_p=0.01, weight_faults=True,
                     drift_every=50),
}
