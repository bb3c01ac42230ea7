"""Seeded synthetic inputs and fault-injection trial specs for the five workloads.

This module holds no arithmetic of the coded-computation method: it only draws
random matrices, picks which nodes straggle, and picks which bits are flipped.
Both the CPU oracle's tests and the GPU path's tests/bench import it so that
they see identical arrays.

The paper (arXiv 1811.10751) uses no dataset and runs no experiment; nothing
here stands in for a public benchmark.  Shapes and distributions follow the
five configurations of this build's benchmark definition:

  cfg0  tiny coded matmul        A,B 256x256 U[-1,1] seed 0, m=n=d=2, P=10
  cfg1  matmul with stragglers   A,B 4096x4096 U[-1,1] seed 0, m=n=d=2, P=16
  cfg2  B=1 coded MLP            4096-4096-4096-10, W~N(0,1/4096), m=4,n=2,P=24
  cfg3  B=256 coded MLP          4096-8192-8192-10, m=2,n=4,P=32, bf16 workers
  cfg4  soft errors              cfg1 inputs + one bit flip per corrupted node
"""
from __future__ import annotations

import numpy as np

CONFIGS = {
    0: dict(kind="matmul", N1=256, N0=256, Nc=256, m=2, n=2, d=2, P=10, seed=0),
    1: dict(kind="matmul", N1=4096, N0=4096, Nc=4096, m=2, n=2, d=2, P=16, seed=0,
            trials=100, trial_seed0=1000),
    2: dict(kind="mlp", sizes=(4096, 4096, 4096, 10), batch=1, m=4, n=2, d1=1, d2=1,
            P=24, seed=2, steps=1000, eta=0.01, decay=0.0, worker="f32"),
    3: dict(kind="mlp", sizes=(4096, 8192, 8192, 10), batch=256, m=2, n=4, d1=1, d2=1,
            P=32, seed=3, steps=20, eta=0.01, decay=0.0, worker="bf16"),
    4: dict(kind="matmul", N1=4096, N0=4096, Nc=4096, m=2, n=2, d=2, P=16, seed=0,
            trials=1000, trial_seed0=5000, flip_prob=0.05),
}


def matmul_inputs(N1: int, N0: int, Nc: int, seed: int = 0):
    """A (N1 x N0) then B (N0 x Nc), uniform on [-1, 1], fp32, C-contiguous."""
    rng = np.random.default_rng(seed)
    A = rng.uniform(-1.0, 1.0, size=(N1, N0)).astype(np.float32)
    B = rng.uniform(-1.0, 1.0, size=(N0, Nc)).astype(np.float32)
    return A, B


def erasure_trial(trial_seed: int, P: int, n_drop: int) -> np.ndarray:
    """uint8[P] presence mask with a seeded random set of n_drop nodes missing."""
    rng = np.random.default_rng(trial_seed)
    dropped = rng.choice(P, size=n_drop, replace=False)
    present = np.ones(P, dtype=np.uint8)
    present[dropped] = 0
    return present


def bitflip_trial(trial_seed: int, P: int, n_elem: int, max_errors: int,
                  prob: float = 0.05):
    """List of (node, flat element index, bit) soft errors for one trial.

    Every node is corrupted independently with probability `prob`, in node
    order, stopping once `max_errors` nodes are corrupted.  A corrupted node
    gets one flipped bit (0..31) in one uniformly chosen fp32 element of its
    output block.
    """
    rng = np.random.default_rng(trial_seed)
    flips = []
    for p in range(P):
        hit = rng.random() < prob
        elem = int(rng.integers(0, n_elem))
        bit = int(rng.integers(0, 32))
        if hit and len(flips) < max_errors:
            flips.append((p, elem, bit))
    return flips


def apply_bitflips(stack: np.ndarray, flips) -> np.ndarray:
    """Return a copy of the fp32 stack [P, rows, cols] with the listed bits flipped."""
    assert stack.dtype == np.float32
    out = np.ascontiguousarray(stack).copy()
    words = out.view(np.uint32).reshape(out.shape[0], -1)
    for (p, elem, bit) in flips:
        words[p, elem] ^= np.uint32(1 << bit)
    return out


def gaussian_node_errors(trial_seed: int, P: int, n_bad: int, shape, scale: float = 1.0):
    """Whole-node additive Gaussian noise: (sorted bad node list, noise[n_bad, *shape])."""
    rng = np.random.default_rng(trial_seed)
    bad = np.sort(rng.choice(P, size=n_bad, replace=False))
    noise = (scale * rng.standard_normal(size=(n_bad,) + tuple(shape))).astype(np.float32)
    return bad, noise


def mlp_init(sizes, seed: int):
    """Weight matrices W^l of shape (sizes[l+1], sizes[l]), N(0, 1/4096) entries, fp32."""
    rng = np.random.default_rng(seed)
    sigma = 1.0 / 64.0
    return [(sigma * rng.standard_normal(size=(sizes[l + 1], sizes[l]))).astype(np.float32)
            for l in range(len(sizes) - 1)]


def mlp_batch(seed: int, step: int, n_in: int, n_classes: int, batch: int):
    """Inputs X (n_in x batch) uniform on [-1,1] and one-hot labels Y (n_classes x batch)."""
    rng = np.random.default_rng([seed, step])
    X = rng.uniform(-1.0, 1.0, size=(n_in, batch)).astype(np.float32)
    cls = rng.integers(0, n_classes, size=batch)
    Y = np.zeros((n_classes, batch), dtype=np.float32)
    Y[cls, np.arange(batch)] = 1.0
    return X, Y
