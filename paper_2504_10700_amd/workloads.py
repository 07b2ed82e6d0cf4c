"""Seeded synthetic inputs for the symmetric contraction.

Holds none of the method's arithmetic: shapes, value distributions and the
element mix only.  Both the HIP path and the CPU oracle are fed from here, so a
parity test compares the two on identical arrays.

The paper trains on eight chemistry datasets (Evaluation, dataset table) that
are not available; the contraction is a per-atom operation that sees only the
node count, the element index of each node, A and W, so the stand-ins below
keep those: batches of a few thousand to 200k atoms, 89 elements with a few
dominant ones, structures of 10..190 atoms concatenated, A ~ N(0,1).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import numpy as np

# indices (atomic number - 1) of the six dominant elements: H C N O Si Fe
DOMINANT_ELEMENTS = (0, 5, 6, 7, 13, 25)


@dataclass(frozen=True)
class Workload:
    name: str
    num_nodes: int
    num_elements: int
    num_channels: int
    l_max: int
    nu_max: int
    out_irreps: Tuple[Tuple[int, int], ...]   # (L, parity)
    dtype: str                                # "f32" | "f64"
    seed: int
    z_mode: str = "skewed"                    # "uniform" | "skewed"
    structures: Optional[int] = None          # concatenated structures (sizes 10..190)
    backward: bool = True

    @property
    def n_lm(self) -> int:
        return (self.l_max + 1) ** 2

    @property
    def n_LM(self) -> int:
        return sum(2 * L + 1 for L, _ in self.out_irreps)


_O01 = ((0, 1), (1, -1))
_O012 = ((0, 1), (1, -1), (2, 1))

WORKLOADS = {
    "tiny": Workload("tiny", 64, 2, 8, 1, 2, ((0, 1),), "f64", 1001, z_mode="uniform"),
    "medium_fwd": Workload("medium_fwd", 10_000, 89, 128, 3, 3, _O01, "f32", 1002, backward=False),
    "training_step": Workload("training_step", 10_000, 89, 128, 3, 3, _O01, "f32", 1003),
    "large_batch": Workload("large_batch", 200_000, 89, 128, 3, 3, _O01, "f32", 1004, structures=2000),
    "wide_high_l": Workload("wide_high_l", 50_000, 89, 256, 3, 3, _O012, "f32", 1005),
    "wide_high_l_f64": Workload("wide_high_l_f64", 5_000, 89, 256, 3, 3, _O012, "f64", 1006),
}


def element_probabilities(num_elements: int, z_mode: str) -> np.ndarray:
    if z_mode == "uniform" or num_elements <= len(DOMINANT_ELEMENTS):
        return np.full(num_elements, 1.0 / num_elements)
    p = np.full(num_elements, 0.0)
    dom = [e for e in DOMINANT_ELEMENTS if e < num_elements]
    p[dom] = 0.10
    rest = [e for e in range(num_elements) if e not in dom]
    p[rest] = (1.0 - 0.10 * len(dom)) / len(rest)
    return p


def structure_sizes(rng: np.random.Generator, n_structures: int, total: int,
                    lo: int = 10, hi: int = 190) -> np.ndarray:
    """Sizes uniform in lo..hi, nudged by +-1 cyclically (within bounds) to sum to total."""
    sizes = rng.integers(lo, hi + 1, size=n_structures)
    diff = int(total - sizes.sum())
    step = 1 if diff > 0 else -1
    i = 0
    while diff != 0:
        if lo <= sizes[i] + step <= hi:
            sizes[i] += step
            diff -= step
        i = (i + 1) % n_structures
    return sizes


@dataclass
class Inputs:
    A: np.ndarray      # (N, K, n_lm)   fp64 master copy
    z: np.ndarray      # (N,) int32
    W: np.ndarray      # (Z, P, K)
    dB: np.ndarray     # (N, K, n_LM)
    structure_sizes: Optional[np.ndarray] = None


def make_inputs(wl: Workload, paths: Sequence[Sequence[int]], num_nodes: Optional[int] = None) -> Inputs:
    """Draw z, A, W, dB (in that order) in fp64 from numpy's default_rng(seed).

    `paths` is the caller's path table, rows (nu, out_index, ...): only used to
    count the paths per (nu, output irrep) for the weight scale
    W ~ N(0,1) / sqrt(#paths of that (nu, output irrep)).
    """
    rng = np.random.default_rng(wl.seed)
    N = wl.num_nodes if num_nodes is None else num_nodes
    sizes = None
    if wl.structures is not None and num_nodes is None:
        sizes = structure_sizes(rng, wl.structures, N)
    z = rng.choice(wl.num_elements, size=N, p=element_probabilities(wl.num_elements, wl.z_mode))
    z = z.astype(np.int32)
    A = rng.standard_normal((N, wl.num_channels, wl.n_lm))
    paths = np.asarray(paths, dtype=np.int64).reshape(-1, 6)
    P = paths.shape[0]
    counts = {}
    for row in paths:
        counts[(row[0], row[1])] = counts.get((row[0], row[1]), 0) + 1
    scale = np.array([1.0 / np.sqrt(counts[(row[0], row[1])]) for row in paths])
    W = rng.standard_normal((wl.num_elements, P, wl.num_channels)) * scale[None, :, None]
    dB = rng.standard_normal((N, wl.num_channels, wl.n_LM))
    return Inputs(A=A, z=z, W=W, dB=dB, structure_sizes=sizes)


def make_cotangent(wl: Workload, num_nodes: Optional[int] = None) -> np.ndarray:
    """H, the cotangent of dA for the second-order pass: N(0,1) of the shape of A, fp64,
    from its own stream default_rng(seed + 7919) so that make_inputs stays unchanged."""
    N = wl.num_nodes if num_nodes is None else num_nodes
    return np.random.default_rng(wl.seed + 7919).standard_normal((N, wl.num_channels, wl.n_lm))
