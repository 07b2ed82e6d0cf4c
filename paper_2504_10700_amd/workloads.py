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
    dtype: str                                # "f32" | "f64" | "bf16" (rows in bfloat16, weights and arithmetic fp32)
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
_O0123 = ((0, 1), (1, -1), (2, 1), (3, -1))

WORKLOADS = {
    "tiny": Workload("tiny", 64, 2, 8, 1, 2, ((0, 1),), "f64", 1001, z_mode="uniform"),
    "medium_fwd": Workload("medium_fwd", 10_000, 89, 128, 3, 3, _O01, "f32", 1002, backward=False),
    "training_step": Workload("training_step", 10_000, 89, 128, 3, 3, _O01, "f32", 1003),
    "large_batch": Workload("large_batch", 200_000, 89, 128, 3, 3, _O01, "f32", 1004, structures=2000),
    "wide_high_l": Workload("wide_high_l", 50_000, 89, 256, 3, 3, _O012, "f32", 1005),
    "wide_high_l_f64": Workload("wide_high_l_f64", 5_000, 89, 256, 3, 3, _O012, "f64", 1006),
    # not one of the task's configurations: every output irrep up to L = 3 at the training-step shape
    "outputs_l3": Workload("outputs_l3", 10_000, 89, 128, 3, 3, _O0123, "f32", 1008),
    # the training step with A, B, dB, dA stored as bfloat16
    "training_step_bf16": Workload("training_step_bf16", 10_000, 89, 128, 3, 3, _O01, "bf16", 1003),
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


# ---------------------------------------------------------------------------------------
# Channelwise tensor product (Algorithm 1): a graph, per-edge Y and R, per-node h.
#
# The paper's graphs come from a 4 Angstrom cutoff on molecules, liquids and crystals
# (Evaluation, dataset description): a few to a few tens of neighbours per atom, and a batch
# is many small structures (1..768 atoms) whose edges never cross structure boundaries.  The
# stand-in cuts the atoms into structures of 10..190 atoms (as for `large_batch`), draws the
# in-degree of every atom from Poisson(mean_degree) (clipped to 4 * mean_degree, and about 1%
# of the atoms receive nothing), senders uniformly among the other atoms of the same
# structure (several edges between one pair stand for periodic images), edges grouped by
# receiver as neighbour lists are.  Y, h, dA ~ N(0,1) (the
# components of spherical harmonics in the usual "component" normalisation have unit rms);
# R ~ N(0,1) / sqrt(mean_degree * #paths into the same l3) so that A is O(1).

@dataclass(frozen=True)
class TPWorkload:
    name: str
    num_nodes: int
    mean_degree: int
    num_channels: int
    l_Y: int
    l_h: int
    L_max: int
    dtype: str
    seed: int

    @property
    def n_Y(self) -> int:
        return (self.l_Y + 1) ** 2

    @property
    def n_h(self) -> int:
        return (self.l_h + 1) ** 2

    @property
    def n_out(self) -> int:
        return (self.L_max + 1) ** 2


TP_WORKLOADS = {
    "tp_tiny": TPWorkload("tp_tiny", 40, 5, 8, 1, 1, 1, "f64", 4001),
    "tp_first_layer": TPWorkload("tp_first_layer", 10_000, 20, 128, 3, 0, 3, "f32", 4002),
    "tp_training_step": TPWorkload("tp_training_step", 10_000, 20, 128, 3, 1, 3, "f32", 4003),
    "tp_large_batch": TPWorkload("tp_large_batch", 50_000, 20, 128, 3, 1, 3, "f32", 4004),
}


@dataclass
class TPInputs:
    Y: np.ndarray          # (E, n_Y)
    h: np.ndarray          # (N, K, n_h)
    R: np.ndarray          # (E, P, K)
    dA: np.ndarray         # (N, K, n_out)
    sender: np.ndarray     # (E,) int32
    receiver: np.ndarray   # (E,) int32, ascending
    row_ptr: np.ndarray    # (N+1,) int32: edges received by node i are row_ptr[i]..row_ptr[i+1]
    send_ptr: np.ndarray   # (N+1,) int32
    send_edge: np.ndarray  # (E,) int32: edge ids grouped by sender, ascending within a sender


def graph_indices(sender: np.ndarray, receiver: np.ndarray, num_nodes: int):
    """row_ptr, send_ptr, send_edge for edges already grouped by receiver."""
    row_ptr = np.zeros(num_nodes + 1, dtype=np.int32)
    row_ptr[1:] = np.cumsum(np.bincount(receiver, minlength=num_nodes))
    send_ptr = np.zeros(num_nodes + 1, dtype=np.int32)
    send_ptr[1:] = np.cumsum(np.bincount(sender, minlength=num_nodes))
    send_edge = np.argsort(sender, kind="stable").astype(np.int32)
    return row_ptr, send_ptr, send_edge


def make_tp_graph(wl: TPWorkload, rng: np.random.Generator):
    """The graph of a tensor-product workload drawn from `rng` (the first draws of make_tp_inputs):
    (sender, receiver) per edge, edges grouped by receiver."""
    N = wl.num_nodes
    deg = np.minimum(rng.poisson(wl.mean_degree, size=N), 4 * wl.mean_degree)
    deg[rng.random(N) < 0.01] = 0
    if N == 1:
        deg[:] = 0
    # structures: consecutive runs of atoms; small graphs are one structure
    if N >= 400:
        sizes = structure_sizes(rng, max(1, N // 100), N)
    else:
        sizes = np.array([N])
    first = np.repeat(np.cumsum(sizes) - sizes, sizes)    # first atom of every atom's structure
    size_of = np.repeat(sizes, sizes)
    deg[size_of == 1] = 0
    receiver = np.repeat(np.arange(N, dtype=np.int32), deg)
    E = int(receiver.size)
    lo, span = first[receiver], size_of[receiver]
    sender = (lo + rng.integers(0, 1 << 30, size=E) % np.maximum(span - 1, 1)).astype(np.int32)
    sender += (sender >= receiver).astype(np.int32)      # never the receiver itself
    return sender, receiver


def make_tp_inputs(wl: TPWorkload, paths: Sequence[Sequence[int]]) -> TPInputs:
    """Draws the graph, then Y, h, R, dA (in that order) in fp64 from default_rng(seed).
    `paths`: the caller's path table, rows (l1, l2, l3), used only to count the paths per l3."""
    rng = np.random.default_rng(wl.seed)
    N = wl.num_nodes
    sender, receiver = make_tp_graph(wl, rng)
    E = int(receiver.size)
    paths = np.asarray(paths, dtype=np.int64).reshape(-1, 3)
    per_l3 = np.bincount(paths[:, 2], minlength=wl.L_max + 1)
    scale = 1.0 / np.sqrt(max(wl.mean_degree, 1) * per_l3[paths[:, 2]])
    Y = rng.standard_normal((E, wl.n_Y))
    h = rng.standard_normal((N, wl.num_channels, wl.n_h))
    R = rng.standard_normal((E, paths.shape[0], wl.num_channels)) * scale[None, :, None]
    dA = rng.standard_normal((N, wl.num_channels, wl.n_out))
    row_ptr, send_ptr, send_edge = graph_indices(sender, receiver, N)
    return TPInputs(Y, h, R, dA, sender, receiver, row_ptr, send_ptr, send_edge)


def make_tp_cotangents(wl: TPWorkload, inp: TPInputs):
    """HY, Hh, HR: cotangents of (dY, dh, dR) for the second-order pass, N(0,1) of the shapes of
    Y, h, R, from their own stream default_rng(seed + 7919)."""
    rng = np.random.default_rng(wl.seed + 7919)
    return rng.standard_normal(inp.Y.shape), rng.standard_normal(inp.h.shape), rng.standard_normal(inp.R.shape)


def make_graph_sizes(n_graphs: int, seed: int = 6001, max_size: int = 768) -> np.ndarray:
    """Vertex counts for the load balancer: half small molecules (1..39 atoms), 40% mid-sized
    cells (40..199), 10% large systems (200..max_size); the paper's combined data set spans
    1..768 atoms per structure with most structures small (Evaluation, data set description)."""
    rng = np.random.default_rng(seed)
    kind = rng.random(n_graphs)
    sizes = np.where(kind < 0.5, rng.integers(1, 40, n_graphs),
                     np.where(kind < 0.9, rng.integers(40, 200, n_graphs), rng.integers(200, max_size + 1, n_graphs)))
    return sizes.astype(np.int32)


def make_linear_inputs(n_nodes: int, k_in: int, k_out: int, l_max: int, seed: int):
    """X, W, dY for the per-order channel-mixing linear: X, dY ~ N(0,1), W ~ N(0,1)/sqrt(k_in)."""
    rng = np.random.default_rng(seed)
    nc = (l_max + 1) ** 2
    X = rng.standard_normal((n_nodes, k_in, nc))
    W = rng.standard_normal((l_max + 1, k_in, k_out)) / np.sqrt(k_in)
    dY = rng.standard_normal((n_nodes, k_out, nc))
    return X, W, dY

