"""Pins for oracle/balanced_batches.py: hand traces of the listing, invariants the algorithm
guarantees, and special cases with a closed-form outcome."""
import os

import numpy as np
import pytest

from oracle import balanced_batches as obb

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "balanced_batches_examples.txt")


def read_examples():
    out = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        sizes, cap, gpus, bins = (x.strip() for x in line.split("|"))
        out.append(([int(x) for x in sizes.split()], int(cap), int(gpus),
                    [[int(x) for x in b.split()] for b in bins.split(";")]))
    return out


@pytest.mark.parametrize("sizes,cap,gpus,bins", read_examples())
def test_hand_traces(sizes, cap, gpus, bins):
    assert obb.create_balanced_batches(sizes, cap, gpus) == bins


def random_sizes(rng, n, lo=1, hi=768):
    # a few small molecules, a bulk of mid-sized cells, some large ones (the paper's data set
    # spans 1..768 atoms per structure)
    kind = rng.random(n)
    return np.where(kind < 0.5, rng.integers(lo, 40, n), np.where(kind < 0.9, rng.integers(40, 200, n),
                                                                  rng.integers(200, hi + 1, n)))


@pytest.mark.parametrize("seed,n,cap,gpus", [(1, 200, 3072, 4), (2, 1000, 3072, 8), (3, 50, 768, 3), (4, 777, 1000, 1)])
def test_invariants(seed, n, cap, gpus):
    rng = np.random.default_rng(seed)
    sizes = random_sizes(rng, n)
    bins = obb.create_balanced_batches(sizes, cap, gpus)
    flat = sorted(i for b in bins for i in b)
    assert flat == list(range(n)), "every graph is assigned exactly once"
    loads = [int(sizes[b].sum()) if b else 0 for b in bins]
    assert max(loads) <= cap, "capacity constraint"
    assert len(bins) % gpus == 0, "a multiple of the GPU count"
    assert len(bins) >= -(-int(sizes.sum()) // cap), "at least ceil(S / C) bins"
    # the bins opened by the first call are balanced: the largest-to-emptiest dealing keeps their
    # loads within one largest graph of each other unless a bin was given up early
    first = -(-(-(-int(sizes.sum()) // cap)) // gpus) * gpus
    assert max(loads[:first]) - min(loads[:first]) <= int(sizes.max())


def test_equal_sizes_are_dealt_round_robin():
    # 12 graphs of size 5, capacity 20: ceil(60/20) = 3 bins, four graphs each, dealt cyclically.
    # In every sweep the bins are visited from emptiest to fullest with ties in the previous
    # order; all bins tie, so the order stays 0, 1, 2.
    bins = obb.create_balanced_batches([5] * 12, 20, 1)
    assert bins == [[0, 3, 6, 9], [1, 4, 7, 10], [2, 5, 8, 11]]


def test_single_graph_and_empty_input():
    assert obb.create_balanced_batches([7], 10, 4) == [[0], [], [], []]
    assert obb.create_balanced_batches([], 10, 4) == []


def test_stable_sort_keeps_the_input_order_of_equal_graphs():
    bins = obb.create_balanced_batches([3, 9, 3, 9], 9, 1)      # S = 24 -> 3 bins
    # sorted: 9 (index 1), 9 (index 3), 3 (index 0), 3 (index 2)
    assert bins[0][0] == 1 and bins[1][0] == 3 and bins[2] == [0, 2]


def test_oversized_graph_is_an_error():
    with pytest.raises(ValueError):
        obb.create_balanced_batches([5, 11], 10, 1)


def test_no_worse_than_one_bin_per_graph_and_close_to_the_lower_bound():
    rng = np.random.default_rng(9)
    sizes = random_sizes(rng, 5000)
    bins = obb.create_balanced_batches(sizes, 3072, 8)
    lower = -(-int(sizes.sum()) // 3072)
    used = sum(1 for b in bins if b)
    assert lower <= used <= int(1.1 * lower) + 8
