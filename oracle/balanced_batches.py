"""Oracle of the load balancer: the iterative multi-objective bin packing of the paper.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Follows Algorithm CREATE-BALANCED-BATCHES (Section 3, the subsection on the iterative
multi-objective bin packing) step by step, in its notation: L the graph sizes (vertex counts), C the bin
capacity, G the number of GPUs, c(B_j) the remaining capacity of bin j, p the pointer into the
sorted list.  Plain Python lists and the language's stable sort; nothing is reorganised for
speed.

Readings of what the paper leaves open:
* the sort of the bins takes the listing's line (stable, by remaining capacity, descending:
  the emptiest bin receives the next - largest remaining - graph); the prose next to it speaks
  of prioritising fuller bins, which contradicts the listing and the stated goal of balance;
* the second-chance test (some bin still accepting graphs has less room left than some bin
  already given up on) compares the smallest remaining capacity among the bins still active
  after the sweep with the largest among the bins marked full in that sweep;
* a bin keeps the identity it was created with: bins of the first call are numbered 0..M-1,
  bins created by the recursive call for the remaining graphs continue the numbering; bins that
  stay empty (M is rounded up to a multiple of G) are kept, so that every call contributes a
  multiple of G bins;
* a graph larger than C cannot be placed at all: that is an error.
"""
from __future__ import annotations

from typing import List, Sequence


def create_balanced_batches(L: Sequence[int], C: int, G: int) -> List[List[int]]:
    """Returns the bins in creation order, each a list of graph indices (positions in L) in the
    order in which they were added."""
    sizes = [int(x) for x in L]
    if C < 1 or G < 1:
        raise ValueError("capacity and number of GPUs must be positive")
    if any(s < 0 or s > C for s in sizes):
        raise ValueError("a graph is larger than the bin capacity (or negative)")
    return _create(sizes, list(range(len(sizes))), C, G)


def _create(L: List[int], index: List[int], C: int, G: int) -> List[List[int]]:
    N = len(L)
    if N == 0:
        return []
    # (L, I) <- StableSort(L, descending)
    order = sorted(range(N), key=lambda i: -L[i])          # Python's sort is stable
    Ls = [L[i] for i in order]
    I = [index[i] for i in order]
    S = sum(Ls)
    M = -(-S // C)                                          # ceil(S / C)
    M = max(M, 1)                                           # all-zero sizes still need a bin
    M = -(-M // G) * G                                      # ceil(M / G) * G
    content: List[List[int]] = [[] for _ in range(M)]       # B_j
    c = [C] * M                                             # c(B_j)
    active = list(range(M))                                 # the bins still in B, as bin ids
    p = 0
    while p < N and active:
        active.sort(key=lambda j: -c[j])                    # stable, by remaining capacity, descending
        full = []
        still = []
        for j in active:
            if p < N and c[j] >= Ls[p]:
                content[j].append(I[p])
                c[j] -= Ls[p]
                p += 1
                still.append(j)
            elif p < N:
                full.append(j)                              # mark B_j as full
            else:
                still.append(j)                             # the sweep ended (break): untouched bins stay
        active = still
        # second chance: a bin that kept accepting graphs is now fuller than a bin given up on
        if full and active and min(c[j] for j in active) < max(c[j] for j in full):
            active = active + full
    bins = content
    if p < N:
        rest = _create(Ls[p:], I[p:], C, G)
        bins = bins + rest
    return bins
