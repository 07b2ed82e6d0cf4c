"""Oracle of the load balancer: the iterative multi-objective bin packing of the paper.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Algorithm CREATE-BALANCED-BATCHES (Section 3): graphs with vertex counts L are distributed
over bins (mini-batches) of capacity C, the number of bins a multiple of the number of GPUs G.
In the words of this file:

  * one ROUND works on the graphs that are still unplaced, largest first (a stable ordering, so
    equal graphs keep their input order).  It opens ceil(ceil(S / C) / G) * G bins, S being the
    vertices still unplaced;
  * a round is a sequence of PASSES over the bins that still accept graphs.  Before a pass
    they are ordered by the room they have left, most room first (stable: ties keep the order
    of the previous pass).  The pass hands the next graph to each bin in turn; a bin without
    room for the graph it is offered is given up for this round, yet the graph stays next in
    line for the following bin.  When the graphs run out mid-pass the remaining bins are
    simply not visited;
  * after a pass, if some bin that is still accepting has less room left than some bin given up
    in that pass, the bins given up in that pass come back (behind the accepting ones): smaller
    graphs are coming and may still fit;
  * a round ends when no bin accepts any more; graphs still unplaced start the next round.

Readings of what the paper leaves open:
* the ordering before a pass is by room left, most first, as the listing has it - the largest
  unplaced graph goes to the emptiest bin; the prose beside it speaks of fuller bins first,
  which contradicts both the listing and the stated goal of balance;
* the come-back test compares the least room among the bins still accepting after the pass
  with the most room among the bins given up in that pass;
* bins keep the number they were opened with: the first round opens 0..M-1, later rounds continue;
  bins that stay empty (M is rounded up to a multiple of G) are kept, so every round
  contributes a multiple of G bins;
* a graph larger than C can never be placed: an error.
"""
from __future__ import annotations

from typing import List, Sequence


class _Bin:
    def __init__(self, number: int, capacity: int):
        self.number = number
        self.room = capacity
        self.graphs: List[int] = []


def create_balanced_batches(L: Sequence[int], C: int, G: int) -> List[List[int]]:
    """Returns the bins in the order they were opened, each a list of graph indices (positions in
    L) in the order in which the bin received them."""
    sizes = [int(x) for x in L]
    if C < 1 or G < 1:
        raise ValueError("capacity and number of GPUs must be positive")
    if any(s < 0 or s > C for s in sizes):
        raise ValueError("a graph is larger than the bin capacity (or negative)")
    unplaced = sorted(range(len(sizes)), key=lambda g: -sizes[g])   # stable: equal sizes keep input order
    bins: List[_Bin] = []
    while unplaced:
        unplaced = _round(sizes, unplaced, C, G, bins)
    return [b.graphs for b in bins]


def _round(sizes: List[int], queue: List[int], C: int, G: int, bins: List[_Bin]) -> List[int]:
    """One round: opens its bins (appended to `bins`), places what it can, returns the rest."""
    total = sum(sizes[g] for g in queue)
    n_bins = max(-(-total // C), 1)          # graphs of size zero still need a bin
    n_bins = -(-n_bins // G) * G
    accepting = [_Bin(len(bins) + k, C) for k in range(n_bins)]
    bins.extend(accepting)
    nxt = 0                                   # position in the queue of the next graph to place
    while nxt < len(queue) and accepting:
        accepting.sort(key=lambda b: -b.room)  # most room first; list.sort is stable
        kept, given_up = [], []
        for b in accepting:
            if nxt == len(queue):
                kept.append(b)                # the graphs ran out: not visited, stays as it is
            elif b.room >= sizes[queue[nxt]]:
                b.graphs.append(queue[nxt])
                b.room -= sizes[queue[nxt]]
                nxt += 1
                kept.append(b)
            else:
                given_up.append(b)
        accepting = kept
        if accepting and given_up and min(b.room for b in accepting) < max(b.room for b in given_up):
            accepting = accepting + given_up
    return queue[nxt:]
