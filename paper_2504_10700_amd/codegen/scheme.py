"""Evaluation scheme of the generated kernels: coupled (irrep-level) Horner form.

Algorithm 2 of arXiv 2504.10700 sums, per output component, over all monomials of
A with a weight and a generalized Clebsch-Gordan coefficient each.  The generated
kernels compute the same polynomial in a factored form:

  1. pair couplings   T(l1,l2,L2)[M2] = sum C(l1,l2,L2)[m1,m2,M2] a_l1[m1] a_l2[m2]
     (shared by every path and output that needs them),
  2. weighted sums    S(L2,l3,L)[M2]  = sum_s w_s T_s[M2]      over the internal paths s
     that couple their pair to L2 and then with a_l3 to the output L,
  3. second coupling  B_L[M]         += sum C(L2,l3,L)[M2,m3,M] S[M2] a_l3[m3],
     plus the nu = 1 and nu = 2 terms  w a_L  and  w T(l1,l2,L).

The internal paths form a minimal basis of the symmetric polynomials (the external,
ordered paths of the C ABI are over-complete): external weights are folded into
internal ones (w' = F w) and internal weight gradients unfolded (dW = F^T dW').
The backward program is the reverse-mode derivative of the same graph.
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

from .program import Program

CG = Callable[[int, int, int], np.ndarray]


@dataclass(frozen=True)
class InternalPath:
    nu: int
    out: int            # output irrep index
    l1: int             # nu=1: the irrep itself
    l2: int = -1        # nu>=2: pair (l1 <= l2)
    L2: int = -1        # nu=3: intermediate
    l3: int = -1        # nu=3: third factor


def sl(l: int) -> slice:
    return slice(l * l, (l + 1) * (l + 1))


class Bilinear:
    """Collects terms coef * x * y -> target and emits them with shared products."""

    def __init__(self, P: Program):
        self.P = P
        self.terms: Dict[Tuple, float] = {}
        self.order: List[Tuple] = []

    def add(self, target, coef: float, x: int, y: int):
        if x > y:
            x, y = y, x
        key = (target, x, y)
        if key not in self.terms:
            self.terms[key] = 0.0
            self.order.append(key)
        self.terms[key] += coef

    def emit(self, acc: Dict, mode: str = "chain") -> None:
        """acc[target] (Optional[int]) is updated in place.

        mode "products": every x*y is an explicit (shared) product, one constant FMA per term.
        mode "chain":    per target, terms of equal |coef| are first summed with signed FMAs
                         (the sign is a free operand modifier), then scaled once.
        """
        P = self.P
        if mode == "products":
            for key in self.order:
                c = self.terms[key]
                if abs(c) < 1e-13:
                    continue
                target, x, y = key
                acc[target] = P.cfma(P.mul(x, y), c, acc.get(target))
            return
        by_target: Dict = {}
        for key in self.order:
            c = self.terms[key]
            if abs(c) < 1e-13:
                continue
            target, x, y = key
            mags = by_target.setdefault(target, {})
            mags.setdefault(round(abs(c), 11), []).append((c, x, y))
        for target, mags in by_target.items():
            # a group of unit magnitude goes first: as the first term of a target it needs no scaling
            for mag, lst in sorted(mags.items(), key=lambda kv: (abs(kv[0] - 1.0) > 1e-9,)):
                c0 = lst[0][0]
                q = P.mul(lst[0][1], lst[0][2])
                for c, x, y in lst[1:]:
                    q = P.fma(x, y, q) if (c > 0) == (c0 > 0) else P.fnma(x, y, q)
                acc[target] = P.cfma(q, c0, acc.get(target))


MODE = "chain"


def couple_into(P: Program, C: np.ndarray, u: Sequence[int], v: Sequence[int], acc: List[Optional[int]]):
    """acc[c] += sum_ab C[a,b,c] u[a] v[b]."""
    bl = Bilinear(P)
    for a, b, c in zip(*np.nonzero(C)):
        bl.add(int(c), float(C[a, b, c]), u[a], v[b])
    d = {i: acc[i] for i in range(len(acc)) if acc[i] is not None}
    bl.emit(d, MODE)
    for i in range(len(acc)):
        acc[i] = d.get(i)


class Scheme:
    def __init__(self, cg: CG, l_max: int, outs: Sequence[Tuple[int, int]], basis: Sequence[InternalPath]):
        self.cg, self.l_max, self.outs, self.basis = cg, l_max, list(outs), list(basis)
        self.n_lm = (l_max + 1) ** 2
        self.out_off = np.cumsum([0] + [2 * L + 1 for L, _ in outs])
        self.n_LM = int(self.out_off[-1])

    # -- shared pieces -----------------------------------------------------------------
    def _pairs(self, P: Program, a: List[int], needed) -> Dict[Tuple[int, int, int], List[int]]:
        T = {}
        for (l1, l2, L2) in needed:
            acc: List[Optional[int]] = [None] * (2 * L2 + 1)
            couple_into(P, self.cg(l1, l2, L2), a[sl(l1)], a[sl(l2)], acc)
            T[(l1, l2, L2)] = acc
        return T

    def _needed_pairs(self):
        need = []
        for s in self.basis:
            if s.nu == 2:
                key = (s.l1, s.l2, self.outs[s.out][0])
            elif s.nu == 3:
                key = (s.l1, s.l2, s.L2)
            else:
                continue
            if key not in need:
                need.append(key)
        return need

    def _groups(self):
        """nu=3 internal paths grouped by (L2, l3, out)."""
        g: Dict[Tuple[int, int, int], List[int]] = {}
        for i, s in enumerate(self.basis):
            if s.nu == 3:
                g.setdefault((s.L2, s.l3, s.out), []).append(i)
        return g

    # -- forward -----------------------------------------------------------------------
    def forward(self) -> Program:
        P = Program()
        a = [P.inp(f"a[{i}]") for i in range(self.n_lm)]
        w = [P.inp(f"w[{i}]") for i in range(len(self.basis))]
        T = self._pairs(P, a, self._needed_pairs())
        B: List[List[Optional[int]]] = [[None] * (2 * L + 1) for L, _ in self.outs]
        for i, s in enumerate(self.basis):
            L = self.outs[s.out][0]
            if s.nu == 1:
                for M in range(2 * L + 1):
                    B[s.out][M] = P.fma(w[i], a[L * L + M], B[s.out][M])
            elif s.nu == 2:
                t = T[(s.l1, s.l2, L)]
                for M in range(2 * L + 1):
                    if t[M] is not None:
                        B[s.out][M] = P.fma(w[i], t[M], B[s.out][M])
        for (L2, l3, out), members in self._groups().items():
            L = self.outs[out][0]
            S: List[Optional[int]] = [None] * (2 * L2 + 1)
            for i in members:
                s = self.basis[i]
                t = T[(s.l1, s.l2, L2)]
                for M2 in range(2 * L2 + 1):
                    if t[M2] is not None:
                        S[M2] = P.fma(w[i], t[M2], S[M2])
            Cc = self.cg(L2, l3, L)
            live = [m for m in range(2 * L2 + 1) if S[m] is not None]
            couple_into(P, Cc[live], [S[m] for m in live], a[sl(l3)], B[out])
        for o in range(len(self.outs)):
            for M in range(len(B[o])):
                P.out(f"b[{self.out_off[o] + M}]", B[o][M])
        return P

    # -- backward ----------------------------------------------------------------------
    def backward(self) -> Program:
        P = Program()
        a = [P.inp(f"a[{i}]") for i in range(self.n_lm)]
        w = [P.inp(f"w[{i}]") for i in range(len(self.basis))]
        g = [P.inp(f"g[{i}]") for i in range(self.n_LM)]
        dw: List[Optional[int]] = [P.inp(f"dw[{i}]") for i in range(len(self.basis))]
        T = self._pairs(P, a, self._needed_pairs())
        dT: Dict[Tuple[int, int, int], List[Optional[int]]] = {k: [None] * len(v) for k, v in T.items()}
        da: Dict[int, Optional[int]] = {}
        for i, s in enumerate(self.basis):
            L = self.outs[s.out][0]
            go = g[self.out_off[s.out]:self.out_off[s.out + 1]]
            if s.nu == 1:
                for M in range(2 * L + 1):
                    dw[i] = P.fma(go[M], a[L * L + M], dw[i])
                    da[L * L + M] = P.fma(w[i], go[M], da.get(L * L + M))
            elif s.nu == 2:
                key = (s.l1, s.l2, L)
                for M in range(2 * L + 1):
                    if T[key][M] is not None:
                        dw[i] = P.fma(go[M], T[key][M], dw[i])
                        dT[key][M] = P.fma(w[i], go[M], dT[key][M])
        for (L2, l3, out), members in self._groups().items():
            L = self.outs[out][0]
            go = g[self.out_off[out]:self.out_off[out + 1]]
            Cc = self.cg(L2, l3, L)                      # [M2, m3, M]
            S: List[Optional[int]] = [None] * (2 * L2 + 1)
            for i in members:
                s = self.basis[i]
                t = T[(s.l1, s.l2, L2)]
                for M2 in range(2 * L2 + 1):
                    if t[M2] is not None:
                        S[M2] = P.fma(w[i], t[M2], S[M2])
            live = [m for m in range(2 * L2 + 1) if S[m] is not None]
            # V[M2] = sum C[M2,m3,M] a_l3[m3] g[M]
            V: List[Optional[int]] = [None] * (2 * L2 + 1)
            couple_into(P, np.transpose(Cc, (1, 2, 0)), a[sl(l3)], go, V)
            for i in members:
                s = self.basis[i]
                key = (s.l1, s.l2, L2)
                for M2 in range(2 * L2 + 1):
                    if T[key][M2] is not None and V[M2] is not None:
                        dw[i] = P.fma(T[key][M2], V[M2], dw[i])
                        dT[key][M2] = P.fma(w[i], V[M2], dT[key][M2])
            # da_l3[m3] += sum C[M2,m3,M] S[M2] g[M]
            acc: List[Optional[int]] = [da.get(l3 * l3 + m) for m in range(2 * l3 + 1)]
            Ct = np.transpose(Cc, (0, 2, 1))[live]        # [M2(live), M, m3]
            couple_into(P, Ct, [S[m] for m in live], go, acc)
            for m in range(2 * l3 + 1):
                if acc[m] is not None:
                    da[l3 * l3 + m] = acc[m]
        # reverse of the pair couplings
        bl = Bilinear(P)
        for (l1, l2, L2), d in dT.items():
            C = self.cg(l1, l2, L2)
            for m1, m2, M2 in zip(*np.nonzero(C)):
                if d[M2] is None:
                    continue
                c = float(C[m1, m2, M2])
                bl.add(l1 * l1 + int(m1), c, a[l2 * l2 + int(m2)], d[M2])
                bl.add(l2 * l2 + int(m2), c, a[l1 * l1 + int(m1)], d[M2])
        bl.emit(da, MODE)
        for i in range(self.n_lm):
            P.out(f"da[{i}]", da.get(i))
        for i in range(len(self.basis)):
            P.out(f"dw[{i}]", dw[i])
        return P
