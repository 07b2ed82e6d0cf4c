"""Forward-mode and reverse-mode differentiation of straight-line Programs.

Used for the second-order pass of the contraction: the directional derivative of the
forward program along a tangent H gives ddB; the reverse-mode derivative of
psi = sum(g * ddB) with respect to A and w' gives dA2 and the dW2 contributions.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

from .program import ADD, CFMA, CMUL, FMA, FNMA, INP, MUL, SUB, Program


def _neg(P: Program, x: Optional[int]) -> Optional[int]:
    return None if x is None else P.cmul(x, -1.0)


def _sub(P: Program, x: Optional[int], y: Optional[int]) -> Optional[int]:
    if y is None:
        return x
    if x is None:
        return _neg(P, y)
    return P.sub(x, y)


def replay_with_tangent(src: Program, dst: Program, inputs: Dict[str, Tuple[int, Optional[int]]]):
    """Re-emits `src` into `dst`, carrying a tangent with every value.

    inputs maps the C++ expression of every input of src to (value id, tangent id or None)
    in dst.  Returns {output lvalue of src: (value id, tangent id or None)}.
    """
    val: List[Optional[int]] = [None] * len(src.ops)
    tan: List[Optional[int]] = [None] * len(src.ops)
    live = src.live_ops()
    for i, op in enumerate(src.ops):
        if not live[i]:
            continue
        k = op[0]
        if k == INP:
            val[i], tan[i] = inputs[op[1]]
        elif k == MUL:
            x, y = op[1], op[2]
            val[i] = dst.mul(val[x], val[y])
            t = None
            if tan[x] is not None:
                t = dst.mul(tan[x], val[y])
            if tan[y] is not None:
                t = dst.fma(val[x], tan[y], t)
            tan[i] = t
        elif k == ADD:
            x, y = op[1], op[2]
            val[i] = dst.add(val[x], val[y])
            tan[i] = dst.add(tan[x], tan[y])
        elif k == SUB:
            x, y = op[1], op[2]
            val[i] = dst.sub(val[x], val[y])
            tan[i] = _sub(dst, tan[x], tan[y])
        elif k in (FMA, FNMA):
            x, y, z = op[1], op[2], op[3]
            if k == FMA:
                val[i] = dst.fma(val[x], val[y], val[z])
                t = tan[z]
                if tan[x] is not None:
                    t = dst.fma(tan[x], val[y], t)
                if tan[y] is not None:
                    t = dst.fma(val[x], tan[y], t)
            else:
                val[i] = dst.fnma(val[x], val[y], val[z])
                t = tan[z]
                for u, v in ((tan[x], val[y]), (val[x], tan[y])):
                    if u is None or v is None:
                        continue
                    t = dst.fnma(u, v, t) if t is not None else _neg(dst, dst.mul(u, v))
            tan[i] = t
        elif k == CMUL:
            val[i] = dst.cmul(val[op[1]], op[2])
            tan[i] = None if tan[op[1]] is None else dst.cmul(tan[op[1]], op[2])
        elif k == CFMA:
            x, c, z = op[1], op[2], op[3]
            val[i] = dst.cfma(val[x], c, val[z])
            tan[i] = tan[z] if tan[x] is None else dst.cfma(tan[x], c, tan[z])
        else:
            raise ValueError(k)
    return {lv: (val[x], tan[x]) if x is not None else (None, None) for lv, x in src.outputs}


def reverse(P: Program, seeds: Dict[int, int]) -> Dict[int, int]:
    """Appends the adjoint computation to P.  seeds: {value id: adjoint id}.  Returns the
    adjoints {value id: adjoint id} of everything the seeded values depend on."""
    adj: Dict[int, Optional[int]] = dict(seeds)
    n0 = len(P.ops)
    ops = list(P.ops[:n0])
    for i in range(n0 - 1, -1, -1):
        g = adj.get(i)
        if g is None:
            continue
        op = ops[i]
        k = op[0]
        if k == INP:
            continue
        if k == MUL:
            x, y = op[1], op[2]
            adj[x] = P.fma(g, y, adj.get(x))
            adj[y] = P.fma(g, x, adj.get(y))
        elif k == ADD:
            adj[op[1]] = P.add(adj.get(op[1]), g)
            adj[op[2]] = P.add(adj.get(op[2]), g)
        elif k == SUB:
            adj[op[1]] = P.add(adj.get(op[1]), g)
            adj[op[2]] = _sub(P, adj.get(op[2]), g)
        elif k == FMA:
            x, y, z = op[1], op[2], op[3]
            adj[x] = P.fma(g, y, adj.get(x))
            adj[y] = P.fma(g, x, adj.get(y))
            adj[z] = P.add(adj.get(z), g)
        elif k == FNMA:  # z - x*y
            x, y, z = op[1], op[2], op[3]
            for u, v in ((x, y), (y, x)):
                cur = adj.get(u)
                adj[u] = P.fnma(g, v, cur) if cur is not None else _neg(P, P.mul(g, v))
            adj[z] = P.add(adj.get(z), g)
        elif k == CMUL:
            adj[op[1]] = P.cfma(g, op[2], adj.get(op[1]))
        elif k == CFMA:
            adj[op[1]] = P.cfma(g, op[2], adj.get(op[1]))
            adj[op[3]] = P.add(adj.get(op[3]), g)
        else:
            raise ValueError(k)
    return {k: v for k, v in adj.items() if v is not None}
