"""Straight-line program builder used by the kernel generator.

A Program is a list of scalar per-lane operations (one lane = one channel of one
node) over named inputs.  It can be evaluated with numpy in any float type (to
validate the algebra and to estimate rounding error before touching a GPU),
counted (VALU operations per (node, channel)) and printed as C++ statements.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

# op codes
INP, MUL, ADD, SUB, FMA, FNMA, CMUL, CFMA = "inp", "mul", "add", "sub", "fma", "fnma", "cmul", "cfma"


class Program:
    def __init__(self):
        self.ops: List[Tuple] = []       # (op, args...) ; result id = index
        self.names: Dict[int, str] = {}  # ids of inputs -> C++ expression
        self.outputs: List[Tuple[str, int]] = []   # (C++ lvalue, id)
        self._memo: Dict[Tuple, int] = {}

    # ---- construction
    def inp(self, cexpr: str) -> int:
        self.ops.append((INP, cexpr))
        self.names[len(self.ops) - 1] = cexpr
        return len(self.ops) - 1

    def _push(self, key: Tuple) -> int:
        if key in self._memo:
            return self._memo[key]
        self.ops.append(key)
        self._memo[key] = len(self.ops) - 1
        return len(self.ops) - 1

    def mul(self, x: int, y: int) -> int:
        if x > y:
            x, y = y, x
        return self._push((MUL, x, y))

    def add(self, x: Optional[int], y: Optional[int]) -> Optional[int]:
        if x is None:
            return y
        if y is None:
            return x
        if x > y:
            x, y = y, x
        return self._push((ADD, x, y))

    def fma(self, x: int, y: int, z: Optional[int]) -> int:
        """x*y + z (z may be None = zero)."""
        if z is None:
            return self.mul(x, y)
        if x > y:
            x, y = y, x
        return self._push((FMA, x, y, z))

    def fnma(self, x: int, y: int, z: int) -> int:
        """z - x*y (the negation is an operand modifier of the hardware FMA)."""
        if x > y:
            x, y = y, x
        return self._push((FNMA, x, y, z))

    def sub(self, x: int, y: int) -> int:
        return self._push((SUB, x, y))

    def cmul(self, x: int, c: float) -> int:
        if c == 1.0:
            return x
        return self._push((CMUL, x, float(c)))

    def cfma(self, x: int, c: float, z: Optional[int]) -> int:
        """x*c + z with a compile-time constant c (z may be None = zero)."""
        if z is None:
            return self.cmul(x, c)
        if c == 1.0:
            return self.add(x, z)
        return self._push((CFMA, x, float(c), z))

    def out(self, lvalue: str, x: Optional[int]) -> None:
        self.outputs.append((lvalue, x))

    # ---- analysis
    def live_ops(self) -> List[bool]:
        live = [False] * len(self.ops)
        stack = [x for _, x in self.outputs if x is not None]
        while stack:
            i = stack.pop()
            if live[i]:
                continue
            live[i] = True
            for a in self.ops[i][1:]:
                if isinstance(a, int) and not isinstance(a, bool):
                    stack.append(a)
        return live

    def count(self) -> Dict[str, int]:
        live = self.live_ops()
        c: Dict[str, int] = {}
        for i, op in enumerate(self.ops):
            if live[i] and op[0] != INP:
                c[op[0]] = c.get(op[0], 0) + 1
        c["total"] = sum(c.values())
        return c

    # ---- rewriting
    def prescale_single_products(self) -> "Program":
        """Returns an equivalent program with fewer operations: a product x*y that is used once, by
        `x*y*c + z` with a literal c, costs two operations for one term.  Where several such terms
        share a factor and |c|, that factor is scaled once (s = y*|c|) and every term becomes one
        fused multiply-add x*s + z (z - x*s for negative c).  Factor-constant pairs are chosen
        greedily, most shared first; pairs used once are left as they are."""
        live = self.live_ops()
        uses = [0] * len(self.ops)
        for i, op in enumerate(self.ops):
            if live[i]:
                for a in op[1:]:
                    if isinstance(a, int) and not isinstance(a, bool) and op[0] != INP:
                        uses[a] += 1
        for _, x in self.outputs:
            if x is not None:
                uses[x] += 1
        cand = {}   # cfma id -> (x, y, c, z, product id)
        for k, op in enumerate(self.ops):
            if live[k] and op[0] == CFMA:
                prod = self.ops[op[1]]
                if prod[0] == MUL and uses[op[1]] == 1:
                    cand[k] = (prod[1], prod[2], op[2], op[3], op[1])
        assign = {}   # cfma id -> (factor to scale, other factor)
        remaining = dict(cand)
        while remaining:
            votes: Dict[Tuple[int, float], int] = {}
            for x, y, c, _, _ in remaining.values():
                for f in {x, y}:
                    votes[(f, abs(c))] = votes.get((f, abs(c)), 0) + 1
            (f, c), n = max(votes.items(), key=lambda kv: (kv[1], -kv[0][0], -kv[0][1]))
            if n < 2:
                break
            for k in [k for k, (x, y, cc, _, _) in remaining.items() if abs(cc) == c and f in (x, y)]:
                x, y = remaining[k][0], remaining[k][1]
                assign[k] = (f, y if f == x else x)
                del remaining[k]
        q = Program()
        new: Dict[int, int] = {}
        scaled: Dict[Tuple[int, float], int] = {}
        skip = {cand[k][4] for k in assign}
        for i, op in enumerate(self.ops):
            if op[0] == INP:
                new[i] = q.inp(op[1])
                continue
            if not live[i] or i in skip:
                continue
            if i in assign:
                f, other = assign[i]
                _, _, c, z, _ = cand[i]
                if (f, abs(c)) not in scaled:
                    scaled[(f, abs(c))] = q.cmul(new[f], abs(c))
                s_ = scaled[(f, abs(c))]
                new[i] = q.fma(new[other], s_, new[z]) if c > 0 else q.fnma(new[other], s_, new[z])
                continue
            k = op[0]
            a = [new[v] if isinstance(v, int) and not isinstance(v, bool) else v for v in op[1:]]
            if k == MUL:
                new[i] = q.mul(a[0], a[1])
            elif k == ADD:
                new[i] = q.add(a[0], a[1])
            elif k == SUB:
                new[i] = q.sub(a[0], a[1])
            elif k == FMA:
                new[i] = q.fma(a[0], a[1], a[2])
            elif k == FNMA:
                new[i] = q.fnma(a[0], a[1], a[2])
            elif k == CMUL:
                new[i] = q.cmul(a[0], a[1])
            elif k == CFMA:
                new[i] = q.cfma(a[0], a[1], a[2])
            else:
                raise ValueError(k)
        for lv, x in self.outputs:
            q.out(lv, new[x] if x is not None else None)
        return q

    # ---- evaluation
    def evaluate(self, inputs: Dict[str, np.ndarray], dtype=np.float64) -> Dict[str, np.ndarray]:
        live = self.live_ops()
        val: List[Optional[np.ndarray]] = [None] * len(self.ops)
        for i, op in enumerate(self.ops):
            if not live[i]:
                continue
            k = op[0]
            if k == INP:
                val[i] = inputs[op[1]].astype(dtype)
            elif k == MUL:
                val[i] = val[op[1]] * val[op[2]]
            elif k == ADD:
                val[i] = val[op[1]] + val[op[2]]
            elif k == FMA:
                val[i] = _fma(val[op[1]], val[op[2]], val[op[3]], dtype)
            elif k == FNMA:
                val[i] = _fma(-val[op[1]], val[op[2]], val[op[3]], dtype)
            elif k == SUB:
                val[i] = val[op[1]] - val[op[2]]
            elif k == CMUL:
                val[i] = val[op[1]] * dtype(op[2])
            elif k == CFMA:
                val[i] = _fma(val[op[1]], dtype(op[2]), val[op[3]], dtype)
            else:
                raise ValueError(k)
        res = {}
        for lv, x in self.outputs:
            res[lv] = val[x] if x is not None else None
        return res

    # ---- C++ emission
    def emit(self, scalar: str = "T", indent: str = "  ") -> str:
        live = self.live_ops()
        lines = []
        name = dict(self.names)

        def n(i):
            return name[i]

        def lit(c):
            return f"{scalar}({repr(float(c))})"
        for i, op in enumerate(self.ops):
            if not live[i] or op[0] == INP:
                continue
            name[i] = f"t{i}"
            k = op[0]
            if k == MUL:
                e = f"{n(op[1])} * {n(op[2])}"
            elif k == ADD:
                e = f"{n(op[1])} + {n(op[2])}"
            elif k == FMA:
                e = f"sc_fma({n(op[1])}, {n(op[2])}, {n(op[3])})"
            elif k == FNMA:
                e = f"sc_fma(-{n(op[1])}, {n(op[2])}, {n(op[3])})"
            elif k == SUB:
                e = f"{n(op[1])} - {n(op[2])}"
            elif k == CMUL:
                e = f"{n(op[1])} * {lit(op[2])}"
            elif k == CFMA:
                e = f"sc_fma({n(op[1])}, {lit(op[2])}, {n(op[3])})"
            lines.append(f"{indent}const {scalar} t{i} = {e};")
        for lv, x in self.outputs:
            lines.append(f"{indent}{lv} = {n(x) if x is not None else scalar + '(0)'};")
        return "\n".join(lines)


def _fma(x, y, z, dtype):
    if dtype == np.float32:
        # emulate a fused multiply-add: exact product in double, one rounding
        return (x.astype(np.float64) * np.float64(y) + z.astype(np.float64)).astype(np.float32)
    return x * y + z
