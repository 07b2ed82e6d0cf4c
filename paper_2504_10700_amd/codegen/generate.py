"""Generator of the straight-line device code of the specialised kernels.

    python -m paper_2504_10700_amd.codegen.generate            # rewrite csrc/generated/*.inc
    python -m paper_2504_10700_amd.codegen.generate --check    # fail if a file would change

For every configuration in SPECS it
  1. asks the library's table builder for the external coupling paths and their
     polynomials (tables.py),
  2. chooses a minimal internal basis of coupled paths (one subset of candidates per
     multiset of l's, found by coordinate descent on the forward + backward operation count),
  3. solves for the fold matrix F (external polynomial p = sum_s F[s,p] * internal polynomial s)
     on random samples and checks the residual,
  4. builds the forward and backward straight-line programs (scheme.py), checks them against
     the external polynomials (values and, by finite differences, gradients) in fp64,
  5. derives the second-order program from the forward one (autodiff.py: tangent along H, then
     the reverse-mode derivative of sum(g * tangent)) and checks it the same way,
  6. writes csrc/generated/sc_gen_<tag>.inc.
Deterministic: the same library gives the same files.
"""
from __future__ import annotations

import argparse
import itertools
import os
import sys
from typing import Dict, List, Sequence, Tuple

import numpy as np

from .autodiff import replay_with_tangent, reverse
from .program import Program
from .scheme import InternalPath, Scheme
from .tables import HOST_LIB, Tables

_HERE = os.path.dirname(os.path.abspath(__file__))
OUT_DIR = os.path.join(os.path.dirname(_HERE), "csrc", "generated")

# tag -> (l_max, nu_max, output irreps)
SPECS = {
    "l3n3_0e1o": (3, 3, ((0, 1), (1, -1))),
    "l3n3_0e1o2e": (3, 3, ((0, 1), (1, -1), (2, 1))),
    "l3n3_0e1o2e3o": (3, 3, ((0, 1), (1, -1), (2, 1), (3, -1))),
    "l1n2_0e": (1, 2, ((0, 1),)),
    "l3n3_0e": (3, 3, ((0, 1),)),      # scalar outputs only: the product of a model's last layer
}


def candidates(tab: Tables, out: int, ms: Tuple[int, ...]) -> List[InternalPath]:
    """Coupled paths (pair first, then the third factor) for a sorted multiset of three l's."""
    L, _ = tab.outs[out]
    res, seen = [], set()
    for i in range(3):
        l3 = ms[i]
        rest = [ms[j] for j in range(3) if j != i]
        l1, l2 = min(rest), max(rest)
        for L2 in range(abs(l1 - l2), l1 + l2 + 1):
            if l1 == l2 and L2 % 2 == 1:
                continue  # antisymmetric coupling of two equal factors vanishes
            if abs(L2 - l3) <= L <= L2 + l3 and (l1, l2, L2, l3) not in seen:
                seen.add((l1, l2, L2, l3))
                res.append(InternalPath(3, out, l1, l2, L2, l3))
    return res


class ScaledCG:
    """The library's coupling tensors, each divided by its most frequent |coefficient|.

    The internal basis polynomials may carry any scale (the fold matrix absorbs it), so every
    coupling tensor is rescaled to make as many of its entries as possible exactly +-1: sums
    of such terms need no multiplication by a constant.
    """

    def __init__(self, tab: Tables):
        self.tab = tab
        self._cache = {}

    def __call__(self, l1: int, l2: int, l3: int) -> np.ndarray:
        key = (l1, l2, l3)
        if key not in self._cache:
            C = np.array(self.tab.cg(l1, l2, l3))
            nz = np.abs(C[C != 0.0])
            if nz.size:
                vals, counts = np.unique(np.round(nz, 12), return_counts=True)
                mode = vals[np.argmax(counts)]               # ties: the smallest magnitude
                kappa = float(nz[np.abs(nz - mode) < 1e-11][0])  # an actual entry, not the rounded value
                C = C / kappa
                unit = np.abs(np.abs(C) - 1.0) < 1e-13
                C[unit] = np.sign(C[unit])
            C.setflags(write=False)
            self._cache[key] = C
        return self._cache[key]


def eval_internal(tab, s: InternalPath, a: np.ndarray) -> np.ndarray:
    """tab: anything with .cg(l1,l2,l3) and .outs"""
    L = tab.outs[s.out][0]

    def al(l):
        return a[:, l * l:(l + 1) ** 2]
    if s.nu == 1:
        return al(s.l1)
    if s.nu == 2:
        return np.einsum("abc,na,nb->nc", tab.cg(s.l1, s.l2, L), al(s.l1), al(s.l2))
    T = np.einsum("abc,na,nb->nc", tab.cg(s.l1, s.l2, s.L2), al(s.l1), al(s.l2))
    return np.einsum("abc,na,nb->nc", tab.cg(s.L2, s.l3, L), T, al(s.l3))


class _Shim:
    """What eval_internal and Scheme need: the (scaled) couplings and the output irreps."""

    def __init__(self, cg, outs):
        self.cg, self.outs = cg, outs


def choose_basis(tab: Tables, samples: np.ndarray, cg=None):
    """Returns (basis, fold) with fold[s] = list of (external path, coefficient)."""
    cg = cg or tab.cg
    shim = _Shim(cg, tab.outs)
    groups: Dict[Tuple, List[int]] = {}
    for p, (nu, out, l1, l2, l3, L2) in enumerate(tab.paths):
        ms = tuple(sorted(l for l in (l1, l2, l3) if l >= 0))
        groups.setdefault((nu, out, ms), []).append(p)
    ext = {p: tab.eval_external(p, samples) for p in range(tab.num_paths)}
    options: Dict[Tuple, List[Tuple[InternalPath, ...]]] = {}
    for key, plist in groups.items():
        nu, out, ms = key
        E = np.stack([ext[p].ravel() for p in plist], 1)
        r = np.linalg.matrix_rank(E, tol=1e-9)
        if r == 0:
            options[key] = [()]
        elif nu == 1:
            options[key] = [(InternalPath(1, out, ms[0]),)]
        elif nu == 2:
            options[key] = [(InternalPath(2, out, ms[0], ms[1]),)]
        else:
            cands = candidates(tab, out, ms)
            Q = {c: eval_internal(shim, c, samples).ravel() for c in cands}
            subs = [sub for sub in itertools.combinations(cands, r)
                    if np.linalg.matrix_rank(np.stack([Q[c] for c in sub], 1), tol=1e-9) == r]
            assert subs, key
            options[key] = subs
    keys = list(options)
    cur = {k: options[k][0] for k in keys}

    def cost(sel):
        sch = Scheme(cg, tab.l_max, tab.outs, [c for k in keys for c in sel[k]])
        return sch.forward().count()["total"] + sch.backward().count()["total"]
    best = cost(cur)
    improved = True
    while improved:
        improved = False
        for k in keys:
            for sub in options[k]:
                if sub == cur[k]:
                    continue
                trial = dict(cur)
                trial[k] = sub
                c = cost(trial)
                if c < best:
                    best, cur, improved = c, trial, True
    basis: List[InternalPath] = []
    fold: List[List[Tuple[int, float]]] = []
    for k in keys:
        if not cur[k]:
            continue
        plist = groups[k]
        E = np.stack([ext[p].ravel() for p in plist], 1)
        Q = np.stack([eval_internal(shim, c, samples).ravel() for c in cur[k]], 1)
        F, *_ = np.linalg.lstsq(Q, E, rcond=None)
        assert np.abs(Q @ F - E).max() < 1e-11, (k, np.abs(Q @ F - E).max())
        for j, c in enumerate(cur[k]):
            basis.append(c)
            fold.append([(plist[i], float(F[j, i])) for i in range(len(plist)) if abs(F[j, i]) > 1e-12])
    return basis, fold


def build_double_backward(fwd: Program, n_lm: int, n_LM: int, S: int) -> Program:
    """Second-order program: with psi = sum_j g[j] * (d b[j] / d a . h),
    ddb = d psi / d g (the tangent of the forward program along h), da = d psi / d a,
    dw += d psi / d w."""
    P = Program()
    a = [P.inp(f"a[{i}]") for i in range(n_lm)]
    h = [P.inp(f"h[{i}]") for i in range(n_lm)]
    w = [P.inp(f"w[{s}]") for s in range(S)]
    g = [P.inp(f"g[{j}]") for j in range(n_LM)]
    dw = [P.inp(f"dw[{s}]") for s in range(S)]
    inputs = {f"a[{i}]": (a[i], h[i]) for i in range(n_lm)}
    inputs.update({f"w[{s}]": (w[s], None) for s in range(S)})
    outs = replay_with_tangent(fwd, P, inputs)
    seeds: Dict[int, int] = {}
    for j in range(n_LM):
        t = outs[f"b[{j}]"][1]
        if t is not None:
            seeds[t] = P.add(seeds.get(t), g[j])
    adj = reverse(P, seeds)
    for j in range(n_LM):
        P.out(f"ddb[{j}]", outs[f"b[{j}]"][1])
    for i in range(n_lm):
        P.out(f"da[{i}]", adj.get(a[i]))
    for s in range(S):
        P.out(f"dw[{s}]", P.add(dw[s], adj.get(w[s])))
    return P


def self_check_double(tab: Tables, basis, fold, dbl: Program, dtype=np.float64):
    """Second-order program against the second derivatives of the external polynomials."""
    rng = np.random.default_rng(54321)
    n = 1000
    a = rng.standard_normal((n, tab.n_lm))
    h = rng.standard_normal((n, tab.n_lm))
    g = rng.standard_normal((n, tab.n_LM))
    counts = {}
    for (nu, out, *_r) in tab.paths:
        counts[(nu, out)] = counts.get((nu, out), 0) + 1
    Wext = np.stack([rng.standard_normal(n) / np.sqrt(counts[(p[0], p[1])]) for p in tab.paths], 1)
    a, h, g, Wext = (x.astype(dtype).astype(np.float64) for x in (a, h, g, Wext))
    S = len(basis)
    w = np.zeros((n, S))
    for s, lst in enumerate(fold):
        for p, c in lst:
            w[:, s] += c * Wext[:, p]
    off = np.cumsum([0] + [2 * L + 1 for L, _ in tab.outs])
    ddB = np.zeros((n, tab.n_LM))
    dA2 = np.zeros((n, tab.n_lm))
    dW2 = np.zeros((n, tab.num_paths))
    for p, path in enumerate(tab.paths):
        nu, out = path[0], path[1]
        M, i1, i2, i3, coef = tab.path_terms(p)
        for t in range(len(M)):
            col = off[out] + M[t]
            idx = (i1[t], i2[t], i3[t])[:nu]
            # tangent of the monomial: one factor replaced by h
            tang = np.zeros(n)
            for k in range(nu):
                f = [h[:, idx[j]] if j == k else a[:, idx[j]] for j in range(nu)]
                tang += np.prod(f, axis=0)
            ddB[:, col] += Wext[:, p] * coef[t] * tang
            dW2[:, p] += g[:, col] * coef[t] * tang
            # derivative of the tangent with respect to the factor in slot m
            for m in range(nu):
                d = np.zeros(n)
                for k in range(nu):
                    if k == m:
                        continue
                    f = [h[:, idx[j]] if j == k else a[:, idx[j]] for j in range(nu) if j != m]
                    d += np.prod(f, axis=0)
                dA2[:, idx[m]] += g[:, col] * Wext[:, p] * coef[t] * d
    inputs = {f"a[{i}]": a[:, i] for i in range(tab.n_lm)}
    inputs.update({f"h[{i}]": h[:, i] for i in range(tab.n_lm)})
    inputs.update({f"w[{s}]": w[:, s] for s in range(S)})
    inputs.update({f"g[{j}]": g[:, j] for j in range(tab.n_LM)})
    inputs.update({f"dw[{s}]": np.zeros(n) for s in range(S)})
    r = dbl.evaluate(inputs, dtype)

    def col(v):
        return np.zeros(n) if v is None else v.astype(np.float64)
    ddBg = np.stack([col(r[f"ddb[{j}]"]) for j in range(tab.n_LM)], 1)
    dAg = np.stack([col(r[f"da[{i}]"]) for i in range(tab.n_lm)], 1)
    dwg = np.stack([col(r[f"dw[{s}]"]) for s in range(S)], 1)
    dWg = np.zeros((n, tab.num_paths))
    for s, lst in enumerate(fold):
        for p, c in lst:
            dWg[:, p] += c * dwg[:, s]

    def err(x, y):
        return float(np.abs(x - y).max() / np.sqrt((y ** 2).mean()))
    return {"ddB": err(ddBg, ddB), "dA2": err(dAg, dA2), "dW2(per node)": err(dWg, dW2)}


def self_check(tab: Tables, basis, fold, fwd: Program, bwd: Program, dtype=np.float64):
    """Generated programs against the library's external polynomials.  Returns error norms."""
    rng = np.random.default_rng(12345)
    n = 2000
    a = rng.standard_normal((n, tab.n_lm))
    g = rng.standard_normal((n, tab.n_LM))
    counts = {}
    for (nu, out, *_r) in tab.paths:
        counts[(nu, out)] = counts.get((nu, out), 0) + 1
    Wext = np.stack([rng.standard_normal(n) / np.sqrt(counts[(p[0], p[1])]) for p in tab.paths], 1)  # [n, P]
    a, g, Wext = (x.astype(dtype).astype(np.float64) for x in (a, g, Wext))
    w = np.zeros((n, len(basis)))
    for s, lst in enumerate(fold):
        for p, c in lst:
            w[:, s] += c * Wext[:, p]
    off = np.cumsum([0] + [2 * L + 1 for L, _ in tab.outs])
    # reference from the external polynomials (fp64), gradients by differentiating the terms
    B = np.zeros((n, tab.n_LM))
    dA = np.zeros((n, tab.n_lm))
    dWext = np.zeros((n, tab.num_paths))
    for p, path in enumerate(tab.paths):
        nu, out = path[0], path[1]
        M, i1, i2, i3, coef = tab.path_terms(p)
        for t in range(len(M)):
            col = off[out] + M[t]
            f = [a[:, i] for i in (i1[t], i2[t], i3[t])[:nu]]
            mono = coef[t] * np.prod(f, axis=0)
            B[:, col] += Wext[:, p] * mono
            dWext[:, p] += g[:, col] * mono
            for k, i in enumerate((i1[t], i2[t], i3[t])[:nu]):
                rest = [f[j] for j in range(nu) if j != k]
                dA[:, i] += g[:, col] * Wext[:, p] * coef[t] * (np.prod(rest, axis=0) if rest else 1.0)
    inputs = {f"a[{i}]": a[:, i] for i in range(tab.n_lm)}
    inputs.update({f"w[{s}]": w[:, s] for s in range(len(basis))})
    rf = fwd.evaluate(inputs, dtype)
    Bg = np.stack([rf[f"b[{j}]"] for j in range(tab.n_LM)], 1).astype(np.float64)
    inputs.update({f"g[{j}]": g[:, j] for j in range(tab.n_LM)})
    inputs.update({f"dw[{s}]": np.zeros(n) for s in range(len(basis))})
    rb = bwd.evaluate(inputs, dtype)
    dAg = np.stack([rb[f"da[{i}]"] for i in range(tab.n_lm)], 1).astype(np.float64)
    dwg = np.stack([rb[f"dw[{s}]"] for s in range(len(basis))], 1).astype(np.float64)
    dWg = np.zeros((n, tab.num_paths))
    for s, lst in enumerate(fold):
        for p, c in lst:
            dWg[:, p] += c * dwg[:, s]

    def err(x, y):
        return float(np.abs(x - y).max() / np.sqrt((y ** 2).mean()))
    return {"B": err(Bg, B), "dA": err(dAg, dA), "dW(per node)": err(dWg, dWext)}


def emit_inc(tag: str, tab: Tables, basis, fold, fwd: Program, bwd: Program, dbl: Program) -> str:
    S, P = len(basis), tab.num_paths
    L = []
    L.append(f"// GENERATED by paper_2504_10700_amd/codegen/generate.py for l_max={tab.l_max}, nu_max={tab.nu_max}, outputs "
             + "+".join(f"{l}{'e' if p > 0 else 'o'}" for l, p in tab.outs) + ".  Do not edit.")
    L.append("//")
    L.append("// Straight-line evaluation of Algorithm 2 of arXiv 2504.10700 (and of its reverse-mode")
    L.append("// derivative) per (node, channel) in the coupled Horner form described in codegen/scheme.py.")
    fc, bc, dc = fwd.count(), bwd.count(), dbl.count()
    L.append(f"// Operation counts per (node, channel): forward {fc['total']}, backward {bc['total']}, "
             f"second-order pass {dc['total']}.")
    L.append("// Internal path basis (index: nu, output irrep, l1, l2, L2, l3):")
    for i, s in enumerate(basis):
        L.append(f"//   {i:2d}: nu={s.nu} out={s.out} l1={s.l1} l2={s.l2} L2={s.L2} l3={s.l3}")
    L.append(f"struct Gen_{tag} {{")
    L.append(f"  static constexpr int kLmax = {tab.l_max}, kNuMax = {tab.nu_max}, kNumOut = {len(tab.outs)};")
    L.append(f"  static constexpr int kNlm = {tab.n_lm}, kNLM = {tab.n_LM}, kP = {P}, kS = {S};")
    L.append("  static constexpr int kOutL[kNumOut] = {" + ", ".join(str(l) for l, _ in tab.outs) + "};")
    L.append("  static constexpr int kOutParity[kNumOut] = {" + ", ".join(str(p) for _, p in tab.outs) + "};")

    def flops(c):
        return 2 * (c.get("fma", 0) + c.get("fnma", 0) + c.get("cfma", 0)) + sum(c.get(k, 0) for k in ("mul", "add", "sub", "cmul"))
    L.append("  // VALU instructions and floating-point operations (a fused multiply-add counts twice) per")
    L.append("  // (node, channel) of forward, backward and the second-order pass.")
    L.append(f"  static constexpr int kOps[3] = {{{fc['total']}, {bc['total']}, {dc['total']}}};")
    L.append(f"  static constexpr int kFlops[3] = {{{flops(fc)}, {flops(bc)}, {flops(dc)}}};")
    L.append("")
    L.append("  // w'[s] = sum_p F[s,p] * W[z,p,k]; Wz points at W[z,0,k], consecutive paths are K apart.")
    L.append("  template <typename T>")
    L.append("  static __device__ __forceinline__ void fold(const T* __restrict__ Wz, int K, T (&w)[kS]) {")
    for s, lst in enumerate(fold):
        terms = " + ".join(f"T({repr(c)}) * Wz[{p} * K]" for p, c in lst)
        L.append(f"    w[{s}] = {terms};")
    L.append("  }")
    L.append("")
    L.append("  template <typename T>")
    L.append("  static __device__ __forceinline__ void forward(const T (&a)[kNlm], const T (&w)[kS], T (&b)[kNLM]) {")
    L.append(fwd.emit("T", "    "))
    L.append("  }")
    L.append("")
    L.append("  // dW[z,p,k] = sum_s F[s,p] * r[s] (the transpose of fold).")
    by_p: Dict[int, List[Tuple[int, float]]] = {p: [] for p in range(P)}
    for s, lst in enumerate(fold):
        for p, c in lst:
            by_p[p].append((s, c))
    # Rows and external paths fall into small independent blocks (connected components of the fold
    # matrix): the paths of a block need the rows of that block only.
    parent = list(range(S))

    def find(x):
        while parent[x] != x:
            parent[x] = parent[parent[x]]
            x = parent[x]
        return x
    for p in range(P):
        rs = [s_ for s_, _ in by_p[p]]
        for r in rs[1:]:
            a, b = find(rs[0]), find(r)
            if a != b:
                parent[max(a, b)] = min(a, b)
    roots = sorted({find(r) for r in range(S)})
    comp_of_row = {r: roots.index(find(r)) for r in range(S)}
    comp_rows = [[r for r in range(S) if comp_of_row[r] == c] for c in range(len(roots))]
    comp_outs = [[] for _ in roots]
    for p in range(P):
        comp_outs[comp_of_row[by_p[p][0][0]] if by_p[p] else 0].append(p)   # identically zero paths ride with block 0
    max_rows = max(len(c) for c in comp_rows)
    max_paths = max(len(c) for c in comp_outs)
    L.append("  // Independent blocks of the fold matrix, one descriptor each (read as one run of scalar loads):")
    L.append("  // the block's internal rows (the last one repeated up to kMaxBlockRows), its external paths and,")
    L.append("  // per path, the coefficients on the block's rows: dW[path[i]] = sum_r coef[i][r] * r[row[r]].")
    L.append(f"  static constexpr int kNumBlocks = {len(roots)}, kMaxBlockRows = {max_rows}, kMaxBlockPaths = {max_paths};")
    L.append("  struct Block {")
    L.append("    int n_rows, n_paths;")
    L.append("    int row[kMaxBlockRows];")
    L.append("    int path[kMaxBlockPaths];")
    L.append("    double coef[kMaxBlockPaths][kMaxBlockRows];")
    L.append("  };")
    L.append("  static constexpr Block kBlocks[kNumBlocks] = {")
    for c in range(len(roots)):
        rws = comp_rows[c] + [comp_rows[c][-1]] * (max_rows - len(comp_rows[c]))
        pths = comp_outs[c] + [comp_outs[c][-1] if comp_outs[c] else 0] * (max_paths - len(comp_outs[c]))
        coef_rows = []
        for i in range(max_paths):
            cs = [0.0] * max_rows
            if i < len(comp_outs[c]):
                for s_, cf in by_p[comp_outs[c][i]]:
                    cs[comp_rows[c].index(s_)] = cf
            coef_rows.append("{" + ", ".join(repr(x) for x in cs) + "}")
        L.append(f"      {{{len(comp_rows[c])}, {len(comp_outs[c])}, {{{', '.join(map(str, rws))}}}, {{{', '.join(map(str, pths))}}},")
        L.append("       {" + ", ".join(coef_rows) + "}},")
    L.append("  };")
    L.append("")
    L.append("  // da is overwritten; dw is accumulated into.")
    L.append("  template <typename T>")
    L.append("  static __device__ __forceinline__ void backward(const T (&a)[kNlm], const T (&w)[kS], const T (&g)[kNLM],")
    L.append("                                                  T (&da)[kNlm], T (&dw)[kS]) {")
    L.append(bwd.emit("T", "    "))
    L.append("  }")
    L.append("")
    L.append("  // Second-order pass: with psi = sum_j g[j] * (d b[j] / d a . h): ddb = d psi / d g,")
    L.append("  // da = d psi / d a (both overwritten); d psi / d w is accumulated into dw.")
    L.append("  template <typename T>")
    L.append("  static __device__ __forceinline__ void double_backward(const T (&a)[kNlm], const T (&w)[kS], const T (&g)[kNLM],")
    L.append("                                                         const T (&h)[kNlm], T (&ddb)[kNLM], T (&da)[kNlm],")
    L.append("                                                         T (&dw)[kS]) {")
    L.append(dbl.emit("T", "    "))
    L.append("  }")
    L.append("};")
    return "\n".join(L) + "\n"


def generate(tag: str, lib_path: str = HOST_LIB, verbose: bool = True) -> str:
    l_max, nu_max, outs = SPECS[tag]
    tab = Tables(lib_path, l_max, nu_max, outs)
    samples = np.random.default_rng(0).standard_normal((40, tab.n_lm))
    cg = ScaledCG(tab)
    basis, fold = choose_basis(tab, samples, cg)
    sch = Scheme(cg, l_max, outs, basis)
    fwd, bwd = sch.forward(), sch.backward()
    dbl = build_double_backward(fwd, tab.n_lm, tab.n_LM, len(basis))
    # Single products scaled by a literal share their scaled factor (about 5% fewer operations): used for the
    # larger bases, whose kernels are bound by the vector ALUs (49-row basis: step -2% at 50k nodes / 256
    # channels).  Not for the small bases: the scaled factors stay live across the program and push the backward
    # instance held to three waves per SIMD from 12 to 36 bytes of scratch (48.5 -> 50.0 us at 10k nodes), and
    # nothing is gained where memory is the bound.
    if len(basis) > 32:
        fwd, bwd, dbl = fwd.prescale_single_products(), bwd.prescale_single_products(), dbl.prescale_single_products()
    e64 = self_check(tab, basis, fold, fwd, bwd, np.float64)
    assert max(e64.values()) < 1e-12, e64
    d64 = self_check_double(tab, basis, fold, dbl, np.float64)
    assert max(d64.values()) < 1e-12, d64
    if verbose:
        e32 = self_check(tab, basis, fold, fwd, bwd, np.float32)
        d32 = self_check_double(tab, basis, fold, dbl, np.float32)
        print(f"[{tag}] S={len(basis)} P={tab.num_paths} ops fwd={fwd.count()['total']} bwd={bwd.count()['total']} "
              f"second-order={dbl.count()['total']}")
        print(f"[{tag}] fp64 self-check max|err|/rms: {e64} {d64}")
        print(f"[{tag}] fp32 emulation  max|err|/rms: {e32} {d32}")
    return emit_inc(tag, tab, basis, fold, fwd, bwd, dbl)


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--check", action="store_true")
    ap.add_argument("--lib", default=HOST_LIB)
    args = ap.parse_args(argv)
    os.makedirs(OUT_DIR, exist_ok=True)
    rc = 0
    for tag in SPECS:
        text = generate(tag, args.lib)
        path = os.path.join(OUT_DIR, f"sc_gen_{tag}.inc")
        old = open(path).read() if os.path.exists(path) else None
        if args.check:
            if old != text:
                print(f"{path} is out of date", file=sys.stderr)
                rc = 1
        elif old != text:
            with open(path, "w") as f:
                f.write(text)
            print("wrote", path)
    return rc


if __name__ == "__main__":
    sys.exit(main())
