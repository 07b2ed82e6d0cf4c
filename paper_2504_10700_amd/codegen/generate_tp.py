"""Generator of the straight-line device code of the channelwise tensor product kernels.

    python -m paper_2504_10700_amd.codegen.generate_tp            # rewrite csrc/generated/tp_gen_*.inc
    python -m paper_2504_10700_amd.codegen.generate_tp --check    # fail if a file would change

Per (edge, channel) Algorithm 1 of arXiv 2504.10700 is a sum over paths (l1,l2,l3) of
R[p] * C(l1,l2,l3) Y_l1 h_l2.  Two programs are emitted per configuration, each a set of
bilinear couplings through the same sparse tensors with a different free index:

  forward   acc[l3] += C . Y_l1 . (R[p] h_l2)
  backward  q[l1]    = C . h_l2 . g_l3 ;  dR[p] = Y_l1 . q ;  dY_l1 += R[p] q
            s[l2]    = C . Y_l1 . g_l3 ;  dh_l2 += R[p] s      (the edge's share of its sender's dh)

A third program, the second-order pass, is derived from the forward one (autodiff.py): the
message's derivative along the cotangents (hy, hh, hr) of (dY, dh, dR) is added to ddA, and
the reverse-mode derivative of sum(g * that derivative) gives d2Y, d2h and d2R.

The sparse terms come from the library's host tables (tp_plan_terms on a host-only plan);
every coupling tensor is divided by its most frequent |coefficient| (the factor is folded
into the one multiplication by R[p]) so that most terms need no constant.  The programs are
checked in fp64 against the terms before anything is written.  Deterministic.
"""
from __future__ import annotations

import argparse
import ctypes as C
import os
import sys
from typing import Dict, List, Optional, Tuple

import numpy as np

from .autodiff import replay_with_tangent, reverse
from .program import Program
from .scheme import couple_into
from .tables import HOST_LIB

_HERE = os.path.dirname(os.path.abspath(__file__))
OUT_DIR = os.path.join(os.path.dirname(_HERE), "csrc", "generated")

# tag -> (l_Y, l_h, L_max)
SPECS = {
    "y3h0o3": (3, 0, 3),
    "y3h1o3": (3, 1, 3),
}


class _Config(C.Structure):
    _fields_ = [("struct_size", C.c_int32), ("num_channels", C.c_int32), ("l_Y", C.c_int32), ("l_h", C.c_int32),
                ("L_max", C.c_int32), ("dtype", C.c_int32), ("device", C.c_int32), ("flags", C.c_uint32)]


class TPTables:
    """Paths and dense per-path coupling tensors from the library's host-side table builder."""

    def __init__(self, lib_path: str, l_Y: int, l_h: int, L_max: int):
        lib = C.CDLL(lib_path)
        lib.sc_last_error.restype = C.c_char_p
        cfg = _Config()
        cfg.struct_size = C.sizeof(_Config)
        cfg.num_channels, cfg.l_Y, cfg.l_h, cfg.L_max = 64, l_Y, l_h, L_max
        cfg.dtype, cfg.device, cfg.flags = 1, 0, 1 | 2      # f64, host only, generic
        plan = C.c_void_p()

        def check(st):
            if st != 0:
                raise RuntimeError(lib.sc_last_error().decode())
        check(lib.tp_plan_create(C.byref(cfg), C.byref(plan)))
        info = (C.c_int32 * 11)()
        check(lib.tp_plan_info(plan, info))
        self.n_Y, self.n_h, self.n_out, self.P = info[0], info[1], info[2], info[3]
        paths = np.zeros((self.P, 3), dtype=np.int32)
        ip = C.POINTER(C.c_int32)
        check(lib.tp_plan_paths(plan, paths.ctypes.data_as(ip)))
        self.paths = [tuple(int(x) for x in r) for r in paths]
        n = C.c_int32()
        check(lib.tp_plan_terms(plan, 0, C.byref(n), None, None, None, None, None))
        arr = [np.zeros(n.value, dtype=np.int32) for _ in range(4)]
        coef = np.zeros(n.value)
        check(lib.tp_plan_terms(plan, n.value, C.byref(n), *[x.ctypes.data_as(ip) for x in arr],
                                coef.ctypes.data_as(C.POINTER(C.c_double))))
        self.terms = (*arr, coef)
        # dense C[p][m1][m2][m3] of every path
        self.C: List[np.ndarray] = []
        for p, (l1, l2, l3) in enumerate(self.paths):
            D = np.zeros((2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1))
            sel = arr[0] == p
            D[arr[1][sel] - l1 * l1, arr[2][sel] - l2 * l2, arr[3][sel] - l3 * l3] = coef[sel]
            self.C.append(D)
        check(lib.tp_plan_destroy(plan))


def split_scale(Cp: np.ndarray) -> Tuple[np.ndarray, float]:
    """Cp = kappa * Cs with the most frequent |entry| of Cs exactly 1."""
    nz = np.abs(Cp[Cp != 0.0])
    vals, counts = np.unique(np.round(nz, 12), return_counts=True)
    mode = vals[np.argmax(counts)]
    kappa = float(nz[np.abs(nz - mode) < 1e-11][0])
    Cs = Cp / kappa
    unit = np.abs(np.abs(Cs) - 1.0) < 1e-13
    Cs[unit] = np.sign(Cs[unit])
    return Cs, kappa


def sl(l: int) -> slice:
    return slice(l * l, (l + 1) * (l + 1))


def build_programs(tab: TPTables) -> Tuple[Program, Program]:
    scaled = [split_scale(Cp) for Cp in tab.C]
    # forward: acc[c] += sum C[a,b,c] y[a] (kappa r[p] h[b])
    F = Program()
    y = [F.inp(f"y[{a}]") for a in range(tab.n_Y)]
    h = [F.inp(f"h[{b}]") for b in range(tab.n_h)]
    r = [F.inp(f"r[{p}]") for p in range(tab.P)]
    acc: List[Optional[int]] = [F.inp(f"acc[{c}]") for c in range(tab.n_out)]
    for p, (l1, l2, l3) in enumerate(tab.paths):
        Cs, kappa = scaled[p]
        rk = F.cmul(r[p], kappa)
        u = [F.mul(rk, hb) for hb in h[sl(l2)]]
        part = acc[sl(l3)]
        couple_into(F, Cs, y[sl(l1)], u, part)
        acc[sl(l3)] = part
    for c in range(tab.n_out):
        F.out(f"acc[{c}]", acc[c])

    # backward of one edge
    Bq = Program()
    y = [Bq.inp(f"y[{a}]") for a in range(tab.n_Y)]
    h = [Bq.inp(f"h[{b}]") for b in range(tab.n_h)]
    r = [Bq.inp(f"r[{p}]") for p in range(tab.P)]
    g = [Bq.inp(f"g[{c}]") for c in range(tab.n_out)]
    dy: List[Optional[int]] = [None] * tab.n_Y
    for p, (l1, l2, l3) in enumerate(tab.paths):
        Cs, kappa = scaled[p]
        q: List[Optional[int]] = [None] * (2 * l1 + 1)
        couple_into(Bq, np.transpose(Cs, (1, 2, 0)), h[sl(l2)], g[sl(l3)], q)   # q[a] = sum C[a,b,c] h[b] g[c]
        dot = None
        for a, qa in zip(y[sl(l1)], q):
            if qa is not None:
                dot = Bq.fma(a, qa, dot)
        Bq.out(f"dr[{p}]", None if dot is None else Bq.cmul(dot, kappa))
        rk = Bq.cmul(r[p], kappa)
        for i, qa in enumerate(q):
            if qa is not None:
                dy[l1 * l1 + i] = Bq.fma(rk, qa, dy[l1 * l1 + i])
    for a in range(tab.n_Y):
        Bq.out(f"dy[{a}]", dy[a])
    # the edge's share of its sender's gradient: dh[b] = sum_p r[p] sum C[a,b,c] y[a] g[c]
    dh: List[Optional[int]] = [None] * tab.n_h
    for p, (l1, l2, l3) in enumerate(tab.paths):
        Cs, kappa = scaled[p]
        s: List[Optional[int]] = [None] * (2 * l2 + 1)
        couple_into(Bq, np.transpose(Cs, (0, 2, 1)), y[sl(l1)], g[sl(l3)], s)   # s[b] = sum C[a,b,c] y[a] g[c]
        rk = Bq.cmul(r[p], kappa)
        for i, sb in enumerate(s):
            if sb is not None:
                dh[l2 * l2 + i] = Bq.fma(rk, sb, dh[l2 * l2 + i])
    for b in range(tab.n_h):
        Bq.out(f"dh[{b}]", dh[b])
    return F, Bq


def build_double_backward(tab: TPTables, F: Program) -> Program:
    """psi = sum_c g[c] * (derivative of the edge's message along (hy, hh, hr)):
    dda += that derivative; d2y, d2h, d2r = d psi / d (y, h, r) (overwritten)."""
    P = Program()
    y = [P.inp(f"y[{a}]") for a in range(tab.n_Y)]
    hy = [P.inp(f"hy[{a}]") for a in range(tab.n_Y)]
    h = [P.inp(f"h[{b}]") for b in range(tab.n_h)]
    hh = [P.inp(f"hh[{b}]") for b in range(tab.n_h)]
    r = [P.inp(f"r[{p}]") for p in range(tab.P)]
    hr = [P.inp(f"hr[{p}]") for p in range(tab.P)]
    g = [P.inp(f"g[{c}]") for c in range(tab.n_out)]
    dda = [P.inp(f"dda[{c}]") for c in range(tab.n_out)]
    unused = P.inp("T(0)")     # primal value of the forward accumulator: never live
    inputs = {f"y[{a}]": (y[a], hy[a]) for a in range(tab.n_Y)}
    inputs.update({f"h[{b}]": (h[b], hh[b]) for b in range(tab.n_h)})
    inputs.update({f"r[{p}]": (r[p], hr[p]) for p in range(tab.P)})
    inputs.update({f"acc[{c}]": (unused, None) for c in range(tab.n_out)})
    outs = replay_with_tangent(F, P, inputs)
    seeds: Dict[int, int] = {}
    for c in range(tab.n_out):
        t = outs[f"acc[{c}]"][1]
        if t is not None:
            seeds[t] = P.add(seeds.get(t), g[c])
    adj = reverse(P, seeds)
    for c in range(tab.n_out):
        P.out(f"dda[{c}]", P.add(dda[c], outs[f"acc[{c}]"][1]))
    for p in range(tab.P):
        P.out(f"d2r[{p}]", adj.get(r[p]))
    for a in range(tab.n_Y):
        P.out(f"d2y[{a}]", adj.get(y[a]))
    for b in range(tab.n_h):
        P.out(f"d2h[{b}]", adj.get(h[b]))
    return P


def self_check_double(tab: TPTables, D: Program, dtype=np.float64) -> Dict[str, float]:
    rng = np.random.default_rng(1357)
    n = 1500
    shapes = {"y": tab.n_Y, "hy": tab.n_Y, "h": tab.n_h, "hh": tab.n_h, "r": tab.P, "hr": tab.P, "g": tab.n_out}
    v = {k: rng.standard_normal((n, m)).astype(dtype).astype(np.float64) for k, m in shapes.items()}
    p, a, b, c, coef = tab.terms
    dda = np.zeros((n, tab.n_out))
    d2r = np.zeros((n, tab.P))
    d2y = np.zeros((n, tab.n_Y))
    d2h = np.zeros((n, tab.n_h))
    for t in range(len(coef)):
        Y, HY, X, HX, R, HR, G = (v["y"][:, a[t]], v["hy"][:, a[t]], v["h"][:, b[t]], v["hh"][:, b[t]],
                                  v["r"][:, p[t]], v["hr"][:, p[t]], v["g"][:, c[t]])
        dda[:, c[t]] += coef[t] * (HR * Y * X + R * HY * X + R * Y * HX)
        d2r[:, p[t]] += coef[t] * G * (HY * X + Y * HX)
        d2y[:, a[t]] += coef[t] * G * (HR * X + R * HX)
        d2h[:, b[t]] += coef[t] * G * (HR * Y + R * HY)
    inputs = {f"{k}[{i}]": v[k][:, i] for k, m in shapes.items() for i in range(m)}
    inputs.update({f"dda[{i}]": np.zeros(n) for i in range(tab.n_out)})
    inputs["T(0)"] = np.zeros(n)
    res = D.evaluate(inputs, dtype)

    def col(x):
        return np.zeros(n) if x is None else x.astype(np.float64)

    def err(x, ref):
        return float(np.abs(x - ref).max() / np.sqrt((ref ** 2).mean()))
    return {
        "ddA": err(np.stack([col(res[f"dda[{i}]"]) for i in range(tab.n_out)], 1), dda),
        "d2R": err(np.stack([col(res[f"d2r[{i}]"]) for i in range(tab.P)], 1), d2r),
        "d2Y": err(np.stack([col(res[f"d2y[{i}]"]) for i in range(tab.n_Y)], 1), d2y),
        "d2h": err(np.stack([col(res[f"d2h[{i}]"]) for i in range(tab.n_h)], 1), d2h),
    }


def self_check(tab: TPTables, F: Program, Bq: Program, dtype=np.float64) -> Dict[str, float]:
    rng = np.random.default_rng(2468)
    n = 1500
    y = rng.standard_normal((n, tab.n_Y))
    h = rng.standard_normal((n, tab.n_h))
    r = rng.standard_normal((n, tab.P))
    g = rng.standard_normal((n, tab.n_out))
    y, h, r, g = (x.astype(dtype).astype(np.float64) for x in (y, h, r, g))
    p, a, b, c, coef = tab.terms
    msg = np.zeros((n, tab.n_out))
    dr = np.zeros((n, tab.P))
    dy = np.zeros((n, tab.n_Y))
    dh = np.zeros((n, tab.n_h))
    for t in range(len(coef)):
        msg[:, c[t]] += coef[t] * r[:, p[t]] * y[:, a[t]] * h[:, b[t]]
        dr[:, p[t]] += coef[t] * y[:, a[t]] * h[:, b[t]] * g[:, c[t]]
        dy[:, a[t]] += coef[t] * r[:, p[t]] * h[:, b[t]] * g[:, c[t]]
        dh[:, b[t]] += coef[t] * r[:, p[t]] * y[:, a[t]] * g[:, c[t]]
    inputs = {f"y[{i}]": y[:, i] for i in range(tab.n_Y)}
    inputs.update({f"h[{i}]": h[:, i] for i in range(tab.n_h)})
    inputs.update({f"r[{i}]": r[:, i] for i in range(tab.P)})
    inputs.update({f"g[{i}]": g[:, i] for i in range(tab.n_out)})
    inputs.update({f"acc[{i}]": np.zeros(n) for i in range(tab.n_out)})

    def col(v):
        return np.zeros(n) if v is None else v.astype(np.float64)

    def err(x, ref):
        return float(np.abs(x - ref).max() / np.sqrt((ref ** 2).mean()))
    rf, rq = F.evaluate(inputs, dtype), Bq.evaluate(inputs, dtype)
    return {
        "msg": err(np.stack([col(rf[f"acc[{i}]"]) for i in range(tab.n_out)], 1), msg),
        "dR": err(np.stack([col(rq[f"dr[{i}]"]) for i in range(tab.P)], 1), dr),
        "dY": err(np.stack([col(rq[f"dy[{i}]"]) for i in range(tab.n_Y)], 1), dy),
        "dh": err(np.stack([col(rq[f"dh[{i}]"]) for i in range(tab.n_h)], 1), dh),
    }


def flops(c: Dict[str, int]) -> int:
    return 2 * (c.get("fma", 0) + c.get("fnma", 0) + c.get("cfma", 0)) + sum(c.get(k, 0) for k in ("mul", "add", "sub", "cmul"))


def emit_inc(tag: str, spec, tab: TPTables, F: Program, Bq: Program, D: Program) -> str:
    l_Y, l_h, L_max = spec
    cs = [F.count(), Bq.count(), D.count()]
    L = []
    L.append(f"// GENERATED by paper_2504_10700_amd/codegen/generate_tp.py for l_Y={l_Y}, l_h={l_h}, L_max={L_max}.  Do not edit.")
    L.append("//")
    L.append("// Straight-line evaluation of Algorithm 1 of arXiv 2504.10700 per (edge, channel) and of its")
    L.append("// derivatives; paths (index of r): " + " ".join(f"{i}:({a},{b},{c})" for i, (a, b, c) in enumerate(tab.paths)))
    L.append(f"struct GenTP_{tag} {{")
    L.append(f"  static constexpr int kLY = {l_Y}, kLh = {l_h}, kLout = {L_max};")
    L.append(f"  static constexpr int kNY = {tab.n_Y}, kNh = {tab.n_h}, kNout = {tab.n_out}, kP = {tab.P};")
    L.append("  // vector instructions / flops (a fused multiply-add counts twice) per (edge, channel):")
    L.append("  // forward, backward, second-order pass")
    L.append("  static constexpr int kOps[3] = {" + ", ".join(str(c["total"]) for c in cs) + "};")
    L.append("  static constexpr int kFlops[3] = {" + ", ".join(str(flops(c)) for c in cs) + "};")
    L.append("")
    L.append("  // acc += message of one edge")
    L.append("  template <typename T>")
    L.append("  static __device__ __forceinline__ void forward(const T (&y)[kNY], const T (&h)[kNh], const T (&r)[kP],")
    L.append("                                                 T (&acc)[kNout]) {")
    L.append(F.emit("T", "    "))
    L.append("  }")
    L.append("")
    L.append("  // g = dA of the receiver; overwritten: dr, dy (this channel's share of the edge's dY) and dh")
    L.append("  // (the edge's share of the gradient of its sender's features)")
    L.append("  template <typename T>")
    L.append("  static __device__ __forceinline__ void backward(const T (&y)[kNY], const T (&h)[kNh], const T (&r)[kP],")
    L.append("                                                  const T (&g)[kNout], T (&dr)[kP], T (&dy)[kNY], T (&dh)[kNh]) {")
    L.append(Bq.emit("T", "    "))
    L.append("  }")
    L.append("")
    L.append("  // Second-order pass of one edge.  hy, hh, hr: cotangents of (dY, dh, dR); g = dA of the receiver.")
    L.append("  // dda += derivative of the edge's message along (hy, hh, hr); with psi = sum(g * that derivative):")
    L.append("  // d2r = d psi / d r, d2y = this channel's share of d psi / d y, d2h = the edge's share of d psi / d h")
    L.append("  // (all three overwritten).")
    L.append("  template <typename T>")
    L.append("  static __device__ __forceinline__ void double_backward(const T (&y)[kNY], const T (&hy)[kNY], const T (&h)[kNh],")
    L.append("                                                         const T (&hh)[kNh], const T (&r)[kP], const T (&hr)[kP],")
    L.append("                                                         const T (&g)[kNout], T (&dda)[kNout], T (&d2r)[kP],")
    L.append("                                                         T (&d2y)[kNY], T (&d2h)[kNh]) {")
    L.append(D.emit("T", "    "))
    L.append("  }")
    L.append("};")
    return "\n".join(L) + "\n"


def generate(tag: str, lib_path: str = HOST_LIB, verbose: bool = True) -> str:
    spec = SPECS[tag]
    tab = TPTables(lib_path, *spec)
    F, Bq = build_programs(tab)
    D = build_double_backward(tab, F)
    e64 = self_check(tab, F, Bq, np.float64)
    assert max(e64.values()) < 1e-12, e64
    d64 = self_check_double(tab, D, np.float64)
    assert max(d64.values()) < 1e-12, d64
    if verbose:
        e32 = self_check(tab, F, Bq, np.float32)
        d32 = self_check_double(tab, D, np.float32)
        print(f"[tp {tag}] P={tab.P} terms={len(tab.terms[4])} ops fwd={F.count()['total']} bwd={Bq.count()['total']} "
              f"second-order={D.count()['total']}")
        print(f"[tp {tag}] fp64 self-check max|err|/rms: {e64} {d64}")
        print(f"[tp {tag}] fp32 emulation  max|err|/rms: {e32} {d32}")
    return emit_inc(tag, spec, tab, F, Bq, D)


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--check", action="store_true")
    ap.add_argument("--lib", default=HOST_LIB)
    args = ap.parse_args(argv)
    os.makedirs(OUT_DIR, exist_ok=True)
    rc = 0
    for tag in SPECS:
        text = generate(tag, args.lib, verbose=not args.check)
        path = os.path.join(OUT_DIR, f"tp_gen_{tag}.inc")
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
