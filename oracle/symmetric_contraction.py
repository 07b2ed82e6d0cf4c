"""fp64 oracle of the MACE symmetric tensor contraction (product basis).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Follows Algorithm 2 of the paper (the product-basis step of MACE, Section 4.1)
and the message equation of Section 2.2 (m = sum_nu sum_eta W^(nu)_{k,eta} B^(nu)_{eta,kLM}):
for every atom i, channel k and output component (L,M)

    B[i,k,(L,M)] = sum_{nu=1..nu_max} sum_{eta} W[z_i, p(nu,L,eta), k]
                   * sum_{a_1..a_nu} U^{(nu,L,eta)}[M, a_1..a_nu] * prod_xi A[i,k,a_xi]

with dense generalized coupling tensors U, no sparsity, no symmetrisation.
The backward is the analytic derivative of that expression.

Readings of what the paper leaves open:
* component index a = l*l + l + m; A carries l = 0..l_max with parity (-1)^l;
* a coupling path eta is an ORDERED l-tuple plus, for nu = 3, the intermediate
  L2 of the chain ((l1 (x) l2) -> L2) (x) l3 -> L; all paths allowed by the
  triangle rule and parity are present (over-complete on purpose);
* U chains the unit-norm invariant tensors of oracle.coupling with no extra factor;
* weights are per (element, path, channel); the nu-sum and the weights are
  inside the operation.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

from .coupling import coupling_tensor


@dataclass(frozen=True)
class OracleConfig:
    num_channels: int
    l_max: int
    nu_max: int
    num_elements: int
    out_irreps: Tuple[Tuple[int, int], ...]  # ((L, parity), ...), parity = +1 (e) / -1 (o)

    @property
    def n_lm(self) -> int:
        return (self.l_max + 1) ** 2

    @property
    def n_LM(self) -> int:
        return sum(2 * L + 1 for L, _ in self.out_irreps)

    def out_slice(self, out_idx: int) -> slice:
        start = sum(2 * L + 1 for L, _ in self.out_irreps[:out_idx])
        return slice(start, start + 2 * self.out_irreps[out_idx][0] + 1)


def enumerate_paths(cfg: OracleConfig) -> List[Tuple[int, int, int, int, int, int]]:
    """All coupling paths as rows (nu, out_idx, l1, l2, l3, L2), unused = -1.

    Order: nu ascending, then output irrep, then (l1, l2, L2, l3) lexicographic.
    """
    paths = []
    ls = range(cfg.l_max + 1)
    for nu in range(1, cfg.nu_max + 1):
        for oi, (L, par) in enumerate(cfg.out_irreps):
            if nu == 1:
                if L <= cfg.l_max and (-1) ** L == par:
                    paths.append((1, oi, L, -1, -1, -1))
            elif nu == 2:
                for l1 in ls:
                    for l2 in ls:
                        if abs(l1 - l2) <= L <= l1 + l2 and (-1) ** (l1 + l2) == par:
                            paths.append((2, oi, l1, l2, -1, -1))
            elif nu == 3:
                block = []
                for l1 in ls:
                    for l2 in ls:
                        for L2 in range(abs(l1 - l2), l1 + l2 + 1):
                            for l3 in ls:
                                if abs(L2 - l3) <= L <= L2 + l3 and (-1) ** (l1 + l2 + l3) == par:
                                    block.append((l1, l2, L2, l3))
                block.sort()
                for l1, l2, L2, l3 in block:
                    paths.append((3, oi, l1, l2, l3, L2))
            else:
                raise ValueError("nu_max > 3 is outside what this oracle covers")
    return paths


def _embed(cfg: OracleConfig, l: int) -> slice:
    return slice(l * l, (l + 1) * (l + 1))


def dense_U(cfg: OracleConfig, path) -> np.ndarray:
    """Generalized coupling tensor of one path, shape (2L+1, n_lm, ..nu times..)."""
    nu, oi, l1, l2, l3, L2 = path
    L = cfg.out_irreps[oi][0]
    n = cfg.n_lm
    if nu == 1:
        U = np.zeros((2 * L + 1, n))
        for M in range(2 * L + 1):
            U[M, L * L + M] = 1.0
        return U
    if nu == 2:
        U = np.zeros((2 * L + 1, n, n))
        C = coupling_tensor(l1, l2, L)  # [m1, m2, M]
        U[:, _embed(cfg, l1), _embed(cfg, l2)] = np.transpose(C, (2, 0, 1))
        return U
    U = np.zeros((2 * L + 1, n, n, n))
    C12 = coupling_tensor(l1, l2, L2)  # [m1, m2, M2]
    C23 = coupling_tensor(L2, l3, L)   # [M2, m3, M]
    blk = np.einsum("abq,qcM->Mabc", C12, C23)
    U[:, _embed(cfg, l1), _embed(cfg, l2), _embed(cfg, l3)] = blk
    return U


@dataclass
class OracleTables:
    cfg: OracleConfig
    paths: list
    # per nu: matrix (n_lm**nu, ncols) and for every column block its path index / out slice
    Umat: dict = field(default_factory=dict)
    cols: dict = field(default_factory=dict)   # nu -> list of (path_index, col_start, col_stop)


def build_tables(cfg: OracleConfig) -> OracleTables:
    paths = enumerate_paths(cfg)
    T = OracleTables(cfg=cfg, paths=paths)
    for nu in range(1, cfg.nu_max + 1):
        blocks, cols, c0 = [], [], 0
        for p, path in enumerate(paths):
            if path[0] != nu:
                continue
            U = dense_U(cfg, path)
            nM = U.shape[0]
            blocks.append(U.reshape(nM, -1).T)  # (n_lm**nu, nM)
            cols.append((p, c0, c0 + nM))
            c0 += nM
        T.Umat[nu] = np.concatenate(blocks, axis=1) if blocks else np.zeros((cfg.n_lm ** nu, 0))
        T.cols[nu] = cols
    return T


def _powers(A: np.ndarray, nu: int) -> np.ndarray:
    """prod_xi A[..., a_xi] for all (a_1..a_nu): shape (..., n**nu)."""
    X = A
    for _ in range(nu - 1):
        X = (X[..., :, None] * A[..., None, :]).reshape(*A.shape[:-1], -1)
    return X


def _path_polys(T: OracleTables, A: np.ndarray):
    """P[nu] of shape (n, K, ncols_nu): the un-weighted path polynomials."""
    return {nu: _powers(A, nu) @ T.Umat[nu] for nu in T.Umat}


def forward(T: OracleTables, A: np.ndarray, z: np.ndarray, W: np.ndarray, chunk: int = 64) -> np.ndarray:
    """B[node, channel, LM] per Algorithm 2.  A: (N,K,n_lm), z: (N,), W: (Z,P,K)."""
    cfg = T.cfg
    A = np.asarray(A, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    N, K, _ = A.shape
    B = np.zeros((N, K, cfg.n_LM))
    for s in range(0, N, chunk):
        a = A[s:s + chunk]
        w = W[z[s:s + chunk]]                       # (c, P, K)
        P = _path_polys(T, a)
        for nu, cols in T.cols.items():
            for p, c0, c1 in cols:
                sl = cfg.out_slice(T.paths[p][1])
                B[s:s + chunk, :, sl] += w[:, p, :, None] * P[nu][:, :, c0:c1]
    return B


def backward(T: OracleTables, A: np.ndarray, z: np.ndarray, W: np.ndarray, dB: np.ndarray,
             chunk: int = 64):
    """(dA, dW) for upstream gradient dB; same layouts as A and W."""
    cfg = T.cfg
    A = np.asarray(A, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    dB = np.asarray(dB, dtype=np.float64)
    N, K, n = A.shape
    dA = np.zeros_like(A)
    dW = np.zeros_like(W)
    for s in range(0, N, chunk):
        a = A[s:s + chunk]
        zz = z[s:s + chunk]
        w = W[zz]
        g = dB[s:s + chunk]
        c = a.shape[0]
        P = _path_polys(T, a)
        for nu, cols in T.cols.items():
            dP = np.zeros((c, K, T.Umat[nu].shape[1]))
            for p, c0, c1 in cols:
                sl = cfg.out_slice(T.paths[p][1])
                dP[:, :, c0:c1] = g[:, :, sl] * w[:, p, :, None]
                # dW[z,p,k] += sum_M dB * P
                np.add.at(dW[:, p, :], zz, (g[:, :, sl] * P[nu][:, :, c0:c1]).sum(axis=2))
            dX = (dP @ T.Umat[nu].T).reshape((c, K) + (n,) * nu)
            if nu == 1:
                dA[s:s + chunk] += dX
            elif nu == 2:
                dA[s:s + chunk] += np.einsum("ikab,ikb->ika", dX, a)
                dA[s:s + chunk] += np.einsum("ikab,ika->ikb", dX, a)
            else:
                dA[s:s + chunk] += np.einsum("ikabc,ikb,ikc->ika", dX, a, a)
                dA[s:s + chunk] += np.einsum("ikabc,ika,ikc->ikb", dX, a, a)
                dA[s:s + chunk] += np.einsum("ikabc,ika,ikb->ikc", dX, a, a)
    return dA, dW


def double_backward(T: OracleTables, A: np.ndarray, z: np.ndarray, W: np.ndarray, dB: np.ndarray,
                    H: np.ndarray, chunk: int = 64):
    """Second-order pass needed when a loss depends on dA (forces are derivatives of the
    energy, Section 2.2, so force training differentiates the backward once more).

    With phi = sum(dB * B(A, W)) and psi = sum(H * dphi/dA) (H has the shape of A) returns
        ddB = dpsi/d(dB)   [n, K, n_LM]   = directional derivative of B along H
        dA2 = dpsi/dA      [n, K, n_lm]   = Hessian of phi applied to H
        dW2 = dpsi/dW      [Z, P, K]
    written out from the definition of B as a polynomial: the derivative along H replaces
    one factor A by H in every slot in turn.
    """
    cfg = T.cfg
    A = np.asarray(A, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    dB = np.asarray(dB, dtype=np.float64)
    H = np.asarray(H, dtype=np.float64)
    N, K, n = A.shape
    ddB = np.zeros_like(dB)
    dA2 = np.zeros_like(A)
    dW2 = np.zeros_like(W)
    for s in range(0, N, chunk):
        a, h, g, zz = A[s:s + chunk], H[s:s + chunk], dB[s:s + chunk], z[s:s + chunk]
        w = W[zz]
        c = a.shape[0]
        for nu, cols in T.cols.items():
            Umat = T.Umat[nu]                                  # [n^nu, col]
            # derivative along h of the monomials a_{a1}..a_{a_nu}: h takes every slot in turn
            if nu == 1:
                Xdot = h
            elif nu == 2:
                Xdot = np.einsum("ika,ikb->ikab", h, a) + np.einsum("ika,ikb->ikab", a, h)
            else:
                aa = np.einsum("ika,ikb->ikab", a, a)
                ha = np.einsum("ika,ikb->ikab", h, a)
                ah = np.einsum("ika,ikb->ikab", a, h)
                Xdot = (np.einsum("ikab,ikd->ikabd", ha, a) + np.einsum("ikab,ikd->ikabd", ah, a)
                        + np.einsum("ikab,ikd->ikabd", aa, h))
            Pdot = Xdot.reshape(c, K, -1) @ Umat               # directional derivative of every path polynomial
            gw = np.zeros((c, K, Umat.shape[1]))               # dB * W per column
            for p, c0, c1 in cols:
                sl = cfg.out_slice(T.paths[p][1])
                ddB[s:s + chunk, :, sl] += w[:, p, :, None] * Pdot[:, :, c0:c1]
                np.add.at(dW2[:, p, :], zz, (g[:, :, sl] * Pdot[:, :, c0:c1]).sum(axis=2))
                gw[:, :, c0:c1] = g[:, :, sl] * w[:, p, :, None]
            # dX[a1..a_nu] = sum_col gw[col] * U[col; a1..a_nu]; in dA2 one slot is the free
            # index, one holds h and (nu = 3) the last keeps a
            dX = (gw @ Umat.T).reshape((c, K) + (n,) * nu)
            if nu == 2:
                dA2[s:s + chunk] += np.einsum("ikab,ika->ikb", dX, h)
                dA2[s:s + chunk] += np.einsum("ikab,ikb->ika", dX, h)
            elif nu == 3:
                for hs, rs, ks in ((0, 1, 2), (0, 2, 1), (1, 0, 2), (1, 2, 0), (2, 0, 1), (2, 1, 0)):
                    # slot hs holds h, slot rs is differentiated (free index), slot ks keeps a
                    idx = ["", "", ""]
                    idx[hs], idx[rs], idx[ks] = "x", "y", "v"
                    dA2[s:s + chunk] += np.einsum("ik" + "".join(idx) + ",ikx,ikv->iky", dX, h, a)
    return ddB, dA2, dW2
