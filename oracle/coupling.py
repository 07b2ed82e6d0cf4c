"""Real-basis SO(3) irreps and three-irrep coupling tensors (oracle side, fp64).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper uses Clebsch-Gordan coefficients C^{l3 m3}_{l1 m1, l2 m2} (notation
table, Section 2.2) and generalized ones C^{LM}_{lm} (Algorithm 2) without
fixing basis, phase or normalisation.  The reading taken here:

* Components of an irrep l are indexed m = -l..l in the real spherical-harmonic
  basis built from Condon-Shortley kets,
      |l, m>_R = ((-1)^m |l,m> + |l,-m>) / sqrt(2)            m > 0
      |l, 0>_R = |l,0>
      |l,-u>_R = ((-1)^u |l,u> - |l,-u>) / (i sqrt(2))        u > 0
  so that l = 1 is ordered (y, z, x).
* C(l1,l2,l3) is THE rotation-invariant tensor of V_l1 (x) V_l2 (x) V_l3 (it is
  unique up to scale when the triangle rule of Section 4.2 holds, and does not
  exist otherwise), scaled to unit Frobenius norm, sign chosen so the first
  non-zero entry in row-major (m1,m2,m3) order is positive.

Here the tensor is obtained as the null vector of the summed infinitesimal
rotation generators, which involves no Wigner-3j / Racah formula at all.
"""
from __future__ import annotations

import functools

import numpy as np
import scipy.linalg


def complex_to_real_matrix(l: int) -> np.ndarray:
    """Q[m', m]: real-basis vector m' expressed in Condon-Shortley kets |l,m>."""
    n = 2 * l + 1
    Q = np.zeros((n, n), dtype=np.complex128)
    s = 1.0 / np.sqrt(2.0)
    Q[l, l] = 1.0
    for u in range(1, l + 1):
        sign = (-1.0) ** u
        # m' = +u
        Q[l + u, l + u] = sign * s
        Q[l + u, l - u] = s
        # m' = -u
        Q[l - u, l + u] = sign * s / 1j
        Q[l - u, l - u] = -s / 1j
    return Q


def complex_generators(l: int):
    """Angular-momentum matrices (Jx, Jy, Jz) on kets |l,m>, m = -l..l."""
    n = 2 * l + 1
    m = np.arange(-l, l + 1)
    Jz = np.diag(m).astype(np.complex128)
    Jp = np.zeros((n, n), dtype=np.complex128)  # J+ |m> = c |m+1>
    for i in range(n - 1):
        mm = m[i]
        Jp[i + 1, i] = np.sqrt(l * (l + 1) - mm * (mm + 1))
    Jm = Jp.conj().T
    Jx = (Jp + Jm) / 2.0
    Jy = (Jp - Jm) / (2.0j)
    return Jx, Jy, Jz


@functools.lru_cache(maxsize=None)
def real_generators(l: int) -> np.ndarray:
    """X[a] (a = x,y,z): real antisymmetric generators acting on real-basis
    component vectors, D^l(exp(theta . L)) = expm(sum_a theta_a X[a])."""
    Q = complex_to_real_matrix(l)
    out = []
    for J in complex_generators(l):
        # a state with real-basis components v has ket components Q^T v;
        # kets rotate with exp(-i theta J).
        X = Q.conj() @ (-1j * J) @ Q.T
        assert np.abs(X.imag).max() < 1e-13
        out.append(X.real)
    X = np.stack(out)
    X.setflags(write=False)
    return X


def rotation_matrix(theta) -> np.ndarray:
    """3x3 rotation exp(theta . L) for an axis-angle vector theta (xyz)."""
    tx, ty, tz = (float(t) for t in theta)
    K = np.array([[0.0, -tz, ty], [tz, 0.0, -tx], [-ty, tx, 0.0]])
    return scipy.linalg.expm(K)


def wigner_D_real(l: int, theta) -> np.ndarray:
    """Real-basis Wigner D matrix of irrep l for axis-angle vector theta."""
    X = real_generators(l)
    G = sum(float(t) * X[a] for a, t in enumerate(theta))
    return scipy.linalg.expm(G)


@functools.lru_cache(maxsize=None)
def coupling_tensor(l1: int, l2: int, l3: int) -> np.ndarray:
    """C(l1,l2,l3)[m1,m2,m3]: unit-norm invariant tensor, zero array if the
    triangle rule |l1-l2| <= l3 <= l1+l2 fails."""
    n1, n2, n3 = 2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1
    if not (abs(l1 - l2) <= l3 <= l1 + l2):
        C = np.zeros((n1, n2, n3))
        C.setflags(write=False)
        return C
    X1, X2, X3 = real_generators(l1), real_generators(l2), real_generators(l3)
    I1, I2, I3 = np.eye(n1), np.eye(n2), np.eye(n3)
    S = np.zeros((n1 * n2 * n3,) * 2)
    for a in range(3):
        G = (np.kron(np.kron(X1[a], I2), I3)
             + np.kron(np.kron(I1, X2[a]), I3)
             + np.kron(np.kron(I1, I2), X3[a]))
        S += G.T @ G
    w, v = np.linalg.eigh(S)
    # exactly one invariant: one (numerically) zero eigenvalue, a gap after it
    assert abs(w[0]) < 1e-10 and (len(w) == 1 or w[1] > 1e-3), (l1, l2, l3, w[:3])
    c = v[:, 0]
    c = c / np.linalg.norm(c)
    c[np.abs(c) < 1e-13] = 0.0
    first = c[np.nonzero(c)[0][0]]
    if first < 0:
        c = -c
    C = c.reshape(n1, n2, n3)
    C.setflags(write=False)
    return C
