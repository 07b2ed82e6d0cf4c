"""Pins for oracle/coupling.py against things it does not compute itself:
textbook real spherical harmonics, the Cartesian form of l=1, a hand-derived
table, sympy's Wigner 3j (an outside library) and group-theory identities."""
import itertools
import os

import numpy as np
import pytest

from oracle import coupling as oc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def real_sh_textbook(l, r):
    """Textbook real spherical harmonics in Cartesian form (orthonormal on the sphere)."""
    x, y, z = r
    r2 = x * x + y * y + z * z
    pi = np.pi
    if l == 0:
        return np.array([0.5 * np.sqrt(1 / pi)])
    if l == 1:
        return np.sqrt(3 / (4 * pi)) * np.array([y, z, x])
    if l == 2:
        return np.array([
            0.5 * np.sqrt(15 / pi) * x * y,
            0.5 * np.sqrt(15 / pi) * y * z,
            0.25 * np.sqrt(5 / pi) * (3 * z * z - r2),
            0.5 * np.sqrt(15 / pi) * x * z,
            0.25 * np.sqrt(15 / pi) * (x * x - y * y),
        ])
    if l == 3:
        return np.array([
            0.25 * np.sqrt(35 / (2 * pi)) * y * (3 * x * x - y * y),
            0.5 * np.sqrt(105 / pi) * x * y * z,
            0.25 * np.sqrt(21 / (2 * pi)) * y * (5 * z * z - r2),
            0.25 * np.sqrt(7 / pi) * (5 * z ** 3 - 3 * z * r2),
            0.25 * np.sqrt(21 / (2 * pi)) * x * (5 * z * z - r2),
            0.25 * np.sqrt(105 / pi) * (x * x - y * y) * z,
            0.25 * np.sqrt(35 / (2 * pi)) * x * (x * x - 3 * y * y),
        ])
    raise ValueError(l)


@pytest.mark.parametrize("l", [0, 1, 2, 3, 4, 6])
def test_generators_are_so3_irrep(l):
    X = oc.real_generators(l)
    for a in range(3):
        assert np.abs(X[a] + X[a].T).max() < 1e-14
    # [X_x, X_y] = X_z and cyclic
    for a, b, c in [(0, 1, 2), (1, 2, 0), (2, 0, 1)]:
        assert np.abs(X[a] @ X[b] - X[b] @ X[a] - X[c]).max() < 1e-12
    cas = sum(X[a] @ X[a] for a in range(3))
    assert np.abs(cas + l * (l + 1) * np.eye(2 * l + 1)).max() < 1e-12


def test_l1_is_yzx_permuted_rotation():
    rng = np.random.default_rng(0)
    P = np.zeros((3, 3))
    P[0, 1] = P[1, 2] = P[2, 0] = 1.0   # (x,y,z) -> (y,z,x)
    for _ in range(5):
        th = rng.normal(size=3)
        R = oc.rotation_matrix(th)
        assert np.abs(R @ R.T - np.eye(3)).max() < 1e-13 and np.linalg.det(R) > 0
        assert np.abs(oc.wigner_D_real(1, th) - P @ R @ P.T).max() < 1e-13


def test_rotation_matrix_is_right_handed():
    # quarter turn about z takes x to y
    R = oc.rotation_matrix([0, 0, np.pi / 2])
    assert np.abs(R @ np.array([1.0, 0, 0]) - np.array([0, 1.0, 0])).max() < 1e-14


@pytest.mark.parametrize("l", [0, 1, 2, 3])
def test_wigner_D_rotates_textbook_real_sh(l):
    rng = np.random.default_rng(10 + l)
    for _ in range(4):
        th = rng.normal(size=3) * 1.3
        R = oc.rotation_matrix(th)
        D = oc.wigner_D_real(l, th)
        assert np.abs(D @ D.T - np.eye(2 * l + 1)).max() < 1e-13
        r = rng.normal(size=3)
        r /= np.linalg.norm(r)
        assert np.abs(real_sh_textbook(l, R @ r) - D @ real_sh_textbook(l, r)).max() < 1e-13


TRIPLES = [(a, b, c) for a in range(4) for b in range(4) for c in range(7) if abs(a - b) <= c <= a + b]


@pytest.mark.parametrize("l1,l2,l3", TRIPLES)
def test_coupling_invariant_unit_norm_sign(l1, l2, l3):
    C = oc.coupling_tensor(l1, l2, l3)
    assert abs(np.linalg.norm(C) - 1.0) < 1e-13
    flat = C.ravel()
    assert flat[np.nonzero(flat)[0][0]] > 0
    th = np.random.default_rng(l1 * 100 + l2 * 10 + l3).normal(size=3)
    D1, D2, D3 = (oc.wigner_D_real(l, th) for l in (l1, l2, l3))
    Crot = np.einsum("ai,bj,ck,ijk->abc", D1, D2, D3, C)
    assert np.abs(Crot - C).max() < 1e-13


def test_coupling_zero_outside_triangle():
    for l1, l2, l3 in [(0, 0, 1), (1, 1, 3), (3, 1, 1), (0, 2, 1), (2, 3, 6)]:
        C = oc.coupling_tensor(l1, l2, l3)
        assert C.shape == (2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1) and not C.any()


def test_coupling_closed_forms():
    assert abs(oc.coupling_tensor(0, 0, 0)[0, 0, 0] - 1.0) < 1e-15
    for l in range(1, 5):
        n = 2 * l + 1
        assert np.abs(oc.coupling_tensor(l, l, 0)[:, :, 0] - np.eye(n) / np.sqrt(n)).max() < 1e-14
        assert np.abs(oc.coupling_tensor(0, l, l)[0] - np.eye(n) / np.sqrt(n)).max() < 1e-14
        assert np.abs(oc.coupling_tensor(l, 0, l)[:, 0, :] - np.eye(n) / np.sqrt(n)).max() < 1e-14
    # C(1,1,1) is the Levi-Civita symbol / sqrt(6); (y,z,x) is an even permutation of (x,y,z)
    eps = np.zeros((3, 3, 3))
    for p in itertools.permutations(range(3)):
        eps[p] = np.linalg.det(np.eye(3)[list(p)])
    assert np.abs(oc.coupling_tensor(1, 1, 1) - eps / np.sqrt(6)).max() < 1e-14


def test_coupling_1_1_2_matches_hand_derived_table():
    want = np.zeros((3, 3, 5))
    with open(os.path.join(GOLDEN, "coupling_1_1_2.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            i, j, k, num, den = line.split()
            want[int(i), int(j), int(k)] = float(num) / np.sqrt(float(den))
    got = oc.coupling_tensor(1, 1, 2)
    assert np.count_nonzero(got) == 11
    assert np.abs(got - want).max() < 1e-14


@pytest.mark.parametrize("l1,l2", [(1, 1), (1, 2), (2, 2), (2, 3), (3, 3)])
def test_coupling_orthogonality(l1, l2):
    # sum_{m1 m2} C(l1,l2,l3)[m1,m2,m3] C(l1,l2,l3')[m1,m2,m3'] = delta delta / (2 l3 + 1)
    for l3 in range(abs(l1 - l2), l1 + l2 + 1):
        for l3p in range(abs(l1 - l2), l1 + l2 + 1):
            G = np.einsum("abc,abd->cd", oc.coupling_tensor(l1, l2, l3), oc.coupling_tensor(l1, l2, l3p))
            want = np.eye(2 * l3 + 1) / (2 * l3 + 1) if l3 == l3p else 0.0
            assert np.abs(G - want).max() < 1e-13
    # completeness: the C(l1,l2,l3) over all l3, rescaled, form an orthogonal basis change
    tot = sum((2 * l3 + 1) * np.einsum("abc,dec->abde", oc.coupling_tensor(l1, l2, l3), oc.coupling_tensor(l1, l2, l3))
              for l3 in range(abs(l1 - l2), l1 + l2 + 1))
    n1, n2 = 2 * l1 + 1, 2 * l2 + 1
    assert np.abs(tot.reshape(n1 * n2, n1 * n2) - np.eye(n1 * n2)).max() < 1e-13


def _complex_to_real_test_side(l):
    """Rows: real SH m' as combinations of complex Y_l^m (textbook relation
    Y_{l,+u} = sqrt2 (-1)^u Re Y_l^u, Y_{l,-u} = sqrt2 (-1)^u Im Y_l^u)."""
    n = 2 * l + 1
    Q = np.zeros((n, n), dtype=complex)
    Q[l, l] = 1
    for u in range(1, l + 1):
        # Re Y^u = (Y^u + (-1)^u Y^-u)/2 ; Im Y^u = (Y^u - (-1)^u Y^-u)/(2i)
        Q[l + u, l + u] = (-1) ** u / np.sqrt(2)
        Q[l + u, l - u] = 1 / np.sqrt(2)
        Q[l - u, l + u] = (-1) ** u / (1j * np.sqrt(2))
        Q[l - u, l - u] = -1 / (1j * np.sqrt(2))
    return Q


@pytest.mark.parametrize("l1,l2,l3", [(1, 1, 0), (1, 1, 1), (1, 1, 2), (1, 2, 1), (1, 2, 3), (2, 2, 2),
                                      (2, 3, 1), (2, 2, 3), (3, 3, 2), (3, 3, 4), (2, 3, 5), (3, 3, 6), (3, 2, 4)])
def test_coupling_against_sympy_wigner_3j(l1, l2, l3):
    from sympy.physics.wigner import wigner_3j
    w = np.zeros((2 * l1 + 1, 2 * l2 + 1, 2 * l3 + 1), dtype=complex)
    for m1 in range(-l1, l1 + 1):
        for m2 in range(-l2, l2 + 1):
            m3 = -m1 - m2
            if abs(m3) <= l3:
                w[m1 + l1, m2 + l2, m3 + l3] = float(wigner_3j(l1, l2, l3, m1, m2, m3))
    # the 3j symbol is the invariant of the ket components; a real-basis tensor
    # t relates to it by contracting each slot with conj(Q) (kets = Q^T real).
    Q1, Q2, Q3 = (_complex_to_real_test_side(l) for l in (l1, l2, l3))
    t = np.einsum("ai,bj,ck,ijk->abc", Q1.conj(), Q2.conj(), Q3.conj(), w)
    t = t.real if np.abs(t.real).max() > np.abs(t.imag).max() else t.imag
    t = t / np.linalg.norm(t)
    flat = t.ravel()
    big = np.nonzero(np.abs(flat) > 1e-12)[0][0]
    if flat[big] < 0:
        t = -t
    assert np.abs(t - oc.coupling_tensor(l1, l2, l3)).max() < 1e-12


def test_coupling_sparsity_is_in_the_range_the_paper_quotes():
    # Section 4.1: non-zeros are "typically less than 20%" of the combinations.
    fr = []
    for l1, l2, l3 in TRIPLES:
        if min(l1, l2, l3) >= 1:
            C = oc.coupling_tensor(l1, l2, l3)
            fr.append(np.count_nonzero(C) / C.size)
    assert np.median(fr) < 0.20 and max(fr) < 0.30
