"""Pins for oracle/symmetric_contraction.py: closed forms, brute-force loops of
Algorithm 2, rotation / inversion equivariance, weight-counting multiplicities,
finite differences and polynomial identities.  None of them re-uses the
oracle's own contraction code to produce the expected value."""
import itertools
import math

import numpy as np
import pytest

from oracle import coupling as oc
from oracle import symmetric_contraction as osc

O01 = ((0, 1), (1, -1))
O012 = ((0, 1), (1, -1), (2, 1))


def rand_inputs(cfg, N, seed):
    rng = np.random.default_rng(seed)
    P = len(osc.enumerate_paths(cfg))
    z = rng.integers(0, cfg.num_elements, size=N).astype(np.int32)
    A = rng.standard_normal((N, cfg.num_channels, cfg.n_lm))
    W = rng.standard_normal((cfg.num_elements, P, cfg.num_channels))
    dB = rng.standard_normal((N, cfg.num_channels, cfg.n_LM))
    return A, z, W, dB


# ---------------------------------------------------------------- path table

def sym_power_multiplicity(l_max, nu, L, parity):
    """Multiplicity of irrep (L,parity) in Sym^nu(0e+1o+..+l_max) by weight counting."""
    basis = [(m, (-1) ** l) for l in range(l_max + 1) for m in range(-l, l + 1)]

    def count(mtot):
        c = 0
        for combo in itertools.combinations_with_replacement(range(len(basis)), nu):
            if sum(basis[i][0] for i in combo) == mtot and np.prod([basis[i][1] for i in combo]) == parity:
                c += 1
        return c
    return count(L) - count(L + 1)


def test_path_counts_and_order():
    cfg = osc.OracleConfig(4, 3, 3, 2, O012)
    paths = osc.enumerate_paths(cfg)
    cnt = {}
    for p in paths:
        cnt[(p[0], p[1])] = cnt.get((p[0], p[1]), 0) + 1
    assert cnt == {(1, 0): 1, (1, 1): 1, (1, 2): 1, (2, 0): 4, (2, 1): 6, (2, 2): 7,
                   (3, 0): 23, (3, 1): 51, (3, 2): 65}
    assert paths == sorted(paths, key=lambda p: (p[0], p[1], p[2], p[3], p[5], p[4]))
    assert len(osc.enumerate_paths(osc.OracleConfig(4, 3, 3, 2, O01))) == 86
    tiny = osc.enumerate_paths(osc.OracleConfig(8, 1, 2, 2, ((0, 1),)))
    assert tiny == [(1, 0, 0, -1, -1, -1), (2, 0, 0, 0, -1, -1), (2, 0, 1, 1, -1, -1)]
    # every path obeys triangle rule(s) and parity
    for nu, oi, l1, l2, l3, L2 in paths:
        L, par = cfg.out_irreps[oi]
        if nu == 2:
            assert abs(l1 - l2) <= L <= l1 + l2 and (-1) ** (l1 + l2) == par
        if nu == 3:
            assert abs(l1 - l2) <= L2 <= l1 + l2 and abs(L2 - l3) <= L <= L2 + l3
            assert (-1) ** (l1 + l2 + l3) == par


@pytest.mark.parametrize("l_max,outs", [(1, ((0, 1), (1, -1), (2, 1), (3, -1))), (3, O012)])
def test_symmetrised_rank_equals_weight_counting_multiplicity(l_max, outs):
    cfg = osc.OracleConfig(1, l_max, 3, 1, outs)
    paths = osc.enumerate_paths(cfg)
    for nu in (2, 3):
        for oi, (L, par) in enumerate(outs):
            vecs = []
            for p in paths:
                if p[0] == nu and p[1] == oi:
                    U = osc.dense_U(cfg, p)
                    Us = sum(np.transpose(U, (0,) + tuple(1 + i for i in s))
                             for s in itertools.permutations(range(nu))) / math.factorial(nu)
                    vecs.append(Us.ravel())
            want = sym_power_multiplicity(l_max, nu, L, par)
            if not vecs:
                assert want == 0
                continue
            rank = np.linalg.matrix_rank(np.array(vecs), tol=1e-10)
            assert rank == want, (nu, L, par, rank, want)


def test_known_multiplicities():
    # independent of the oracle: the numbers the design relies on
    assert [sym_power_multiplicity(3, 2, L, p) for L, p in O012] == [4, 3, 5]
    assert [sym_power_multiplicity(3, 3, L, p) for L, p in O012] == [8, 12, 14]
    assert [sym_power_multiplicity(1, 3, L, p) for L, p in ((0, 1), (1, -1), (2, 1), (3, -1))] == [2, 2, 1, 1]


# ---------------------------------------------------------------- closed forms

def test_tiny_config_closed_form():
    cfg = osc.OracleConfig(8, 1, 2, 2, ((0, 1),))
    T = osc.build_tables(cfg)
    A, z, W, dB = rand_inputs(cfg, 64, 1)
    Wn = W[z]                                     # (N, 3, K)
    a0, a1 = A[:, :, 0], A[:, :, 1:4]
    n1 = (a1 ** 2).sum(-1)
    B = Wn[:, 0] * a0 + Wn[:, 1] * a0 ** 2 + Wn[:, 2] * n1 / np.sqrt(3)
    assert np.abs(osc.forward(T, A, z, W)[:, :, 0] - B).max() < 1e-13
    g = dB[:, :, 0]
    dA = np.zeros_like(A)
    dA[:, :, 0] = g * (Wn[:, 0] + 2 * Wn[:, 1] * a0)
    dA[:, :, 1:4] = (g * Wn[:, 2] * 2 / np.sqrt(3))[:, :, None] * a1
    dW = np.zeros_like(W)
    for i in range(64):
        dW[z[i], 0] += g[i] * a0[i]
        dW[z[i], 1] += g[i] * a0[i] ** 2
        dW[z[i], 2] += g[i] * n1[i] / np.sqrt(3)
    gA, gW = osc.backward(T, A, z, W, dB)
    assert np.abs(gA - dA).max() < 1e-13 and np.abs(gW - dW).max() < 1e-12


def test_scalar_only_input_closed_form():
    cfg = osc.OracleConfig(3, 3, 3, 2, O012)
    T = osc.build_tables(cfg)
    A, z, W, _ = rand_inputs(cfg, 5, 2)
    A[:, :, 1:] = 0.0
    a = A[:, :, 0]
    idx = {(p[0], p[1], p[2], p[3], p[4], p[5]): i for i, p in enumerate(T.paths)}
    w1 = W[z][:, idx[(1, 0, 0, -1, -1, -1)]]
    w2 = W[z][:, idx[(2, 0, 0, 0, -1, -1)]]
    w3 = W[z][:, idx[(3, 0, 0, 0, 0, 0)]]
    B = osc.forward(T, A, z, W)
    assert np.abs(B[:, :, 0] - (w1 * a + w2 * a ** 2 + w3 * a ** 3)).max() < 1e-13
    assert np.abs(B[:, :, 1:]).max() < 1e-14


def test_invariant_quadratic_block_closed_form():
    # 0e, nu = 2 only: sum_l W_(l,l) |A_l|^2 / sqrt(2l+1)
    cfg = osc.OracleConfig(2, 3, 2, 3, ((0, 1),))
    T = osc.build_tables(cfg)
    A, z, W, _ = rand_inputs(cfg, 7, 3)
    W[:, 0] = 0.0  # drop nu = 1
    want = 0.0
    for p, path in enumerate(T.paths):
        if path[0] == 2:
            l = path[2]
            assert path[3] == l
            want = want + W[z][:, p] * (A[:, :, l * l:(l + 1) ** 2] ** 2).sum(-1) / np.sqrt(2 * l + 1)
    assert np.abs(osc.forward(T, A, z, W)[:, :, 0] - want).max() < 1e-13


def test_vector_triple_products_closed_form():
    """l_max = 1, nu = 3, output 1o: with v = (A_y,A_z,A_x) and s = A_00 the path
    ((1 x 1)->0) x 1 gives |v|^2 v / 3 and ((1 x 1)->1) x 1 gives (v x v) x v = 0."""
    cfg = osc.OracleConfig(1, 1, 3, 1, ((1, -1),))
    T = osc.build_tables(cfg)
    rng = np.random.default_rng(5)
    A = rng.standard_normal((3, 1, 4))
    z = np.zeros(3, dtype=np.int32)
    v = A[:, 0, 1:4]
    for p, path in enumerate(T.paths):
        W = np.zeros((1, len(T.paths), 1))
        W[0, p, 0] = 1.0
        B = osc.forward(T, A, z, W)[:, 0, :]
        if path[0] == 3 and path[2:] == (1, 1, 1, 0):
            # C(1,1,0) = delta/sqrt3 ; C(0,1,1) = delta/sqrt3
            assert np.abs(B - (v ** 2).sum(-1, keepdims=True) * v / 3.0).max() < 1e-14
        if path[0] == 3 and path[2:] == (1, 1, 1, 1):
            assert np.abs(B).max() < 1e-14
        if path[0] == 3 and path[2:] == (0, 0, 1, 0):
            assert np.abs(B - A[:, 0, :1] ** 2 * v / np.sqrt(3)).max() < 1e-14
        if path[0] == 2 and path[2:4] == (0, 1):
            assert np.abs(B - A[:, 0, :1] * v / np.sqrt(3)).max() < 1e-14


# ---------------------------------------------------------------- brute force

def brute_force_forward(cfg, A, z, W):
    """Literal loop nest of Algorithm 2 with coefficients read straight from the
    three-irrep tensors (no dense U, no matmul)."""
    paths = osc.enumerate_paths(cfg)
    N, K, n = A.shape
    lm = [(l, m) for l in range(cfg.l_max + 1) for m in range(-l, l + 1)]
    B = np.zeros((N, K, cfg.n_LM))
    for i in range(N):
        for k in range(K):
            col = 0
            for oi, (L, par) in enumerate(cfg.out_irreps):
                for M in range(-L, L + 1):
                    acc = 0.0
                    for p, (nu, po, l1, l2, l3, L2) in enumerate(paths):
                        if po != oi:
                            continue
                        w = W[z[i], p, k]
                        if nu == 1:
                            acc += w * A[i, k, L * L + L + M]
                        elif nu == 2:
                            C = oc.coupling_tensor(l1, l2, L)
                            for a1, (la, ma) in enumerate(lm):
                                for a2, (lb, mb) in enumerate(lm):
                                    if la == l1 and lb == l2:
                                        acc += w * C[ma + l1, mb + l2, M + L] * A[i, k, a1] * A[i, k, a2]
                        else:
                            C12 = oc.coupling_tensor(l1, l2, L2)
                            C23 = oc.coupling_tensor(L2, l3, L)
                            for a1, (la, ma) in enumerate(lm):
                                if la != l1:
                                    continue
                                for a2, (lb, mb) in enumerate(lm):
                                    if lb != l2:
                                        continue
                                    for a3, (lc, mc) in enumerate(lm):
                                        if lc != l3:
                                            continue
                                        cg = 0.0
                                        for M2 in range(-L2, L2 + 1):
                                            cg += C12[ma + l1, mb + l2, M2 + L2] * C23[M2 + L2, mc + l3, M + L]
                                        acc += w * cg * A[i, k, a1] * A[i, k, a2] * A[i, k, a3]
                    B[i, k, col] = acc
                    col += 1
    return B


@pytest.mark.parametrize("l_max,nu_max,outs,N,K", [
    (1, 2, ((0, 1),), 3, 2),
    (2, 3, O012, 2, 2),
    (3, 3, O01, 1, 2),
])
def test_forward_matches_brute_force(l_max, nu_max, outs, N, K):
    cfg = osc.OracleConfig(K, l_max, nu_max, 2, outs)
    T = osc.build_tables(cfg)
    A, z, W, _ = rand_inputs(cfg, N, 7)
    assert np.abs(osc.forward(T, A, z, W) - brute_force_forward(cfg, A, z, W)).max() < 1e-12


# ---------------------------------------------------------------- symmetries

def block_diag_D(cfg_ls, th):
    import scipy.linalg
    return scipy.linalg.block_diag(*[oc.wigner_D_real(l, th) for l in cfg_ls])


@pytest.mark.parametrize("outs", [O01, O012, ((3, -1), (2, -1), (1, 1))])
def test_rotation_and_inversion_equivariance(outs):
    cfg = osc.OracleConfig(3, 3, 3, 4, outs)
    T = osc.build_tables(cfg)
    A, z, W, dB = rand_inputs(cfg, 6, 11)
    th = np.array([0.7, -1.1, 0.4])
    Din = block_diag_D(range(cfg.l_max + 1), th)
    Dout = block_diag_D([L for L, _ in outs], th)
    B = osc.forward(T, A, z, W)
    Brot = osc.forward(T, A @ Din.T, z, W)
    assert np.abs(Brot - B @ Dout.T).max() < 1e-12
    # gradients: dA rotates like A, dW is invariant
    dA, dW = osc.backward(T, A, z, W, dB)
    dA2, dW2 = osc.backward(T, A @ Din.T, z, W, dB @ Dout.T)
    assert np.abs(dA2 - dA @ Din.T).max() < 1e-12
    assert np.abs(dW2 - dW).max() < 1e-11
    # inversion: A_l -> (-1)^l A_l  =>  B_(L,p) -> p B
    sgn_in = np.concatenate([np.full(2 * l + 1, (-1.0) ** l) for l in range(cfg.l_max + 1)])
    sgn_out = np.concatenate([np.full(2 * L + 1, float(p)) for L, p in outs])
    assert np.abs(osc.forward(T, A * sgn_in, z, W) - B * sgn_out).max() < 1e-12
    assert np.abs(B).max() > 0.1


def test_permutation_symmetry_and_vanishing_paths():
    cfg = osc.OracleConfig(2, 3, 3, 2, O01)
    T = osc.build_tables(cfg)
    A, z, W, dB = rand_inputs(cfg, 8, 13)
    B = osc.forward(T, A, z, W)
    dA, dW = osc.backward(T, A, z, W, dB)
    # replace every U by its average over slot permutations: nothing may change
    Ts = osc.build_tables(cfg)
    for nu in (2, 3):
        n = cfg.n_lm
        U = Ts.Umat[nu].T.reshape((-1,) + (n,) * nu)
        Us = sum(np.transpose(U, (0,) + tuple(1 + i for i in s))
                 for s in itertools.permutations(range(nu))) / math.factorial(nu)
        Ts.Umat[nu] = Us.reshape(U.shape[0], -1).T
    assert np.abs(osc.forward(Ts, A, z, W) - B).max() < 1e-12
    dAs, dWs = osc.backward(Ts, A, z, W, dB)
    assert np.abs(dAs - dA).max() < 1e-12 and np.abs(dWs - dW).max() < 1e-12
    # paths that couple two EQUAL l's to an odd L2 first are antisymmetric: their
    # polynomial is identically zero, hence dW = 0
    n_vanish = 0
    for p, (nu, oi, l1, l2, l3, L2) in enumerate(T.paths):
        if nu == 3 and l1 == l2 and L2 % 2 == 1:
            assert np.abs(dW[:, p]).max() < 1e-12
            n_vanish += 1
        elif nu == 3 and (l1, l2, l3) == (1, 1, 1) and oi == 1:
            assert np.abs(dW[:, p]).max() > 1e-3
    assert n_vanish >= 5


# ---------------------------------------------------------------- derivatives

@pytest.mark.parametrize("l_max,nu_max,outs", [(1, 2, ((0, 1),)), (3, 3, O01), (2, 3, O012)])
def test_backward_matches_finite_differences(l_max, nu_max, outs):
    cfg = osc.OracleConfig(2, l_max, nu_max, 3, outs)
    T = osc.build_tables(cfg)
    A, z, W, dB = rand_inputs(cfg, 5, 17)
    dA, dW = osc.backward(T, A, z, W, dB)

    def loss(A_, W_):
        return (osc.forward(T, A_, z, W_) * dB).sum()
    rng = np.random.default_rng(3)
    h = 1e-5
    for _ in range(12):
        i, k, a = rng.integers(5), rng.integers(2), rng.integers(cfg.n_lm)
        Ap, Am = A.copy(), A.copy()
        Ap[i, k, a] += h
        Am[i, k, a] -= h
        fd = (loss(Ap, W) - loss(Am, W)) / (2 * h)
        assert abs(fd - dA[i, k, a]) < 1e-7 * max(1.0, abs(fd))
    for _ in range(12):
        e, p, k = rng.integers(3), rng.integers(W.shape[1]), rng.integers(2)
        Wp, Wm = W.copy(), W.copy()
        Wp[e, p, k] += h
        Wm[e, p, k] -= h
        fd = (loss(A, Wp) - loss(A, Wm)) / (2 * h)
        assert abs(fd - dW[e, p, k]) < 1e-7 * max(1.0, abs(fd))


def test_polynomial_identities():
    cfg = osc.OracleConfig(2, 3, 3, 3, O01)
    T = osc.build_tables(cfg)
    A, z, W, dB = rand_inputs(cfg, 6, 19)
    # absent element: dW row is exactly zero; dW does not depend on W (B linear in W)
    z[z == 2] = 0
    dA, dW = osc.backward(T, A, z, W, dB)
    assert not dW[2].any()
    _, dW2 = osc.backward(T, A, z, 3.0 * W + 1.0, dB)
    assert np.abs(dW2 - dW).max() < 1e-12
    # Euler: per correlation order nu, sum_a A_a dB_nu/dA_a = nu * B_nu
    for nu in (1, 2, 3):
        Wnu = np.zeros_like(W)
        sel = [p for p, path in enumerate(T.paths) if path[0] == nu]
        Wnu[:, sel] = W[:, sel]
        Bnu = osc.forward(T, A, z, Wnu)
        dAnu, _ = osc.backward(T, A, z, Wnu, dB)
        lhs = (A * dAnu).sum(-1)
        rhs = nu * (Bnu * dB).sum(-1)
        assert np.abs(lhs - rhs).max() < 1e-11
        # homogeneity of degree nu
        assert np.abs(osc.forward(T, 1.7 * A, z, Wnu) - 1.7 ** nu * Bnu).max() < 1e-11
    # chunking does not change the result
    assert np.abs(osc.forward(T, A, z, W, chunk=4) - osc.forward(T, A, z, W, chunk=64)).max() < 1e-13
