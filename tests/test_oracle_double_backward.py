"""Pins for the oracle's second-order pass: closed form of the tiny configuration, finite
differences of the (already pinned) first-order backward, symmetry of the Hessian, linearity
and rotation equivariance."""
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
    H = rng.standard_normal((N, cfg.num_channels, cfg.n_lm))
    return A, z, W, dB, H


def test_tiny_config_closed_form():
    cfg = osc.OracleConfig(8, 1, 2, 2, ((0, 1),))
    T = osc.build_tables(cfg)
    A, z, W, dB, H = rand_inputs(cfg, 40, 1)
    Wn = W[z]
    a0, a1, h0, h1, g = A[:, :, 0], A[:, :, 1:4], H[:, :, 0], H[:, :, 1:4], dB[:, :, 0]
    ha = (h1 * a1).sum(-1)
    s3 = np.sqrt(3.0)
    ddB = h0 * (Wn[:, 0] + 2 * Wn[:, 1] * a0) + 2 * Wn[:, 2] * ha / s3
    dA2 = np.zeros_like(A)
    dA2[:, :, 0] = 2 * g * Wn[:, 1] * h0
    dA2[:, :, 1:4] = (2 * g * Wn[:, 2] / s3)[:, :, None] * h1
    dW2 = np.zeros_like(W)
    for i in range(40):
        dW2[z[i], 0] += g[i] * h0[i]
        dW2[z[i], 1] += 2 * g[i] * h0[i] * a0[i]
        dW2[z[i], 2] += 2 * g[i] * ha[i] / s3
    got = osc.double_backward(T, A, z, W, dB, H)
    assert np.abs(got[0][:, :, 0] - ddB).max() < 1e-13
    assert np.abs(got[1] - dA2).max() < 1e-13
    assert np.abs(got[2] - dW2).max() < 1e-12


@pytest.mark.parametrize("l_max,nu_max,outs", [(1, 2, ((0, 1),)), (3, 3, O01), (2, 3, O012)])
def test_matches_finite_differences_of_the_backward(l_max, nu_max, outs):
    cfg = osc.OracleConfig(2, l_max, nu_max, 3, outs)
    T = osc.build_tables(cfg)
    A, z, W, dB, H = rand_inputs(cfg, 4, 7)
    ddB, dA2, dW2 = osc.double_backward(T, A, z, W, dB, H)

    def psi(A_, W_, dB_):
        return (osc.backward(T, A_, z, W_, dB_)[0] * H).sum()
    rng = np.random.default_rng(5)
    h = 1e-5
    for _ in range(10):
        i, k, a = rng.integers(4), rng.integers(2), rng.integers(cfg.n_lm)
        Ap, Am = A.copy(), A.copy()
        Ap[i, k, a] += h
        Am[i, k, a] -= h
        fd = (psi(Ap, W, dB) - psi(Am, W, dB)) / (2 * h)
        assert abs(fd - dA2[i, k, a]) < 1e-7 * max(1.0, abs(fd))
    for _ in range(10):
        e, p, k = rng.integers(3), rng.integers(W.shape[1]), rng.integers(2)
        Wp, Wm = W.copy(), W.copy()
        Wp[e, p, k] += h
        Wm[e, p, k] -= h
        fd = (psi(A, Wp, dB) - psi(A, Wm, dB)) / (2 * h)
        assert abs(fd - dW2[e, p, k]) < 1e-7 * max(1.0, abs(fd))
    for _ in range(10):   # psi is linear in dB: the difference quotient is exact up to rounding
        i, k, c = rng.integers(4), rng.integers(2), rng.integers(cfg.n_LM)
        Gp = dB.copy()
        Gp[i, k, c] += 1.0
        fd = psi(A, W, Gp) - psi(A, W, dB)
        assert abs(fd - ddB[i, k, c]) < 1e-10 * max(1.0, abs(fd))


def test_ddB_is_the_directional_derivative_of_the_forward():
    cfg = osc.OracleConfig(2, 3, 3, 3, O01)
    T = osc.build_tables(cfg)
    A, z, W, dB, H = rand_inputs(cfg, 5, 9)
    ddB, _, _ = osc.double_backward(T, A, z, W, dB, H)
    e = 1e-6
    fd = (osc.forward(T, A + e * H, z, W) - osc.forward(T, A - e * H, z, W)) / (2 * e)
    assert np.abs(fd - ddB).max() < 1e-7 * max(1.0, np.abs(ddB).max())


def test_hessian_symmetry_linearity_and_absent_elements():
    cfg = osc.OracleConfig(2, 3, 3, 4, O01)
    T = osc.build_tables(cfg)
    A, z, W, dB, H = rand_inputs(cfg, 6, 11)
    z[z == 3] = 1
    H2 = np.random.default_rng(3).standard_normal(H.shape)
    r1 = osc.double_backward(T, A, z, W, dB, H)
    r2 = osc.double_backward(T, A, z, W, dB, H2)
    # H2 . Hess . H == H . Hess . H2
    assert abs((H2 * r1[1]).sum() - (H * r2[1]).sum()) < 1e-9
    # linear in H and in dB
    r3 = osc.double_backward(T, A, z, W, dB, 2.0 * H - 0.5 * H2)
    for x1, x2, x3 in zip(r1, r2, r3):
        assert np.abs(x3 - (2.0 * x1 - 0.5 * x2)).max() < 1e-10
    r4 = osc.double_backward(T, A, z, W, 3.0 * dB, H)
    assert np.abs(r4[0] - r1[0]).max() < 1e-12 and np.abs(r4[1] - 3 * r1[1]).max() < 1e-10
    assert not r1[2][3].any()
    # Euler: phi is a sum of homogeneous parts; for the cubic part alone  A . Hess . H = 2 * H . grad
    Wc = np.zeros_like(W)
    sel = [p for p, path in enumerate(T.paths) if path[0] == 3]
    Wc[:, sel] = W[:, sel]
    _, dA2c, _ = osc.double_backward(T, A, z, Wc, dB, H)
    dAc, _ = osc.backward(T, A, z, Wc, dB)
    assert abs((A * dA2c).sum() - 2.0 * (H * dAc).sum()) < 1e-9


def test_rotation_equivariance():
    import scipy.linalg
    outs = O012
    cfg = osc.OracleConfig(2, 3, 3, 3, outs)
    T = osc.build_tables(cfg)
    A, z, W, dB, H = rand_inputs(cfg, 4, 13)
    th = np.array([0.3, 0.9, -0.6])
    Din = scipy.linalg.block_diag(*[oc.wigner_D_real(l, th) for l in range(4)])
    Dout = scipy.linalg.block_diag(*[oc.wigner_D_real(L, th) for L, _ in outs])
    r = osc.double_backward(T, A, z, W, dB, H)
    rr = osc.double_backward(T, A @ Din.T, z, W, dB @ Dout.T, H @ Din.T)
    assert np.abs(rr[0] - r[0] @ Dout.T).max() < 1e-11
    assert np.abs(rr[1] - r[1] @ Din.T).max() < 1e-11
    assert np.abs(rr[2] - r[2]).max() < 1e-10
