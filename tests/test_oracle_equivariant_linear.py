"""Pins for oracle/equivariant_linear.py: a literal loop nest, closed forms, equivariance and
finite differences."""
import numpy as np

from oracle import coupling as oc
from oracle import equivariant_linear as oel


def case(seed, N=5, Kin=6, Kout=4, l_max=3):
    rng = np.random.default_rng(seed)
    n = (l_max + 1) ** 2
    return (rng.standard_normal((N, Kin, n)), rng.standard_normal((l_max + 1, Kin, Kout)),
            rng.standard_normal((N, Kout, n)))


def test_against_the_literal_loop_nest():
    X, W, _ = case(1, l_max=2)
    Y = np.zeros((X.shape[0], W.shape[2], X.shape[2]))
    for i in range(X.shape[0]):
        for kp in range(W.shape[2]):
            for l in range(3):
                for m in range(2 * l + 1):
                    for k in range(W.shape[1]):
                        Y[i, kp, l * l + m] += W[l, k, kp] * X[i, k, l * l + m]
    assert np.allclose(oel.forward(X, W), Y, rtol=0, atol=1e-13)


def test_closed_forms():
    X, W, _ = case(2, Kin=5, Kout=5)
    W[:] = np.eye(5)[None]
    assert np.array_equal(oel.forward(X, W), X)                 # identity matrices copy
    W[2] *= 0                                                   # zero matrix for l = 2 removes components 4..8
    Y = oel.forward(X, W)
    assert not Y[:, :, 4:9].any() and np.array_equal(Y[:, :, :4], X[:, :, :4])
    P = np.eye(5)[[1, 0, 2, 3, 4]]                              # a permutation of the channels
    Wp = np.stack([P] * 4)
    assert np.array_equal(oel.forward(X, Wp), X[:, [1, 0, 2, 3, 4], :])


def test_rotation_equivariance_and_channel_linearity():
    X, W, _ = case(3)
    theta = np.array([0.5, -0.2, 1.1])
    D = [oc.wigner_D_real(l, theta) for l in range(4)]

    def rot(x):
        out = np.empty_like(x)
        for l in range(4):
            out[..., l * l:(l + 1) ** 2] = x[..., l * l:(l + 1) ** 2] @ D[l].T
        return out
    assert np.allclose(oel.forward(rot(X), W), rot(oel.forward(X, W)), atol=1e-12)
    X2 = case(4)[0]
    assert np.allclose(oel.forward(2 * X - 3 * X2, W), 2 * oel.forward(X, W) - 3 * oel.forward(X2, W), atol=1e-12)


def test_backward_against_finite_differences_and_euler():
    X, W, dY = case(5)
    dX, dW = oel.backward(X, W, dY)
    rng = np.random.default_rng(6)
    phi = lambda X_, W_: float((dY * oel.forward(X_, W_)).sum())
    eps = 1e-6
    for name, x, g in (("X", X, dX), ("W", W, dW)):
        for _ in range(10):
            idx = tuple(rng.integers(0, s) for s in x.shape)
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            fd = (phi(xp, W) - phi(xm, W)) / (2 * eps) if name == "X" else (phi(X, xp) - phi(X, xm)) / (2 * eps)
            assert abs(fd - g[idx]) <= 1e-7 * max(1.0, abs(fd))
    assert np.isclose((X * dX).sum(), phi(X, W)) and np.isclose((W * dW).sum(), phi(X, W))
