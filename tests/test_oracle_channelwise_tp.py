"""Pins for oracle/channelwise_tp.py (Algorithm 1 and the pooling over neighbours) against
things it does not compute itself: closed forms, textbook spherical harmonics, a literal
loop nest, finite differences and symmetry properties."""
import numpy as np
import pytest

from oracle import channelwise_tp as otp
from oracle import coupling as oc
from test_oracle_coupling import real_sh_textbook


def random_case(cfg, N, E, seed):
    rng = np.random.default_rng(seed)
    P = len(otp.enumerate_paths(cfg))
    Y = rng.standard_normal((E, cfg.n_Y))
    h = rng.standard_normal((N, cfg.num_channels, cfg.n_h))
    R = rng.standard_normal((E, P, cfg.num_channels))
    sender = rng.integers(0, N, E)
    receiver = np.sort(rng.integers(0, N, E))
    return Y, h, R, sender, receiver


def test_paths_of_the_mace_configurations():
    # scalar sender features (first layer): one path per l1; with vectors (second layer): ten
    assert otp.enumerate_paths(otp.TPConfig(4, 3, 0, 3)) == [(0, 0, 0), (1, 0, 1), (2, 0, 2), (3, 0, 3)]
    assert otp.enumerate_paths(otp.TPConfig(4, 3, 1, 3)) == [
        (0, 0, 0), (0, 1, 1), (1, 0, 1), (1, 1, 0), (1, 1, 2), (2, 0, 2), (2, 1, 1), (2, 1, 3), (3, 0, 3), (3, 1, 2)]
    # parity: the cross product (1,1,1) is not a path; the triangle rule caps l3
    assert (1, 1, 1) not in otp.enumerate_paths(otp.TPConfig(4, 3, 3, 3))
    assert all(abs(a - b) <= c <= a + b for a, b, c in otp.enumerate_paths(otp.TPConfig(4, 3, 3, 3)))


def test_scalar_sender_features_closed_form():
    # l2 = 0: C(l,0,l) = delta / sqrt(2l+1), so msg[l block] = R_l * h * Y[l block] / sqrt(2l+1)
    cfg = otp.TPConfig(5, 3, 0, 3)
    Y, h, R, sender, receiver = random_case(cfg, 7, 23, 1)
    msg = otp.edge_messages(cfg, Y, h, R, sender)
    for l in range(4):
        want = R[:, l, :, None] * h[sender][:, :, 0:1] * Y[:, None, l * l:(l + 1) ** 2] / np.sqrt(2 * l + 1)
        assert np.allclose(msg[:, :, l * l:(l + 1) ** 2], want, rtol=0, atol=1e-13)


def test_scalar_output_closed_form():
    # L_max = 0 with vectors on both sides: msg = R0*Y0*h0 + R1 * (Y1 . h1) / sqrt(3)
    cfg = otp.TPConfig(3, 1, 1, 0)
    assert otp.enumerate_paths(cfg) == [(0, 0, 0), (1, 1, 0)]
    Y, h, R, sender, receiver = random_case(cfg, 5, 17, 2)
    hj = h[sender]
    want = R[:, 0] * Y[:, 0:1] * hj[:, :, 0] + R[:, 1] * np.einsum("ea,eka->ek", Y[:, 1:4], hj[:, :, 1:4]) / np.sqrt(3)
    assert np.allclose(otp.edge_messages(cfg, Y, h, R, sender)[:, :, 0], want, rtol=0, atol=1e-13)


def test_vector_times_vector_to_l2_is_the_traceless_symmetric_product():
    # path (1,1,2) alone: in Cartesian terms the symmetric traceless part of y (x) v, whose squared
    # norm is |y|^2 |v|^2 minus the trace part (y.v)^2 / 3 minus the antisymmetric part
    # |y x v|^2 / 2, i.e. |y|^2 |v|^2 / 2 + (y.v)^2 / 6; the unit-norm coupling tensor is the
    # isometric projection divided by sqrt(2*2+1)
    cfg = otp.TPConfig(1, 1, 1, 2)
    paths = otp.enumerate_paths(cfg)
    rng = np.random.default_rng(3)
    Y = np.zeros((9, 4)); Y[:, 1:] = rng.standard_normal((9, 3))
    h = np.zeros((9, 1, 4)); h[:, 0, 1:] = rng.standard_normal((9, 3))
    R = np.zeros((9, len(paths), 1)); R[:, paths.index((1, 1, 2)), 0] = 1.0
    msg = otp.edge_messages(cfg, Y, h, R, np.arange(9))[:, 0, 4:9]
    y, v = Y[:, 1:], h[:, 0, 1:]
    yy, vv, yv = (y * y).sum(1), (v * v).sum(1), (y * v).sum(1)
    assert np.allclose((msg ** 2).sum(1), (0.5 * yy * vv + yv * yv / 6.0) / 5.0, rtol=1e-12)


@pytest.mark.parametrize("l1,l2,l3", [(1, 1, 0), (1, 1, 2), (2, 1, 1), (2, 1, 3), (3, 1, 2), (2, 2, 2), (3, 2, 1)])
def test_product_of_spherical_harmonics_of_one_direction(l1, l2, l3):
    # Y_l1(r) (x) Y_l2(r) coupled to l3 is proportional to Y_l3(r), with one factor for all r
    cfg = otp.TPConfig(1, 3, 2, 3)
    paths = otp.enumerate_paths(cfg)
    rng = np.random.default_rng(4)
    ratios = []
    for _ in range(6):
        r = rng.standard_normal(3)
        r /= np.linalg.norm(r)
        Y = np.concatenate([real_sh_textbook(l, r) for l in range(4)])[None]
        h = np.concatenate([real_sh_textbook(l, r) for l in range(3)])[None, None]
        R = np.zeros((1, len(paths), 1)); R[0, paths.index((l1, l2, l3)), 0] = 1.0
        msg = otp.edge_messages(cfg, Y, h, R, np.zeros(1, dtype=int))[0, 0]
        want = real_sh_textbook(l3, r)
        got = msg[l3 * l3:(l3 + 1) ** 2]
        ratio = got @ want / (want @ want)
        assert np.allclose(got, ratio * want, atol=1e-13)
        other = np.delete(msg, np.s_[l3 * l3:(l3 + 1) ** 2])
        assert not other.any()
        ratios.append(ratio)
    assert np.allclose(ratios, ratios[0], rtol=1e-12) and abs(ratios[0]) > 1e-3
    if (l1, l2, l3) == (1, 1, 0):
        # (1/sqrt3) |Y_1|^2 / Y_0 with |Y_1|^2 = 3/(4 pi), Y_0 = 1/(2 sqrt pi)
        assert np.isclose(ratios[0], np.sqrt(3.0) / (2.0 * np.sqrt(np.pi)), rtol=1e-12)


def test_against_the_literal_loop_nest_of_algorithm_1():
    cfg = otp.TPConfig(2, 2, 1, 2)
    N, E = 4, 9
    Y, h, R, sender, receiver = random_case(cfg, N, E, 5)
    paths = otp.enumerate_paths(cfg)
    A = np.zeros((N, cfg.num_channels, cfg.n_out))
    for e in range(E):
        for k in range(cfg.num_channels):
            for l3 in range(cfg.L_max + 1):
                for m3 in range(2 * l3 + 1):
                    acc = 0.0
                    for p, (l1, l2, L) in enumerate(paths):
                        if L != l3:
                            continue
                        C = oc.coupling_tensor(l1, l2, l3)
                        for m1 in range(2 * l1 + 1):
                            for m2 in range(2 * l2 + 1):
                                acc += (C[m1, m2, m3] * R[e, p, k] * Y[e, l1 * l1 + m1]
                                        * h[sender[e], k, l2 * l2 + m2])
                    A[receiver[e], k, l3 * l3 + m3] += acc
    assert np.allclose(otp.forward(cfg, Y, h, R, sender, receiver, N), A, rtol=0, atol=1e-13)


def test_pooling_sums_the_edges_of_each_receiver_and_ignores_edge_order():
    cfg = otp.TPConfig(3, 3, 1, 3)
    N, E = 6, 40
    Y, h, R, sender, receiver = random_case(cfg, N, E, 6)
    receiver[receiver == 2] = 3                      # node 2 receives nothing
    A = otp.forward(cfg, Y, h, R, sender, receiver, N)
    msg = otp.edge_messages(cfg, Y, h, R, sender)
    for i in range(N):
        assert np.allclose(A[i], msg[receiver == i].sum(0), atol=1e-13)
    assert not A[2].any()
    perm = np.random.default_rng(7).permutation(E)
    A2 = otp.forward(cfg, Y[perm], h, R[perm], sender[perm], receiver[perm], N)
    assert np.allclose(A, A2, atol=1e-12)


def test_rotation_equivariance():
    cfg = otp.TPConfig(3, 3, 1, 3)
    N, E = 5, 21
    Y, h, R, sender, receiver = random_case(cfg, N, E, 8)
    theta = np.array([0.3, -1.1, 0.7])
    D = [oc.wigner_D_real(l, theta) for l in range(4)]

    def rot(x, lmax):
        out = np.empty_like(x)
        for l in range(lmax + 1):
            out[..., l * l:(l + 1) ** 2] = x[..., l * l:(l + 1) ** 2] @ D[l].T
        return out
    A = otp.forward(cfg, Y, h, R, sender, receiver, N)
    A_rot = otp.forward(cfg, rot(Y, 3), rot(h, 1), R, sender, receiver, N)
    assert np.allclose(A_rot, rot(A, 3), atol=1e-12)
    # inversion: natural parity on both inputs gives natural parity on the output
    sgnY = np.concatenate([np.full(2 * l + 1, (-1.0) ** l) for l in range(4)])
    A_inv = otp.forward(cfg, Y * sgnY, h * sgnY[:4], R, sender, receiver, N)
    assert np.allclose(A_inv, A * sgnY, atol=1e-12)


def test_backward_against_finite_differences_and_euler():
    cfg = otp.TPConfig(3, 3, 1, 3)
    N, E = 5, 14
    Y, h, R, sender, receiver = random_case(cfg, N, E, 9)
    rng = np.random.default_rng(10)
    dA = rng.standard_normal((N, cfg.num_channels, cfg.n_out))
    dY, dh, dR = otp.backward(cfg, Y, h, R, sender, receiver, dA)

    def phi(Y_, h_, R_):
        return float((dA * otp.forward(cfg, Y_, h_, R_, sender, receiver, N)).sum())
    eps = 1e-6
    for name, x, g in (("Y", Y, dY), ("h", h, dh), ("R", R, dR)):
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in x.shape)
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = {"Y": Y, "h": h, "R": R}
            args_m = dict(args_p)
            args_p[name], args_m[name] = xp, xm
            fd = (phi(args_p["Y"], args_p["h"], args_p["R"]) - phi(args_m["Y"], args_m["h"], args_m["R"])) / (2 * eps)
            assert abs(fd - g[idx]) <= 1e-7 * max(1.0, abs(fd)), (name, idx, fd, g[idx])
    # the operation is linear in each of Y, h and R
    p0 = phi(Y, h, R)
    for x, g in ((Y, dY), (h, dh), (R, dR)):
        assert np.isclose((x * g).sum(), p0, rtol=1e-12)
    # senders without outgoing edges and edges-less receivers
    unused = np.setdiff1d(np.arange(N), sender)
    assert not dh[unused].any()


def test_double_backward_against_finite_differences_of_the_backward():
    cfg = otp.TPConfig(3, 3, 1, 3)
    N, E = 5, 13
    Y, h, R, sender, receiver = random_case(cfg, N, E, 11)
    rng = np.random.default_rng(12)
    dA = rng.standard_normal((N, cfg.num_channels, cfg.n_out))
    HY, Hh, HR = rng.standard_normal(Y.shape), rng.standard_normal(h.shape), rng.standard_normal(R.shape)
    ddA, d2Y, d2h, d2R = otp.double_backward(cfg, Y, h, R, sender, receiver, dA, HY, Hh, HR)

    def psi(Y_, h_, R_, dA_):
        dY, dh, dR = otp.backward(cfg, Y_, h_, R_, sender, receiver, dA_)
        return float((HY * dY).sum() + (Hh * dh).sum() + (HR * dR).sum())
    eps = 1e-6
    base = {"Y": Y, "h": h, "R": R, "dA": dA}
    for name, grad in (("Y", d2Y), ("h", d2h), ("R", d2R), ("dA", ddA)):
        for _ in range(10):
            idx = tuple(rng.integers(0, s) for s in base[name].shape)
            ap, am = dict(base), dict(base)
            ap[name], am[name] = base[name].copy(), base[name].copy()
            ap[name][idx] += eps
            am[name][idx] -= eps
            fd = (psi(ap["Y"], ap["h"], ap["R"], ap["dA"]) - psi(am["Y"], am["h"], am["R"], am["dA"])) / (2 * eps)
            assert abs(fd - grad[idx]) <= 2e-7 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])


def test_double_backward_identities():
    cfg = otp.TPConfig(2, 3, 1, 3)
    N, E = 6, 17
    Y, h, R, sender, receiver = random_case(cfg, N, E, 13)
    rng = np.random.default_rng(14)
    dA = rng.standard_normal((N, cfg.num_channels, cfg.n_out))
    HY, Hh, HR = rng.standard_normal(Y.shape), rng.standard_normal(h.shape), rng.standard_normal(R.shape)
    ddA, d2Y, d2h, d2R = otp.double_backward(cfg, Y, h, R, sender, receiver, dA, HY, Hh, HR)
    dY, dh, dR = otp.backward(cfg, Y, h, R, sender, receiver, dA)
    psi = (HY * dY).sum() + (Hh * dh).sum() + (HR * dR).sum()
    # psi is linear in dA, and of degree two in (Y, h, R) jointly with the cotangents taking one
    # slot: Euler gives sum(Y*d2Y) + sum(h*d2h) + sum(R*d2R) = 2 * psi
    assert np.isclose((dA * ddA).sum(), psi, rtol=1e-12)
    assert np.isclose((Y * d2Y).sum() + (h * d2h).sum() + (R * d2R).sum(), 2 * psi, rtol=1e-12)
    # choosing the cotangents equal to the inputs makes ddA three times the forward result
    A = otp.forward(cfg, Y, h, R, sender, receiver, N)
    ddA_same = otp.double_backward(cfg, Y, h, R, sender, receiver, dA, Y, h, R)[0]
    assert np.allclose(ddA_same, 3.0 * A, atol=1e-12)
    # a cotangent on one argument only leaves that argument's second derivative at zero
    only_Y = otp.double_backward(cfg, Y, h, R, sender, receiver, dA, HY, 0 * Hh, 0 * HR)
    assert not only_Y[1].any() and only_Y[2].any() and only_Y[3].any()
    # rotating Y, h and their cotangents rotates ddA and d2Y, d2h; d2R is invariant
    theta = np.array([-0.4, 0.9, 1.3])
    D = [oc.wigner_D_real(l, theta) for l in range(4)]

    def rot(x, lmax):
        out = np.empty_like(x)
        for l in range(lmax + 1):
            out[..., l * l:(l + 1) ** 2] = x[..., l * l:(l + 1) ** 2] @ D[l].T
        return out
    r = otp.double_backward(cfg, rot(Y, 3), rot(h, 1), R, sender, receiver, rot(dA, 3), rot(HY, 3), rot(Hh, 1), HR)
    assert np.allclose(r[0], rot(ddA, 3), atol=1e-12) and np.allclose(r[1], rot(d2Y, 3), atol=1e-12)
    assert np.allclose(r[2], rot(d2h, 1), atol=1e-12) and np.allclose(r[3], d2R, atol=1e-12)
