"""fp64 oracle of the MACE channelwise tensor product (construction of the messages).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Follows Algorithm 1 of the paper (the message construction of MACE, Section 4.1): for
every edge ji (sender j, receiver i), channel k and output component (l3, m3)

    msg[ji,k,(l3,m3)] = sum over (l1,m1), (l2,m2) of
        C(l1,l2,l3)[m1,m2,m3] * R[ji, p(l1,l2,l3), k] * Y[ji,(l1,m1)] * h[j,k,(l2,m2)]

followed by the pooling over the neighbours of the receiving atom that Section 4.1
describes before Algorithm 2 (the messages are summed over j on the receiving vertex):

    A[i,k,(l3,m3)] = sum over the edges ji with receiver i of msg[ji,k,(l3,m3)].

Readings of what the paper leaves open:
* Y carries l1 = 0..l_Y, h carries l2 = 0..l_h, the output l3 = 0..L_max, all in the real
  basis with component index l*l + l + m and parity (-1)^l (spherical harmonics and the
  irreps MACE keeps have this "natural" parity);
* C(l1,l2,l3) is the unit-norm invariant tensor of oracle.coupling (the same reading as for
  Algorithm 2); a triple (l1,l2,l3) is a path iff the triangle rule holds and l1+l2+l3 is
  even (parity is conserved; odd sums would produce pseudo-tensors, which are not among the
  natural-parity outputs);
* the radial weights R are per (edge, path, channel); paths are ordered by (l1,l2,l3)
  ascending, as in the index order of R in Algorithm 1;
* contributions of different paths to the same (l3,m3) are summed, as the accumulation
  line of Algorithm 1 states.
The backward functions are the analytic derivatives of these expressions.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

from .coupling import coupling_tensor


@dataclass(frozen=True)
class TPConfig:
    num_channels: int
    l_Y: int       # spherical harmonics carry l1 = 0..l_Y
    l_h: int       # sender features carry l2 = 0..l_h
    L_max: int     # messages carry l3 = 0..L_max

    @property
    def n_Y(self) -> int:
        return (self.l_Y + 1) ** 2

    @property
    def n_h(self) -> int:
        return (self.l_h + 1) ** 2

    @property
    def n_out(self) -> int:
        return (self.L_max + 1) ** 2


def irrep_slice(l: int) -> slice:
    return slice(l * l, (l + 1) * (l + 1))


def enumerate_paths(cfg: TPConfig) -> List[Tuple[int, int, int]]:
    """(l1, l2, l3) allowed by the triangle rule (Section 4.2) and parity, ascending."""
    paths = []
    for l1 in range(cfg.l_Y + 1):
        for l2 in range(cfg.l_h + 1):
            for l3 in range(cfg.L_max + 1):
                if abs(l1 - l2) <= l3 <= l1 + l2 and (l1 + l2 + l3) % 2 == 0:
                    paths.append((l1, l2, l3))
    return paths


def edge_messages(cfg: TPConfig, Y: np.ndarray, h: np.ndarray, R: np.ndarray, sender: np.ndarray) -> np.ndarray:
    """msg[E, K, n_out] of Algorithm 1.  Y: (E, n_Y), h: (N, K, n_h), R: (E, P, K), sender: (E,)."""
    Y = np.asarray(Y, dtype=np.float64)
    h = np.asarray(h, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    E = Y.shape[0]
    msg = np.zeros((E, cfg.num_channels, cfg.n_out))
    hj = h[sender]                                        # (E, K, n_h): features of the sending atom
    for p, (l1, l2, l3) in enumerate(enumerate_paths(cfg)):
        C = coupling_tensor(l1, l2, l3)
        msg[:, :, irrep_slice(l3)] += np.einsum("abc,ek,ea,ekb->ekc", C, R[:, p, :], Y[:, irrep_slice(l1)],
                                                hj[:, :, irrep_slice(l2)], optimize=True)
    return msg


def forward(cfg: TPConfig, Y, h, R, sender, receiver, num_nodes: int) -> np.ndarray:
    """A[N, K, n_out]: the messages of Algorithm 1 summed over the edges of each receiver."""
    msg = edge_messages(cfg, Y, h, R, sender)
    A = np.zeros((num_nodes, cfg.num_channels, cfg.n_out))
    np.add.at(A, np.asarray(receiver), msg)
    return A


def backward(cfg: TPConfig, Y, h, R, sender, receiver, dA):
    """Gradients of sum(dA * A) with respect to Y (E, n_Y), h (N, K, n_h) and R (E, P, K)."""
    Y = np.asarray(Y, dtype=np.float64)
    h = np.asarray(h, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    dA = np.asarray(dA, dtype=np.float64)
    sender = np.asarray(sender)
    g = dA[np.asarray(receiver)]                          # (E, K, n_out): gradient of every edge's message
    hj = h[sender]
    dY = np.zeros_like(Y)
    dR = np.zeros_like(R)
    dhj = np.zeros_like(hj)
    for p, (l1, l2, l3) in enumerate(enumerate_paths(cfg)):
        C = coupling_tensor(l1, l2, l3)
        y, x, gg, r = Y[:, irrep_slice(l1)], hj[:, :, irrep_slice(l2)], g[:, :, irrep_slice(l3)], R[:, p, :]
        dR[:, p, :] = np.einsum("abc,ea,ekb,ekc->ek", C, y, x, gg, optimize=True)
        dY[:, irrep_slice(l1)] += np.einsum("abc,ek,ekb,ekc->ea", C, r, x, gg, optimize=True)
        dhj[:, :, irrep_slice(l2)] += np.einsum("abc,ek,ea,ekc->ekb", C, r, y, gg, optimize=True)
    dh = np.zeros_like(h)
    np.add.at(dh, sender, dhj)
    return dY, dh, dR


def double_backward(cfg: TPConfig, Y, h, R, sender, receiver, dA, HY, Hh, HR):
    """Second-order pass needed when a loss depends on the gradients (forces are derivatives of
    the energy, Section 2.2, and reach the loss through dY).

    With (dY, dh, dR) = backward(..., dA) and psi = sum(HY*dY) + sum(Hh*dh) + sum(HR*dR) returns
        ddA = dpsi/d(dA)  (N, K, n_out)      d2Y = dpsi/dY  (E, n_Y)
        d2h = dpsi/dh     (N, K, n_h)        d2R = dpsi/dR  (E, P, K)
    written out from the definition: every message is linear in each of Y, h and R, so psi is
    the sum over edges of dA[receiver] contracted with the message in which, in turn, Y, h or R
    is replaced by its cotangent, and the gradients differentiate those three terms.
    """
    Y, h, R, dA, HY, Hh, HR = (np.asarray(x, dtype=np.float64) for x in (Y, h, R, dA, HY, Hh, HR))
    sender, receiver = np.asarray(sender), np.asarray(receiver)
    g = dA[receiver]                                     # (E, K, n_out)
    x, hx = h[sender], Hh[sender]                        # (E, K, n_h)
    E = Y.shape[0]
    tdot = np.zeros((E, cfg.num_channels, cfg.n_out))    # derivative of every message along (HY, Hh, HR)
    d2Y = np.zeros_like(Y)
    d2R = np.zeros_like(R)
    d2x = np.zeros_like(x)
    for p, (l1, l2, l3) in enumerate(enumerate_paths(cfg)):
        C = coupling_tensor(l1, l2, l3)
        s1, s2, s3 = irrep_slice(l1), irrep_slice(l2), irrep_slice(l3)
        y, hy, xx, hxx, r, hr, gg = Y[:, s1], HY[:, s1], x[:, :, s2], hx[:, :, s2], R[:, p, :], HR[:, p, :], g[:, :, s3]
        tdot[:, :, s3] += (np.einsum("abc,ek,ea,ekb->ekc", C, r, hy, xx, optimize=True)
                           + np.einsum("abc,ek,ea,ekb->ekc", C, r, y, hxx, optimize=True)
                           + np.einsum("abc,ek,ea,ekb->ekc", C, hr, y, xx, optimize=True))
        # psi_e = sum_c g[c] * tdot[c]; its derivatives with respect to y, x and r
        d2Y[:, s1] += (np.einsum("abc,ek,ekb,ekc->ea", C, r, hxx, gg, optimize=True)
                       + np.einsum("abc,ek,ekb,ekc->ea", C, hr, xx, gg, optimize=True))
        d2x[:, :, s2] += (np.einsum("abc,ek,ea,ekc->ekb", C, r, hy, gg, optimize=True)
                          + np.einsum("abc,ek,ea,ekc->ekb", C, hr, y, gg, optimize=True))
        d2R[:, p, :] = (np.einsum("abc,ea,ekb,ekc->ek", C, hy, xx, gg, optimize=True)
                        + np.einsum("abc,ea,ekb,ekc->ek", C, y, hxx, gg, optimize=True))
    ddA = np.zeros_like(dA)
    np.add.at(ddA, receiver, tdot)
    d2h = np.zeros_like(h)
    np.add.at(d2h, sender, d2x)
    return ddA, d2Y, d2h, d2R
