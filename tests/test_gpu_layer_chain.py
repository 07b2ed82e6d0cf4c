"""The two kernels chained as in a MACE interaction + product block, through the C ABI:

    A = tensor product + pooling (Algorithm 1)      B = symmetric contraction (Algorithm 2)
    energy  E = sum(c * B)                          forces-like gradient  dY = dE/dY

Checks, against the same chain in the fp64 oracles, the first-order gradients of E and the
gradient with respect to the contraction weights W of a force-type loss L = sum(HY * dY), which
needs the second-order passes of both kernels (tp_double_backward gives dL/d(dA), which is
the cotangent H of sc_double_backward).  The layouts fit without any copy:
A[node][channel][16] is the output of the one and the input of the other.
"""
import sys

import numpy as np
import pytest

from oracle import channelwise_tp as otp
from oracle import symmetric_contraction as osc
from paper_2504_10700_amd import workloads
from gpu_util import check

pytestmark = pytest.mark.gpu

O01 = ((0, 1), (1, -1))


def test_interaction_and_product_chain_first_and_second_order():
    import torch
    from paper_2504_10700_amd import binding as sc
    from paper_2504_10700_amd import tp_binding as tp
    dev = torch.device("cuda:0")
    N, K, Z = 160, 128, 5
    twl = workloads.TPWorkload("chain_tp", N, 8, K, 3, 1, 3, "f64", 7101)
    swl = workloads.Workload("chain_sc", N, Z, K, 3, 3, O01, "f64", 7102, z_mode="uniform")
    tcfg = otp.TPConfig(K, 3, 1, 3)
    tin = workloads.make_tp_inputs(twl, otp.enumerate_paths(tcfg))
    scfg = osc.OracleConfig(K, 3, 3, Z, O01)
    T = osc.build_tables(scfg)
    sin = workloads.make_inputs(swl, T.paths)
    E = int(tin.Y.shape[0])
    print(f"chain: N={N} E={E} K={K}", flush=True)
    sys.stdout.flush()
    f64 = torch.float64
    f = lambda x: torch.tensor(x, dtype=f64, device=dev)
    i32 = lambda x: torch.tensor(x, dtype=torch.int32, device=dev)
    Y, h, R = f(tin.Y), f(tin.h), f(tin.R)
    snd, rowp, sndp, snde = i32(tin.sender), i32(tin.row_ptr), i32(tin.send_ptr), i32(tin.send_edge)
    z, W, c = i32(sin.z), f(sin.W), f(sin.dB)            # c: the readout weights, E = sum(c * B)
    HY = f(np.random.default_rng(7103).standard_normal(tin.Y.shape))

    tplan = tp.tp_plan_create(K, 3, 1, 3, tp.SC_F64, 0)
    splan = sc.sc_plan_create(K, 3, 3, Z, O01, sc.SC_F64, 0)
    tws_b = tp.tp_workspace_bytes(tplan, E)
    tws = torch.empty(tws_b, dtype=torch.uint8, device=dev)
    sws_b = sc.sc_workspace_bytes(splan, N)
    sws = torch.empty(sws_b, dtype=torch.uint8, device=dev)

    # forward chain
    A = torch.empty((N, K, 16), dtype=f64, device=dev)
    B = torch.empty((N, K, 4), dtype=f64, device=dev)
    tp.tp_forward(tplan, N, N, E, Y, h, R, snd, rowp, A)
    sc.sc_forward(splan, N, A, z, W, B, sws, sws_b)
    # backward chain of E = sum(c * B)
    dA, dW = torch.empty_like(A), torch.empty_like(W)
    sc.sc_backward(splan, N, A, z, W, c, dA, dW, sws, sws_b, sc.SC_REUSE_GROUPING)
    dY, dh, dR = torch.empty_like(Y), torch.empty_like(h), torch.empty_like(R)
    tp.tp_backward(tplan, N, N, E, Y, h, R, snd, rowp, sndp, snde, dA, dY, dh, dR, tws, tws_b)
    # force-type loss L = sum(HY * dY): dL/d(dA) from the tensor product's second-order pass ...
    zero_h, zero_R = torch.zeros_like(h), torch.zeros_like(R)
    ddA, d2Y, d2h, d2R = torch.empty_like(A), torch.empty_like(Y), torch.empty_like(h), torch.empty_like(R)
    tp.tp_double_backward(tplan, N, N, E, Y, h, R, snd, rowp, sndp, snde, dA, HY, zero_h, zero_R, ddA, d2Y, d2h, d2R,
                          tws, tws_b)
    # ... is the cotangent of dA in the contraction's second-order pass, which yields dL/dW
    ddB, dA2, dW2 = torch.empty_like(B), torch.empty_like(A), torch.empty_like(W)
    sc.sc_double_backward(splan, N, A, z, W, c, ddA, ddB, dA2, dW2, sws, sws_b, sc.SC_REUSE_GROUPING)
    torch.cuda.synchronize()
    tp.tp_plan_destroy(tplan)
    sc.sc_plan_destroy(splan)

    # the same chain in the oracles
    A_ref = otp.forward(tcfg, tin.Y, tin.h, tin.R, tin.sender, tin.receiver, N)
    B_ref = osc.forward(T, A_ref, sin.z, sin.W)
    dA_ref, dW_ref = osc.backward(T, A_ref, sin.z, sin.W, sin.dB)
    dY_ref, dh_ref, dR_ref = otp.backward(tcfg, tin.Y, tin.h, tin.R, tin.sender, tin.receiver, dA_ref)
    HYn = HY.cpu().numpy()
    ddA_ref = otp.double_backward(tcfg, tin.Y, tin.h, tin.R, tin.sender, tin.receiver, dA_ref, HYn,
                                  np.zeros_like(tin.h), np.zeros_like(tin.R))[0]
    dW2_ref = osc.double_backward(T, A_ref, sin.z, sin.W, sin.dB, ddA_ref)[2]
    got = lambda x: x.cpu().numpy()
    has_edges = np.diff(tin.row_ptr) > 0
    check("A", got(A)[has_edges], A_ref[has_edges], "f64")
    check("B", got(B), B_ref, "f64")
    check("dW", got(dW), dW_ref, "f64")
    check("dY", got(dY), dY_ref, "f64")
    check("dh", got(dh)[np.diff(tin.send_ptr) > 0], dh_ref[np.diff(tin.send_ptr) > 0], "f64")
    check("dR", got(dR), dR_ref, "f64")
    check("dL/dW", got(dW2), dW2_ref, "f64")

    # and dL/dW against a finite difference of the oracle chain (L is linear in HY, smooth in W)
    def loss(Wp):
        dA_p, _ = osc.backward(T, A_ref, sin.z, Wp, sin.dB)
        return float((HYn * otp.backward(tcfg, tin.Y, tin.h, tin.R, tin.sender, tin.receiver, dA_p)[0]).sum())
    rng = np.random.default_rng(7104)
    present = np.unique(sin.z)
    for _ in range(3):
        idx = (int(rng.choice(present)), int(rng.integers(0, sin.W.shape[1])), int(rng.integers(0, K)))
        eps = 1e-5
        Wp, Wm = sin.W.copy(), sin.W.copy()
        Wp[idx] += eps
        Wm[idx] -= eps
        fd = (loss(Wp) - loss(Wm)) / (2 * eps)
        assert abs(fd - got(dW2)[idx]) <= 1e-6 * max(1.0, abs(fd)), (idx, fd, got(dW2)[idx])
