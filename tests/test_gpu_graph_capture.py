"""The compute entry points only enqueue kernels on the caller's stream (no allocation, no
synchronisation, no memset nodes), so a training step can be captured into a HIP graph and
replayed: the launch-bound regime of the paper's batches (capacity 3072 atoms per GPU, Section 5).
Every replay is compared bitwise with the eager result on the same data (the kernels are
deterministic), with eager work and synchronisations between the replays."""
import sys

import numpy as np
import pytest

from paper_2504_10700_amd import workloads

pytestmark = pytest.mark.gpu

O01 = ((0, 1), (1, -1))


def test_contraction_step_and_fused_forward_replay_bitwise():
    import torch
    from paper_2504_10700_amd import binding as sc
    from paper_2504_10700_amd import el_binding as el
    dev = torch.device("cuda:0")
    N, K, Z = 3072, 128, 89
    print(f"graph capture: N={N} K={K} Z={Z}", flush=True)
    sys.stdout.flush()
    wl = workloads.Workload("graph", N, Z, K, 3, 3, O01, "f32", 9501)
    plan = sc.sc_plan_create(K, 3, 3, Z, O01, sc.SC_F32, 0)
    try:
        inp = workloads.make_inputs(wl, sc.sc_plan_paths(plan))
        X, Wlin, _ = workloads.make_linear_inputs(N, K, K, 3, 9502)
        f = lambda x: torch.tensor(x, dtype=torch.float32, device=dev)
        A, W, dB, Xd, Wl = f(inp.A), f(inp.W), f(inp.dB), f(X), f(Wlin)
        z = torch.tensor(inp.z, dtype=torch.int32, device=dev)
        nb = sc.sc_workspace_bytes(plan, N)
        ws = torch.empty(nb, dtype=torch.uint8, device=dev)
        fb = el.el_sc_workspace_bytes(plan, K, N)
        fws = torch.empty(fb, dtype=torch.uint8, device=dev)
        outs = lambda: (torch.full((N, K, 4), float("nan"), device=dev), torch.full_like(A, float("nan")),
                        torch.full_like(W, float("nan")), torch.full((N, K, 4), float("nan"), device=dev))

        def step(B, dA, dW, B2):
            sc.sc_forward(plan, N, A, z, W, B, ws, nb)
            sc.sc_backward(plan, N, A, z, W, dB, dA, dW, ws, nb, sc.SC_REUSE_GROUPING)
            el.el_sc_forward(plan, K, N, Xd, Wl, z, W, B2, fws, fb)

        def eager():
            o = outs()
            step(*o)
            torch.cuda.synchronize()
            return [t.clone() for t in o]

        ref = eager()
        g_out = outs()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):                # warm-up on the capture stream, as torch asks
            step(*g_out)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(*g_out)
        for replay in range(3):
            if replay:                               # new data in the same buffers, eager work in between
                A.copy_(torch.roll(A, replay, 0))
                dB.mul_(1.5)
                Xd.add_(0.25)
                ref = eager()
            for t in g_out:
                t.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for name, got, want in zip(("B", "dA", "dW", "B fused"), g_out, ref):
                assert torch.equal(got, want), f"replay {replay}: {name} differs from the eager result"
    finally:
        sc.sc_plan_destroy(plan)


def test_tensor_product_step_replay_bitwise():
    import torch
    from oracle import channelwise_tp as otp          # only its path enumeration, for the input generator
    from paper_2504_10700_amd import tp_binding as tp
    dev = torch.device("cuda:0")
    twl = workloads.TPWorkload("graph_tp", 1500, 16, 128, 3, 1, 3, "f32", 9511)
    tin = workloads.make_tp_inputs(twl, otp.enumerate_paths(otp.TPConfig(128, 3, 1, 3)))
    N, E = twl.num_nodes, int(tin.Y.shape[0])
    print(f"graph capture tp: N={N} E={E}", flush=True)
    sys.stdout.flush()
    plan = tp.tp_plan_create(128, 3, 1, 3, tp.SC_F32, 0)
    try:
        f = lambda x: torch.tensor(x, dtype=torch.float32, device=dev)
        i32 = lambda x: torch.tensor(x, dtype=torch.int32, device=dev)
        Y, h, R, dA = f(tin.Y), f(tin.h), f(tin.R), f(tin.dA)
        snd, rowp, sndp, snde = i32(tin.sender), i32(tin.row_ptr), i32(tin.send_ptr), i32(tin.send_edge)
        wb = tp.tp_workspace_bytes(plan, E)
        ws = torch.empty(wb, dtype=torch.uint8, device=dev)
        outs = lambda: (torch.full((N, 128, 16), float("nan"), device=dev), torch.full_like(Y, float("nan")),
                        torch.full_like(h, float("nan")), torch.full_like(R, float("nan")))

        def step(A, dY, dh, dR):
            tp.tp_forward(plan, N, N, E, Y, h, R, snd, rowp, A)
            tp.tp_backward(plan, N, N, E, Y, h, R, snd, rowp, sndp, snde, dA, dY, dh, dR, ws, wb)

        def eager():
            o = outs()
            step(*o)
            torch.cuda.synchronize()
            return [t.clone() for t in o]

        ref = eager()
        g_out = outs()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(*g_out)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(*g_out)
        for replay in range(3):
            if replay:
                R.mul_(0.9)
                h.add_(0.1)
                ref = eager()
            for t in g_out:
                t.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for name, got, want in zip(("A", "dY", "dh", "dR"), g_out, ref):
                assert torch.equal(got, want), f"replay {replay}: {name} differs from the eager result"
    finally:
        tp.tp_plan_destroy(plan)
