"""Parity of the channelwise tensor product (tp_forward / tp_backward through the C ABI) with
the fp64 CPU oracle of Algorithm 1.  Tolerances as for the contraction: fp32
max|err|/rms(ref) <= 1e-5 per output tensor, fp64 max(|err| / max(|ref|, rms(ref))) <= 1e-12.
"""
import sys

import numpy as np
import pytest

from oracle import channelwise_tp as otp
from paper_2504_10700_amd import workloads
from gpu_util import check

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tp():
    import torch
    assert torch.cuda.is_available()
    from paper_2504_10700_amd import tp_binding
    return tp_binding


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


class TPRun:
    def __init__(self, tp, wl, inp, flags=0):
        import torch
        self.tp, self.wl, self.torch = tp, wl, torch
        dev = torch.device("cuda:0")
        self.tdt = torch.float32 if wl.dtype == "f32" else torch.float64
        self.plan = tp.tp_plan_create(wl.num_channels, wl.l_Y, wl.l_h, wl.L_max,
                                      tp.SC_F32 if wl.dtype == "f32" else tp.SC_F64, 0, flags)
        self.N, self.E = inp.h.shape[0], inp.Y.shape[0]
        f = lambda x: torch.tensor(x, dtype=self.tdt, device=dev)
        i = lambda x: torch.tensor(x, dtype=torch.int32, device=dev)
        self.Y, self.h, self.R, self.dA = f(inp.Y), f(inp.h), f(inp.R), f(inp.dA)
        self.sender, self.row_ptr = i(inp.sender), i(inp.row_ptr)
        self.send_ptr, self.send_edge = i(inp.send_ptr), i(inp.send_edge)
        self.A = torch.full((self.N, wl.num_channels, wl.n_out), float("nan"), dtype=self.tdt, device=dev)
        self.dY, self.dh, self.dR = (torch.full_like(x, float("nan")) for x in (self.Y, self.h, self.R))
        self.ws_bytes = tp.tp_workspace_bytes(self.plan, self.E)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev)

    def forward(self):
        self.tp.tp_forward(self.plan, self.N, self.N, self.E, self.Y, self.h, self.R, self.sender, self.row_ptr, self.A)
        self.torch.cuda.synchronize()
        return self.A.cpu().numpy()

    def backward(self):
        self.tp.tp_backward(self.plan, self.N, self.N, self.E, self.Y, self.h, self.R, self.sender, self.row_ptr,
                            self.send_ptr, self.send_edge, self.dA, self.dY, self.dh, self.dR, self.ws, self.ws_bytes)
        self.torch.cuda.synchronize()
        return self.dY.cpu().numpy(), self.dh.cpu().numpy(), self.dR.cpu().numpy()

    def double_backward(self, HY, Hh, HR):
        """Returns (ddA, d2Y, d2h, d2R) and the cotangents as computed (fp64 numpy)."""
        torch = self.torch
        H = [torch.tensor(x, dtype=self.tdt, device=self.A.device) for x in (HY, Hh, HR)]
        out = [torch.full_like(x, float("nan")) for x in (self.A, self.Y, self.h, self.R)]
        self.tp.tp_double_backward(self.plan, self.N, self.N, self.E, self.Y, self.h, self.R, self.sender, self.row_ptr,
                                   self.send_ptr, self.send_edge, self.dA, H[0], H[1], H[2], out[0], out[1], out[2],
                                   out[3], self.ws, self.ws_bytes)
        torch.cuda.synchronize()
        return [x.cpu().numpy() for x in out], [x.double().cpu().numpy() for x in H]

    def inputs_as_computed(self):
        return tuple(x.double().cpu().numpy() for x in (self.Y, self.h, self.R, self.dA))

    def close(self):
        self.tp.tp_plan_destroy(self.plan)


def oracle_cfg(wl):
    return otp.TPConfig(wl.num_channels, wl.l_Y, wl.l_h, wl.L_max)


def check_rows(name, got, ref, zero_rows, dtype, whole_tensor=True):
    """Rows listed in zero_rows (atoms without incoming / outgoing edges) must be exactly zero.  The
    tolerance is read literally - error scale = rms of the WHOLE reference tensor, zero rows included -
    unless whole_tensor is False (degenerate graphs where almost every row is zero)."""
    assert not got[zero_rows].any(), f"{name}: rows without edges must be exactly zero"
    if whole_tensor:
        check(name, got, ref, dtype)
    else:
        check(name, got[~zero_rows], ref[~zero_rows], dtype)


def full_parity(tp, wl, flags=0, mutate=None, whole_tensor=True):
    say(f"case {wl.name}: N={wl.num_nodes} deg~{wl.mean_degree} K={wl.num_channels} "
        f"l=({wl.l_Y},{wl.l_h},{wl.L_max}) {wl.dtype} flags={flags}")
    cfg = oracle_cfg(wl)
    paths = otp.enumerate_paths(cfg)
    inp = workloads.make_tp_inputs(wl, paths)
    if mutate:
        mutate(inp)
    run = TPRun(tp, wl, inp, flags)
    assert [tuple(r) for r in tp.tp_plan_paths(run.plan).tolist()] == paths
    Y, h, R, dA = run.inputs_as_computed()
    A = run.forward()
    no_edges = np.diff(inp.row_ptr) == 0
    check_rows("A", A, otp.forward(cfg, Y, h, R, inp.sender, inp.receiver, run.N), no_edges, wl.dtype, whole_tensor)
    dY, dh, dR = run.backward()
    dY_ref, dh_ref, dR_ref = otp.backward(cfg, Y, h, R, inp.sender, inp.receiver, dA)
    check("dY", dY, dY_ref, wl.dtype)
    silent = np.diff(inp.send_ptr) == 0
    check_rows("dh", dh, dh_ref, silent, wl.dtype, whole_tensor)
    check("dR", dR, dR_ref, wl.dtype)
    # bitwise reproducible
    A2 = run.forward()
    again = run.backward()
    assert np.array_equal(A, A2) and all(np.array_equal(x, y) for x, y in zip((dY, dh, dR), again))
    # second-order pass
    got, (HY, Hh, HR) = run.double_backward(*workloads.make_tp_cotangents(wl, inp))
    ref = otp.double_backward(cfg, Y, h, R, inp.sender, inp.receiver, dA, HY, Hh, HR)
    check_rows("ddA", got[0], ref[0], no_edges, wl.dtype, whole_tensor)
    check("d2Y", got[1], ref[1], wl.dtype)
    check_rows("d2h", got[2], ref[2], silent, wl.dtype, whole_tensor)
    check("d2R", got[3], ref[3], wl.dtype)
    got2, _ = run.double_backward(HY, Hh, HR)
    assert all(np.array_equal(x, y) for x, y in zip(got, got2))
    info = tp.tp_plan_info(run.plan)
    run.close()
    return info


def wl_of(name, N, deg, K, l_Y, l_h, L_max, dtype, seed):
    return workloads.TPWorkload(name, N, deg, K, l_Y, l_h, L_max, dtype, seed)


@pytest.mark.parametrize("flags", [0, 2])
def test_tiny_config_fp64(tp, flags):
    full_parity(tp, workloads.TP_WORKLOADS["tp_tiny"], flags)


@pytest.mark.parametrize("flags", [0, 2])
@pytest.mark.parametrize("dtype", ["f32", "f64"])
@pytest.mark.parametrize("l_h", [0, 1])
def test_mace_shapes_small_graph(tp, flags, dtype, l_h):
    full_parity(tp, wl_of("mace_small", 300, 12, 128, 3, l_h, 3, dtype, 5000 + l_h), flags)


@pytest.mark.parametrize("K", [8, 96, 192])
def test_channel_counts_that_do_not_fill_a_wave(tp, K):
    full_parity(tp, wl_of(f"k{K}", 60, 6, K, 3, 1, 3, "f32", 5100 + K))


@pytest.mark.parametrize("l_Y,l_h,L_max", [(0, 0, 0), (2, 3, 1), (3, 3, 3), (1, 2, 3)])
def test_other_configurations(tp, l_Y, l_h, L_max):
    full_parity(tp, wl_of("other", 50, 5, 64, l_Y, l_h, L_max, "f64", 5200))


def test_degenerate_graphs(tp):
    # one node without edges; a star (every edge into node 0); a high-degree tail
    full_parity(tp, wl_of("one_node", 1, 3, 128, 3, 1, 3, "f32", 5301))

    def star(inp):
        E = inp.sender.size
        inp.receiver[:] = 0
        inp.sender[:] = 1 + np.arange(E) % 29
        inp.row_ptr[:], inp.send_ptr[:], inp.send_edge[:] = workloads.graph_indices(inp.sender, inp.receiver, 30)
    # one receiver of 30 atoms: 29 of 30 rows of A are zero, so the rows with edges set the error scale
    full_parity(tp, wl_of("star", 30, 8, 128, 3, 1, 3, "f32", 5302), mutate=star, whole_tensor=False)


def test_per_edge_messages_without_pooling(tp):
    # the literal output of Algorithm 1: every edge is its own output row
    import torch
    wl = wl_of("per_edge", 40, 6, 128, 3, 1, 3, "f32", 5401)
    cfg = oracle_cfg(wl)
    inp = workloads.make_tp_inputs(wl, otp.enumerate_paths(cfg))
    run = TPRun(tp, wl, inp)
    E = run.E
    ident = torch.arange(E + 1, dtype=torch.int32, device="cuda:0")
    msg = torch.empty((E, wl.num_channels, wl.n_out), dtype=torch.float32, device="cuda:0")
    tp.tp_forward(run.plan, run.N, E, E, run.Y, run.h, run.R, run.sender, ident, msg)
    torch.cuda.synchronize()
    Y, h, R, _ = run.inputs_as_computed()
    check("msg", msg.cpu().numpy(), otp.edge_messages(cfg, Y, h, R, inp.sender), "f32")
    run.close()


def test_empty_graph_and_argument_errors(tp):
    import torch
    wl = wl_of("err", 20, 4, 128, 3, 1, 3, "f32", 5501)
    cfg = oracle_cfg(wl)
    inp = workloads.make_tp_inputs(wl, otp.enumerate_paths(cfg))
    run = TPRun(tp, wl, inp)
    # no edges: A and dh are zeroed
    zeros = torch.zeros(run.N + 1, dtype=torch.int32, device="cuda:0")
    tp.tp_forward(run.plan, run.N, run.N, 0, None, run.h, None, None, zeros, run.A)
    tp.tp_backward(run.plan, run.N, run.N, 0, None, run.h, None, None, zeros, zeros, None, run.dA, None, run.dh,
                   None, None, 0)
    torch.cuda.synchronize()
    assert not run.A.cpu().numpy().any() and not run.dh.cpu().numpy().any()
    tp.tp_forward(run.plan, 0, 0, 0, None, None, None, None, None, None)
    with pytest.raises(tp.ScError) as e:
        tp.tp_forward(run.plan, run.N, run.N, run.E, run.Y, run.h, None, run.sender, run.row_ptr, run.A)
    assert e.value.status == 1
    with pytest.raises(tp.ScError) as e:
        tp.tp_forward(run.plan, run.N, run.N, run.E, run.Y.data_ptr() + 4, run.h, run.R, run.sender, run.row_ptr, run.A)
    assert e.value.status == 1
    with pytest.raises(tp.ScError) as e:
        tp.tp_backward(run.plan, run.N, run.N, run.E, run.Y, run.h, run.R, run.sender, run.row_ptr,
                       run.send_ptr, run.send_edge, run.dA, run.dY, run.dh, run.dR, run.ws, 16)
    assert e.value.status == 3
    # the plan still works
    Y, h, R, _ = run.inputs_as_computed()
    check("A", run.forward(), otp.forward(cfg, Y, h, R, inp.sender, inp.receiver, run.N), "f32")
    run.close()


def oracle_over_receivers(cfg, inp, Y, h, R, dA, cot=None, chunk=200):
    """The oracle on consecutive chunks of receiving atoms (edges are grouped by receiver, so a chunk of
    atoms owns a contiguous range of edges), from several threads; per-atom and per-edge results are
    concatenated, the per-sender sums (dh, d2h) added over the chunks.  The oracle itself is unchanged."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    from threadpoolctl import threadpool_limits
    N = h.shape[0]

    def one(a0):
        a1 = min(N, a0 + chunk)
        e0, e1 = int(inp.row_ptr[a0]), int(inp.row_ptr[a1])
        es = slice(e0, e1)
        recv = inp.receiver[es] - a0
        A = otp.forward(cfg, Y[es], h, R[es], inp.sender[es], recv, a1 - a0)
        dY, dh, dR = otp.backward(cfg, Y[es], h, R[es], inp.sender[es], recv, dA[a0:a1])
        out = [A, dY, dh, dR]
        if cot is not None:
            HY, Hh, HR = cot
            out += list(otp.double_backward(cfg, Y[es], h, R[es], inp.sender[es], recv, dA[a0:a1], HY[es], Hh, HR[es]))
        return out

    threads = max(1, min(16, len(os.sched_getaffinity(0))))
    with threadpool_limits(limits=1):
        with ThreadPoolExecutor(threads) as ex:
            parts = list(ex.map(one, range(0, N, chunk)))
    cat = lambda k: np.concatenate([p[k] for p in parts], axis=0)
    add = lambda k: sum(p[k] for p in parts)
    res = {"A": cat(0), "dY": cat(1), "dh": add(2), "dR": cat(3)}
    if cot is not None:
        res.update({"ddA": cat(4), "d2Y": cat(5), "d2h": add(6), "d2R": cat(7)})
    return res


@pytest.mark.parametrize("name", ["tp_training_step", "tp_first_layer"])
def test_full_size_every_atom_and_edge(tp, name):
    """The workloads bench.py times, in its launch configuration, compared on every atom and edge:
    A, dY, dh, dR of forward + backward and ddA, d2Y, d2h, d2R of the second-order pass."""
    wl = workloads.TP_WORKLOADS[name]
    say(f"case {wl.name}: N={wl.num_nodes} deg~{wl.mean_degree} K={wl.num_channels}")
    cfg = oracle_cfg(wl)
    inp = workloads.make_tp_inputs(wl, otp.enumerate_paths(cfg))
    run = TPRun(tp, wl, inp)
    info = tp.tp_plan_info(run.plan)
    assert info.specialised == 1
    A = run.forward()
    dY, dh, dR = run.backward()
    Y, h, R, dA = run.inputs_as_computed()
    (ddA, d2Y, d2h, d2R), cot = run.double_backward(*workloads.make_tp_cotangents(wl, inp))
    ref = oracle_over_receivers(cfg, inp, Y, h, R, dA, cot)
    no_edges, silent = np.diff(inp.row_ptr) == 0, np.diff(inp.send_ptr) == 0
    check_rows("A", A, ref["A"], no_edges, wl.dtype)
    check("dY", dY, ref["dY"], wl.dtype)
    check_rows("dh", dh, ref["dh"], silent, wl.dtype)
    check("dR", dR, ref["dR"], wl.dtype)
    check_rows("ddA", ddA, ref["ddA"], no_edges, wl.dtype)
    check("d2Y", d2Y, ref["d2Y"], wl.dtype)
    check_rows("d2h", d2h, ref["d2h"], silent, wl.dtype)
    check("d2R", d2R, ref["d2R"], wl.dtype)
    A2 = run.forward()
    again = run.backward()
    assert np.array_equal(A, A2) and all(np.array_equal(x, y) for x, y in zip((dY, dh, dR), again)), "not reproducible"
    run.close()


def test_edge_tensors_that_pass_two_to_the_31_elements(tp):
    """Maximum sizes: 90 000 atoms, ~1.78 M edges, so R and dR hold 2.3e9 elements (9 GB each):
    element offsets pass 2^31 and byte offsets 2^33 in the kernels.  The graph comes from the
    workload generator, the tensors are drawn on the device (seeded).  The oracle sees three
    ranges of receiving atoms - the first, the ones whose edges straddle element offset 2^31 of R,
    the last - for A, dY and dR, and three sets of sending atoms with every edge they send for dh."""
    import torch
    wl = wl_of("tp_two_to_the_31", 90_000, 20, 128, 3, 1, 3, "f32", 5401)
    cfg = oracle_cfg(wl)
    paths = otp.enumerate_paths(cfg)
    sender, receiver = workloads.make_tp_graph(wl, np.random.default_rng(wl.seed))
    N, E, P = wl.num_nodes, int(receiver.size), len(paths)
    row_ptr, send_ptr, send_edge = workloads.graph_indices(sender, receiver, N)
    say(f"case {wl.name}: N={N} E={E} K={wl.num_channels}")
    assert E * P * wl.num_channels > (1 << 31)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.seed)
    rnd = lambda *shape: torch.randn(shape, generator=gen, device=dev, dtype=torch.float32)
    per_l3 = np.bincount(np.asarray(paths)[:, 2], minlength=wl.L_max + 1)
    scale = torch.tensor(1.0 / np.sqrt(wl.mean_degree * per_l3[np.asarray(paths)[:, 2]]), dtype=torch.float32, device=dev)
    Y, h = rnd(E, wl.n_Y), rnd(N, wl.num_channels, wl.n_h)
    R = rnd(E, P, wl.num_channels)
    R *= scale[None, :, None]
    dA = rnd(N, wl.num_channels, wl.n_out)
    i32 = lambda x: torch.tensor(x, dtype=torch.int32, device=dev)
    d_sender, d_row_ptr, d_send_ptr, d_send_edge = i32(sender), i32(row_ptr), i32(send_ptr), i32(send_edge)
    A = torch.full((N, wl.num_channels, wl.n_out), float("nan"), dtype=torch.float32, device=dev)
    dY, dh, dR = (torch.full_like(x, float("nan")) for x in (Y, h, R))
    plan = tp.tp_plan_create(wl.num_channels, wl.l_Y, wl.l_h, wl.L_max, tp.SC_F32, 0, 0)
    assert tp.tp_plan_info(plan).specialised == 1
    nbytes = tp.tp_workspace_bytes(plan, E)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    tp.tp_forward(plan, N, N, E, Y, h, R, d_sender, d_row_ptr, A)
    tp.tp_backward(plan, N, N, E, Y, h, R, d_sender, d_row_ptr, d_send_ptr, d_send_edge, dA, dY, dh, dR, ws, nbytes)
    torch.cuda.synchronize()
    assert all(bool(torch.isfinite(x).all()) for x in (A, dY, dh, dR))
    no_edges, silent = np.diff(row_ptr) == 0, np.diff(send_ptr) == 0
    assert not bool(A[i32(np.flatnonzero(no_edges)).long()].any()) and not bool(dh[i32(np.flatnonzero(silent)).long()].any())
    f64 = lambda x: x.double().cpu().numpy()
    h_host = f64(h)
    e_mid = (1 << 31) // (P * wl.num_channels)        # the edge whose rows of R start at element offset 2^31
    a_mid = int(receiver[e_mid])
    for name, a0, a1 in (("first atoms", 0, 40), ("atoms around 2^31", a_mid - 20, a_mid + 20), ("last atoms", N - 40, N)):
        e0, e1 = int(row_ptr[a0]), int(row_ptr[a1])
        if name == "atoms around 2^31":
            assert e0 < e_mid < e1
        es = slice(e0, e1)
        recv = receiver[es] - a0
        A_ref = otp.forward(cfg, f64(Y[es]), h_host, f64(R[es]), sender[es], recv, a1 - a0)
        dY_ref, _, dR_ref = otp.backward(cfg, f64(Y[es]), h_host, f64(R[es]), sender[es], recv, f64(dA[a0:a1]))
        check(f"A({name})", A[a0:a1].cpu().numpy(), A_ref, "f32")
        check(f"dY({name})", dY[es].cpu().numpy(), dY_ref, "f32")
        check(f"dR({name})", dR[es].cpu().numpy(), dR_ref, "f32")
    # dh of some senders: the oracle on the sub-graph of every edge they send
    for name, j0, j1 in (("first senders", 0, 30), ("senders around 2^31", a_mid - 15, a_mid + 15), ("last senders", N - 30, N)):
        edges = send_edge[send_ptr[j0]:send_ptr[j1]].astype(np.int64)
        recv_atoms, recv = np.unique(receiver[edges], return_inverse=True)
        sel = torch.tensor(edges, device=dev)
        _, dh_ref, _ = otp.backward(cfg, f64(Y[sel]), h_host, f64(R[sel]), sender[edges], recv.astype(np.int32),
                                    f64(dA[torch.tensor(recv_atoms, device=dev).long()]))
        check(f"dh({name})", dh[j0:j1].cpu().numpy(), dh_ref[j0:j1], "f32")
    tp.tp_plan_destroy(plan)
    del Y, h, R, dA, A, dY, dh, dR, ws
    torch.cuda.empty_cache()


@pytest.mark.parametrize("flags", [0, 2])
def test_wrong_index_arrays_stay_inside_the_buffers(tp, flags):
    """The index arrays are not validated, but every index is clamped where it is read: a list with
    senders, offsets and edge ids out of range gives meaningless numbers for the edges concerned and
    leaves the device healthy - the correct list gives the oracle's result right afterwards."""
    import torch
    wl = wl_of("bad_indices", 40, 6, 128, 3, 1, 3, "f32", 5301)
    cfg = oracle_cfg(wl)
    inp = workloads.make_tp_inputs(wl, otp.enumerate_paths(cfg))
    run = TPRun(tp, wl, inp, flags)
    good = [x.clone() for x in (run.sender, run.row_ptr, run.send_ptr, run.send_edge)]
    E = run.E
    say(f"case bad_indices: N={run.N} E={E} flags={flags}")
    run.sender[::7] = -5
    run.sender[3::11] = run.N + 1000
    run.row_ptr[5] = E + 12345
    run.row_ptr[9] = -4
    run.send_ptr[7] = 2 * E
    run.send_edge[::5] = E + 7
    run.send_edge[2::9] = -1
    run.forward()
    run.backward()
    HY, Hh, HR = workloads.make_tp_cotangents(wl, inp)
    run.double_backward(HY, Hh, HR)
    for dst, src in zip((run.sender, run.row_ptr, run.send_ptr, run.send_edge), good):
        dst.copy_(src)
    torch.cuda.synchronize()
    Y, h, R, dA = run.inputs_as_computed()
    no_edges = np.diff(inp.row_ptr) == 0
    A = run.forward()
    check("A", A[~no_edges], otp.forward(cfg, Y, h, R, inp.sender, inp.receiver, run.N)[~no_edges], wl.dtype)
    dY, dh, dR = run.backward()
    dY_ref, dh_ref, dR_ref = otp.backward(cfg, Y, h, R, inp.sender, inp.receiver, dA)
    check("dY", dY, dY_ref, wl.dtype)
    check("dR", dR, dR_ref, wl.dtype)
    run.close()
