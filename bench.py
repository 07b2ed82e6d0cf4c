#!/usr/bin/env python3
"""Benchmark of the symmetric-contraction hot path on one MI355X.

One "step" = sc_forward + sc_backward (the grouping of the nodes by element and the
preparation of the weights done once, in the forward, and reused by the backward) over
one batch of synthetic atoms that is already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W]
                  [--workload training_step|large_batch|wide_high_l|wide_high_l_f64|medium_fwd|outputs_l3|tiny]

Default workload: `training_step` (10 000 nodes, 89 elements, 128 channels, l<=3, nu<=3,
outputs 0e+1o, fp32, forward+backward) - the configuration the metric "atoms/sec
symmetric-contraction fwd+bwd (128ch, l<=3, nu=3)" is quoted on.  With the default
workload the same line also carries, under "also", a shorter measurement of
`large_batch` (200 000 nodes, same shapes): at 10 000 nodes a step is ~0.09 ms and
launch / fixed costs weigh as much as the data movement, at 200 000 nodes they do not;
of `medium_fwd`, `wide_high_l`, `outputs_l3` and the bfloat16-row variant; of the training
step in the other layout (--component-major), on the same buffers every step (cache-resident,
labelled so) and with batches ordered by element (--z-grouped); of the second-order pass
(sc_double_backward alone) on both workloads; and of the operations around the contraction.
"attainable" holds streaming probes of the same run (what this machine reaches without arithmetic,
for plain reads / writes / copies and for the access patterns of the two main kernels).

value          nodes (atoms) per second, forward + backward, whole step (all launches)
roofline       the dominant kernel (fused backward: dA + per-tile dW) against the HBM
               peak: algorithmic bytes per launch / its mean duration, the duration
               taken with HIP events recorded by the library on the launch stream
cpu_baseline   the fp64 oracle timed on this machine's host cores on a bounded sample

Cache hygiene: buffer sets (A, dB, B, dA) are rotated so that >= 1 GB of other traffic
passes before a buffer is touched again, and the backward of a step reads a different
copy of A than its forward did (in training the two are far apart in time): the
256 MB last-level cache cannot serve any of the reads.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published
FP32_PEAK_TFLOPS = 157.3   # MI355X vector fp32, published (256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz x 2 (FMA) x 2 (packed))
VALU_ISSUE_PEAK = 256 * 4 * 16 * 2.4e9   # per-lane vector instructions per second at the published clock
METRIC = "atoms/sec symmetric-contraction fwd+bwd (128ch, l<=3, nu=3); % HBM peak"


def algorithmic_bytes(wl, n_nodes, elem):
    """Bytes that must cross HBM per launch: A, dB in and dA out (backward);
    A in, B out and 4 B of z per node (forward)."""
    K = wl.num_channels
    fwd = n_nodes * (K * (wl.n_lm + wl.n_LM) * elem + 4)
    bwd = n_nodes * K * (2 * wl.n_lm + wl.n_LM) * elem
    return fwd, bwd


def cpu_baseline(wl, n_sample):
    from oracle import symmetric_contraction as osc
    from paper_2504_10700_amd import workloads
    cfg = osc.OracleConfig(wl.num_channels, wl.l_max, wl.nu_max, wl.num_elements, wl.out_irreps)
    T = osc.build_tables(cfg)
    inp = workloads.make_inputs(wl, T.paths, num_nodes=n_sample)
    t0 = time.perf_counter()
    osc.forward(T, inp.A, inp.z, inp.W)
    if wl.backward:
        osc.backward(T, inp.A, inp.z, inp.W, inp.dB)
    dt = time.perf_counter() - t0
    return {"value": n_sample / dt, "unit": "nodes/s", "cores": len(os.sched_getaffinity(0)), "kind": "oracle",
            "sample": f"first {n_sample} nodes of the workload, fp64 dense-tensor oracle (numpy/BLAS), "
                      f"{'forward+backward' if wl.backward else 'forward'}, {dt:.1f} s"}


def describe(wl):
    return (f"{wl.name}: {wl.num_nodes} nodes, {wl.num_elements} elements ({wl.z_mode} z, unsorted), "
            f"{wl.num_channels} channels, l_max={wl.l_max}, nu_max={wl.nu_max}, outputs "
            + "+".join(f"{L}{'e' if p > 0 else 'o'}" for L, p in wl.out_irreps)
            + (", forward+backward" if wl.backward else ", forward only"))


def measure(wl, steps, warmup, generic=False, tile_nodes=0, component_major=False, z_grouped=False, rotate=True):
    import numpy as np
    import torch
    from paper_2504_10700_amd import binding as sc
    from paper_2504_10700_amd import workloads

    dev = torch.device("cuda:0")
    # tdt / elem: the per-node tensors; W and dW are fp32 when those are stored as bfloat16
    tdt = {"f32": torch.float32, "f64": torch.float64, "bf16": torch.bfloat16}[wl.dtype]
    wdt = torch.float64 if wl.dtype == "f64" else torch.float32
    elem = {"f32": 4, "f64": 8, "bf16": 2}[wl.dtype]
    plan = sc.sc_plan_create(wl.num_channels, wl.l_max, wl.nu_max, wl.num_elements, wl.out_irreps,
                             {"f32": sc.SC_F32, "f64": sc.SC_F64, "bf16": sc.SC_BF16}[wl.dtype], 0,
                             sc.SC_PLAN_FORCE_GENERIC if generic else 0, tile_nodes)
    info = sc.sc_plan_info(plan)
    inp = workloads.make_inputs(wl, sc.sc_plan_paths(plan))
    N, K = wl.num_nodes, wl.num_channels

    per_set = N * K * (2 * wl.n_lm + 2 * wl.n_LM) * elem
    n_sets = max(2, min(8, int(np.ceil(1.0e9 / per_set))))
    if not rotate:     # every step on the same buffers: what fits stays in the 256 MB last-level cache
        n_sets = 1
    A0 = torch.tensor(inp.A, dtype=tdt, device=dev)
    dB0 = torch.tensor(inp.dB, dtype=tdt, device=dev)
    W = torch.tensor(inp.W, dtype=wdt, device=dev)
    z = torch.tensor(inp.z, dtype=torch.int32, device=dev)
    del inp
    call_flags = sc.SC_COMPONENT_MAJOR if component_major else 0
    if z_grouped:   # a batch whose nodes the caller has ordered by element (A, dB are iid: only z changes)
        z = torch.sort(z).values.contiguous()
        call_flags |= sc.SC_Z_GROUPED
    if component_major:   # the same rows as [node][component][channel]
        A0, dB0 = A0.transpose(1, 2).contiguous(), dB0.transpose(1, 2).contiguous()
    sets = []
    for s in range(n_sets):
        sets.append({
            "A": A0 if s == 0 else A0.roll(s, 0).contiguous(),
            "dB": dB0 if s == 0 else dB0.roll(s, 0).contiguous(),
            "B": torch.empty_like(dB0),
            "dA": torch.empty_like(A0),
        })
    dW = torch.empty_like(W)
    ws_bytes = sc.sc_workspace_bytes(plan, N)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    def step(i):
        f = sets[i % n_sets]
        sc.sc_forward(plan, N, f["A"], z, W, f["B"], ws, ws_bytes, call_flags)
        if wl.backward:
            b = sets[(i + n_sets // 2) % n_sets]   # another copy of A: no cache reuse across fwd -> bwd
            sc.sc_backward(plan, N, b["A"], z, W, b["dB"], b["dA"], dW, ws, ws_bytes,
                           sc.SC_REUSE_GROUPING | sc.SC_REUSE_WEIGHTS | call_flags)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    value = N / (dt / steps)

    # Second pass with the library's event brackets around the main kernels.
    sc.sc_profile_enable(plan, True)
    fwd_ms, bwd_ms = [], []
    for i in range(min(steps, 50)):
        step(i)
        f, b = sc.sc_profile_read(plan)
        fwd_ms.append(f)
        bwd_ms.append(b)
    sc.sc_profile_enable(plan, False)
    sc.sc_plan_destroy(plan)
    fwd_bytes, bwd_bytes = algorithmic_bytes(wl, N, elem)
    fwd_mean = float(np.mean(fwd_ms))
    if wl.backward:
        k_ms, k_bytes, k_name = float(np.mean(bwd_ms)), bwd_bytes, "backward (dA + per-tile dW)"
    else:
        k_ms, k_bytes, k_name = fwd_mean, fwd_bytes, "forward"
    achieved = k_bytes / (k_ms * 1e-3) / 1e9
    step_bytes = fwd_bytes + (bwd_bytes if wl.backward else 0)
    k_ops = info.ops[1 if wl.backward else 0]     # 0 for the table-driven kernels
    valu_issue_frac = N * K * k_ops / (k_ms * 1e-3) / VALU_ISSUE_PEAK if k_ops else None

    # HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter runs
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath) and wl.backward and info.specialised and tile_nodes == 0 and not component_major and not z_grouped:
        ent = json.load(open(tpath)).get(wl.name)
        if ent:
            traffic = 1024.0 * (ent["fetch_kib"] * ent["fetch_scale"] + ent["write_kib"] * ent["write_scale"])
    del sets, A0, dB0, ws
    torch.cuda.empty_cache()
    return {
        "value": value, "unit": "nodes/s", "steps": steps, "warmup": warmup, "ms_per_step": dt / steps * 1e3,
        "dtype": wl.dtype,
        "config": {"workload": describe(wl), "num_paths": int(info.num_paths),
                   "kernel": "generated" if info.specialised else "table-driven",
                   "buffer_sets_rotated": n_sets, "tile_nodes": tile_nodes,
                   "layout": "[node][component][channel]" if component_major else "[node][channel][component]",
                   "z_order": "grouped by element (SC_Z_GROUPED)" if z_grouped else "as drawn"},
        "step_hbm_fraction": value * (step_bytes / N) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "kernel": k_name, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "kernel_ms": k_ms,
                     "forward_kernel_ms": fwd_mean, "algorithmic_bytes_per_launch": k_bytes,
                     "valu_issue_frac": valu_issue_frac},
    }


def measure_attainable(n_nodes=10_000, chblocks=2, reps=20):
    """Streaming probes of the library (kernels without arithmetic, known byte counts), timed
    with events on the launch stream in this same run: what the box attains for plain reads,
    writes, copies, and for the access pattern of the fused backward kernel (gathered 4 KB + 1 KB
    rows in, 4 KB rows out) at the batch size of the workload and at 20x that size.  Buffers are
    rotated so that no launch finds its data in the 256 MB last-level cache."""
    import numpy as np
    import torch
    from paper_2504_10700_amd import binding as sc

    dev = torch.device("cuda:0")

    def timed(launch, n_variants):
        for i in range(3):
            launch(i % n_variants)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        torch.cuda.synchronize()
        ev[0].record()
        for i in range(reps):
            launch(i % n_variants)
        ev[1].record()
        torch.cuda.synchronize()
        return ev[0].elapsed_time(ev[1]) / reps * 1e-3

    out = {"unit": "GB/s", "note": "library streaming probes, same run; rows = the backward kernel's access "
                                   "pattern (9216 B per row of 64 channels) without arithmetic; forward_rows = the "
                                   "forward kernel's (5120 B per row, batch order)"}
    nbytes = 1 << 30
    bufs = [torch.empty(nbytes // 4, dtype=torch.float32, device=dev).normal_() for _ in range(3)]
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    t = timed(lambda i: sc.sc_probe_stream(sc.SC_PROBE_READ, bufs[i], None, sink, None, nbytes), 3)
    out["read"] = nbytes / t / 1e9
    t = timed(lambda i: sc.sc_probe_stream(sc.SC_PROBE_WRITE, None, None, bufs[i], None, nbytes), 3)
    out["write"] = nbytes / t / 1e9
    t = timed(lambda i: sc.sc_probe_stream(sc.SC_PROBE_COPY, bufs[i], None, bufs[(i + 1) % 3], None, nbytes), 3)
    out["copy"] = 2 * nbytes / t / 1e9
    del bufs
    torch.cuda.empty_cache()
    for label, rows, n_sets in (("rows_at_batch_size", n_nodes * chblocks, 6), ("rows_at_20x_batch_size", 20 * n_nodes * chblocks, 2)):
        rng = np.random.default_rng(5)
        sets = []
        for s in range(n_sets):
            sets.append((torch.empty(rows * 1024, dtype=torch.float32, device=dev).normal_(),
                         torch.empty(rows * 256, dtype=torch.float32, device=dev).normal_(),
                         torch.empty(rows * 1024, dtype=torch.float32, device=dev)))
        perm = torch.tensor(rng.permutation(rows).astype(np.int32), device=dev)
        t = timed(lambda i: sc.sc_probe_stream(sc.SC_PROBE_ROWS, sets[i][0], sets[i][1], sets[i][2], perm, rows), n_sets)
        out[label] = rows * 9216 / t / 1e9
        out[label + "_us"] = t * 1e6
        # the forward's traffic (4 KB in, 1 KB out per row) in the order of the batch
        ident = torch.arange(rows, dtype=torch.int32, device=dev)
        t = timed(lambda i: sc.sc_probe_stream(sc.SC_PROBE_ROWS_FORWARD, sets[i][0], None, sets[i][1], ident, rows), n_sets)
        out["forward_" + label] = rows * 5120 / t / 1e9
        out["forward_" + label + "_us"] = t * 1e6
        del sets
        torch.cuda.empty_cache()
    out["frac_of_peak"] = {k: out[k] / HBM_PEAK_GBS for k in ("read", "write", "copy", "rows_at_batch_size",
                                                              "rows_at_20x_batch_size", "forward_rows_at_batch_size",
                                                              "forward_rows_at_20x_batch_size")}
    return out


def measure_double_backward(wl, steps, warmup, tile_nodes=0):
    """The second-order pass alone: one step = sc_double_backward (grouping included)."""
    import numpy as np
    import torch
    from paper_2504_10700_amd import binding as sc
    from paper_2504_10700_amd import workloads

    dev = torch.device("cuda:0")
    tdt = torch.float32 if wl.dtype == "f32" else torch.float64
    elem = 4 if wl.dtype == "f32" else 8
    plan = sc.sc_plan_create(wl.num_channels, wl.l_max, wl.nu_max, wl.num_elements, wl.out_irreps,
                             sc.SC_F32 if wl.dtype == "f32" else sc.SC_F64, 0, 0, tile_nodes)
    info = sc.sc_plan_info(plan)
    inp = workloads.make_inputs(wl, sc.sc_plan_paths(plan))
    N, K = wl.num_nodes, wl.num_channels
    per_set = N * K * (3 * wl.n_lm + 2 * wl.n_LM) * elem
    n_sets = max(2, min(8, int(np.ceil(1.0e9 / per_set))))
    A0 = torch.tensor(inp.A, dtype=tdt, device=dev)
    dB0 = torch.tensor(inp.dB, dtype=tdt, device=dev)
    H0 = torch.tensor(workloads.make_cotangent(wl), dtype=tdt, device=dev)
    W = torch.tensor(inp.W, dtype=tdt, device=dev)
    z = torch.tensor(inp.z, dtype=torch.int32, device=dev)
    del inp
    sets = []
    for s in range(n_sets):
        sets.append({
            "A": A0 if s == 0 else A0.roll(s, 0).contiguous(),
            "dB": dB0 if s == 0 else dB0.roll(s, 0).contiguous(),
            "H": H0 if s == 0 else H0.roll(s, 0).contiguous(),
            "ddB": torch.empty((N, K, wl.n_LM), dtype=tdt, device=dev),
            "dA2": torch.empty((N, K, wl.n_lm), dtype=tdt, device=dev),
        })
    dW2 = torch.empty_like(W)
    ws_bytes = sc.sc_workspace_bytes(plan, N)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    def step(i):
        b = sets[i % n_sets]
        sc.sc_double_backward(plan, N, b["A"], z, W, b["dB"], b["H"], b["ddB"], b["dA2"], dW2, ws, ws_bytes, 0)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    sc.sc_profile_enable(plan, True)
    k_ms = []
    for i in range(min(steps, 50)):
        step(i)
        k_ms.append(sc.sc_profile_read_double_backward(plan))
    sc.sc_profile_enable(plan, False)
    sc.sc_plan_destroy(plan)
    k_ms = float(np.mean(k_ms))
    k_bytes = N * K * (3 * wl.n_lm + 2 * wl.n_LM) * elem   # A, H, dB in; dA2, ddB out
    achieved = k_bytes / (k_ms * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath) and info.specialised and tile_nodes == 0:
        ent = json.load(open(tpath)).get("double_backward:" + wl.name)
        if ent:
            traffic = 1024.0 * (ent["fetch_kib"] * ent["fetch_scale"] + ent["write_kib"] * ent["write_scale"])
    # The second-order kernel needs more time on the vector ALUs than on HBM (see "alu"):
    # both figures are reported, the larger fraction names the bound.
    hbm = {"achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
           "traffic": traffic, "algorithmic_bytes_per_launch": k_bytes}
    if info.specialised and wl.dtype == "f32":
        tflops = N * K * info.flops[2] / (k_ms * 1e-3) / 1e12
        roof = {"bound": "alu", "kernel": "double backward (ddB + dA2 + per-tile dW2)", "achieved": tflops,
                "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tflops / FP32_PEAK_TFLOPS, "traffic": traffic,
                "kernel_ms": k_ms, "flops_per_node_channel": int(info.flops[2]),
                "valu_issue_frac": N * K * info.ops[2] / (k_ms * 1e-3) / VALU_ISSUE_PEAK, "hbm": hbm}
    else:
        roof = dict(hbm, bound="hbm", kernel="double backward (ddB + dA2 + per-tile dW2)", kernel_ms=k_ms)
    del sets, A0, dB0, H0, ws
    torch.cuda.empty_cache()
    return {
        "value": N / (dt / steps), "unit": "nodes/s", "steps": steps, "warmup": warmup,
        "ms_per_step": dt / steps * 1e3, "dtype": wl.dtype,
        "config": {"workload": describe(wl).replace("forward+backward", "second-order pass only"),
                   "kernel": "generated" if info.specialised else "table-driven", "buffer_sets_rotated": n_sets,
                   "tile_nodes": tile_nodes},
        "roofline": roof,
    }


def measure_tp(wl, steps, warmup):
    """Channelwise tensor product (Algorithm 1 with pooling): one step = tp_forward + tp_backward."""
    import numpy as np
    import torch
    from paper_2504_10700_amd import tp_binding as tp
    from paper_2504_10700_amd import workloads

    dev = torch.device("cuda:0")
    tdt = torch.float32 if wl.dtype == "f32" else torch.float64
    elem = 4 if wl.dtype == "f32" else 8
    plan = tp.tp_plan_create(wl.num_channels, wl.l_Y, wl.l_h, wl.L_max, tp.SC_F32 if wl.dtype == "f32" else tp.SC_F64, 0)
    info = tp.tp_plan_info(plan)
    inp = workloads.make_tp_inputs(wl, tp.tp_plan_paths(plan))
    N, K, E, P = wl.num_nodes, wl.num_channels, int(inp.Y.shape[0]), int(info.num_paths)
    f = lambda x: torch.tensor(x, dtype=tdt, device=dev)
    i32 = lambda x: torch.tensor(x, dtype=torch.int32, device=dev)
    Y, h, dA = f(inp.Y), f(inp.h), f(inp.dA)
    sender, row_ptr = i32(inp.sender), i32(inp.row_ptr)
    send_ptr, send_edge = i32(inp.send_ptr), i32(inp.send_edge)
    # R and dR are the large tensors (E*P*K): two copies of each are rotated so that a step never
    # finds the previous step's rows in the 256 MB last-level cache
    R0 = f(inp.R)
    del inp
    Rs = [R0, R0.clone()]
    dRs = [torch.empty_like(R0), torch.empty_like(R0)]
    A = torch.empty((N, K, wl.n_out), dtype=tdt, device=dev)
    dY, dh = torch.empty_like(Y), torch.empty_like(h)
    ws_bytes = tp.tp_workspace_bytes(plan, E)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    def step(i):
        tp.tp_forward(plan, N, N, E, Y, h, Rs[i % 2], sender, row_ptr, A)
        tp.tp_backward(plan, N, N, E, Y, h, Rs[(i + 1) % 2], sender, row_ptr, send_ptr, send_edge, dA, dY, dh,
                       dRs[i % 2], ws, ws_bytes)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tp.tp_profile_enable(plan, True)
    ms = []
    for i in range(min(steps, 30)):
        step(i)
        ms.append(tp.tp_profile_read(plan))
    tp.tp_profile_enable(plan, False)
    tp.tp_plan_destroy(plan)
    fwd_ms, bwd_ms, dhs_ms = (float(x) for x in np.mean(np.array(ms), axis=0))
    # algorithmic bytes per launch: the per-edge tensors once each (R, Y, one index; dR out) plus
    # the per-node tensors once (h, dA in; A out); gathered rows are counted once per node.  The
    # backward kernel also writes dY partials per channel block into the workspace (and, table-driven
    # kernels only, per-edge shares of dh), which small sum kernels read back: that is overhead of this
    # implementation, reported separately and not counted as algorithmic bytes (it shows up in `traffic`).
    # The generated backward writes dh itself (one more per-node tensor out).
    node_h, node_A = N * K * wl.n_h * elem, N * K * wl.n_out * elem
    chblocks = (K + 63) // 64
    fwd_bytes = E * (P * K * elem + wl.n_Y * elem + 4) + node_h + node_A
    bwd_bytes = E * (2 * P * K * elem + wl.n_Y * elem + 4) + node_h + node_A + (node_h if info.specialised else 0)
    bwd_ws_bytes = E * ((0 if info.specialised else K * wl.n_h) + chblocks * wl.n_Y) * elem   # not algorithmic bytes
    bwd_rate = bwd_bytes / (bwd_ms * 1e-3) / 1e9
    step_bytes = fwd_bytes + bwd_bytes + E * wl.n_Y * elem + (0 if info.specialised else node_h)   # + dY (and dh) out
    k_ops = info.ops[1]
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath) and info.specialised:
        ent = json.load(open(tpath)).get("tp:" + wl.name)
        if ent:
            traffic = 1024.0 * (ent["fetch_kib"] * ent["fetch_scale"] + ent["write_kib"] * ent["write_scale"])
    del Rs, dRs, R0, ws
    torch.cuda.empty_cache()
    return {
        "metric": "edges/sec channelwise tensor product fwd+bwd", "value": E / (dt / steps), "unit": "edges/s",
        "steps": steps, "warmup": warmup, "ms_per_step": dt / steps * 1e3, "dtype": wl.dtype,
        "config": {"workload": f"{wl.name}: {N} nodes, {E} edges (in-degree ~Poisson({wl.mean_degree})), {K} channels, "
                               f"l_Y={wl.l_Y}, l_h={wl.l_h}, L_max={wl.L_max}, {P} paths, forward+backward",
                   "kernel": "generated" if info.specialised else "table-driven"},
        "step_hbm_fraction": step_bytes / (dt / steps) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm",
                     "kernel": "backward over the edges grouped by sender (dR, dY partials, dh)" if info.specialised
                               else "backward over the edges (dR, dY partials, per-edge dh shares)",
                     "achieved": bwd_rate, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": bwd_rate / HBM_PEAK_GBS,
                     "traffic": traffic, "kernel_ms": bwd_ms, "algorithmic_bytes_per_launch": bwd_bytes,
                     "workspace_bytes_written_per_launch": bwd_ws_bytes,
                     "valu_issue_frac": E * K * k_ops / (bwd_ms * 1e-3) / VALU_ISSUE_PEAK if k_ops else None,
                     "forward": {"kernel_ms": fwd_ms, "algorithmic_bytes_per_launch": fwd_bytes,
                                 "achieved": fwd_bytes / (fwd_ms * 1e-3) / 1e9},
                     # only the table-driven kernels sum per-edge shares of dh in a launch of its own
                     "dh_sum": None if info.specialised else
                               {"kernel_ms": dhs_ms, "bytes_per_launch": E * K * wl.n_h * elem + node_h,
                                "achieved": (E * K * wl.n_h * elem + node_h) / (dhs_ms * 1e-3) / 1e9}},
    }


def measure_tp_double_backward(wl, steps, warmup):
    """Second-order pass of the channelwise tensor product alone: one step = tp_double_backward."""
    import numpy as np
    import torch
    from paper_2504_10700_amd import tp_binding as tp
    from paper_2504_10700_amd import workloads

    dev = torch.device("cuda:0")
    tdt = torch.float32 if wl.dtype == "f32" else torch.float64
    elem = 4 if wl.dtype == "f32" else 8
    plan = tp.tp_plan_create(wl.num_channels, wl.l_Y, wl.l_h, wl.L_max, tp.SC_F32 if wl.dtype == "f32" else tp.SC_F64, 0)
    info = tp.tp_plan_info(plan)
    inp = workloads.make_tp_inputs(wl, tp.tp_plan_paths(plan))
    cot = workloads.make_tp_cotangents(wl, inp)
    N, K, E, P = wl.num_nodes, wl.num_channels, int(inp.Y.shape[0]), int(info.num_paths)
    f = lambda x: torch.tensor(x, dtype=tdt, device=dev)
    i32 = lambda x: torch.tensor(x, dtype=torch.int32, device=dev)
    Y, h, dA, HY, Hh = f(inp.Y), f(inp.h), f(inp.dA), f(cot[0]), f(cot[1])
    sender, row_ptr, send_ptr, send_edge = i32(inp.sender), i32(inp.row_ptr), i32(inp.send_ptr), i32(inp.send_edge)
    R0, HR0 = f(inp.R), f(cot[2])
    del inp, cot
    Rs, HRs = [R0, R0.clone()], [HR0, HR0.clone()]    # rotated: no reuse of the last step's rows from cache
    d2Rs = [torch.empty_like(R0), torch.empty_like(R0)]
    ddA, d2Y, d2h = torch.empty((N, K, wl.n_out), dtype=tdt, device=dev), torch.empty_like(Y), torch.empty_like(h)
    ws_bytes = tp.tp_workspace_bytes(plan, E)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    def step(i):
        tp.tp_double_backward(plan, N, N, E, Y, h, Rs[i % 2], sender, row_ptr, send_ptr, send_edge, dA, HY, Hh,
                              HRs[i % 2], ddA, d2Y, d2h, d2Rs[i % 2], ws, ws_bytes)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tp.tp_profile_enable(plan, True)
    ms = []
    for i in range(min(steps, 30)):
        step(i)
        ms.append(tp.tp_profile_read_double_backward(plan))
    tp.tp_profile_enable(plan, False)
    tp.tp_plan_destroy(plan)
    k_ms = float(np.mean(ms))
    chblocks = (K + 63) // 64
    # R, HR in and d2R out per edge, Y, HY, index; h, Hh, dA in and ddA out per node; plus the
    # workspace rows this kernel writes (d2h shares, d2Y partials)
    k_bytes = (E * (3 * P * K * elem + 2 * wl.n_Y * elem + 4) + N * K * (2 * wl.n_h + 2 * wl.n_out) * elem
               + E * (K * wl.n_h + chblocks * wl.n_Y) * elem)
    rate = k_bytes / (k_ms * 1e-3) / 1e9
    k_ops = info.ops[2]
    del Rs, HRs, d2Rs, R0, HR0, ws
    torch.cuda.empty_cache()
    return {
        "metric": "edges/sec channelwise tensor product, second-order pass", "value": E / (dt / steps),
        "unit": "edges/s", "steps": steps, "warmup": warmup, "ms_per_step": dt / steps * 1e3, "dtype": wl.dtype,
        "config": {"workload": f"{wl.name}: {N} nodes, {E} edges, {K} channels, l_Y={wl.l_Y}, l_h={wl.l_h}, "
                               f"L_max={wl.L_max}, {P} paths, second-order pass only",
                   "kernel": "generated" if info.specialised else "table-driven"},
        "roofline": {"bound": "hbm", "kernel": "second-order pass over the edges", "achieved": rate,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": rate / HBM_PEAK_GBS, "traffic": None,
                     "kernel_ms": k_ms, "algorithmic_bytes_per_launch": k_bytes,
                     "valu_issue_frac": E * K * k_ops / (k_ms * 1e-3) / VALU_ISSUE_PEAK if k_ops else None},
    }


def measure_linear(n_nodes=10_000, k_in=128, k_out=128, l_max=3, steps=50, warmup=5):
    """Per-order channel-mixing linear on the matrix cores: one step = el_forward + el_backward."""
    import numpy as np
    import torch
    from paper_2504_10700_amd import el_binding as el
    from paper_2504_10700_amd import workloads

    dev = torch.device("cuda:0")
    X, W, dY = (torch.tensor(x, dtype=torch.float32, device=dev)
                for x in workloads.make_linear_inputs(n_nodes, k_in, k_out, l_max, 9001))
    cfg = el.make_config(k_in, k_out, l_max, el.SC_F32)
    nc = (l_max + 1) ** 2
    n_sets = 6     # rotated so that a step does not find the previous step's tensors in the last-level cache
    Xs = [X] + [X.clone() for _ in range(n_sets - 1)]
    dYs = [dY] + [dY.clone() for _ in range(n_sets - 1)]
    Ys = [torch.empty((n_nodes, k_out, nc), dtype=torch.float32, device=dev) for _ in range(n_sets)]
    dXs = [torch.empty_like(X) for _ in range(n_sets)]
    dW = torch.empty_like(W)
    nbytes = el.el_workspace_bytes(cfg, n_nodes)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def fwd(i):
        el.el_forward(cfg, n_nodes, Xs[i % n_sets], W, Ys[i % n_sets])

    def bwd(i):
        j = (i + n_sets // 2) % n_sets
        el.el_backward(cfg, n_nodes, Xs[j], W, dYs[j], dXs[j], dW, ws, nbytes)

    for i in range(warmup):
        fwd(i)
        bwd(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fwd(i)
        bwd(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    f_ms, b_ms = [], []
    for i in range(min(steps, 30)):      # the library launches on torch's current stream: its events see the kernels
        ev[0].record()
        fwd(i)
        ev[1].record()
        bwd(i)
        ev[2].record()
        torch.cuda.synchronize()
        f_ms.append(ev[0].elapsed_time(ev[1]))
        b_ms.append(ev[1].elapsed_time(ev[2]))
    f_ms, b_ms = float(np.mean(f_ms)), float(np.mean(b_ms))
    gemm_flops = 2.0 * n_nodes * nc * k_in * k_out          # one product; the backward is two of them
    tf = gemm_flops / (f_ms * 1e-3) / 1e12
    return {"metric": "atoms/sec per-order channel-mixing linear fwd+bwd", "value": n_nodes / (dt / steps),
            "unit": "nodes/s", "steps": steps, "warmup": warmup, "ms_per_step": dt / steps * 1e3, "dtype": "f32",
            "config": {"workload": f"{n_nodes} nodes, {k_in} -> {k_out} channels, l_max={l_max}, forward+backward",
                       "kernel": "MFMA 16x16x4 f32"},
            "roofline": {"bound": "mfma", "kernel": "forward (Y = X W per order)", "achieved": tf,
                         "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / FP32_PEAK_TFLOPS, "traffic": None,
                         "kernel_ms": f_ms, "flops_per_launch": gemm_flops,
                         "backward": {"ms": b_ms, "flops": 2 * gemm_flops,
                                      "achieved": 2 * gemm_flops / (b_ms * 1e-3) / 1e12}}}


def measure_fused_forward(wl, steps=50, warmup=5):
    """Forward of linear + contraction: el_sc_forward (one kernel, A stays in registers) next to the two calls
    el_forward + sc_forward through A in memory."""
    import numpy as np
    import torch
    from paper_2504_10700_amd import binding as sc
    from paper_2504_10700_amd import el_binding as el
    from paper_2504_10700_amd import workloads

    dev = torch.device("cuda:0")
    N, K, k_in = wl.num_nodes, wl.num_channels, wl.num_channels
    plan = sc.sc_plan_create(K, wl.l_max, wl.nu_max, wl.num_elements, wl.out_irreps, sc.SC_F32, 0)
    paths = sc.sc_plan_paths(plan)
    inp = workloads.make_inputs(wl, paths)
    Xn, Wln, _ = workloads.make_linear_inputs(N, k_in, K, wl.l_max, wl.seed + 1)
    f = lambda x: torch.tensor(x, dtype=torch.float32, device=dev)
    W, Wl, z = f(inp.W), f(Wln), torch.tensor(inp.z, dtype=torch.int32, device=dev)
    n_sets = 6
    Xs = [f(Xn)]
    Xs += [Xs[0].clone() for _ in range(n_sets - 1)]
    Bs = [torch.empty((N, K, wl.n_LM), dtype=torch.float32, device=dev) for _ in range(n_sets)]
    A = torch.empty((N, K, wl.n_lm), dtype=torch.float32, device=dev)
    fused = el.el_sc_is_fused(plan, k_in)
    fb = el.el_sc_workspace_bytes(plan, k_in, N)
    fws = torch.empty(fb, dtype=torch.uint8, device=dev)
    sb = sc.sc_workspace_bytes(plan, N)
    sws = torch.empty(sb, dtype=torch.uint8, device=dev)
    cfg = el.make_config(k_in, K, wl.l_max, el.SC_F32)

    def one(i):
        el.el_sc_forward(plan, k_in, N, Xs[i % n_sets], Wl, z, W, Bs[i % n_sets], fws, fb)

    def two(i):
        el.el_forward(cfg, N, Xs[i % n_sets], Wl, A)
        sc.sc_forward(plan, N, A, z, W, Bs[i % n_sets], sws, sb)

    def timed(fn):
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    t_one, t_two = timed(one), timed(two)
    sc.sc_plan_destroy(plan)
    nc = wl.n_lm
    gemm_flops = 2.0 * N * nc * k_in * K
    tf = gemm_flops / t_one / 1e12
    return {"metric": "atoms/sec channel-mixing linear + symmetric contraction, forward", "value": N / t_one,
            "unit": "nodes/s", "steps": steps, "warmup": warmup, "ms_per_step": t_one * 1e3, "dtype": "f32",
            "config": {"workload": wl.name, "k_in": k_in, "single_kernel": bool(fused)},
            "two_calls": {"value": N / t_two, "ms_per_step": t_two * 1e3},
            "roofline": {"bound": "mfma", "kernel": "linear on MFMA + contraction from the accumulators",
                         "achieved": tf, "peak": FP32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / FP32_PEAK_TFLOPS,
                         "traffic": None, "flops_per_launch": gemm_flops,
                         "note": "flops of the matrix product only, duration of the whole call (fold + kernel)"}}


def measure_graph_step(n_nodes=3072, steps=300, warmup=20):
    """The paper's per-GPU batch (capacity 3072 atoms, Section 5) is launch-bound: contraction forward + backward
    as eager calls and as one captured HIP graph (the entry points only enqueue kernels)."""
    import torch
    from paper_2504_10700_amd import binding as sc
    from paper_2504_10700_amd import workloads

    dev = torch.device("cuda:0")
    base = workloads.WORKLOADS["training_step"]
    wl = workloads.Workload("paper_batch", n_nodes, base.num_elements, base.num_channels, base.l_max, base.nu_max,
                            base.out_irreps, "f32", 1007)
    plan = sc.sc_plan_create(wl.num_channels, wl.l_max, wl.nu_max, wl.num_elements, wl.out_irreps, sc.SC_F32, 0)
    inp = workloads.make_inputs(wl, sc.sc_plan_paths(plan))
    f = lambda x: torch.tensor(x, dtype=torch.float32, device=dev)
    A, W, dB = f(inp.A), f(inp.W), f(inp.dB)
    z = torch.tensor(inp.z, dtype=torch.int32, device=dev)
    B = torch.empty((n_nodes, wl.num_channels, wl.n_LM), dtype=torch.float32, device=dev)
    dA, dW = torch.empty_like(A), torch.empty_like(W)
    nb = sc.sc_workspace_bytes(plan, n_nodes)
    ws = torch.empty(nb, dtype=torch.uint8, device=dev)

    def step():
        sc.sc_forward(plan, n_nodes, A, z, W, B, ws, nb)
        sc.sc_backward(plan, n_nodes, A, z, W, dB, dA, dW, ws, nb, sc.SC_REUSE_GROUPING | sc.SC_REUSE_WEIGHTS)

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    t_eager = timed(step)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    t_graph = timed(graph.replay)
    sc.sc_plan_destroy(plan)
    return {"metric": METRIC, "value": n_nodes / t_graph, "unit": "nodes/s", "steps": steps, "warmup": warmup,
            "ms_per_step": t_graph * 1e3, "dtype": "f32",
            "config": {"workload": f"{n_nodes} nodes (the paper's batch capacity), otherwise training_step; "
                                   "forward+backward replayed as one HIP graph, inputs resident in cache"},
            "eager": {"value": n_nodes / t_eager, "ms_per_step": t_eager * 1e3}}


def measure_balanced_batches(n_graphs=1_000_000, capacity=3072, n_gpus=8, oracle_sample=200_000):
    """Load balancer (host code): graphs/s of the C++ implementation, the oracle beside it."""
    import numpy as np
    from oracle import balanced_batches as obb
    from paper_2504_10700_amd import bb_binding as bb
    from paper_2504_10700_amd import workloads

    sizes = workloads.make_graph_sizes(n_graphs)
    bb.bb_create_balanced_batches(sizes[:1000], capacity, n_gpus)
    t0 = time.perf_counter()
    bins, slots, n_bins = bb.bb_create_balanced_batches(sizes, capacity, n_gpus)
    dt = time.perf_counter() - t0
    loads = np.bincount(bins, weights=sizes, minlength=n_bins)
    t0 = time.perf_counter()
    obb.create_balanced_batches(sizes[:oracle_sample], capacity, n_gpus)
    dto = time.perf_counter() - t0
    return {"metric": "graphs/sec CREATE-BALANCED-BATCHES (host)", "value": n_graphs / dt, "unit": "graphs/s",
            "seconds": dt,
            "config": {"workload": f"{n_graphs} graphs of 1..768 vertices, capacity {capacity}, {n_gpus} GPUs",
                       "bins": int(n_bins), "lower_bound_bins": int(np.ceil(sizes.sum() / capacity)),
                       "mean_fill": float(loads.mean() / capacity), "min_fill": float(loads.min() / capacity)},
            "cpu_baseline": {"value": oracle_sample / dto, "unit": "graphs/s", "cores": 1, "kind": "oracle",
                             "sample": f"first {oracle_sample} graphs, {dto:.1f} s"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="training_step")
    ap.add_argument("--cpu-sample", type=int, default=3072, help="nodes the oracle is timed on (0 = skip); 3072 take about 12 s")
    ap.add_argument("--generic", action="store_true", help="force the table-driven kernels")
    ap.add_argument("--tile-nodes", type=int, default=0, help="tuning: nodes per tile (0 = library default)")
    ap.add_argument("--component-major", action="store_true",
                    help="per-node tensors laid out [node][component][channel] (SC_COMPONENT_MAJOR)")
    ap.add_argument("--z-grouped", action="store_true",
                    help="the batch arrives ordered by element and the calls say so (SC_Z_GROUPED)")
    ap.add_argument("--no-also", action="store_true", help="skip the extra measurements under \"also\"")
    ap.add_argument("--no-probe", action="store_true", help="skip the streaming probes (\"attainable\")")
    ap.add_argument("--linear", action="store_true",
                    help="measure only the channel-mixing linear (10k nodes, 128 -> 128 channels, l <= 3)")
    ap.add_argument("--graph", action="store_true",
                    help="measure only the 3072-atom step as eager calls and as a replayed HIP graph")
    ap.add_argument("--fused", action="store_true",
                    help="measure only the forward of linear + contraction as one call (--workload)")
    ap.add_argument("--balanced-batches", action="store_true",
                    help="measure only the host load balancer (1M graphs) and print its object")
    ap.add_argument("--tp", action="store_true",
                    help="measure only the channelwise tensor product (--workload tp_training_step|tp_large_batch|tp_first_layer|tp_tiny)")
    ap.add_argument("--attainable", action="store_true",
                    help="measure only the streaming probes (read, write, copy, backward-like rows) and print their object")
    ap.add_argument("--double-backward", action="store_true",
                    help="measure only the second-order pass of --workload and print its object")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    from paper_2504_10700_amd import workloads

    if args.balanced_batches:
        print(json.dumps(measure_balanced_batches()))
        return
    if args.attainable:
        print(json.dumps(measure_attainable()))
        return
    if args.linear:
        print(json.dumps(measure_linear()))
        return
    if args.graph:
        print(json.dumps(measure_graph_step()))
        return
    if args.tp:
        name = args.workload if args.workload in workloads.TP_WORKLOADS else "tp_training_step"
        fn = measure_tp_double_backward if args.double_backward else measure_tp
        print(json.dumps(fn(workloads.TP_WORKLOADS[name], args.steps, args.warmup)))
        return
    wl = workloads.WORKLOADS[args.workload]
    if args.fused:
        print(json.dumps(measure_fused_forward(wl, args.steps, args.warmup)))
        return
    if args.double_backward:
        print(json.dumps(measure_double_backward(wl, args.steps, args.warmup, args.tile_nodes)))
        return
    m = measure(wl, args.steps, args.warmup, args.generic, args.tile_nodes, args.component_major, args.z_grouped)
    out = {"metric": METRIC, "value": m["value"], "unit": m["unit"], "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": m["dtype"], "data": "synthetic", "config": m["config"],
           "step_hbm_fraction": m["step_hbm_fraction"], "roofline": m["roofline"]}
    if not args.generic and not args.no_probe:
        out["attainable"] = measure_attainable(wl.num_nodes, (wl.num_channels + 63) // 64)
    if args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(wl, min(args.cpu_sample, wl.num_nodes))
    if (args.workload == "training_step" and not args.no_also and not args.generic and args.tile_nodes == 0
            and not args.component_major and not args.z_grouped):
        keys = ("value", "unit", "steps", "warmup", "ms_per_step", "dtype", "config", "step_hbm_fraction", "roofline")
        big = measure(workloads.WORKLOADS["large_batch"], 30, 5)
        out["also"] = {"large_batch": {k: big[k] for k in keys}}
        # the other configurations of the benchmark spec: forward only at the training-step shape, and the wide one
        # (256 channels, outputs 0e+1o+2e); then every output irrep up to L = 3 (not one of the task's)
        # and the training step with the per-node tensors stored as bfloat16 (half the bytes)
        for name, st, wu in (("medium_fwd", 100, 10), ("wide_high_l", 20, 3), ("outputs_l3", 40, 5),
                             ("training_step_bf16", 100, 10)):
            m2 = measure(workloads.WORKLOADS[name], st, wu)
            out["also"][name] = {k: m2[k] for k in keys}
        m2 = measure(wl, 100, 10, component_major=True)     # the other layout of the per-node tensors
        out["also"]["training_step_component_major"] = {k: m2[k] for k in keys}
        m2 = measure(wl, 100, 10, rotate=False)             # same buffers every step (cache-resident: not the headline)
        out["also"]["training_step_cache_resident"] = {k: m2[k] for k in keys}
        m2 = measure(wl, 100, 10, z_grouped=True)           # nodes ordered by element by the caller
        out["also"]["training_step_z_grouped"] = {k: m2[k] for k in keys}
        m2 = measure(workloads.WORKLOADS["large_batch"], 30, 5, z_grouped=True)
        out["also"]["large_batch_z_grouped"] = {k: m2[k] for k in keys}
        out["also"]["double_backward_training_step"] = measure_double_backward(wl, 100, 10)
        out["also"]["double_backward_large_batch"] = measure_double_backward(workloads.WORKLOADS["large_batch"], 20, 3)
        out["also"]["channelwise_tp_training_step"] = measure_tp(workloads.TP_WORKLOADS["tp_training_step"], 20, 3)
        out["also"]["channelwise_tp_large_batch"] = measure_tp(workloads.TP_WORKLOADS["tp_large_batch"], 10, 2)
        out["also"]["channelwise_tp_double_backward_training_step"] = measure_tp_double_backward(
            workloads.TP_WORKLOADS["tp_training_step"], 20, 3)
        out["also"]["channel_mixing_linear"] = measure_linear()
        out["also"]["linear_plus_contraction_forward"] = measure_fused_forward(wl, 50, 5)
        out["also"]["paper_batch_3072_atoms_graph"] = measure_graph_step()
        out["also"]["balanced_batches"] = measure_balanced_batches()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
