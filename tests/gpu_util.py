"""Helpers for the GPU parity tests: run the HIP library on numpy inputs and
compare with the oracle under the acceptance tolerances."""
import numpy as np

F32_TOL = 1e-5     # max|got - ref| / rms(ref)                      (fp32 results)
F64_TOL = 1e-12    # max(|got - ref| / max(|ref|, rms(ref)))        (fp64 results)


def rel_err_f32(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    rms = np.sqrt((ref ** 2).mean()) if ref.size else 1.0
    if rms == 0.0:
        return float(np.abs(got).max()) if got.size else 0.0
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / rms) if ref.size else 0.0


def rel_err_f64(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    if not ref.size:
        return 0.0
    rms = np.sqrt((ref ** 2).mean())
    den = np.maximum(np.abs(ref), rms if rms > 0 else 1.0)
    return float((np.abs(np.asarray(got, dtype=np.float64) - ref) / den).max())


BF16_REL = 2.0 ** -8   # bfloat16 keeps 8 significant bits: rounding to nearest is within 2^-9 of the value


def check_bf16_rows(name, got, ref):
    """Per-node results of a plan with bfloat16 rows: the fp32 result rounded to bfloat16, against
    the oracle evaluated on the bfloat16-rounded inputs.  Element by element
    |got - ref| <= 2^-8 |ref| + 1e-5 rms(ref): one bfloat16 rounding (2^-9 relative, doubled for
    values the fp32 error moves across a rounding boundary) on top of the fp32 bar."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    rms = np.sqrt((ref ** 2).mean()) if ref.size else 1.0
    excess = np.abs(got - ref) - (BF16_REL * np.abs(ref) + F32_TOL * rms)
    worst = float(excess.max()) if ref.size else 0.0
    assert worst <= 0.0, f"{name}: exceeds the bfloat16 bound by {worst:.3e} (rms {rms:.3e})"


def check(name, got, ref, dtype):
    if dtype == "bf16":
        return check_bf16_rows(name, got, ref)
    if dtype == "f32":
        err, tol = rel_err_f32(got, ref), F32_TOL
    else:
        err, tol = rel_err_f64(got, ref), F64_TOL
    assert err <= tol, f"{name}: error {err:.3e} exceeds {tol:.1e}"
    return err


# Largest whole-tensor error of a weight gradient seen so far, per case name (printed by
# check_dw; the session summary in conftest.py lists them).
DW_ERRORS = {}


def check_dw(name, dW, dW_ref, z, dtype, case="", whole_tensor=True):
    """Weight gradient against the oracle, under the tolerance read literally: the error
    scale is the rms of the WHOLE reference tensor, rows of absent elements (all zero)
    included.  Those rows must be exactly zero in the result.  The error against the rms
    of the present rows alone (smaller by sqrt(present / all)) is printed next to it.
    whole_tensor=False (batches in which almost every element is absent, where the zero
    rows shrink the scale several times): the present-rows error is the one asserted."""
    num_elements = dW_ref.shape[0]
    present = np.unique(z[(z >= 0) & (z < num_elements)])
    absent = np.setdiff1d(np.arange(num_elements), present)
    assert not np.asarray(dW)[absent].any(), f"{name}: rows of absent elements must be exactly zero"
    fn, tol = (rel_err_f32, F32_TOL) if dtype in ("f32", "bf16") else (rel_err_f64, F64_TOL)   # dW is fp32 with bf16 rows
    whole = fn(dW, dW_ref)
    rows = fn(np.asarray(dW)[present], np.asarray(dW_ref)[present]) if present.size else 0.0
    print(f"{case} {name}: whole-tensor error {whole:.3e}, present-rows error {rows:.3e} "
          f"({present.size}/{num_elements} elements present)", flush=True)
    DW_ERRORS[f"{case} {name}".strip()] = max(whole, DW_ERRORS.get(f"{case} {name}".strip(), 0.0))
    if whole_tensor:
        assert whole <= tol, f"{name}: whole-tensor error {whole:.3e} exceeds {tol:.1e}"
    else:
        assert rows <= tol, f"{name}: present-rows error {rows:.3e} exceeds {tol:.1e}"
    return whole


def oracle_over_chunks(fn, T, node_arrays, shared, n_out_per_node, chunk=64, threads=None):
    """Calls the oracle function `fn(T, *node_arrays[chunk], *shared)` on consecutive chunks
    of nodes from several threads (numpy releases the interpreter lock; every node is
    independent) and puts the results together: the first `n_out_per_node` results are
    per-node arrays (concatenated), the others are sums over nodes (added in chunk order).
    The oracle itself is unchanged; this only spreads its calls over the host's cores.
    node_arrays: arrays with the node axis first; the element index array must be among them
    in the position `fn` expects.  shared: (position, array) pairs inserted as they are."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    from threadpoolctl import threadpool_limits
    n = node_arrays[0].shape[0]
    threads = threads or max(1, min(16, len(os.sched_getaffinity(0))))

    def one(s):
        args = [a[s:s + chunk] for a in node_arrays]
        for pos, arr in shared:
            args.insert(pos, arr)
        out = fn(T, *args)
        return out if isinstance(out, tuple) else (out,)

    with threadpool_limits(limits=1):
        with ThreadPoolExecutor(threads) as ex:
            parts = list(ex.map(one, range(0, n, chunk)))
    outs = []
    for k in range(len(parts[0])):
        if k < n_out_per_node:
            outs.append(np.concatenate([p[k] for p in parts], axis=0))
        else:
            acc = np.zeros_like(parts[0][k])
            for p in parts:
                acc += p[k]
            outs.append(acc)
    return tuple(outs)


def oracle_forward(osc, T, A, z, W):
    return oracle_over_chunks(osc.forward, T, [A, z], [(2, W)], 1)[0]


def oracle_backward(osc, T, A, z, W, dB):
    return oracle_over_chunks(osc.backward, T, [A, z, dB], [(2, W)], 1)


def oracle_double_backward(osc, T, A, z, W, dB, H):
    return oracle_over_chunks(osc.double_backward, T, [A, z, dB, H], [(2, W)], 2)


class GpuRun:
    """Device buffers + plan for one workload; forward()/backward() return numpy arrays."""

    def __init__(self, sc, wl, inp, flags=0, n_nodes=None):
        import torch
        self.sc, self.wl, self.torch = sc, wl, torch
        self.dev = torch.device("cuda:0")
        # tdt: the per-node tensors; wdt: W and dW (fp32 when the rows are bfloat16)
        self.tdt = {"f32": torch.float32, "f64": torch.float64, "bf16": torch.bfloat16}[wl.dtype]
        self.wdt = torch.float64 if wl.dtype == "f64" else torch.float32
        self.plan = sc.sc_plan_create(wl.num_channels, wl.l_max, wl.nu_max, wl.num_elements, wl.out_irreps,
                                      {"f32": sc.SC_F32, "f64": sc.SC_F64, "bf16": sc.SC_BF16}[wl.dtype], 0, flags)
        self.N = inp.A.shape[0] if n_nodes is None else n_nodes
        self.A = torch.tensor(inp.A, dtype=self.tdt, device=self.dev)
        self.W = torch.tensor(inp.W, dtype=self.wdt, device=self.dev)
        self.dB = torch.tensor(inp.dB, dtype=self.tdt, device=self.dev)
        self.z = torch.tensor(inp.z, dtype=torch.int32, device=self.dev)
        self.B = torch.full((self.N, wl.num_channels, wl.n_LM), float("nan"), dtype=self.tdt, device=self.dev)
        self.dA = torch.full_like(self.A, float("nan"))
        self.dW = torch.full_like(self.W, float("nan"))
        self.ws_bytes = sc.sc_workspace_bytes(self.plan, self.N)
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=self.dev)

    def forward(self, flags=0):
        self.sc.sc_forward(self.plan, self.N, self.A, self.z, self.W, self.B, self.ws, self.ws_bytes, flags)
        self.torch.cuda.synchronize()
        return self.B.float().cpu().numpy() if self.wl.dtype == "bf16" else self.B.cpu().numpy()

    def backward(self, flags=0):
        self.sc.sc_backward(self.plan, self.N, self.A, self.z, self.W, self.dB, self.dA, self.dW, self.ws,
                            self.ws_bytes, flags)
        self.torch.cuda.synchronize()
        return (self.dA.float().cpu().numpy() if self.wl.dtype == "bf16" else self.dA.cpu().numpy()), self.dW.cpu().numpy()

    def double_backward(self, H, flags=0):
        """H: numpy array of the shape of A.  Returns (ddB, dA2, dW2, H as computed in fp64)."""
        torch = self.torch
        Hd = torch.tensor(H, dtype=self.tdt, device=self.dev)
        ddB = torch.full_like(self.B, float("nan"))
        dA2 = torch.full_like(self.A, float("nan"))
        dW2 = torch.full_like(self.W, float("nan"))
        self.sc.sc_double_backward(self.plan, self.N, self.A, self.z, self.W, self.dB, Hd, ddB, dA2, dW2, self.ws,
                                   self.ws_bytes, flags)
        torch.cuda.synchronize()
        if self.wl.dtype == "bf16":
            ddB, dA2 = ddB.float(), dA2.float()
        return ddB.cpu().numpy(), dA2.cpu().numpy(), dW2.cpu().numpy(), Hd.double().cpu().numpy()

    def inputs_as_computed(self):
        """The inputs rounded to the run dtype, as fp64 numpy (what the oracle must see)."""
        return (self.A.double().cpu().numpy(), self.z.cpu().numpy(), self.W.double().cpu().numpy(),
                self.dB.double().cpu().numpy())

    def close(self):
        self.sc.sc_plan_destroy(self.plan)
