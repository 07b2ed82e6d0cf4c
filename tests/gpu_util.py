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


def check(name, got, ref, dtype):
    if dtype == "f32":
        err, tol = rel_err_f32(got, ref), F32_TOL
    else:
        err, tol = rel_err_f64(got, ref), F64_TOL
    assert err <= tol, f"{name}: error {err:.3e} exceeds {tol:.1e}"
    return err


class GpuRun:
    """Device buffers + plan for one workload; forward()/backward() return numpy arrays."""

    def __init__(self, sc, wl, inp, flags=0, n_nodes=None):
        import torch
        self.sc, self.wl, self.torch = sc, wl, torch
        self.dev = torch.device("cuda:0")
        self.tdt = torch.float32 if wl.dtype == "f32" else torch.float64
        self.plan = sc.sc_plan_create(wl.num_channels, wl.l_max, wl.nu_max, wl.num_elements, wl.out_irreps,
                                      sc.SC_F32 if wl.dtype == "f32" else sc.SC_F64, 0, flags)
        self.N = inp.A.shape[0] if n_nodes is None else n_nodes
        self.A = torch.tensor(inp.A, dtype=self.tdt, device=self.dev)
        self.W = torch.tensor(inp.W, dtype=self.tdt, device=self.dev)
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
        return self.B.cpu().numpy()

    def backward(self, flags=0):
        self.sc.sc_backward(self.plan, self.N, self.A, self.z, self.W, self.dB, self.dA, self.dW, self.ws,
                            self.ws_bytes, flags)
        self.torch.cuda.synchronize()
        return self.dA.cpu().numpy(), self.dW.cpu().numpy()

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
        return ddB.cpu().numpy(), dA2.cpu().numpy(), dW2.cpu().numpy(), Hd.double().cpu().numpy()

    def inputs_as_computed(self):
        """The inputs rounded to the run dtype, as fp64 numpy (what the oracle must see)."""
        return (self.A.double().cpu().numpy(), self.z.cpu().numpy(), self.W.double().cpu().numpy(),
                self.dB.double().cpu().numpy())

    def close(self):
        self.sc.sc_plan_destroy(self.plan)
