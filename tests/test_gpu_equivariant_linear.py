"""Parity of the per-order channel-mixing linear (el_forward / el_backward through the C ABI,
MFMA kernels and the plain fallback) with the fp64 CPU oracle.  Tolerances as everywhere: fp32
max|err|/rms(ref) <= 1e-5 per output tensor, fp64 max(|err| / max(|ref|, rms(ref))) <= 1e-12."""
import sys

import numpy as np
import pytest

from oracle import equivariant_linear as oel
from paper_2504_10700_amd import workloads
from gpu_util import check

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def el():
    import torch
    assert torch.cuda.is_available()
    from paper_2504_10700_amd import el_binding
    return el_binding


def run_case(el, N, k_in, k_out, l_max, dtype, seed):
    import torch
    print(f"case N={N} k_in={k_in} k_out={k_out} l_max={l_max} {dtype}", flush=True)
    sys.stdout.flush()
    dev = torch.device("cuda:0")
    tdt = torch.float32 if dtype == "f32" else torch.float64
    X, W, dY = workloads.make_linear_inputs(N, k_in, k_out, l_max, seed)
    Xd, Wd, dYd = (torch.tensor(x, dtype=tdt, device=dev) for x in (X, W, dY))
    cfg = el.make_config(k_in, k_out, l_max, el.SC_F32 if dtype == "f32" else el.SC_F64)
    Y = torch.full((N, k_out, (l_max + 1) ** 2), float("nan"), dtype=tdt, device=dev)
    dX, dW = torch.full_like(Xd, float("nan")), torch.full_like(Wd, float("nan"))
    nbytes = el.el_workspace_bytes(cfg, N)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    el.el_forward(cfg, N, Xd, Wd, Y)
    el.el_backward(cfg, N, Xd, Wd, dYd, dX, dW, ws, nbytes)
    torch.cuda.synchronize()
    X64, W64, dY64 = (x.double().cpu().numpy() for x in (Xd, Wd, dYd))
    errs = [check("Y", Y.cpu().numpy(), oel.forward(X64, W64), dtype)]
    dX_ref, dW_ref = oel.backward(X64, W64, dY64)
    errs.append(check("dX", dX.cpu().numpy(), dX_ref, dtype))
    errs.append(check("dW", dW.cpu().numpy(), dW_ref, dtype))
    print("  errors Y, dX, dW: " + ", ".join(f"{e:.2e}" for e in errs), flush=True)
    Y2, dX2, dW2 = torch.empty_like(Y), torch.empty_like(dX), torch.empty_like(dW)
    el.el_forward(cfg, N, Xd, Wd, Y2)
    el.el_backward(cfg, N, Xd, Wd, dYd, dX2, dW2, ws, nbytes)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2) and torch.equal(dX, dX2) and torch.equal(dW, dW2), "not reproducible"


@pytest.mark.parametrize("dtype", ["f32", "f64"])
@pytest.mark.parametrize("l_max", [0, 1, 2, 3])
def test_mfma_kernels_small(el, dtype, l_max):
    # 333 atoms: 20 full row tiles and a ragged one, several ranges in the dW kernel
    run_case(el, 333, 128, 128, l_max, dtype, 8000 + l_max)


@pytest.mark.parametrize("k_in,k_out", [(64, 192), (256, 64), (128, 256), (4, 64)])
def test_mfma_kernels_other_channel_counts(el, k_in, k_out):
    run_case(el, 90, k_in, k_out, 3, "f32", 8100 + k_in)
    run_case(el, 50, k_in, k_out, 1, "f64", 8200 + k_out)


@pytest.mark.parametrize("k_in,k_out", [(96, 40), (7, 5), (128, 100)])
def test_plain_fallback(el, k_in, k_out):
    run_case(el, 70, k_in, k_out, 3, "f32", 8300 + k_in)
    run_case(el, 33, k_in, k_out, 2, "f64", 8400 + k_out)


def test_degenerate_sizes_and_errors(el):
    import torch
    run_case(el, 1, 128, 128, 3, "f32", 8501)
    run_case(el, 16, 128, 128, 3, "f32", 8502)
    cfg = el.make_config(128, 128, 3)
    dW = torch.full((4, 128, 128), float("nan"), device="cuda:0")
    el.el_forward(cfg, 0, None, None, None)
    el.el_backward(cfg, 0, None, None, None, None, dW, None, 0)
    torch.cuda.synchronize()
    assert not dW.cpu().numpy().any()
    X = torch.zeros((8, 128, 16), device="cuda:0")
    W = torch.zeros((4, 128, 128), device="cuda:0")
    with pytest.raises(el.ScError) as e:
        el.el_backward(cfg, 8, X, W, X, X.clone(), dW, None, 0)
    assert e.value.status == 3
    with pytest.raises(el.ScError) as e:
        el.el_forward(cfg, 8, X.data_ptr() + 4, W, X.clone())
    assert e.value.status == 1


def test_full_size(el):
    # the shape bench.py times: 10 000 atoms, 128 -> 128 channels, l <= 3
    run_case(el, 10_000, 128, 128, 3, "f32", 8601)
