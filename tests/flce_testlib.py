"""Shared helpers of the GPU parity tests: upload a workload, call the C ABI
through the Python binding, compare with the CPU oracle at the stated bars."""
import numpy as np
import torch

import workloads

# Tolerances (relative loss error, gradient max-abs error relative to max|ref|).
TOL = {"f32": (1e-5, 1e-4), "bf16": (2e-3, 2e-2)}


def to_device(a: np.ndarray, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        bits = workloads.bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def upload(w):
    return to_device(w.X, w.dtype), to_device(w.W, w.dtype), torch.from_numpy(w.targets).cuda()


def run_gpu(w, flags=0, poison=True):
    import paper_2410_10989_amd as flce
    X, W, t = upload(w)
    dX = torch.empty_like(X)
    dW = torch.empty_like(W)
    loss = torch.empty((), dtype=torch.float32, device="cuda")
    if poison:   # outputs must be fully overwritten
        dX.fill_(float("nan"))
        dW.fill_(float("nan"))
        loss.fill_(float("nan"))
    flce.flce_fwd_bwd(X, W, t, w.ignore_index, loss=loss, dX=dX, dW=dW, flags=flags)
    torch.cuda.synchronize()
    return float(loss.item()), dX, dW


def assert_close(name, got: np.ndarray, ref: np.ndarray, rel_to_max: float, ref_max=None):
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{name}: non-finite values"
    scale = float(np.abs(ref).max()) if ref_max is None else float(ref_max)
    err = float(np.abs(got - ref).max()) if got.size else 0.0
    bound = rel_to_max * scale
    assert err <= bound or (scale == 0.0 and err == 0.0), \
        f"{name}: max-abs error {err:.3e} > {rel_to_max:g} x max|ref| = {bound:.3e}"
    return err / scale if scale > 0 else 0.0


def assert_loss(got: float, ref: float, rel: float):
    assert np.isfinite(got), "loss is not finite"
    assert abs(got - ref) <= rel * abs(ref) or (ref == 0.0 and got == 0.0), \
        f"loss {got!r} vs oracle {ref!r}: rel err {abs(got - ref) / max(abs(ref), 1e-300):.3e} > {rel:g}"
