"""Helpers for the GPU parity tests: host arrays -> device tensors and the error metric.

PyTorch is used for device memory only; no torch arithmetic takes part in any comparison
(the float() widening of a bf16 result on its way back to the host is exact).
"""
import numpy as np

import hapgen

TOL = {"bf16": 2e-2, "f32": 1e-5}


def torch_mod():
    import torch
    return torch


def gen(seed, tensor, shape, sigma, dtype):
    """Returns (float64 host values exactly as the device will see them, device tensor)."""
    torch = torch_mod()
    if dtype == "bf16":
        vals, bits = hapgen.normal_bf16(seed, tensor, shape, sigma)
        dev = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
        return vals.astype(np.float64), dev
    vals = hapgen.normal(seed, tensor, shape, sigma, dtype=np.float32)
    return vals.astype(np.float64), torch.from_numpy(vals).cuda()


def upload(vals64, dtype):
    """Uploads host float64 values that are already representable in dtype."""
    torch = torch_mod()
    t = torch.from_numpy(np.ascontiguousarray(vals64, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def empty(shape, dtype, fill=None):
    torch = torch_mod()
    td = {"bf16": torch.bfloat16, "f32": torch.float32, "u8": torch.uint8}[dtype]
    t = torch.empty(shape, dtype=td, device="cuda")
    if fill is not None:
        t.fill_(fill)
    return t


def host(t):
    torch = torch_mod()
    torch.cuda.synchronize()
    return t.detach().float().cpu().numpy().astype(np.float64)


def relerr(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    if not np.isfinite(got).all():
        return float("inf")
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def check(name, got, ref, dtype):
    e = relerr(got, ref)
    print(f"parity {name}: max|err|/max|ref| = {e:.3e} (bar {TOL[dtype]:.0e})")
    assert e <= TOL[dtype], f"{name}: max|err|/max|ref| = {e:.3e} > {TOL[dtype]:.0e}"
    return e
