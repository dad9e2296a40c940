"""Helpers shared by the GPU parity tests: error metrics and tensor marshalling.

Parity metric (stated tolerance of the path): per output tensor
    E_inf = max_i |gpu_i - oracle_i| / max_j |oracle_j|   <=  1e-2 (bf16 storage, fp32 accumulate)
                                                           <=  1e-4 (fp32 path)
An element-wise relative error is undefined on post-ReLU tensors (half the entries are zero).
"""
import numpy as np
import torch

TOL = {torch.bfloat16: 1e-2, torch.float32: 1e-4}
DEV = "cuda:0"


def to_dev(a, dtype):
    """numpy -> device tensor of the storage dtype (round-to-nearest-even for bf16)."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.float32).to(dtype).to(DEV)


def as64(t):
    """device tensor -> float64 numpy (exact widening of the stored values)."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def einf(gpu, ora, ignore=None):
    gpu = np.asarray(gpu, dtype=np.float64)
    ora = np.asarray(ora, dtype=np.float64)
    assert gpu.shape == ora.shape, (gpu.shape, ora.shape)
    assert np.all(np.isfinite(gpu)), "non-finite values in the GPU result"
    diff = np.abs(gpu - ora)
    if ignore is not None:
        diff = np.where(ignore, 0.0, diff)
    scale = np.max(np.abs(ora))
    return float(np.max(diff) / scale) if scale > 0 else float(np.max(diff))


def e2(gpu, ora):
    gpu = np.asarray(gpu, dtype=np.float64)
    ora = np.asarray(ora, dtype=np.float64)
    n = np.linalg.norm(ora)
    return float(np.linalg.norm(gpu - ora) / n) if n > 0 else float(np.linalg.norm(gpu - ora))


def check(gpu, ora, dtype, what, ignore=None, tol=None):
    tol = TOL[dtype] if tol is None else tol
    e = einf(gpu, ora, ignore)
    assert e <= tol, f"{what}: E_inf = {e:.3e} > {tol:g} (E2 = {e2(gpu, ora):.3e})"
    return e
