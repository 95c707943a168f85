"""Shared helpers for the parity tests (CPU side: oracle calls and error metrics)."""
import numpy as np
import torch

import oracle
import smoe_inputs as si

TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}   # max |gpu - ref| / max |ref| per tensor


def rel_err(gpu, ref) -> float:
    """max_i |gpu_i - ref_i| / max_i |ref_i| (error normalised by the tensor's max-abs)."""
    g = gpu.detach().to(torch.float32).cpu().numpy().astype(np.float64) if isinstance(gpu, torch.Tensor) else np.asarray(gpu, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    assert g.shape == r.shape, (g.shape, r.shape)
    if r.size == 0:
        return 0.0
    assert np.isfinite(g).all(), "non-finite values in GPU result"
    denom = np.abs(r).max()
    return float(np.abs(g - r).max() / (denom if denom > 0 else 1.0))


def assert_close(gpu, ref, dtype, what=""):
    e = rel_err(gpu, ref)
    assert e <= TOL[dtype], f"{what}: relative error {e:.3e} > {TOL[dtype]:.0e}"
    return e


def torch_dtype(name: str):
    return torch.float32 if name == "f32" else torch.bfloat16


def oracle_routing(logits: torch.Tensor, k: int, E: int):
    ei, g = oracle.topk_gate(logits.numpy(), k)
    se, o, off = oracle.route(ei, E)
    return ei, g, se, o, off


def dev(t):
    return t.cuda() if isinstance(t, torch.Tensor) else torch.from_numpy(np.ascontiguousarray(t)).cuda()
