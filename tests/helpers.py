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


def row_rel_err(gpu, ref) -> float:
    """Largest per-row error, each row of the last axis normalised by that row's own max-abs: a wrong row of
    small magnitude cannot hide behind the tensor's largest entry.  Rows whose reference is all zero must be
    zero.  Meant for rows that are sums of one scale (outputs of a product); short rows such as the [T, k]
    routing-weight gradients are judged on the tensor's scale only."""
    g = gpu.detach().to(torch.float32).cpu().numpy().astype(np.float64) if isinstance(gpu, torch.Tensor) else np.asarray(gpu, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    if r.size == 0:
        return 0.0
    g, r = g.reshape(-1, g.shape[-1]), r.reshape(-1, r.shape[-1])
    scale = np.abs(r).max(axis=1)
    err = np.abs(g - r).max(axis=1)
    assert (err[scale == 0] == 0).all(), "a row that must be zero is not"
    nz = scale > 0
    return float((err[nz] / scale[nz]).max()) if nz.any() else 0.0


ROW_MIN_WIDTH = 16


def assert_close(gpu, ref, dtype, what=""):
    e = rel_err(gpu, ref)
    assert e <= TOL[dtype], f"{what}: relative error {e:.3e} > {TOL[dtype]:.0e}"
    r = np.asarray(ref)
    if r.ndim >= 2 and r.shape[-1] >= ROW_MIN_WIDTH:
        er = row_rel_err(gpu, ref)
        assert er <= TOL[dtype], f"{what}: per-row relative error {er:.3e} > {TOL[dtype]:.0e}"
    return e


def torch_dtype(name: str):
    return torch.float32 if name == "f32" else torch.bfloat16


def oracle_routing(logits: torch.Tensor, k: int, E: int):
    ei, g = oracle.topk_gate(logits.numpy(), k)
    se, o, off = oracle.route(ei, E)
    return ei, g, se, o, off


def oracle_gates_f32(g):
    """The oracle's own gates rounded once to fp32, the precision the routing weights are stored in
    (the checker's inputs never come from the GPU; the GPU's gates are compared with these at 1e-6)."""
    return np.asarray(g, dtype=np.float64).astype(np.float32).astype(np.float64)


def dev(t):
    return t.cuda() if isinstance(t, torch.Tensor) else torch.from_numpy(np.ascontiguousarray(t)).cuda()
