"""Seeded synthetic inputs shared by the oracle-side tests and the HIP path.

This module only draws random tensors and fits router biases; none of the
method's arithmetic (expert transforms, activations, sorting, gradients) lives
here, so the CPU oracle and the GPU library can both be fed from it without
sharing any code of their own.

Tensors come back as CPU torch tensors in their storage dtype (fp32, or bf16
obtained by one round-to-nearest-even of the fp32 draw).  `as_f64` turns any of
them into the exact float64 numpy array the oracle consumes.

Workloads follow the Mixtral-style SMoE MLP shapes the paper benchmarks
(Sec. 4 and 4.1: d_model 1024..4096, k = 2..8, E = 8k); the real model weights
and corpora are not used, values are N(0,1) activations / N(0,0.02) weights.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import numpy as np
import torch

ACT_NONE, ACT_GELU, ACT_SWIGLU = 0, 1, 2


@dataclass(frozen=True)
class MLPConfig:
    name: str
    T: int
    d_model: int
    d_expert: int
    E: int
    k: int
    act: int
    dtype: str = "bf16"          # "f32" or "bf16"
    zipf_s: float = 0.0          # >0: expert loads follow Zipf(s) via a fitted router bias
    masked_experts: int = 0      # this many highest-numbered experts get -inf logits (never chosen)

    @property
    def d_h(self) -> int:
        return 2 * self.d_expert if self.act == ACT_SWIGLU else self.d_expert

    @property
    def Tk(self) -> int:
        return self.T * self.k

    def gemm_flops_fwd(self) -> float:
        return 2.0 * self.Tk * self.d_model * (self.d_h + self.d_expert)


CONFIGS = {
    # the five workloads of the benchmark plan
    "C1": MLPConfig("C1", 256, 64, 128, 4, 2, ACT_GELU, "f32"),
    "C2": MLPConfig("C2", 4096, 1024, 2816, 8, 2, ACT_SWIGLU),
    "C3": MLPConfig("C3", 16384, 4096, 14336, 8, 2, ACT_SWIGLU, zipf_s=1.2),
    "C4": MLPConfig("C4", 8192, 2048, 512, 64, 8, ACT_SWIGLU),
    "C4-decode": MLPConfig("C4-decode", 64, 2048, 512, 64, 8, ACT_SWIGLU),
    "C4-decode-masked": MLPConfig("C4-decode-masked", 64, 2048, 512, 64, 8, ACT_SWIGLU, masked_experts=16),
    # reduced C3 (all dims / 16, Zipf loads kept) that the oracle finishes whole in seconds
    "C3-small": MLPConfig("C3-small", 1024, 256, 896, 8, 2, ACT_SWIGLU, zipf_s=1.2),
    "C3-small-f32": MLPConfig("C3-small-f32", 1024, 256, 896, 8, 2, ACT_SWIGLU, "f32", zipf_s=1.2),
}
# Unit-benchmark shapes of Sec. 4.1 / 4.2: d_model = 4096, d_ff = 2 d_model active hidden units,
# d_expert = d_ff / k, E = 8k, T = 30 * 2048 tokens, granularity k in {1, 2, 4, 8, 16}; "G-dense" is
# the dense MLP with the same active parameters (one expert of width d_ff that every token uses).
GRANULARITY_KS = (1, 2, 4, 8, 16)
for _k in GRANULARITY_KS:
    CONFIGS[f"G{_k}"] = MLPConfig(f"G{_k}", 30 * 2048, 4096, 8192 // _k, 8 * _k, _k, ACT_GELU)
CONFIGS["G-dense"] = MLPConfig("G-dense", 30 * 2048, 4096, 8192, 1, 1, ACT_GELU)
# Decreasing sparsity, Sec. 4.3: E = 64 experts of the unit benchmark's width at E = 64 (d_expert = 1024), k growing
# to 30; "S-dense" is the fully dense MLP holding all E * d_expert hidden units.
SPARSITY_KS = (1, 2, 4, 8, 16, 30)
for _k in SPARSITY_KS:
    CONFIGS[f"S{_k}"] = MLPConfig(f"S{_k}", 30 * 2048, 4096, 1024, 64, _k, ACT_GELU)
CONFIGS["S-dense"] = MLPConfig("S-dense", 30 * 2048, 4096, 64 * 1024, 1, 1, ACT_GELU)

# Mixture-of-Attention projections (Alg. 4): W_Q [E,d_model,d_out], W_O [E,d_out,d_model]
MOA_C5 = dict(T=8192, d_model=2048, E=16, k=4, d_out=512)


def _gen(seed: int, tensor_id: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed((int(seed) * 1000003 + tensor_id * 7919 + 12345) & 0x7FFFFFFFFFFF)
    return g


def normal(shape, std: float, seed: int, tensor_id: int, dtype: str) -> torch.Tensor:
    """N(0, std) draw in fp32, stored as fp32 or rounded once (RNE) to bf16."""
    x = torch.randn(*shape, generator=_gen(seed, tensor_id), dtype=torch.float32)
    if std != 1.0:
        x.mul_(std)
    if dtype == "bf16":
        return x.to(torch.bfloat16)
    if dtype == "f32":
        return x
    raise ValueError(dtype)


def as_f64(t) -> np.ndarray:
    """Exact float64 copy of a tensor (bf16 and fp32 values are representable)."""
    if isinstance(t, torch.Tensor):
        if t.dtype in (torch.int32, torch.int64):
            return t.numpy()
        return t.to(torch.float32).numpy().astype(np.float64)
    return np.asarray(t, dtype=np.float64)


def as_f32(t: torch.Tensor) -> np.ndarray:
    """Exact float32 numpy view of a tensor (half the memory of as_f64, same values)."""
    return t.to(torch.float32).numpy()


def zipf_shares(E: int, s: float) -> np.ndarray:
    w = 1.0 / np.arange(1, E + 1, dtype=np.float64) ** s
    return w / w.sum()


def _topk_loads(logits: np.ndarray, k: int) -> np.ndarray:
    """Share of routed slots per expert when every token keeps its k largest logits."""
    E = logits.shape[1]
    top = np.argpartition(-logits, k - 1, axis=1)[:, :k]
    return np.bincount(top.reshape(-1), minlength=E) / float(top.size)


def fit_router_bias(base_logits: np.ndarray, k: int, target: np.ndarray, iters: int = 300) -> np.ndarray:
    """Per-expert bias b so that top-k routing of base_logits + b has loads ~ target.

    Damped fixed point on log-loads; it only shapes the synthetic input (the
    imbalance of the workload), the router itself is computed elsewhere.
    """
    b = np.zeros(base_logits.shape[1], dtype=np.float64)
    for _ in range(iters):
        load = np.maximum(_topk_loads(base_logits + b, k), 1e-6)
        b += 0.5 * (np.log(target) - np.log(load))
        b -= b[0]
    return b


def router_logits(cfg: MLPConfig, seed: int) -> torch.Tensor:
    """[T,E] fp32 logits ~ N(0,1), plus the Zipf bias / expert mask the config asks for."""
    logits = torch.randn(cfg.T, cfg.E, generator=_gen(seed, 1), dtype=torch.float32)
    if cfg.zipf_s > 0:
        b = fit_router_bias(logits.numpy().astype(np.float64), cfg.k, zipf_shares(cfg.E, cfg.zipf_s))
        logits = logits + torch.from_numpy(b.astype(np.float32))
    if cfg.masked_experts > 0:
        logits[:, cfg.E - cfg.masked_experts:] = -float("inf")
    return logits


def mlp_case(cfg: MLPConfig, seed: int = 0, with_grad: bool = True) -> dict:
    """All tensors of one SMoE MLP problem: X, W1, W2, logits, and the upstream gradient dY."""
    case = dict(cfg=cfg)
    case["logits"] = router_logits(cfg, seed)
    case["X"] = normal((cfg.T, cfg.d_model), 1.0, seed, 2, cfg.dtype)
    case["W1"] = normal((cfg.E, cfg.d_model, cfg.d_h), 0.02, seed, 3, cfg.dtype)
    case["W2"] = normal((cfg.E, cfg.d_expert, cfg.d_model), 0.02, seed, 4, cfg.dtype)
    if with_grad:
        case["dY"] = normal((cfg.T, cfg.d_model), 1.0, seed, 5, cfg.dtype)
    return case


def custom(name="custom", **kw) -> MLPConfig:
    base = MLPConfig(name, 64, 32, 32, 4, 2, ACT_GELU, "f32")
    return replace(base, **kw)


def plinear_case(T, d_in, d_out, E, k, dtype="f32", seed=0, x_rows=None, zipf_s=0.0) -> dict:
    """Tensors for one ParallelLinear call: logits, X [x_rows,d_in], W [E,d_in,d_out], dY rows.
    zipf_s > 0 adds the fitted per-expert bias that makes the expert loads follow Zipf(s)."""
    x_rows = T if x_rows is None else x_rows
    logits = torch.randn(T, E, generator=_gen(seed, 11), dtype=torch.float32)
    if zipf_s > 0:
        b = fit_router_bias(logits.numpy().astype(np.float64), k, zipf_shares(E, zipf_s), iters=100)
        logits = logits + torch.from_numpy(b.astype(np.float32))
    return dict(
        logits=logits,
        X=normal((x_rows, d_in), 1.0, seed, 12, dtype),
        W=normal((E, d_in, d_out), 1.0 / math.sqrt(d_in), seed, 13, dtype),
        dY_T=normal((T, d_out), 1.0, seed, 14, dtype),
        dY_Tk=normal((T * k, d_out), 1.0, seed, 15, dtype),
    )
