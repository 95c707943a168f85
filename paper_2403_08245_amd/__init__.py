"""Python binding of libsmoe (ScatterMoE's ParallelLinear hot path on MI355X).

Argument marshalling only: every function here checks tensor dtypes/contiguity, allocates
outputs and scratch with torch, and calls the C entry point of the same name
(smoe_<name>, declared in include/smoe.h) on torch's current HIP stream.  There is no
Python or PyTorch fallback: if libsmoe.so is missing, importing this package fails.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

ACT_NONE, ACT_GELU, ACT_SWIGLU = 0, 1, 2
F32, BF16 = 0, 1

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsmoe.so")

EXPORTS = [
    "smoe_create", "smoe_destroy", "smoe_strerror", "smoe_abi_version", "smoe_set_kernel_mode", "smoe_set_clock_probe", "smoe_set_tile_group",
    "smoe_topk_gate", "smoe_topk_gate_bwd", "smoe_route_workspace_bytes", "smoe_route", "smoe_route_noalloc",
    "smoe_plinear_fwd", "smoe_plinear_bwd_workspace_bytes", "smoe_plinear_bwd",
    "smoe_plinear_act_fwd_workspace_bytes", "smoe_plinear_act_fwd", "smoe_mlp_fwd_workspace_bytes", "smoe_mlp_fwd", "smoe_mlp_saves_yhat", "smoe_mlp_bwd_workspace_bytes", "smoe_mlp_bwd",
    "smoe_group", "smoe_attention_fwd", "smoe_attention_bwd_workspace_bytes", "smoe_attention_bwd",
    "smoe_momha_fwd_workspace_bytes", "smoe_momha_fwd", "smoe_momha_bwd_workspace_bytes", "smoe_momha_bwd",
]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} not found: build it first (python __graft_entry__.py); "
            "this package has no fallback path")
    return ctypes.CDLL(LIB_PATH)


lib = _load()

_vp, _i, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t


class smoe_routing(ctypes.Structure):
    _fields_ = [("sorted_expert_idxs", _vp), ("sorted_scattered_idxs", _vp), ("expert_offsets", _vp),
                ("Tk", ctypes.c_int32), ("E", ctypes.c_int32)]


_rp = ctypes.POINTER(smoe_routing)
lib.smoe_create.argtypes = [ctypes.POINTER(_vp), _i]
lib.smoe_destroy.argtypes = [_vp]
lib.smoe_destroy.restype = None
lib.smoe_strerror.argtypes = [_i]
lib.smoe_strerror.restype = ctypes.c_char_p
lib.smoe_set_kernel_mode.argtypes = [_vp, _i]
lib.smoe_set_clock_probe.argtypes = [_vp, _vp]
lib.smoe_set_tile_group.argtypes = [_vp, _i]
lib.smoe_topk_gate.argtypes = [_vp, _vp, _vp, _i, _i, _i, _vp, _vp]
lib.smoe_topk_gate_bwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _vp]
lib.smoe_attention_fwd.argtypes = [_vp, _vp, _i, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _vp]
lib.smoe_attention_bwd_workspace_bytes.argtypes = [_i, _i, _i, _i]
lib.smoe_attention_bwd_workspace_bytes.restype = _sz
lib.smoe_attention_bwd.argtypes = [_vp, _vp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _sz]
lib.smoe_momha_fwd_workspace_bytes.argtypes = [_i] * 7
lib.smoe_momha_fwd_workspace_bytes.restype = _sz
lib.smoe_momha_fwd.argtypes = [_vp, _vp, _i, _vp, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _rp, _i, _vp, _vp,
                               _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz]
lib.smoe_momha_bwd_workspace_bytes.argtypes = [_i] * 6
lib.smoe_momha_bwd_workspace_bytes.restype = _sz
lib.smoe_momha_bwd.argtypes = [_vp, _vp, _i, _vp, _vp, _i, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _rp, _i, _vp,
                               _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz]
lib.smoe_route_workspace_bytes.argtypes = [_i, _i, _i]
lib.smoe_route_workspace_bytes.restype = _sz
lib.smoe_route.argtypes = [_vp, _vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _sz]
lib.smoe_route_noalloc.argtypes = [_vp, _vp, _vp, _i, _i, _i, _vp, _vp, _vp]
lib.smoe_plinear_fwd.argtypes = [_vp, _vp, _i, _vp, _i, _i, _vp, _i, _rp, _i, _vp, _i, _i, _i, _vp, _vp]
lib.smoe_plinear_bwd_workspace_bytes.argtypes = [_i] * 9
lib.smoe_plinear_bwd_workspace_bytes.restype = _sz
lib.smoe_plinear_bwd.argtypes = [_vp, _vp, _i, _vp, _vp, _i, _i, _vp, _i, _vp, _rp, _i, _vp, _i, _i, _i,
                                 _vp, _vp, _vp, _vp, _sz]
lib.smoe_plinear_act_fwd_workspace_bytes.argtypes = [_i] * 7
lib.smoe_plinear_act_fwd_workspace_bytes.restype = _sz
lib.smoe_plinear_act_fwd.argtypes = [_vp, _vp, _i, _i, _vp, _i, _i, _i, _vp, _rp, _i, _vp, _vp, _vp, _sz]
lib.smoe_mlp_fwd_workspace_bytes.argtypes = [_i] * 7
lib.smoe_mlp_fwd_workspace_bytes.restype = _sz
lib.smoe_mlp_fwd.argtypes = [_vp, _vp, _i, _i, _vp, _i, _i, _i, _vp, _vp, _rp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _sz]
lib.smoe_mlp_bwd_workspace_bytes.argtypes = [_i] * 6
lib.smoe_mlp_saves_yhat.argtypes = [_vp, _i, _i, _i, _i, _i, _i, _i]
lib.smoe_mlp_bwd_workspace_bytes.restype = _sz
lib.smoe_mlp_bwd.argtypes = [_vp, _vp, _i, _i, _vp, _vp, _i, _i, _i, _vp, _vp, _rp, _i, _vp, _vp, _vp, _vp,
                             _vp, _vp, _vp, _vp, _vp, _sz]
lib.smoe_group.argtypes = [_vp, _vp, _i, _vp, _i, _rp, _i, _vp, _vp]


class SmoeError(RuntimeError):
    pass


def _check(rc: int, what: str):
    if rc != 0:
        raise SmoeError(f"{what}: {lib.smoe_strerror(rc).decode()} ({rc})")


_ctx_by_device: dict[int, ctypes.c_void_p] = {}


def ctx(device: int | None = None) -> ctypes.c_void_p:
    """The library context of a device (created on first use)."""
    dev = torch.cuda.current_device() if device is None else device
    if dev not in _ctx_by_device:
        h = _vp()
        _check(lib.smoe_create(ctypes.byref(h), dev), "smoe_create")
        _ctx_by_device[dev] = h
    return _ctx_by_device[dev]


def set_kernel_mode(mode: int):
    _check(lib.smoe_set_kernel_mode(ctx(), mode), "smoe_set_kernel_mode")


def set_tile_group(group_m: int):
    _check(lib.smoe_set_tile_group(ctx(), group_m), "smoe_set_tile_group")


def set_clock_probe(buf: torch.Tensor | None):
    """Device int64 tensor of 512 entries that the persistent scatter2scatter kernels report their clocks to
    (see smoe_set_clock_probe), or None to turn the probe off."""
    if buf is not None and (buf.dtype != torch.int64 or buf.numel() < 512 or not buf.is_cuda):
        raise ValueError("need a device int64 tensor of 512 entries")
    _check(lib.smoe_set_clock_probe(ctx(), _p(buf)), "smoe_set_clock_probe")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _p(t):
    return None if t is None else t.data_ptr()


def _chk(t: torch.Tensor, dtype=None):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return t


def _new(*shape, dtype, device) -> torch.Tensor:
    """Every output and scratch tensor of this binding comes from here (uninitialised device memory).
    Tests replace this one function to poison new tensors and to put guard bands around them."""
    return torch.empty(*shape, dtype=dtype, device=device)


def _like(t: torch.Tensor) -> torch.Tensor:
    return _new(*t.shape, dtype=t.dtype, device=t.device)


def _ws(nbytes: int, device) -> torch.Tensor | None:
    return _new(max(nbytes, 256), dtype=torch.uint8, device=device)


@dataclass
class Routing:
    """Device arrays of Sec. 3.1 step 2 plus the ctypes view the C ABI takes."""
    sorted_expert_idxs: torch.Tensor
    sorted_scattered_idxs: torch.Tensor
    expert_offsets: torch.Tensor
    Tk: int
    E: int

    def c(self) -> smoe_routing:
        return smoe_routing(self.sorted_expert_idxs.data_ptr(), self.sorted_scattered_idxs.data_ptr(),
                            self.expert_offsets.data_ptr(), self.Tk, self.E)


def topk_gate(logits: torch.Tensor, k: int):
    _chk(logits, torch.float32)
    T, E = logits.shape
    idx = _new(T, k, dtype=torch.int32, device=logits.device)
    gates = _new(T, k, dtype=torch.float32, device=logits.device)
    _check(lib.smoe_topk_gate(ctx(), _stream(), _p(logits), T, E, k, _p(idx), _p(gates)), "smoe_topk_gate")
    return idx, gates


def topk_gate_bwd(expert_idxs: torch.Tensor, gates: torch.Tensor, dgates: torch.Tensor, E: int) -> torch.Tensor:
    _chk(expert_idxs, torch.int32)
    _chk(gates, torch.float32)
    _chk(dgates, torch.float32)
    T, k = expert_idxs.shape
    if gates.numel() != T * k or dgates.numel() != T * k:
        raise ValueError("gates and dgates must hold T*k entries")
    dlogits = _new(T, E, dtype=torch.float32, device=gates.device)
    _check(lib.smoe_topk_gate_bwd(ctx(), _stream(), _p(expert_idxs), _p(gates), _p(dgates), T, E, k, _p(dlogits)),
           "smoe_topk_gate_bwd")
    return dlogits


def attention_fwd(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor):
    """Q [B,T,G,h,d], K and V [B,T,h,d] (bf16) -> O like Q, LSE [B,T,G,h] fp32."""
    for t in (Q, K, V):
        _chk(t, torch.bfloat16)
    B, T, G, h, d = Q.shape
    if K.shape != (B, T, h, d) or V.shape != K.shape:
        raise ValueError("K and V must be [B, T, h, d]")
    O = _like(Q)
    LSE = _new(B, T, G, h, dtype=torch.float32, device=Q.device)
    _check(lib.smoe_attention_fwd(ctx(), _stream(), BF16, _p(Q), _p(K), _p(V), B, T, G, h, d, _p(O), _p(LSE)),
           "smoe_attention_fwd")
    return O, LSE


def attention_bwd(dO, Q, K, V, O, LSE):
    for t in (dO, Q, K, V, O):
        _chk(t, torch.bfloat16)
    _chk(LSE, torch.float32)
    B, T, G, h, d = Q.shape
    dQ, dK, dV = _like(Q), _like(K), _like(V)
    nb = lib.smoe_attention_bwd_workspace_bytes(B, T, G, h)
    ws = _ws(nb, Q.device)
    _check(lib.smoe_attention_bwd(ctx(), _stream(), BF16, _p(dO), _p(Q), _p(K), _p(V), _p(O), _p(LSE), B, T, G, h, d,
                                  _p(dQ), _p(dK), _p(dV), _p(ws), nb), "smoe_attention_bwd")
    return dQ, dK, dV


@dataclass
class MomhaBuffers:
    """Tensors smoe_momha_fwd keeps for the backward pass (Alg. 4's intermediates)."""
    K: torch.Tensor
    V: torch.Tensor
    Q: torch.Tensor
    Ohat: torch.Tensor
    LSE: torch.Tensor
    Yhat: torch.Tensor


def momha_fwd(X, W_K, W_V, W_Q, W_O, r: Routing, k: int, gates, B: int, T: int, h_expert: int, d_head: int):
    for t in (X, W_K, W_V, W_Q, W_O):
        _chk(t, torch.bfloat16)
    _chk(gates, torch.float32)
    N, d_model = X.shape
    d_out = h_expert * d_head
    dev = X.device
    bf = dict(dtype=torch.bfloat16, device=dev)
    buf = MomhaBuffers(_new(N, d_out, **bf), _new(N, d_out, **bf), _new(N * k, d_out, **bf),
                       _new(N * k, d_out, **bf), _new(N * k, h_expert, dtype=torch.float32, device=dev),
                       _new(N * k, d_model, **bf))
    O = _new(N, d_model, **bf)
    nb = lib.smoe_momha_fwd_workspace_bytes(B, T, k, d_model, h_expert, d_head, 1)
    ws = _ws(nb, dev)
    rc = r.c()
    _check(lib.smoe_momha_fwd(ctx(), _stream(), BF16, _p(X), B, T, d_model, h_expert, d_head, _p(W_K), _p(W_V),
                              _p(W_Q), _p(W_O), ctypes.byref(rc), k, _p(gates), _p(O), _p(buf.K), _p(buf.V),
                              _p(buf.Q), _p(buf.Ohat), _p(buf.LSE), _p(buf.Yhat), _p(ws), nb), "smoe_momha_fwd")
    return O, buf


def momha_bwd(dO, X, W_K, W_V, W_Q, W_O, r: Routing, k: int, gates, B: int, T: int, h_expert: int, d_head: int,
              buf: MomhaBuffers):
    _chk(dO, torch.bfloat16)
    N, d_model = X.shape
    dX, dW_K, dW_V = _like(X), _like(W_K), _like(W_V)
    dW_Q, dW_O = _like(W_Q), _like(W_O)
    dgates = _new(N, k, dtype=torch.float32, device=X.device)
    nb = lib.smoe_momha_bwd_workspace_bytes(B, T, k, d_model, h_expert, d_head)
    ws = _ws(nb, X.device)
    rc = r.c()
    _check(lib.smoe_momha_bwd(ctx(), _stream(), BF16, _p(dO), _p(X), B, T, d_model, h_expert, d_head, _p(W_K), _p(W_V),
                              _p(W_Q), _p(W_O), ctypes.byref(rc), k, _p(gates), _p(buf.K), _p(buf.V), _p(buf.Q),
                              _p(buf.Ohat), _p(buf.LSE), _p(buf.Yhat), _p(dX), _p(dW_K), _p(dW_V), _p(dW_Q), _p(dW_O),
                              _p(dgates), _p(ws), nb), "smoe_momha_bwd")
    return dX, dW_K, dW_V, dW_Q, dW_O, dgates


def route(expert_idxs: torch.Tensor, E: int) -> Routing:
    _chk(expert_idxs, torch.int32)
    T, k = expert_idxs.shape
    dev = expert_idxs.device
    se = _new(T * k, dtype=torch.int32, device=dev)
    so = _new(T * k, dtype=torch.int32, device=dev)
    off = _new(E + 1, dtype=torch.int32, device=dev)
    nb = lib.smoe_route_workspace_bytes(T, k, E)
    ws = _ws(nb, dev)
    _check(lib.smoe_route(ctx(), _stream(), _p(expert_idxs), T, k, E, _p(se), _p(so), _p(off), _p(ws), ws.numel()),
           "smoe_route")
    return Routing(se, so, off, T * k, E)


def route_noalloc(expert_idxs: torch.Tensor, E: int, out: Routing) -> Routing:
    """smoe_route_noalloc: routing into the caller's arrays `out`, scratch inside the library."""
    _chk(expert_idxs, torch.int32)
    T, k = expert_idxs.shape
    if out.sorted_expert_idxs.numel() < T * k or out.expert_offsets.numel() < E + 1:
        raise ValueError("output arrays too small")
    _check(lib.smoe_route_noalloc(ctx(), _stream(), _p(expert_idxs), T, k, E, _p(out.sorted_expert_idxs),
                                  _p(out.sorted_scattered_idxs), _p(out.expert_offsets)), "smoe_route_noalloc")
    return Routing(out.sorted_expert_idxs, out.sorted_scattered_idxs, out.expert_offsets, T * k, E)


def group(x: torch.Tensor, r: Routing, fan: int, gates: torch.Tensor | None = None) -> torch.Tensor:
    _chk(x)
    out = _new(r.Tk, x.shape[1], dtype=x.dtype, device=x.device)
    rc = r.c()
    _check(lib.smoe_group(ctx(), _stream(), _dt(x), _p(x), x.shape[1], ctypes.byref(rc), fan,
                          _p(None if gates is None else _chk(gates, torch.float32)), _p(out)), "smoe_group")
    return out


def plinear_fwd(X, W, r: Routing, k: int, gates=None, grouped_in=False, grouped_out=False):
    """Alg. 1.  Returns (Y, Yhat); Y is Yhat when no gates are given."""
    _chk(X); _chk(W, X.dtype)
    d_in, d_out = W.shape[1], W.shape[2]
    Yhat = _new(r.Tk, d_out, dtype=X.dtype, device=X.device)
    Y, gk = None, 0
    if gates is not None:
        _chk(gates, torch.float32)
        gk = gates.shape[1]
        Y = _new(r.Tk // gk, d_out, dtype=X.dtype, device=X.device)
    rc = r.c()
    _check(lib.smoe_plinear_fwd(ctx(), _stream(), _dt(X), _p(X), X.shape[0], d_in, _p(W), d_out, ctypes.byref(rc), k,
                                _p(gates), gk, int(grouped_in), int(grouped_out), _p(Yhat), _p(Y)), "smoe_plinear_fwd")
    return (Yhat if Y is None else Y), Yhat


def plinear_bwd(dY, X, W, Yhat, r: Routing, k: int, gates=None, grouped_in=False, grouped_out=False,
                need_dX=True, need_dW=True):
    """Alg. 2.  Returns (dX, dW, dgates)."""
    _chk(dY, X.dtype); _chk(X); _chk(W, X.dtype)
    d_in, d_out = W.shape[1], W.shape[2]
    dX = _like(X) if need_dX else None
    dW = _like(W) if need_dW else None
    dg, gk = None, 0
    if gates is not None:
        _chk(gates, torch.float32)
        gk = gates.shape[1]
        dg = _like(gates)
    nb = lib.smoe_plinear_bwd_workspace_bytes(_dt(X), X.shape[0], d_in, d_out, r.Tk, k, int(gates is not None),
                                              int(grouped_in), int(grouped_out))
    ws = _ws(nb, X.device)
    rc = r.c()
    _check(lib.smoe_plinear_bwd(ctx(), _stream(), _dt(X), _p(dY), _p(X), X.shape[0], d_in, _p(W), d_out, _p(Yhat),
                                ctypes.byref(rc), k, _p(gates), gk, int(grouped_in), int(grouped_out), _p(dX), _p(dW),
                                _p(dg), _p(ws), ws.numel()), "smoe_plinear_bwd")
    return dX, dW, dg


def hidden_width(act: int, d_expert: int) -> int:
    return 2 * d_expert if act == ACT_SWIGLU else d_expert


def plinear_act_fwd(X, W1, r: Routing, k: int, act: int, keep_hpre=True, out=None, ws=None):
    """Alg. 3 lines 1-2: returns (H, Hpre or None) in expert-sorted order.  `out` = (H, Hpre) and `ws` reuse
    preallocated tensors (repeated calls then allocate nothing)."""
    _chk(X); _chk(W1, X.dtype)
    T, d_model = X.shape
    d_expert = W1.shape[2] // 2 if act == ACT_SWIGLU else W1.shape[2]
    if out is None:
        H = _new(r.Tk, d_expert, dtype=X.dtype, device=X.device)
        Hpre = _new(r.Tk, W1.shape[2], dtype=X.dtype, device=X.device) if keep_hpre else None
    else:
        H, Hpre = out
    nb = lib.smoe_plinear_act_fwd_workspace_bytes(_dt(X), act, T, k, d_model, d_expert, int(Hpre is not None))
    if ws is None:
        ws = _ws(nb, X.device)
    rc = r.c()
    _check(lib.smoe_plinear_act_fwd(ctx(), _stream(), _dt(X), act, _p(X), T, d_model, d_expert, _p(W1), ctypes.byref(rc), k,
                                    _p(Hpre), _p(H), _p(ws), ws.numel()), "smoe_plinear_act_fwd")
    return H, Hpre


class MLPBuffers:
    """Preallocated outputs, saved activations and scratch of one SMoE MLP shape, so that
    repeated calls (training steps, benchmarks) do not allocate."""

    def __init__(self, T, k, E, d_model, d_expert, act, dtype, device, training=True):
        Tk, d_h = T * k, hidden_width(act, d_expert)
        dt = F32 if dtype == torch.float32 else BF16
        mk = lambda *s: _new(*s, dtype=dtype, device=device)
        self.T, self.k, self.E, self.d_model, self.d_expert, self.act, self.dtype = T, k, E, d_model, d_expert, act, dtype
        self.Y = mk(T, d_model)
        self.training = training
        mode = 0
        if training:
            needs = lib.smoe_mlp_saves_yhat(ctx(), dt, act, T, k, E, d_model, d_expert)
            _check(min(needs, 0), "smoe_mlp_saves_yhat")
            mode = 1 if needs else 2
            # the unweighted second product is kept only when the backward pass of this shape reads it
            self.Hpre, self.H, self.Yhat = mk(Tk, d_h), mk(Tk, d_expert), (mk(Tk, d_model) if needs else None)
            self.dX, self.dW1, self.dW2 = mk(T, d_model), mk(E, d_model, d_h), mk(E, d_expert, d_model)
            self.dgates = _new(T, k, dtype=torch.float32, device=device)
            self.ws_bwd = _ws(lib.smoe_mlp_bwd_workspace_bytes(dt, act, T, k, d_model, d_expert), device)
        else:
            self.Hpre = self.H = self.Yhat = None
        self.ws_fwd = _ws(lib.smoe_mlp_fwd_workspace_bytes(dt, act, T, k, d_model, d_expert, mode), device)


def mlp_fwd(X, W1, W2, r: Routing, k: int, gates, act: int, buf: MLPBuffers | None = None, training=True):
    """Alg. 3.  Returns (Y, buf); buf carries the tensors the backward pass needs."""
    _chk(X); _chk(W1, X.dtype); _chk(W2, X.dtype); _chk(gates, torch.float32)
    T, d_model = X.shape
    E, d_expert = W2.shape[0], W2.shape[1]
    if buf is None:
        buf = MLPBuffers(T, k, E, d_model, d_expert, act, X.dtype, X.device, training)
    rc = r.c()
    _check(lib.smoe_mlp_fwd(ctx(), _stream(), _dt(X), act, _p(X), T, d_model, d_expert, _p(W1), _p(W2),
                            ctypes.byref(rc), k, _p(gates), _p(buf.Y), _p(buf.Hpre), _p(buf.H), _p(buf.Yhat),
                            _p(buf.ws_fwd), buf.ws_fwd.numel()), "smoe_mlp_fwd")
    return buf.Y, buf


def mlp_bwd(dY, X, W1, W2, r: Routing, k: int, gates, act: int, buf: MLPBuffers):
    """Backward of mlp_fwd.  Returns (dX, dW1, dW2, dgates), views of buf."""
    _chk(dY, X.dtype)
    T, d_model = X.shape
    d_expert = W2.shape[1]
    rc = r.c()
    _check(lib.smoe_mlp_bwd(ctx(), _stream(), _dt(X), act, _p(dY), _p(X), T, d_model, d_expert, _p(W1), _p(W2),
                            ctypes.byref(rc), k, _p(gates), _p(buf.Hpre), _p(buf.H), _p(buf.Yhat), _p(buf.dX),
                            _p(buf.dW1), _p(buf.dW2), _p(buf.dgates), _p(buf.ws_bwd), buf.ws_bwd.numel()),
           "smoe_mlp_bwd")
    return buf.dX, buf.dW1, buf.dW2, buf.dgates
