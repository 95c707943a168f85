"""GPU parity of the attention kernels and of the SMoE attention layer (Alg. 4) against the fp64 oracle."""
import sys

import numpy as np
import pytest
import torch

import oracle
import smoe_inputs as si
from helpers import TOL

pytestmark = pytest.mark.gpu


def _log(*a):
    print(*a, flush=True, file=sys.stderr)


@pytest.fixture(scope="module")
def smoe():
    import paper_2403_08245_amd as m
    return m


def _bf16(shape, seed, std=1.0):
    x = torch.randn(*shape, generator=torch.Generator().manual_seed(seed), dtype=torch.float32) * std
    return x.to(torch.bfloat16)


def _rel(got, ref):
    return np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-3)   # a lone position has an exactly zero dQ and dK


ATTN_SHAPES = [(1, 1, 1, 1), (2, 77, 3, 2), (1, 300, 4, 1), (3, 33, 1, 2), (1, 130, 5, 1), (1, 64, 16, 1)]


@pytest.mark.parametrize("B,T,G,h", ATTN_SHAPES)
def test_attention_forward(smoe, B, T, G, h):
    _log(f"attention fwd B={B} T={T} G={G} h={h}")
    Q, K, V = _bf16((B, T, G, h, 128), 1), _bf16((B, T, h, 128), 2), _bf16((B, T, h, 128), 3)
    O, L = smoe.attention_fwd(Q.cuda(), K.cuda(), V.cuda())
    Oref, Lref = oracle.attention_fwd(si.as_f64(Q), si.as_f64(K), si.as_f64(V))
    assert _rel(O.float().cpu().numpy().astype(np.float64), Oref) <= TOL[torch.bfloat16]
    assert np.abs(L.cpu().numpy() - Lref).max() <= 2e-2        # log-sum-exp of O(10) scores from bf16 products


@pytest.mark.parametrize("B,T,G,h", ATTN_SHAPES)
def test_attention_backward(smoe, B, T, G, h):
    _log(f"attention bwd B={B} T={T} G={G} h={h}")
    Q, K, V = _bf16((B, T, G, h, 128), 1), _bf16((B, T, h, 128), 2), _bf16((B, T, h, 128), 3)
    dO = _bf16((B, T, G, h, 128), 4)
    Qd, Kd, Vd = Q.cuda(), K.cuda(), V.cuda()
    O, L = smoe.attention_fwd(Qd, Kd, Vd)
    dQ, dK, dV = smoe.attention_bwd(dO.cuda(), Qd, Kd, Vd, O, L)
    rq, rk, rv = oracle.attention_bwd(si.as_f64(dO), si.as_f64(Q), si.as_f64(K), si.as_f64(V))
    for name, got, ref in (("dQ", dQ, rq), ("dK", dK, rk), ("dV", dV, rv)):
        err = _rel(got.float().cpu().numpy().astype(np.float64), ref)
        _log(f"  {name} rel err {err:.2e}")
        assert err <= TOL[torch.bfloat16], name
