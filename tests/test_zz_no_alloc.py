"""The routing entry point that allocates nothing (scratch in a static device array inside the library),
called through the C ABI and compared bit for bit with smoe_route, twice in a row with the second
problem smaller than the first (the array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def smoe():
    import paper_2403_08245_amd as m
    assert torch.cuda.is_available(), "needs the MI355X"
    m.ctx()
    return m


def _experts(T, k, E, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.stack([torch.randperm(E, generator=g)[:k] for _ in range(T)]).to(torch.int32).cuda()


def _route_both(smoe, ei, E):
    """(smoe_route's arrays, smoe_route_noalloc's arrays), both through the C ABI on the current stream."""
    lib, T, k = smoe.lib, ei.shape[0], ei.shape[1]
    stream = torch.cuda.current_stream().cuda_stream
    outs = []
    for noalloc in (False, True):
        se = torch.full((T * k,), -7, dtype=torch.int32, device="cuda")
        so = torch.full((T * k,), -7, dtype=torch.int32, device="cuda")
        off = torch.full((E + 1,), -7, dtype=torch.int32, device="cuda")
        if noalloc:
            before = torch.cuda.memory_allocated()
            rc = lib.smoe_route_noalloc(smoe.ctx(), stream, ei.data_ptr(), T, k, E, se.data_ptr(), so.data_ptr(), off.data_ptr())
            assert torch.cuda.memory_allocated() == before
        else:
            nb = lib.smoe_route_workspace_bytes(T, k, E)
            ws = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")
            rc = lib.smoe_route(smoe.ctx(), stream, ei.data_ptr(), T, k, E, se.data_ptr(), so.data_ptr(), off.data_ptr(),
                                ws.data_ptr(), ws.numel())
        assert rc == 0, lib.smoe_strerror(rc)
        torch.cuda.synchronize()
        outs.append((se.cpu().numpy(), so.cpu().numpy(), off.cpu().numpy()))
    return outs


def test_route_noalloc_matches_route_on_two_calls_in_a_row(smoe):
    for T, k, E, seed in ((20000, 8, 64, 1), (3000, 2, 8, 2), (100, 2, 8, 3)):     # 157 chunks, then 6, then one
        print(f"route_noalloc T={T} k={k} E={E}", flush=True)
        ei = _experts(T, k, E, seed)
        (se, so, off), (se2, so2, off2) = _route_both(smoe, ei, E)
        assert np.array_equal(se, se2) and np.array_equal(so, so2) and np.array_equal(off, off2)
        assert off2[-1] == T * k and (np.sort(so2) == np.arange(T * k)).all()


def test_route_noalloc_rejects_problems_beyond_its_scratch(smoe):
    lib = smoe.lib
    stream = torch.cuda.current_stream().cuda_stream
    T, k, E = 300000, 4, 256            # 1172 chunks x 256 experts x 4 B > 1 MiB
    ei = torch.zeros(T, k, dtype=torch.int32, device="cuda")
    se = torch.full((T * k,), -7, dtype=torch.int32, device="cuda")
    off = torch.full((E + 1,), -7, dtype=torch.int32, device="cuda")
    rc = lib.smoe_route_noalloc(smoe.ctx(), stream, ei.data_ptr(), T, k, E, se.data_ptr(), se.data_ptr(), off.data_ptr())
    assert rc == -5 and b"scratch" in lib.smoe_strerror(rc)
    torch.cuda.synchronize()
    assert (off == -7).all() and (se == -7).all()      # nothing was enqueued
    assert lib.smoe_route_noalloc(smoe.ctx(), stream, None, 0, 2, 8, None, None, off.data_ptr()) == 0   # empty input
    torch.cuda.synchronize()
    assert off[:9].cpu().tolist() == [0] * 9
