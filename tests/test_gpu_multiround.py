"""GPU parity over several rounds of the persistent grid.

The persistent matrix-core kernels (one block per compute unit, 256 blocks) walk a list of 256 x 256
output tiles each; everything that happens between two tiles of one block (the ring of order indices,
the loader running ahead into the next tile, the hand-over of the accumulators to the epilogue) is only
exercised when a launch has more tiles than blocks.  Every case here has at least two, most four or more,
tiles per block, Zipf-distributed expert loads (ragged last tiles in every expert) and is compared
with the oracle on EVERY row: either the whole tensor, or -- where the fp64 per-row oracle would take
minutes -- every row restricted to sampled columns that hit every tile (a restriction of the same
problem: column c of a product depends on column c of the matrix only; row c of a weight gradient on
column c of the input only).  Outputs and workspaces are poisoned and guard-banded (conftest.py).
"""
import time

import numpy as np
import pytest
import torch

import oracle
import smoe_inputs as si
from helpers import TOL, assert_close, oracle_gates_f32, oracle_routing

pytestmark = pytest.mark.gpu
TB = 256          # tile edge of the persistent kernels
GRID = 256        # persistent blocks


def _log(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def smoe():
    import paper_2403_08245_amd as m
    assert torch.cuda.is_available(), "these tests need the MI355X"
    m.ctx()
    return m


def _m_tiles(off):
    return int(((np.diff(off) + TB - 1) // TB).sum())


def _per_tile_columns(width, per_tile, rng, tile=TB):
    """`per_tile` distinct columns out of every tile-wide column block, the last (ragged) one included."""
    cols = []
    for c0 in range(0, width, tile):
        hi = min(c0 + tile, width)
        cols += sorted(rng.choice(np.arange(c0, hi), size=min(per_tile, hi - c0), replace=False).tolist())
    return np.asarray(cols, dtype=np.int64)


# T, k, d_in, d_out, E, gin, gout, with_p, min forward tiles, min input-gradient tiles
MULTIROUND_CASES = [
    # the shortest contractions the persistent kernels take, scattered output, > 4 tiles per block
    pytest.param(32768, 2, 96, 1024, 8, 0, 0, 0, 1024, 0, id="fwd-K96-scatter-out"),
    pytest.param(32768, 2, 128, 1024, 8, 0, 0, 1, 1024, 0, id="fwd-K128-scatter-out-weighted"),
    pytest.param(32768, 2, 1024, 96, 8, 0, 1, 0, 0, 1024, id="dX-K96-scatter-out"),
    pytest.param(65536, 1, 1024, 128, 8, 1, 0, 0, 0, 1024, id="dX-K128-sorted-out"),
    # mid-size contraction, all four (transposed, scattered-output) instantiations over 2+ rounds
    pytest.param(8192, 2, 256, 2048, 8, 0, 1, 0, 512, 0, id="fwd-K256-scatter-to-sorted"),
    pytest.param(8192, 2, 2048, 256, 8, 0, 0, 0, 0, 512, id="dX-K256-scatter-to-scatter"),
    pytest.param(16384, 1, 256, 2048, 8, 1, 1, 0, 512, 0, id="fwd-K256-sorted-to-sorted"),
    pytest.param(16384, 1, 2080, 288, 5, 1, 0, 0, 0, 512, id="dX-K288-ragged-widths"),
]


@pytest.mark.parametrize("T,k,d_in,d_out,E,gin,gout,with_p,min_fwd,min_dx", MULTIROUND_CASES)
def test_plinear_every_row_over_several_rounds(smoe, T, k, d_in, d_out, E, gin, gout, with_p, min_fwd, min_dx):
    t0 = time.time()
    Tk = T * k
    c = si.plinear_case(T, d_in, d_out, E, k, "bf16", seed=31, x_rows=Tk if gin else T, zipf_s=1.2)
    ei, g, se, o, off = oracle_routing(c["logits"], k, E)
    gi, gg = smoe.topk_gate(c["logits"].cuda(), k)
    r = smoe.route(gi, E)
    assert np.array_equal(r.sorted_scattered_idxs.cpu().numpy(), o) and np.array_equal(r.expert_offsets.cpu().numpy(), off)
    assert np.abs(gg.cpu().numpy() - g).max() <= 1e-6
    mt = _m_tiles(off)
    fwd_tiles, dx_tiles = mt * -(-d_out // TB), mt * -(-d_in // TB)
    _log(f"rows per expert {np.diff(off).tolist()}, forward tiles {fwd_tiles}, input-gradient tiles {dx_tiles}")
    assert fwd_tiles >= min_fwd and dx_tiles >= min_dx
    fan = 1 if gin else k
    p64 = oracle_gates_f32(g) if with_p else None
    X, W = c["X"].cuda(), c["W"].cuda()
    Y, Yhat = smoe.plinear_fwd(X, W, r, fan, gg if with_p else None, bool(gin), bool(gout))
    dY_t = c["dY_T"] if with_p else c["dY_Tk"]
    dX, dW, dg = smoe.plinear_bwd(dY_t.cuda(), X, W, Yhat, r, fan, gg if with_p else None, bool(gin), bool(gout))
    torch.cuda.synchronize()
    X64, W64, dY64 = si.as_f64(c["X"]), si.as_f64(c["W"]), si.as_f64(dY_t)
    td = torch.bfloat16
    # forward: every row, every column
    Y_ref, Yhat_ref = oracle.plinear_fwd(X64, W64, se, o, fan, p64, bool(gin), bool(gout))
    assert_close(Yhat, Yhat_ref, td, "Yhat")
    assert_close(Y, Y_ref, td, "Y")
    _log(f"forward compared at {time.time() - t0:.1f}s")
    # backward: every row of dX and dgates; dW rows from every tile (restriction to sampled input features)
    rng = np.random.default_rng(5)
    cin = _per_tile_columns(d_in, 8, rng)
    dX_ref, dW_ref, _ = oracle.plinear_bwd(dY64, X64[:, cin], W64[:, cin, :], se, o, fan, p64, bool(gin), bool(gout))
    ct = torch.from_numpy(cin).cuda()
    assert_close(dX[:, ct], dX_ref, td, "dX (sampled input features, every row)")
    assert_close(dW[:, ct, :], dW_ref, td, "dW (sampled rows of every tile)")
    if with_p:
        # the routing-weight gradient of a token needs its whole input row: the oracle runs a token subset instead
        S = np.sort(rng.choice(T, size=1024, replace=False))
        se_s, o_s, _ = oracle.route(ei[S], E)
        _, _, dp_ref = oracle.plinear_bwd(dY64[S], X64[S], W64, se_s, o_s, fan, p64[S], bool(gin), bool(gout))
        assert_close(dg[torch.from_numpy(S).cuda()], dp_ref, td, "dgates (sampled tokens)")
        assert bool(torch.isfinite(dg).all())
    # the untouched columns cannot hide a hole: poisoned outputs must have been overwritten everywhere
    for name, t in (("Yhat", Yhat), ("Y", Y), ("dX", dX), ("dW", dW)):
        assert bool(torch.isfinite(t.float()).all()), f"{name} holds entries no kernel wrote"
    _log(f"done at {time.time() - t0:.1f}s")


def test_weight_gradient_every_tile_over_several_rounds(smoe):
    """groupXTY with 720 output tiles (twenty experts, 6 x 6 tiles each, ~200 rows per expert): blocks run
    two or three tiles each, experts in largest-first order; eight rows of every tile are compared."""
    T, k, d_in, d_out, E = 4096, 1, 1536, 1536, 20
    c = si.plinear_case(T, d_in, d_out, E, k, "bf16", seed=41, zipf_s=0.6)
    ei, g, se, o, off = oracle_routing(c["logits"], k, E)
    gi, gg = smoe.topk_gate(c["logits"].cuda(), k)
    r = smoe.route(gi, E)
    assert E * (d_in // TB) * (d_out // TB) >= 2 * GRID + 128
    X, W, dY = c["X"].cuda(), c["W"].cuda(), c["dY_Tk"].cuda()
    _, Yhat = smoe.plinear_fwd(X, W, r, k, None, False, True)
    dX, dW, _ = smoe.plinear_bwd(dY, X, W, Yhat, r, k, None, False, True)
    rng = np.random.default_rng(6)
    cin = _per_tile_columns(d_in, 8, rng)
    dX_ref, dW_ref, _ = oracle.plinear_bwd(si.as_f64(c["dY_Tk"]), si.as_f64(c["X"])[:, cin], si.as_f64(c["W"])[:, cin, :],
                                           se, o, k, None, False, True)
    ct = torch.from_numpy(cin).cuda()
    assert_close(dW[:, ct, :], dW_ref, torch.bfloat16, "dW (eight rows of every tile)")
    assert_close(dX[:, ct], dX_ref, torch.bfloat16, "dX")
    assert bool(torch.isfinite(dW.float()).all()) and bool(torch.isfinite(dX.float()).all())


@pytest.mark.parametrize("d_model,d_expert,training", [(256, 2048, True), (256, 2048, False), (160, 1896, True)])
def test_fused_swiglu_forward_every_row_over_several_rounds(smoe, d_model, d_expert, training):
    """The first ParallelLinear with SwiGLU in its epilogue, 500+ tiles (128 gate + 128 up columns each):
    pre-activation and H of EVERY routed row at two hidden units of every tile (the oracle runs the problem
    restricted to those units), Y on sampled tokens; the second case has ragged widths and a contraction
    that is not a multiple of 128."""
    cfg = si.custom("fused-rounds", T=4096, d_model=d_model, d_expert=d_expert, E=8, k=2, act=si.ACT_SWIGLU, dtype="bf16",
                    zipf_s=1.2)
    case = si.mlp_case(cfg, 17, with_grad=False)
    ei, g, se, o, off = oracle_routing(case["logits"], cfg.k, cfg.E)
    gi, gg = smoe.topk_gate(case["logits"].cuda(), cfg.k)
    r = smoe.route(gi, cfg.E)
    assert np.array_equal(r.sorted_scattered_idxs.cpu().numpy(), o)
    tiles = _m_tiles(off) * -(-d_expert // (TB // 2))
    _log(f"fused forward tiles {tiles}")
    assert tiles >= 2 * GRID - 40
    X, W1, W2 = (case[n].cuda() for n in ("X", "W1", "W2"))
    Y, buf = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act, training=training)
    torch.cuda.synchronize()
    g64 = oracle_gates_f32(g)
    rng = np.random.default_rng(8)
    units = _per_tile_columns(d_expert, 2, rng, tile=TB // 2)
    X64, W164, W264 = si.as_f64(case["X"]), si.as_f64(case["W1"]), si.as_f64(case["W2"])
    w1r = W164[:, :, np.concatenate([units, units + d_expert])]
    sub = oracle.mlp_fwd(X64, w1r, W264[:, units, :], ei, g64, cfg.act)        # same rows, only these hidden units
    ut = torch.from_numpy(units).cuda()
    if training:
        got_pre = torch.cat([buf.Hpre[:, ut], buf.Hpre[:, ut + d_expert]], 1)
        assert_close(got_pre, sub["Hpre"][o], torch.bfloat16, "Hpre (every row, two units per tile)")
        assert_close(buf.H[:, ut], sub["H"][o], torch.bfloat16, "H (every row, two units per tile)")
        assert bool(torch.isfinite(buf.H.float()).all()) and bool(torch.isfinite(buf.Hpre.float()).all())
    toks = np.sort(rng.choice(cfg.T, size=48, replace=False))
    Yref = np.stack([oracle.mlp_token_fwd(X64[t], ei[t], g64[t], W164, W264, cfg.act)[0] for t in toks])
    assert_close(Y[torch.from_numpy(toks).cuda()], Yref, torch.bfloat16, "Y (sampled tokens)")
    assert bool(torch.isfinite(Y.float()).all())


@pytest.mark.parametrize("act,T,d_model,d_expert", [
    pytest.param(si.ACT_SWIGLU, 4096, 128, 4096, id="swiglu-derivative-in-epilogue"),
    pytest.param(si.ACT_GELU, 4096, 128, 4096, id="gelu-weighted-sorted-copy"),
    pytest.param(si.ACT_GELU, 16384, 1280, 1024, id="gelu-weighted-hidden-rows"),
    pytest.param(si.ACT_NONE, 4096, 160, 3848, id="identity-ragged-width"),
])
def test_backward_with_dp_in_epilogue_over_several_rounds(smoe, act, T, d_model, d_expert):
    """The W2^T input-gradient product with the routing-weight gradient (and for SwiGLU the activation's derivative)
    in its epilogue, 500+ tiles; for the other activations the two ways of forming dW2 (from a routing-weighted sorted
    copy of dY, or from a plain one and routing-weighted hidden rows when those are narrower).  The intermediate tensors are scratch; what they
    feed is compared: dgates and dX on tokens drawn from every tile of every expert, two column pairs of dW1 and two
    rows of dW2 from every 256-unit tile for every expert (each sums over all the expert's rows), and every output
    must be free of the poison the workspace and outputs start with.  The forward's unweighted second product is not
    kept for such shapes."""
    cfg = si.custom("bwd-epilogue-rounds", T=T, d_model=d_model, d_expert=d_expert, E=8, k=2, act=act, dtype="bf16", zipf_s=1.2)
    case = si.mlp_case(cfg, 23)
    ei, g, se, o, off = oracle_routing(case["logits"], cfg.k, cfg.E)
    gi, gg = smoe.topk_gate(case["logits"].cuda(), cfg.k)
    r = smoe.route(gi, cfg.E)
    assert np.array_equal(r.sorted_scattered_idxs.cpu().numpy(), o)
    tiles = _m_tiles(off) * -(-cfg.d_expert // TB)
    _log(f"input-gradient tiles {tiles}")
    assert tiles >= 2 * GRID
    X, W1, W2, dY = (case[n].cuda() for n in ("X", "W1", "W2", "dY"))
    Y, buf = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act)
    assert buf.Yhat is None
    dX, dW1, dW2, dg = smoe.mlp_bwd(dY, X, W1, W2, r, cfg.k, gg, cfg.act, buf)
    torch.cuda.synchronize()
    for name, t in (("dX", dX), ("dW1", dW1), ("dW2", dW2), ("dgates", dg), ("Y", Y)):
        assert bool(torch.isfinite(t.float()).all()), f"{name} holds entries no kernel wrote"
    g64 = oracle_gates_f32(g)
    X64, W164, W264, dY64 = (si.as_f64(case[n]) for n in ("X", "W1", "W2", "dY"))
    rng = np.random.default_rng(9)
    rows = np.concatenate([rng.choice(np.arange(a, min(a + TB, int(off[e + 1]))), size=min(6 if T <= 4096 else 2, int(off[e + 1]) - a), replace=False)
                           for e in range(cfg.E) for a in range(int(off[e]), int(off[e + 1]), TB)])
    toks = np.unique(o[rows] // cfg.k)
    _log(f"{len(toks)} tokens from {len(rows)} sampled rows")
    ref = [oracle.mlp_token_bwd(X64[t], dY64[t], ei[t], g64[t], W164, W264, cfg.act) for t in toks]
    tt = torch.from_numpy(toks).cuda()
    assert_close(dX[tt], np.stack([q[0] for q in ref]), torch.bfloat16, "dX (tokens from every tile)")
    assert_close(dg[tt], np.stack([q[1] for q in ref]), torch.bfloat16, "dgates (tokens from every tile)")
    units = _per_tile_columns(cfg.d_expert, 2, rng)
    ut = torch.from_numpy(units).cuda()
    r1, g1, r2, g2 = [], [], [], []
    for e in range(cfg.E):
        r1.append(oracle.mlp_dW1_cols(dY64, X64, W164, W264, ei, g64, cfg.act, e, units))
        cols = [ut] + ([ut + cfg.d_expert] if act == si.ACT_SWIGLU else [])
        g1.append(torch.stack([dW1[e][:, c].T for c in cols], 1).float().cpu().numpy())
        r2.append(oracle.mlp_dW2_rows(dY64, X64, W164, W264, ei, g64, cfg.act, e, units))
        g2.append(dW2[e][ut].float().cpu().numpy())
    assert_close(np.stack(g1), np.stack(r1), torch.bfloat16, "dW1 (two unit pairs per tile)")
    assert_close(np.stack(g2), np.stack(r2), torch.bfloat16, "dW2 (two rows per tile)")
