"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs.

Bar: bit-exact for routing indices and offsets; max |gpu - ref| / max |ref| <= 1e-5 (fp32)
or 2e-2 (bf16 inputs, fp32 accumulation) per tensor for outputs and gradients; gates at
1e-6 absolute.
"""
import numpy as np
import pytest
import torch

import oracle
import smoe_inputs as si
from helpers import TOL, assert_close, dev, oracle_gates_f32, oracle_routing, rel_err, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def smoe():
    import paper_2403_08245_amd as m
    assert torch.cuda.is_available(), "these tests need the MI355X"
    m.ctx()
    return m


def _log(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------ routing (bit-exact)
ROUTING_CASES = [
    (1, 1, 1), (3, 4, 4), (64, 64, 8), (4, 64, 8), (256, 4, 2), (1000, 7, 3), (1023, 8, 1),
    (1025, 8, 2), (16384, 8, 2), (8192, 64, 8), (5000, 130, 5), (777, 1, 1),
    (3000, 128, 16), (2000, 200, 70), (500, 256, 3), (300, 300, 4), (70000, 65, 2),
]


@pytest.mark.parametrize("T,E,k", ROUTING_CASES)
def test_topk_and_route_bit_exact(smoe, T, E, k):
    _log(f"routing T={T} E={E} k={k}")
    logits = torch.randn(T, E, generator=torch.Generator().manual_seed(T * 131 + E), dtype=torch.float32)
    ei, g, se, o, off = oracle_routing(logits, k, E)
    gi, gg = smoe.topk_gate(logits.cuda(), k)
    assert np.array_equal(gi.cpu().numpy(), ei)
    assert np.abs(gg.cpu().numpy().astype(np.float64) - g).max() <= 1e-6
    r = smoe.route(gi, E)
    assert np.array_equal(r.sorted_expert_idxs.cpu().numpy(), se)
    assert np.array_equal(r.sorted_scattered_idxs.cpu().numpy(), o)
    assert np.array_equal(r.expert_offsets.cpu().numpy(), off)


@pytest.mark.parametrize("T,E,k", [(1, 1, 1), (257, 8, 2), (1000, 64, 8), (333, 130, 16), (64, 5, 5)])
def test_router_gradient(smoe, T, E, k):
    """dlogits from Alg. 2's dp through the softmax over the kept logits (fp32 against the fp64 definition)."""
    gen = torch.Generator().manual_seed(T + 7 * E + k)
    logits = torch.randn(T, E, generator=gen, dtype=torch.float32)
    dp = torch.randn(T, k, generator=gen, dtype=torch.float32)
    gi, gg = smoe.topk_gate(logits.cuda(), k)
    got = smoe.topk_gate_bwd(gi, gg, dp.cuda(), E).cpu().numpy().astype(np.float64)
    ei, g = oracle.topk_gate(logits.numpy(), k)
    ref = oracle.topk_gate_bwd(ei, g, dp.numpy().astype(np.float64), E)
    assert got.shape == ref.shape
    assert np.abs(got - ref).max() <= TOL[torch.float32] * max(np.abs(ref).max(), 1e-30)
    mask = np.ones_like(ref, dtype=bool)
    np.put_along_axis(mask, ei.astype(np.int64), False, axis=1)
    assert (got[mask] == 0).all()                     # experts that were not kept get an exact zero


@pytest.mark.parametrize("E,k", [(16, 4), (130, 9), (256, 70), (300, 5)])
def test_topk_ties_and_quantised_logits(smoe, E, k):
    g = torch.Generator().manual_seed(5)
    logits = torch.randint(-2, 3, (2048, E), generator=g).to(torch.float32)     # many exact ties
    ei, gates, se, o, off = oracle_routing(logits, k, E)
    gi, gg = smoe.topk_gate(logits.cuda(), k)
    assert np.array_equal(gi.cpu().numpy(), ei)
    assert np.abs(gg.cpu().numpy() - gates).max() <= 1e-6


@pytest.mark.parametrize("E,k", [(4, 3), (70, 8), (130, 5), (256, 256), (300, 7)])
def test_topk_with_nan_and_infinite_logits(smoe, E, k):
    """NaN counts as -inf, kept logits that are all -inf share the weight equally: every slot of every token is
    written (outputs are poisoned beforehand) and equals the oracle's, in the wavefront-per-token and the
    thread-per-token kernels alike."""
    gen = torch.Generator().manual_seed(E)
    logits = torch.randn(600, E, generator=gen, dtype=torch.float32)
    u = torch.rand(600, E, generator=gen)
    logits[u < 0.2] = float("nan")
    logits[(u >= 0.2) & (u < 0.35)] = -float("inf")
    logits[0] = float("nan")                       # nothing to choose from
    logits[1] = -float("inf")
    logits[2, 1:] = float("nan")                   # exactly one number
    ei, gates, se, o, off = oracle_routing(logits, k, E)
    gi, gg = smoe.topk_gate(logits.cuda(), k)
    assert np.array_equal(gi.cpu().numpy(), ei)
    got = gg.cpu().numpy()
    assert np.isfinite(got).all() and np.abs(got - gates).max() <= 1e-6


@pytest.mark.parametrize("pattern", ["one_expert", "empty_middle", "k_equals_E", "masked"])
def test_route_degenerate_distributions(smoe, pattern):
    T, E, k = 300, 8, 2
    if pattern == "one_expert":
        ei = np.full((T, 1), 5, dtype=np.int32); k = 1
    elif pattern == "empty_middle":
        ei = np.stack([np.zeros(T), np.full(T, 7)], 1).astype(np.int32)
    elif pattern == "k_equals_E":
        k = E
        ei = np.stack([np.random.default_rng(t).permutation(E) for t in range(T)]).astype(np.int32)
    else:
        cfg = si.CONFIGS["C4-decode-masked"]
        logits = si.router_logits(cfg, 3)
        ei, _ = oracle.topk_gate(logits.numpy(), cfg.k)
        E = cfg.E
        assert (np.bincount(ei.reshape(-1), minlength=E) == 0).sum() >= 16
    se, o, off = oracle.route(ei, E)
    r = smoe.route(dev(ei), E)
    assert np.array_equal(r.sorted_expert_idxs.cpu().numpy(), se)
    assert np.array_equal(r.sorted_scattered_idxs.cpu().numpy(), o)
    assert np.array_equal(r.expert_offsets.cpu().numpy(), off)


def test_route_empty_input(smoe):
    r = smoe.route(torch.empty(0, 2, dtype=torch.int32, device="cuda"), 4)
    assert r.expert_offsets.cpu().tolist() == [0, 0, 0, 0, 0]


# ------------------------------------------------------------------ ParallelLinear
def _plinear_setup(smoe, T, d_in, d_out, E, k, dtype, seed, grouped_in):
    x_rows = T * k if grouped_in else T
    c = si.plinear_case(T, d_in, d_out, E, k, dtype, seed, x_rows=x_rows)
    ei, g, se, o, off = oracle_routing(c["logits"], k, E)
    gi, gg = smoe.topk_gate(c["logits"].cuda(), k)
    r = smoe.route(gi, E)
    return c, (ei, g, se, o, off), (gi, gg, r)


PL_SHAPES = [
    # T, d_in, d_out, E, k   (several tiles, ragged tails, more experts than rows)
    (96, 64, 128, 4, 2),
    (333, 72, 40, 5, 3),
    (7, 16, 24, 16, 2),
    (520, 256, 136, 3, 1),
    (20, 64, 72, 16, 2),      # a couple of rows per expert: the forward takes the 32-row-tile kernels
    (90, 96, 264, 3, 1),      # the same kernels with several tiles per expert and three column tiles
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("gin,gout,with_p", [(0, 0, 0), (0, 1, 0), (1, 0, 0), (1, 1, 0), (0, 0, 1), (1, 0, 1)])
@pytest.mark.parametrize("shape", PL_SHAPES)
def test_plinear_forward_and_backward(smoe, shape, gin, gout, with_p, dtype):
    T, d_in, d_out, E, k = shape
    _log(f"plinear shape={shape} gin={gin} gout={gout} p={with_p} {dtype}")
    td = torch_dtype(dtype)
    c, (ei, g, se, o, off), (gi, gg, r) = _plinear_setup(smoe, T, d_in, d_out, E, k, dtype, 7, gin)
    fan = 1 if gin else k
    X, W = si.as_f64(c["X"]), si.as_f64(c["W"])
    assert np.abs(gg.cpu().numpy().astype(np.float64) - g).max() <= 1e-6
    p64 = oracle_gates_f32(g) if with_p else None       # the oracle's own gates, in the precision they are stored in
    Y_ref, Yhat_ref = oracle.plinear_fwd(X, W, se, o, fan, p64, bool(gin), bool(gout))
    Y, Yhat = smoe.plinear_fwd(c["X"].cuda(), c["W"].cuda(), r, fan, gg if with_p else None, bool(gin), bool(gout))
    assert_close(Yhat, Yhat_ref, td, "Yhat")
    assert_close(Y, Y_ref, td, "Y")
    dY_t = c["dY_T"] if with_p else c["dY_Tk"]
    dX_ref, dW_ref, dp_ref = oracle.plinear_bwd(si.as_f64(dY_t), X, W, se, o, fan, p64, bool(gin), bool(gout))
    dX, dW, dg = smoe.plinear_bwd(dY_t.cuda(), c["X"].cuda(), c["W"].cuda(), Yhat, r, fan,
                                  gg if with_p else None, bool(gin), bool(gout))
    assert_close(dX, dX_ref, td, "dX")
    assert_close(dW, dW_ref, td, "dW")
    if with_p:
        assert_close(dg, dp_ref, td, "dgates")


@pytest.mark.parametrize("E,gin,gout,with_p", [(2, 0, 0, 1), (1, 1, 1, 0), (3, 0, 1, 0)])
def test_plinear_weight_gradient_with_few_tiles_and_many_rows(smoe, E, gin, gout, with_p):
    """A handful of output tiles per expert and thousands of rows: the weight gradient cuts every expert's rows
    into chunks (fp32 partial tiles, added in chunk order by a second kernel) so that the chip is not left idle;
    the third case has a width that is not a multiple of the tile."""
    T, d_in, d_out, k = 8192, 256, 264 if E == 3 else 256, 1
    td = torch.bfloat16
    c, (ei, g, se, o, off), (gi, gg, r) = _plinear_setup(smoe, T, d_in, d_out, E, k, "bf16", 21, gin)
    X, W = si.as_f64(c["X"]), si.as_f64(c["W"])
    p64 = oracle_gates_f32(g) if with_p else None
    Y, Yhat = smoe.plinear_fwd(c["X"].cuda(), c["W"].cuda(), r, k, gg if with_p else None, bool(gin), bool(gout))
    dY_t = c["dY_T"] if with_p else c["dY_Tk"]
    dX_ref, dW_ref, dp_ref = oracle.plinear_bwd(si.as_f64(dY_t), X, W, se, o, k, p64, bool(gin), bool(gout))
    outs = [smoe.plinear_bwd(dY_t.cuda(), c["X"].cuda(), c["W"].cuda(), Yhat, r, k, gg if with_p else None, bool(gin), bool(gout))
            for _ in range(2)]
    dX, dW, dg = outs[0]
    assert_close(dW, dW_ref, td, "dW")
    assert_close(dX, dX_ref, td, "dX")
    assert torch.equal(outs[0][1], outs[1][1])       # fixed summation order


def test_group_matches_definition(smoe):
    c, (ei, g, se, o, off), (gi, gg, r) = _plinear_setup(smoe, 200, 64, 64, 6, 2, "bf16", 3, 0)
    out = smoe.group(c["X"].cuda(), r, 2)
    assert torch.equal(out.cpu(), c["X"][torch.from_numpy(o.astype(np.int64)) // 2])
    outw = smoe.group(c["dY_T"].cuda(), r, 2, gg)
    ref = g.reshape(-1)[o][:, None] * si.as_f64(c["dY_T"])[o // 2]
    assert_close(outw, ref, torch.bfloat16, "weighted group")


# ------------------------------------------------------------------ SMoE MLP, whole-tensor parity
def _mlp_parity(smoe, cfg, seed, plain=False, mode=None):
    td = torch_dtype(cfg.dtype)
    case = si.mlp_case(cfg, seed)
    smoe.set_kernel_mode(mode if mode is not None else (1 if plain else 0))
    try:
        gi, gg = smoe.topk_gate(case["logits"].cuda(), cfg.k)
        r = smoe.route(gi, cfg.E)
        ei, g, se, o, off = oracle_routing(case["logits"], cfg.k, cfg.E)
        assert np.array_equal(gi.cpu().numpy(), ei)
        assert np.array_equal(r.sorted_scattered_idxs.cpu().numpy(), o)
        assert np.array_equal(r.expert_offsets.cpu().numpy(), off)
        X, W1, W2, dYc = (case[n].cuda() for n in ("X", "W1", "W2", "dY"))
        Y, buf = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act)
        dX, dW1, dW2, dg = smoe.mlp_bwd(dYc, X, W1, W2, r, cfg.k, gg, cfg.act, buf)
        torch.cuda.synchronize()
    finally:
        smoe.set_kernel_mode(0)
    assert np.abs(gg.cpu().numpy().astype(np.float64) - g).max() <= 1e-6
    g64 = oracle_gates_f32(g)
    X64, W164, W264, dY64 = (si.as_f64(case[n]) for n in ("X", "W1", "W2", "dY"))
    ref = oracle.mlp_fwd(X64, W164, W264, ei, g64, cfg.act)
    errs = {}
    errs["Y"] = assert_close(Y, ref["Y"], td, "Y")
    errs["Hpre"] = assert_close(buf.Hpre, ref["Hpre"][o], td, "Hpre (grouped)")
    errs["H"] = assert_close(buf.H, ref["H"][o], td, "H (grouped)")
    if buf.Yhat is not None:         # not kept when the backward pass of this shape forms dp in a product's epilogue
        errs["Yhat"] = assert_close(buf.Yhat, ref["Yhat"], td, "Yhat (scattered)")
    gref = oracle.mlp_bwd(dY64, X64, W164, W264, ei, g64, cfg.act)
    errs["dX"] = assert_close(dX, gref["dX"], td, "dX")
    errs["dW1"] = assert_close(dW1, gref["dW1"], td, "dW1")
    errs["dW2"] = assert_close(dW2, gref["dW2"], td, "dW2")
    errs["dgates"] = assert_close(dg, gref["dgates"], td, "dgates")
    _log(cfg.name, {k: f"{v:.2e}" for k, v in errs.items()})
    return case, (X, W1, W2, dYc, r, gg)


def test_mlp_C1_fp32_full(smoe):
    _mlp_parity(smoe, si.CONFIGS["C1"], 0)


@pytest.mark.parametrize("name", ["C3-small", "C3-small-f32"])
def test_mlp_reduced_mixtral_shape_full(smoe, name):
    _mlp_parity(smoe, si.CONFIGS[name], 1)


def test_mlp_bf16_plain_kernels_full(smoe):
    _mlp_parity(smoe, si.CONFIGS["C3-small"], 2, plain=True)


def test_mlp_bf16_one_block_per_tile_kernels_full(smoe):
    """The non-persistent matrix-core kernels (fallback for short contractions / many experts)."""
    _mlp_parity(smoe, si.CONFIGS["C3-small"], 3, mode=2)


def test_mlp_more_experts_than_the_offset_cache(smoe):
    cfg = si.custom("E300", T=700, d_model=128, d_expert=64, E=300, k=2, act=si.ACT_SWIGLU, dtype="bf16")
    _mlp_parity(smoe, cfg, 8)


def test_mlp_short_contraction_falls_back(smoe):
    cfg = si.custom("K64", T=600, d_model=64, d_expert=32, E=4, k=2, act=si.ACT_GELU, dtype="bf16")
    _mlp_parity(smoe, cfg, 9)


@pytest.mark.parametrize("act", [si.ACT_NONE, si.ACT_GELU, si.ACT_SWIGLU])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_mlp_ragged_shapes_with_empty_experts(smoe, act, dtype):
    # T*k < E rows for some experts, widths that are not multiples of the GEMM tiles
    cfg = si.custom("ragged", T=37, d_model=72, d_expert=40, E=12, k=3, act=act, dtype=dtype, masked_experts=4)
    _mlp_parity(smoe, cfg, 4)


@pytest.mark.parametrize("d_model,d_expert", [(160, 200), (384, 72), (128, 136)])
def test_mlp_fused_swiglu_ragged_widths(smoe, d_model, d_expert):
    """bf16 SwiGLU through the persistent kernels (activation in the first product's epilogue) with hidden
    widths that leave the last gate/up tile partly empty, contractions that are and are not a multiple of
    128, training and inference."""
    cfg = si.custom(f"fused{d_model}x{d_expert}", T=301, d_model=d_model, d_expert=d_expert, E=5, k=2, act=si.ACT_SWIGLU,
                    dtype="bf16")
    case, (X, W1, W2, dYc, r, gg) = _mlp_parity(smoe, cfg, 11)
    Yt, _ = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act, training=True)
    Yi, _ = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act, training=False)
    assert torch.equal(Yt, Yi)


@pytest.mark.parametrize("act", [si.ACT_GELU, si.ACT_SWIGLU])
@pytest.mark.parametrize("shape", [(40, 4, 16, 160, 96, 0), (100, 2, 8, 256, 224, 5), (3, 2, 64, 64, 32, 0)])
def test_mlp_small_batches_take_the_decode_kernels(smoe, shape, act):
    """At most 32 routed rows per expert on average: the forward products run as 32-row tiles, one
    wavefront each.  Widths that leave the last 128-column tile (64 gate columns for SwiGLU) partly empty,
    experts with several tiles (five of eight experts masked out) and with none, training and inference."""
    T, k, E, d_model, d_expert, masked = shape
    cfg = si.custom(f"decode{T}", T=T, d_model=d_model, d_expert=d_expert, E=E, k=k, act=act, dtype="bf16",
                    masked_experts=masked)
    assert T * k <= 32 * E
    case, (X, W1, W2, dYc, r, gg) = _mlp_parity(smoe, cfg, 13)
    Yt, _ = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act, training=True)
    Yi, _ = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act, training=False)
    assert torch.equal(Yt, Yi)


def test_mlp_k1_and_k_equals_E(smoe):
    _mlp_parity(smoe, si.custom("k1", T=130, d_model=64, d_expert=64, E=4, k=1, act=si.ACT_SWIGLU, dtype="bf16"), 5)
    _mlp_parity(smoe, si.custom("kE", T=50, d_model=64, d_expert=32, E=4, k=4, act=si.ACT_GELU, dtype="f32"), 6)


@pytest.mark.parametrize("act", [si.ACT_SWIGLU, si.ACT_GELU])
@pytest.mark.parametrize("k", [1, 2])
def test_routing_weight_gradient_with_vanishing_weights(smoe, act, k):
    """dgates where the persistent kernels form it in a product's epilogue (contraction >= 96): k = 1 (every weight is
    exactly 1), and k = 2 with half of the tokens routed so lopsidedly that their second weight is exactly 0 in fp32 --
    its gradient <dY_t, Yhat> is still a plain dot product of order one, and no step may divide by the weight."""
    cfg = si.custom(f"dp-k{k}", T=700, d_model=128, d_expert=160, E=6, k=k, act=act, dtype="bf16")
    case = si.mlp_case(cfg, 19)
    logits = case["logits"].clone()
    logits[::2, 3] += 200.0                       # exp(-200) underflows: the other kept expert's weight is 0
    ei, g, se, o, off = oracle_routing(logits, cfg.k, cfg.E)
    gi, gg = smoe.topk_gate(logits.cuda(), cfg.k)
    assert np.array_equal(gi.cpu().numpy(), ei) and np.abs(gg.cpu().numpy() - g).max() <= 1e-6
    g32 = oracle_gates_f32(g)
    if k == 2:
        assert (g32[::2, 1] == 0).all() and (gg.cpu().numpy()[::2, 1] == 0).all()
    r = smoe.route(gi, cfg.E)
    X, W1, W2, dY = (case[n].cuda() for n in ("X", "W1", "W2", "dY"))
    Y, buf = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act)
    assert buf.Yhat is None                        # this shape does not keep the unweighted second product
    dX, dW1, dW2, dg = smoe.mlp_bwd(dY, X, W1, W2, r, cfg.k, gg, cfg.act, buf)
    X64, W164, W264, dY64 = (si.as_f64(case[n]) for n in ("X", "W1", "W2", "dY"))
    ref = oracle.mlp_bwd(dY64, X64, W164, W264, ei, g32, cfg.act)
    td = torch.bfloat16
    assert_close(dg, ref["dgates"], td, "dgates")
    if k == 2:
        zero_w = ref["dgates"][::2, 1]
        assert np.abs(zero_w).max() > 0.1           # the gradient of a vanished weight is not small
        assert np.abs(dg.cpu().numpy()[::2, 1] - zero_w).max() <= TOL[td] * np.abs(ref["dgates"]).max()
    assert_close(dX, ref["dX"], td, "dX")
    assert_close(dW1, ref["dW1"], td, "dW1")
    assert_close(dW2, ref["dW2"], td, "dW2")
    assert_close(Y, oracle.mlp_fwd(X64, W164, W264, ei, g32, cfg.act)["Y"], td, "Y")


def test_mlp_is_deterministic(smoe):
    cfg = si.CONFIGS["C3-small"]
    case, (X, W1, W2, dYc, r, gg) = _mlp_parity(smoe, cfg, 9)
    outs = []
    for _ in range(2):
        Y, buf = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act)
        g = smoe.mlp_bwd(dYc, X, W1, W2, r, cfg.k, gg, cfg.act, buf)
        outs.append([t.clone() for t in (Y,) + tuple(g)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("name", ["C1", "C3-small"])
def test_mlp_inference_mode_matches_training_forward(smoe, name):
    """Without saved tensors the pre-activation is not kept (for bf16 SwiGLU it is never written: the
    activation is applied in the first product's epilogue); the output is the same either way."""
    cfg = si.CONFIGS[name]
    case = si.mlp_case(cfg, 0)
    gi, gg = smoe.topk_gate(case["logits"].cuda(), cfg.k)
    r = smoe.route(gi, cfg.E)
    X, W1, W2 = (case[n].cuda() for n in ("X", "W1", "W2"))
    Yt, _ = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act, training=True)
    Yi, _ = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act, training=False)
    assert torch.equal(Yt, Yi)
    ei, g = oracle.topk_gate(case["logits"].numpy(), cfg.k)
    ref = oracle.mlp_fwd(si.as_f64(case["X"]), si.as_f64(case["W1"]), si.as_f64(case["W2"]), ei,
                         oracle_gates_f32(g), cfg.act)
    assert_close(Yi, ref["Y"], torch_dtype(cfg.dtype), f"{name} inference Y")


@pytest.mark.parametrize("name", ["C1", "C3-small", "C3-small-f32"])
def test_hidden_activations_entry_point(smoe, name):
    """smoe_plinear_act_fwd (Alg. 3 lines 1-2) against the oracle, with and without keeping the pre-activation."""
    cfg = si.CONFIGS[name]
    case = si.mlp_case(cfg, 4)
    gi, gg = smoe.topk_gate(case["logits"].cuda(), cfg.k)
    r = smoe.route(gi, cfg.E)
    ei, g, se, o, off = oracle_routing(case["logits"], cfg.k, cfg.E)
    X, W1 = case["X"].cuda(), case["W1"].cuda()
    H, Hpre = smoe.plinear_act_fwd(X, W1, r, cfg.k, cfg.act, keep_hpre=True)
    H2, none = smoe.plinear_act_fwd(X, W1, r, cfg.k, cfg.act, keep_hpre=False)
    assert none is None and torch.equal(H, H2)
    ref = oracle.mlp_fwd(si.as_f64(case["X"]), si.as_f64(case["W1"]), si.as_f64(case["W2"]), ei, oracle_gates_f32(g), cfg.act)
    td = torch_dtype(cfg.dtype)
    assert_close(Hpre, ref["Hpre"][o], td, "Hpre (grouped)")
    assert_close(H, ref["H"][o], td, "H (grouped)")


def test_mlp_empty_batch(smoe):
    cfg = si.CONFIGS["C1"]
    case = si.mlp_case(cfg, 0)
    W1, W2 = case["W1"].cuda(), case["W2"].cuda()
    # T = 0: nothing to do, weight gradients are zeros
    e = torch.empty(0, cfg.k, dtype=torch.int32, device="cuda")
    r0 = smoe.route(e, cfg.E)
    X0 = torch.empty(0, cfg.d_model, device="cuda")
    g0 = torch.empty(0, cfg.k, device="cuda")
    Y0, buf0 = smoe.mlp_fwd(X0, W1, W2, r0, cfg.k, g0, cfg.act)
    buf0.dW1.fill_(7.0); buf0.dW2.fill_(7.0)
    dX0, dW1, dW2, dg0 = smoe.mlp_bwd(X0, X0, W1, W2, r0, cfg.k, g0, cfg.act, buf0)
    assert Y0.shape[0] == 0 and float(dW1.abs().max()) == 0.0 and float(dW2.abs().max()) == 0.0


def test_argument_errors_leave_nothing_enqueued(smoe):
    """Shape, argument and workspace errors are found before the first launch: the outputs of a refused call still hold
    the pattern they were filled with (checked through the C ABI, with undersized / misaligned workspaces, a routing
    problem with more experts than the sort keeps counters for, and inconsistent row counts)."""
    import ctypes
    lib, cx = smoe.lib, smoe.ctx()
    stream = torch.cuda.current_stream().cuda_stream
    cfg = si.CONFIGS["C3-small"]
    case = si.mlp_case(cfg, 0)
    gi, gg = smoe.topk_gate(case["logits"].cuda(), cfg.k)
    r = smoe.route(gi, cfg.E)
    rc_ = r.c()
    X, W1, W2, dY = (case[n].cuda() for n in ("X", "W1", "W2", "dY"))
    mark = lambda *shape: torch.full(shape, 7.0, dtype=torch.bfloat16, device="cuda")
    Y, Hpre, H = mark(cfg.T, cfg.d_model), mark(cfg.Tk, cfg.d_h), mark(cfg.Tk, cfg.d_expert)
    need = lib.smoe_mlp_fwd_workspace_bytes(1, cfg.act, cfg.T, cfg.k, cfg.d_model, cfg.d_expert, 2)
    ws = torch.empty(need + 512, dtype=torch.uint8, device="cuda")
    fwd = lambda wsp, nbytes, T=cfg.T: lib.smoe_mlp_fwd(cx, stream, 1, cfg.act, X.data_ptr(), T, cfg.d_model, cfg.d_expert,
                                                        W1.data_ptr(), W2.data_ptr(), ctypes.byref(rc_), cfg.k, gg.data_ptr(),
                                                        Y.data_ptr(), Hpre.data_ptr(), H.data_ptr(), None, wsp, nbytes)
    assert fwd(ws.data_ptr(), need - 256) == -3              # too small
    assert fwd(ws.data_ptr() + 16, need) == -3               # misaligned
    assert fwd(None, need) == -3
    assert fwd(ws.data_ptr(), need, T=cfg.T - 1) == -1       # T * k does not match the routing
    dX, dW1, dW2 = mark(cfg.T, cfg.d_model), mark(*W1.shape), mark(*W2.shape)
    dg = torch.full((cfg.T, cfg.k), 7.0, device="cuda")
    needb = lib.smoe_mlp_bwd_workspace_bytes(1, cfg.act, cfg.T, cfg.k, cfg.d_model, cfg.d_expert)
    wsb = torch.empty(needb, dtype=torch.uint8, device="cuda")
    bwd = lambda nbytes: lib.smoe_mlp_bwd(cx, stream, 1, cfg.act, dY.data_ptr(), X.data_ptr(), cfg.T, cfg.d_model, cfg.d_expert,
                                          W1.data_ptr(), W2.data_ptr(), ctypes.byref(rc_), cfg.k, gg.data_ptr(), Hpre.data_ptr(),
                                          H.data_ptr(), None, dX.data_ptr(), dW1.data_ptr(), dW2.data_ptr(), dg.data_ptr(),
                                          wsb.data_ptr(), nbytes)
    assert bwd(needb - 256) == -3
    # routing: more experts than the per-expert counters in LDS allow
    E_big = 20000
    se = torch.full((64,), -7, dtype=torch.int32, device="cuda")
    off = torch.full((E_big + 1,), -7, dtype=torch.int32, device="cuda")
    eib = torch.zeros(32, 2, dtype=torch.int32, device="cuda")
    wsr = torch.empty(max(lib.smoe_route_workspace_bytes(32, 2, E_big), 256), dtype=torch.uint8, device="cuda")
    assert lib.smoe_route(cx, stream, eib.data_ptr(), 32, 2, E_big, se.data_ptr(), se.data_ptr(), off.data_ptr(), wsr.data_ptr(),
                          wsr.numel()) == -2
    assert lib.smoe_route_noalloc(cx, stream, eib.data_ptr(), 32, 2, E_big, se.data_ptr(), se.data_ptr(), off.data_ptr()) == -2
    torch.cuda.synchronize()
    for t in (Y, Hpre, H, dX, dW1, dW2, dg):
        assert bool((t == 7.0).all()), "a refused call wrote to an output"
    assert bool((se == -7).all()) and bool((off == -7).all())
    # the same calls with valid arguments go through
    assert fwd(ws.data_ptr(), need) == 0 and bwd(needb) == 0
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Y.float()).all()) and not bool((dW1 == 7.0).all())


def test_error_codes(smoe):
    cfg = si.CONFIGS["C1"]
    case = si.mlp_case(cfg, 0)
    gi, gg = smoe.topk_gate(case["logits"].cuda(), cfg.k)
    r = smoe.route(gi, cfg.E)
    X, W1 = case["X"].cuda(), case["W1"].cuda()
    with pytest.raises(smoe.SmoeError, match="invalid"):
        smoe.topk_gate(case["logits"].cuda(), cfg.E + 1)
    with pytest.raises(smoe.SmoeError, match="invalid"):
        smoe.plinear_fwd(X, W1, r, cfg.k + 1)                       # fan-out does not match Tk
    with pytest.raises(smoe.SmoeError, match="invalid"):
        smoe.plinear_fwd(X, W1, r, cfg.k, gg, False, True)          # gates need scattered output
    Xodd = torch.zeros(cfg.T, 66, device="cuda")
    Wodd = torch.zeros(cfg.E, 66, 66, device="cuda")
    with pytest.raises(smoe.SmoeError, match="unsupported"):
        smoe.plinear_fwd(Xodd, Wodd, r, cfg.k)                      # width not a multiple of 16 bytes
