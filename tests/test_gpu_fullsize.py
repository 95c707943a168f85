"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The oracle cannot run a whole pass at these sizes, so it evaluates what it can compute one by
one: complete rows of Y / dX / dgates / Hpre / H for a seeded sample of tokens that covers
every expert, and sampled rows of dW2[e] and columns of dW1[e] for every expert (each needs
all tokens routed to e).  Routing is compared whole and bit-exact.  Same tolerances as the
small cases.
"""
import time

import numpy as np
import pytest
import torch

import oracle
import smoe_inputs as si
from helpers import ROW_MIN_WIDTH, TOL, oracle_gates_f32, oracle_routing, rel_err, row_rel_err

pytestmark = pytest.mark.gpu


def _log(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def smoe():
    import paper_2403_08245_amd as m
    assert torch.cuda.is_available()
    m.ctx()
    return m


class ExpertCache:
    """float64 views of the experts' matrices (conversion is the slow part of a sampled check): all of them
    when they fit a few GB, else the most recent two."""

    def __init__(self, w32: np.ndarray, keep: int | None = None):
        if keep is None:
            keep = w32.shape[0] if w32.size * 8 <= 12e9 else 2
        self.w, self.keep, self.cache, self.shape = w32, keep, {}, w32.shape

    def __getitem__(self, e):
        e = int(e)
        if e not in self.cache:
            if len(self.cache) >= self.keep:
                self.cache.pop(next(iter(self.cache)))
            self.cache[e] = self.w[e].astype(np.float64)
        return self.cache[e]


def _sample_tokens(ei, E, per_expert, seed, o, off, k):
    """Tokens covering every non-empty expert (rarest included), ordered by expert pair for cache reuse.  The
    routed rows are taken from the first, a middle and the last (usually ragged) 256-row tile of every
    expert's segment in equal shares, so that every position of a persistent block's tile list is visited."""
    rng = np.random.default_rng(seed)
    chosen = set()
    for e in range(E):
        lo, hi = int(off[e]), int(off[e + 1])
        if hi == lo:
            continue
        tiles = (hi - lo + 255) // 256
        picks = sorted({0, tiles // 2, tiles - 1})
        for n, tile in enumerate(picks):
            a, b = lo + tile * 256, min(lo + tile * 256 + 256, hi)
            want = max(per_expert // len(picks) + (1 if n < per_expert % len(picks) else 0), 1)
            here = o[a:b] // k
            have = sum(1 for t in here.tolist() if t in chosen)      # tokens picked for other experts count too
            fresh = np.asarray([t for t in here.tolist() if t not in chosen], dtype=np.int64)
            if want > have and len(fresh):
                chosen.update(rng.choice(fresh, size=min(want - have, len(fresh)), replace=False).tolist())
    return sorted(chosen, key=lambda t: tuple(sorted(ei[t].tolist())))


def _sample_units(d_expert, n, rng):
    """n hidden units from n different 256-wide column tiles (all of them when there are fewer tiles)."""
    tiles = (d_expert + 255) // 256
    units = []
    for t in rng.choice(tiles, size=min(n, tiles), replace=False):
        units.append(int(rng.integers(t * 256, min(t * 256 + 256, d_expert))))
    return np.asarray(sorted(units), dtype=np.int64)


def _check(name, gpu, ref, tol, scale=None, rows=True):
    g = gpu.detach().to(torch.float32).cpu().numpy().astype(np.float64) if isinstance(gpu, torch.Tensor) else gpu
    assert np.isfinite(g).all(), name
    denom = scale if scale is not None else np.abs(ref).max()
    err = float(np.abs(g - ref).max() / (denom if denom > 0 else 1.0))
    assert err <= tol, f"{name}: {err:.3e} > {tol}"
    if rows and scale is None and np.ndim(ref) >= 2 and np.shape(ref)[-1] >= ROW_MIN_WIDTH:
        er = row_rel_err(g, ref)            # every sampled row against its own scale
        assert er <= tol, f"{name}: per-row {er:.3e} > {tol}"
    return err


def _run_fullsize(smoe, cfg, seed, tokens_per_expert, dw_samples, backward=True, last_rows=0):
    t0 = time.time()
    td = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    tol = TOL[td]
    case = si.mlp_case(cfg, seed, with_grad=backward)
    _log(f"{cfg.name}: inputs generated in {time.time() - t0:.1f}s")
    logits = case["logits"].cuda()
    gi, gg = smoe.topk_gate(logits, cfg.k)
    r = smoe.route(gi, cfg.E)
    ei, g, se, o, off = oracle_routing(case["logits"], cfg.k, cfg.E)
    assert np.array_equal(gi.cpu().numpy(), ei)
    assert np.abs(gg.cpu().numpy() - g).max() <= 1e-6
    assert np.array_equal(r.sorted_expert_idxs.cpu().numpy(), se)
    assert np.array_equal(r.sorted_scattered_idxs.cpu().numpy(), o)
    assert np.array_equal(r.expert_offsets.cpu().numpy(), off)
    _log(f"{cfg.name}: routing bit-exact, rows per expert {np.diff(off).tolist()[:16]}")

    X, W1, W2 = (case[n].cuda() for n in ("X", "W1", "W2"))
    buf = smoe.MLPBuffers(cfg.T, cfg.k, cfg.E, cfg.d_model, cfg.d_expert, cfg.act, td, X.device, training=backward)
    Y, _ = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act, buf, training=backward)
    if backward:
        dYd = case["dY"].cuda()
        dX, dW1, dW2, dg = smoe.mlp_bwd(dYd, X, W1, W2, r, cfg.k, gg, cfg.act, buf)
    torch.cuda.synchronize()
    _log(f"{cfg.name}: GPU pass done at {time.time() - t0:.1f}s")

    g64 = oracle_gates_f32(g)
    X32 = si.as_f32(case["X"])
    W1c, W2c = ExpertCache(si.as_f32(case["W1"])), ExpertCache(si.as_f32(case["W2"]))
    dY32 = si.as_f32(case["dY"]) if backward else None
    inv = np.empty(cfg.Tk, dtype=np.int64)
    inv[o] = np.arange(cfg.Tk)                     # sorted position of every slot
    toks = _sample_tokens(ei, cfg.E, tokens_per_expert, seed, o, off, cfg.k)
    if last_rows:
        # tokens with a slot among the last expert-sorted rows: the output tiles the persistent kernels reach
        # last, where a partly filled last round has its contraction split over several blocks
        tail = np.unique(o[cfg.Tk - last_rows:] // cfg.k)
        extra = np.random.default_rng(seed + 2).choice(tail, size=min(8, len(tail)), replace=False).tolist()
        toks = toks + sorted(set(extra) - set(toks), key=lambda t: tuple(sorted(ei[t].tolist())))
    Yc, dXc, dgc = Y.float().cpu().numpy(), None, None
    if backward:
        dXc, dgc = dX.float().cpu().numpy(), dg.cpu().numpy()
        Hpre_c, H_c = buf.Hpre, buf.H
    # per-tensor scales for the normalised error come from the sampled reference rows themselves
    refs = {"Y": [], "dX": [], "dg": [], "Hpre": [], "H": []}
    gots = {k: [] for k in refs}
    for n, t in enumerate(toks):
        y, hpre, h, yhat = oracle.mlp_token_fwd(X32[t], ei[t], g64[t], W1c, W2c, cfg.act)
        refs["Y"].append(y); gots["Y"].append(Yc[t])
        if backward:
            dx, dgt, dhpre, _ = oracle.mlp_token_bwd(X32[t], dY32[t], ei[t], g64[t], W1c, W2c, cfg.act)
            refs["dX"].append(dx); gots["dX"].append(dXc[t])
            refs["dg"].append(dgt); gots["dg"].append(dgc[t])
            rows = inv[t * cfg.k:(t + 1) * cfg.k]
            refs["Hpre"].append(hpre); gots["Hpre"].append(Hpre_c[torch.from_numpy(rows).cuda()].float().cpu().numpy())
            refs["H"].append(h); gots["H"].append(H_c[torch.from_numpy(rows).cuda()].float().cpu().numpy())
        if n % 8 == 0:
            _log(f"{cfg.name}: oracle token {n + 1}/{len(toks)} at {time.time() - t0:.1f}s")
    errs = {}
    for k in refs:
        if refs[k]:
            errs[k] = _check(f"{cfg.name} {k}", np.stack(gots[k]).astype(np.float64), np.stack(refs[k]), tol)
    if backward:
        # sampled entries of one weight-gradient tensor are pooled over all experts and judged
        # against the largest sampled reference magnitude (the per-tensor normalisation of the
        # tolerance; a single expert with one routed token is not a tensor-wide scale)
        rng = np.random.default_rng(seed + 1)
        r2, g2, r1, g1 = [], [], [], []
        for e in range(cfg.E):
            units = _sample_units(cfg.d_expert, dw_samples, rng)
            ref2 = oracle.mlp_dW2_rows(dY32, X32, W1c, W2c, ei, g64, cfg.act, e, units)
            got2 = dW2[e][torch.from_numpy(units).cuda()].float().cpu().numpy().astype(np.float64)
            ref1 = oracle.mlp_dW1_cols(dY32, X32, W1c, W2c, ei, g64, cfg.act, e, units)
            cols = [units] + ([units + cfg.d_expert] if cfg.act == si.ACT_SWIGLU else [])
            got1 = np.stack([dW1[e][:, torch.from_numpy(c).cuda()].float().cpu().numpy().T for c in cols], 1)
            if off[e + 1] == off[e]:
                assert np.abs(got2).max() == 0 and np.abs(got1).max() == 0      # empty expert: zeros written
            r2.append(ref2); g2.append(got2); r1.append(ref1); g1.append(got1.astype(np.float64))
            if e % 8 == 0:
                _log(f"{cfg.name}: dW samples expert {e} at {time.time() - t0:.1f}s")
        # (no per-row scale here: a sampled row of dW2 / column of dW1 is a hidden-unit scalar per token times a
        # token row, and with one or two tokens in an expert that scalar can be a near-cancelled sum)
        errs["dW2"] = _check(f"{cfg.name} dW2 rows", np.stack(g2), np.stack(r2), tol, rows=False)
        errs["dW1"] = _check(f"{cfg.name} dW1 cols", np.stack(g1), np.stack(r1), tol, rows=False)
    _log(cfg.name, "max rel err:", {k: f"{v:.2e}" for k, v in errs.items()}, f"({time.time() - t0:.1f}s)")


def test_C2_small_bf16_sampled(smoe):
    _run_fullsize(smoe, si.CONFIGS["C2"], 0, tokens_per_expert=6, dw_samples=4)


def test_C3_mixtral_layer_sampled(smoe):
    _run_fullsize(smoe, si.CONFIGS["C3"], 0, tokens_per_expert=8, dw_samples=8, last_rows=512)


@pytest.mark.parametrize("d_model,d_expert", [(3072, 2816), (3104, 2848)])
def test_partial_last_round_split_sampled(smoe, d_model, d_expert):
    """Just over 256 output tiles per product, so the persistent kernels run one full round of whole tiles
    and then a round under a quarter full, whose long contraction is cut into chunks run by the idle blocks
    (fp32 partial tiles added by a second kernel).  Contractions that are and are not a multiple of 128;
    the sample takes rows from the first tiles and from the last ones."""
    cfg = si.custom(f"tail{d_model}", T=2560, d_model=d_model, d_expert=d_expert, E=8, k=2, act=si.ACT_GELU, dtype="bf16")
    _, off = np.unique(oracle.topk_gate(si.mlp_case(cfg, 12)["logits"].numpy(), cfg.k)[0], return_counts=True)
    m_tiles = int(((off + 255) // 256).sum())
    for width in (d_model, d_expert):     # output widths of the second product / first input gradient, and of dH
        tiles = m_tiles * ((width + 255) // 256)
        assert tiles > 256 and tiles % 256 <= 64, (m_tiles, tiles)
    _run_fullsize(smoe, cfg, 12, tokens_per_expert=2, dw_samples=1, last_rows=600)
    # the chunks' partial tiles are added in a fixed order: two runs agree bit for bit
    case = si.mlp_case(cfg, 12)
    gi, gg = smoe.topk_gate(case["logits"].cuda(), cfg.k)
    r = smoe.route(gi, cfg.E)
    X, W1, W2, dY = (case[n].cuda() for n in ("X", "W1", "W2", "dY"))
    runs = []
    for _ in range(2):
        Y, buf = smoe.mlp_fwd(X, W1, W2, r, cfg.k, gg, cfg.act)
        grads = smoe.mlp_bwd(dY, X, W1, W2, r, cfg.k, gg, cfg.act, buf)
        runs.append([t.clone() for t in (Y,) + tuple(grads)])
    for a, b in zip(*runs):
        assert torch.equal(a, b)


def test_C4_granular_sampled(smoe):
    _run_fullsize(smoe, si.CONFIGS["C4"], 0, tokens_per_expert=4, dw_samples=2)


@pytest.mark.parametrize("name", ["G4", "G16"])
def test_unit_benchmark_shapes_sampled(smoe, name):
    """Sec. 4.1 / 4.2 shapes (d_model 4096, d_expert = 8192/k, E = 8k, 61440 tokens): the headline k = 4 and the
    finest granularity k = 16 (128 experts, 983040 routed rows)."""
    _run_fullsize(smoe, si.CONFIGS[name], 0, tokens_per_expert=4, dw_samples=2)


@pytest.mark.parametrize("name", ["C4-decode", "C4-decode-masked"])
def test_C4_decode_forward_only(smoe, name):
    cfg = si.CONFIGS[name]
    _run_fullsize(smoe, cfg, 1, tokens_per_expert=1, dw_samples=1, backward=False)


def test_decode_with_four_tokens_mostly_empty_experts(smoe):
    cfg = si.custom("decode-T4", T=4, d_model=2048, d_expert=512, E=64, k=8, act=si.ACT_SWIGLU, dtype="bf16")
    _run_fullsize(smoe, cfg, 2, tokens_per_expert=1, dw_samples=1, backward=True)


# ------------------------------------------------------------------ Mixture-of-Attention projections (Alg. 4)
def test_C5_moa_projections_scatter_to_scatter(smoe):
    """Both ParallelLinears of Alg. 4 run scattered -> scattered: Q = PL(X, W_Q) with fan-out k and no
    weights, O = PL(Ohat, W_O, p).  The attention between them is replaced by seeded values."""
    p = si.MOA_C5
    T, dm, E, k, do = p["T"], p["d_model"], p["E"], p["k"], p["d_out"]
    t0 = time.time()
    cq = si.plinear_case(T, dm, do, E, k, "bf16", seed=5)
    co = si.plinear_case(T, do, dm, E, k, "bf16", seed=6, x_rows=T * k)
    ei, g, se, o, off = oracle_routing(cq["logits"], k, E)
    gi, gg = smoe.topk_gate(cq["logits"].cuda(), k)
    r = smoe.route(gi, E)
    assert np.array_equal(r.sorted_scattered_idxs.cpu().numpy(), o)
    Xd, WQ, Oh, WO = cq["X"].cuda(), cq["W"].cuda(), co["X"].cuda(), co["W"].cuda()
    Q, _ = smoe.plinear_fwd(Xd, WQ, r, k, None, False, False)                 # [Tk, 512] scattered
    Oout, Ohat_y = smoe.plinear_fwd(Oh, WO, r, 1, gg, False, False)           # [T, 2048]
    dQ = cq["dY_Tk"].cuda()
    dXq, dWQ, _ = smoe.plinear_bwd(dQ, Xd, WQ, Q, r, k, None, False, False)
    dO = co["dY_T"].cuda()
    dOh, dWO, dgo = smoe.plinear_bwd(dO, Oh, WO, Ohat_y, r, 1, gg, False, False)
    torch.cuda.synchronize()
    _log(f"C5: GPU done at {time.time() - t0:.1f}s")
    tol = TOL[torch.bfloat16]
    # The oracle runs on restrictions of the same problem: a subset of tokens (rows of the
    # outputs and input gradients depend on one token only) and, for the weight gradients,
    # all tokens but a single input feature (row c of dW[e] depends on column c of the input only).
    X64, WQ64, Oh64, WO64 = (si.as_f64(t) for t in (cq["X"], cq["W"], co["X"], co["W"]))
    dQ64, dO64 = si.as_f64(cq["dY_Tk"]), si.as_f64(co["dY_T"])
    assert np.abs(gg.cpu().numpy() - g).max() <= 1e-6
    g64 = oracle_gates_f32(g)
    rng = np.random.default_rng(7)
    S = np.sort(rng.choice(T, size=48, replace=False))
    slots = (S[:, None] * k + np.arange(k)[None, :]).reshape(-1)
    se_s, o_s, off_s = oracle.route(ei[S], E)
    Q_ref, _ = oracle.plinear_fwd(X64[S], WQ64, se_s, o_s, k, None, False, False)
    O_ref, _ = oracle.plinear_fwd(Oh64[slots], WO64, se_s, o_s, 1, g64[S], False, False)
    dX_ref, _, _ = oracle.plinear_bwd(dQ64[slots], X64[S], WQ64, se_s, o_s, k, None, False, False)
    dOh_ref, _, dg_ref = oracle.plinear_bwd(dO64[S], Oh64[slots], WO64, se_s, o_s, 1, g64[S], False, False)
    St, sl = torch.from_numpy(S).cuda(), torch.from_numpy(slots).cuda()
    errs = dict(Q=_check("Q", Q[sl], Q_ref, tol), O=_check("O", Oout[St], O_ref, tol),
                dX=_check("dX", dXq[St], dX_ref, tol), dOhat=_check("dOhat", dOh[sl], dOh_ref, tol),
                dgates=_check("dgates", dgo[St], dg_ref, tol))
    _log(f"C5: row checks done at {time.time() - t0:.1f}s")
    c = int(rng.integers(0, dm))
    _, dWQ_ref, _ = oracle.plinear_bwd(dQ64, X64[:, [c]], WQ64[:, [c], :], se, o, k, None, False, False)
    errs["dWQ"] = _check("dW_Q row", dWQ[:, c, :], dWQ_ref[:, 0, :], tol)
    c2 = int(rng.integers(0, do))
    _, dWO_ref, _ = oracle.plinear_bwd(dO64, Oh64[:, [c2]], WO64[:, [c2], :], se, o, 1, g64, False, False)
    errs["dWO"] = _check("dW_O row", dWO[:, c2, :], dWO_ref[:, 0, :], tol)
    _log("C5 max rel err:", {k_: f"{v:.2e}" for k_, v in errs.items()}, f"({time.time() - t0:.1f}s)")
