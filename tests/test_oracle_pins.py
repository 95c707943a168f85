"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle is checked against things other than itself: hand-derived worked
examples (tests/golden), scalar brute force, reductions to a dense MLP computed
with a library matmul, permutation invariance, central finite differences,
routing invariants and a counting-sort brute force, grouped/scattered flag
consistency, and Alg. 2 evaluated step by step.  A final group plants typical
mistakes into copies of the oracle and checks that the pins catch each one.
"""
import json
import math
import os

import numpy as np
import pytest

import oracle
from oracle import ACT_GELU, ACT_NONE, ACT_SWIGLU

RNG = np.random.default_rng


def _load(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return json.load(f)


def _rand_problem(seed, T=7, d_model=5, d_expert=6, E=3, k=2, act=ACT_GELU):
    r = RNG(seed)
    d_h = oracle.hidden_width(act, d_expert)
    X = r.standard_normal((T, d_model))
    W1 = r.standard_normal((E, d_model, d_h)) * 0.5
    W2 = r.standard_normal((E, d_expert, d_model)) * 0.5
    logits = r.standard_normal((T, E)).astype(np.float32)
    dY = r.standard_normal((T, d_model))
    ei, g = oracle.topk_gate(logits, k)
    return X, W1, W2, ei, g, dY


# ---------------------------------------------------------------- goldens
def test_golden_mlp_k1(golden_dir):
    G = _load(golden_dir, "smoe_mlp_hand_examples.json")
    c = G["k1"]
    out = oracle.mlp_fwd(c["X"], G["W1"], G["W2"], np.array(c["expert_idxs"]), np.array(c["gates"]), ACT_NONE)
    np.testing.assert_allclose(out["Y"], c["Y"], atol=1e-14)
    np.testing.assert_allclose(out["H"], c["H"], atol=1e-14)


def test_golden_mlp_k2_forward_and_gradients(golden_dir):
    G = _load(golden_dir, "smoe_mlp_hand_examples.json")
    c = G["k2"]
    ei, g = np.array(c["expert_idxs"]), np.array(c["gates"])
    out = oracle.mlp_fwd(c["X"], G["W1"], G["W2"], ei, g, ACT_NONE)
    np.testing.assert_allclose(out["Y"], c["Y"], atol=1e-14)
    np.testing.assert_allclose(out["H"], c["H"], atol=1e-14)
    np.testing.assert_allclose(out["Yhat"], c["Yhat"], atol=1e-14)
    grads = oracle.mlp_bwd(c["dY"], c["X"], G["W1"], G["W2"], ei, g, ACT_NONE)
    np.testing.assert_allclose(grads["dgates"], c["dgates"], atol=1e-14)
    np.testing.assert_allclose(grads["dX"], c["dX"], atol=1e-14)
    np.testing.assert_allclose(grads["dW1"], c["dW1"], atol=1e-14)
    np.testing.assert_allclose(grads["dW2"], c["dW2"], atol=1e-14)


def test_golden_plinear_matches_hand_example(golden_dir):
    """Alg. 3 composed from two Alg. 1 calls reproduces the hand example."""
    G = _load(golden_dir, "smoe_mlp_hand_examples.json")
    c = G["k2"]
    ei = np.array(c["expert_idxs"])
    se, o, off = oracle.route(ei, 2)
    H, _ = oracle.plinear_fwd(c["X"], G["W1"], se, o, 2, None, False, True)
    np.testing.assert_allclose(H, np.array(c["H"])[o], atol=1e-14)
    Y, Yhat = oracle.plinear_fwd(H, G["W2"], se, o, 1, np.array(c["gates"]), True, False)
    np.testing.assert_allclose(Y, c["Y"], atol=1e-14)
    np.testing.assert_allclose(Yhat, c["Yhat"], atol=1e-14)


def test_golden_routing(golden_dir):
    G = _load(golden_dir, "routing_hand_examples.json")
    s = G["sort"]
    se, o, off = oracle.route(np.array(s["expert_idxs"]), s["E"])
    assert se.tolist() == s["sorted_expert_idxs"]
    assert o.tolist() == s["sorted_scattered_idxs"]
    assert off.tolist() == s["expert_offsets"]
    t = G["topk"]
    logits = np.log(np.array(t["logits_exp"])).astype(np.float32)
    ei, g = oracle.topk_gate(logits, t["k"])
    assert ei.tolist() == t["expert_idxs"]
    np.testing.assert_allclose(g, t["gates"], atol=1e-6)


def test_golden_activations(golden_dir):
    G = _load(golden_dir, "activation_textbook_values.json")
    np.testing.assert_allclose(oracle.act_fwd(ACT_GELU, np.array(G["gelu"]["x"])), G["gelu"]["y"], atol=1e-14)
    x = np.array(G["silu"]["x"])
    pre = np.concatenate([x, np.ones_like(x)])            # gate = x, up = 1  -> silu(x)
    np.testing.assert_allclose(oracle.act_fwd(ACT_SWIGLU, pre), G["silu"]["y"], atol=1e-14)
    pre2 = np.concatenate([x, np.full_like(x, -3.0)])     # up scales linearly
    np.testing.assert_allclose(oracle.act_fwd(ACT_SWIGLU, pre2), -3.0 * np.array(G["silu"]["y"]), atol=1e-14)


# ---------------------------------------------------------------- brute force
def _scalar_act(act, pre, d_expert):
    if act == ACT_NONE:
        return list(pre)
    if act == ACT_GELU:
        return [0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in pre]
    return [pre[c] / (1.0 + math.exp(-pre[c])) * pre[c + d_expert] for c in range(d_expert)]


def _brute_mlp(X, W1, W2, ei, g, act):
    """Scalar loops over (t, j, c, r): no numpy arithmetic."""
    T, dm = X.shape
    d_expert = W2.shape[1]
    d_h = W1.shape[2]
    Y = [[0.0] * dm for _ in range(T)]
    for t in range(T):
        for j in range(ei.shape[1]):
            e = int(ei[t, j])
            pre = [sum(float(X[t, r]) * float(W1[e, r, c]) for r in range(dm)) for c in range(d_h)]
            h = _scalar_act(act, pre, d_expert)
            for r in range(dm):
                Y[t][r] += float(g[t, j]) * sum(h[c] * float(W2[e, c, r]) for c in range(d_expert))
    return np.array(Y)


@pytest.mark.parametrize("act", [ACT_NONE, ACT_GELU, ACT_SWIGLU])
def test_forward_vs_scalar_brute_force(act):
    X, W1, W2, ei, g, _ = _rand_problem(1, T=6, d_model=4, d_expert=3, E=3, k=2, act=act)
    out = oracle.mlp_fwd(X, W1, W2, ei, g, act)
    np.testing.assert_allclose(out["Y"], _brute_mlp(X, W1, W2, ei, g, act), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- dense reductions
def _dense_mlp(X, w1, w2, act):
    pre = np.matmul(X, w1)
    if act == ACT_GELU:
        from scipy.stats import norm
        h = pre * norm.cdf(pre)
    elif act == ACT_SWIGLU:
        d = pre.shape[1] // 2
        from scipy.special import expit
        h = pre[:, :d] * expit(pre[:, :d]) * pre[:, d:]
    else:
        h = pre
    return np.matmul(h, w2)


@pytest.mark.parametrize("act", [ACT_NONE, ACT_GELU, ACT_SWIGLU])
def test_single_expert_is_dense_mlp(act):
    X, W1, W2, _, _, _ = _rand_problem(2, T=9, E=1, k=1, act=act)
    ei = np.zeros((9, 1), dtype=np.int32)
    g = np.ones((9, 1))
    out = oracle.mlp_fwd(X, W1, W2, ei, g, act)
    np.testing.assert_allclose(out["Y"], _dense_mlp(X, W1[0], W2[0], act), atol=1e-12)


@pytest.mark.parametrize("act", [ACT_GELU, ACT_SWIGLU])
def test_identical_experts_with_gates_summing_to_one_is_dense(act):
    X, W1, W2, ei, g, _ = _rand_problem(3, T=8, E=4, k=3, act=act)
    W1[:] = W1[0]
    W2[:] = W2[0]
    assert np.allclose(g.sum(1), 1.0)
    out = oracle.mlp_fwd(X, W1, W2, ei, g, act)
    np.testing.assert_allclose(out["Y"], _dense_mlp(X, W1[0], W2[0], act), atol=1e-12)


def test_identity_activation_collapses_to_product_of_matrices():
    X, W1, W2, ei, g, _ = _rand_problem(4, T=8, E=3, k=2, act=ACT_NONE)
    out = oracle.mlp_fwd(X, W1, W2, ei, g, ACT_NONE)
    P = np.einsum("eij,ejk->eik", W1, W2)
    ref = np.zeros_like(out["Y"])
    for t in range(8):
        for j in range(2):
            ref[t] += g[t, j] * (X[t] @ P[ei[t, j]])
    np.testing.assert_allclose(out["Y"], ref, atol=1e-12)


def test_plinear_single_expert_is_matmul():
    r = RNG(5)
    X = r.standard_normal((10, 4))
    W = r.standard_normal((1, 4, 3))
    se = np.zeros(10, dtype=np.int32)
    o = np.arange(10)
    Y, _ = oracle.plinear_fwd(X, W, se, o, 1)
    np.testing.assert_allclose(Y, np.matmul(X, W[0]), atol=1e-13)
    dY = r.standard_normal((10, 3))
    dX, dW, dp = oracle.plinear_bwd(dY, X, W, se, o, 1)
    np.testing.assert_allclose(dX, np.matmul(dY, W[0].T), atol=1e-13)       # Sec. 3.2.1
    np.testing.assert_allclose(dW[0], np.matmul(X.T, dY), atol=1e-13)
    assert dp is None


# ---------------------------------------------------------------- permutation invariance
@pytest.mark.parametrize("act", [ACT_GELU, ACT_SWIGLU])
def test_token_permutation_invariance(act):
    X, W1, W2, ei, g, dY = _rand_problem(6, T=11, E=4, k=2, act=act)
    perm = RNG(60).permutation(11)
    a = oracle.mlp_fwd(X, W1, W2, ei, g, act)
    b = oracle.mlp_fwd(X[perm], W1, W2, ei[perm], g[perm], act)
    np.testing.assert_allclose(b["Y"], a["Y"][perm], atol=1e-12)
    ga = oracle.mlp_bwd(dY, X, W1, W2, ei, g, act)
    gb = oracle.mlp_bwd(dY[perm], X[perm], W1, W2, ei[perm], g[perm], act)
    np.testing.assert_allclose(gb["dX"], ga["dX"][perm], atol=1e-12)
    np.testing.assert_allclose(gb["dgates"], ga["dgates"][perm], atol=1e-12)
    np.testing.assert_allclose(gb["dW1"], ga["dW1"], atol=1e-12)
    np.testing.assert_allclose(gb["dW2"], ga["dW2"], atol=1e-12)


# ---------------------------------------------------------------- finite differences
def _fd(f, arr, idx, h=1e-6):
    old = arr[idx]
    arr[idx] = old + h
    fp = f()
    arr[idx] = old - h
    fm = f()
    arr[idx] = old
    return (fp - fm) / (2 * h)


@pytest.mark.parametrize("act", [ACT_NONE, ACT_GELU, ACT_SWIGLU])
def test_mlp_gradients_vs_finite_differences(act):
    X, W1, W2, ei, g, dY = _rand_problem(7, T=5, d_model=4, d_expert=3, E=3, k=2, act=act)
    grads = oracle.mlp_bwd(dY, X, W1, W2, ei, g, act)
    loss = lambda: float((oracle.mlp_fwd(X, W1, W2, ei, g, act)["Y"] * dY).sum())
    r = RNG(70)
    for name, arr, garr in (("dX", X, grads["dX"]), ("dW1", W1, grads["dW1"]),
                            ("dW2", W2, grads["dW2"]), ("dgates", g, grads["dgates"])):
        for _ in range(12):
            idx = tuple(int(r.integers(0, s)) for s in arr.shape)
            num = _fd(loss, arr, idx)
            assert abs(num - garr[idx]) <= 1e-6 * max(1.0, abs(num)), (name, idx, num, garr[idx])


@pytest.mark.parametrize("gin,gout,with_p", [(False, False, False), (False, True, False), (True, False, False),
                                             (True, True, False), (False, False, True), (True, False, True)])
def test_plinear_gradients_vs_finite_differences(gin, gout, with_p):
    r = RNG(8)
    T, k, E, d_in, d_out = 6, 2, 3, 4, 3
    logits = r.standard_normal((T, E)).astype(np.float32)
    ei, g = oracle.topk_gate(logits, k)
    se, o, off = oracle.route(ei, E)
    X = r.standard_normal((T * k if gin else T, d_in))
    W = r.standard_normal((E, d_in, d_out))
    p = g.copy() if with_p else None
    fan = 1 if gin else k
    Y0, _ = oracle.plinear_fwd(X, W, se, o, fan, p, gin, gout)
    dY = r.standard_normal(Y0.shape)
    dX, dW, dp = oracle.plinear_bwd(dY, X, W, se, o, fan, p, gin, gout)
    loss = lambda: float((oracle.plinear_fwd(X, W, se, o, fan, p, gin, gout)[0] * dY).sum())
    checks = [(X, dX), (W, dW)] + ([(p, dp)] if with_p else [])
    for arr, garr in checks:
        for _ in range(10):
            idx = tuple(int(r.integers(0, s)) for s in arr.shape)
            num = _fd(loss, arr, idx)
            assert abs(num - garr[idx]) <= 1e-6 * max(1.0, abs(num))


def test_activation_derivatives_vs_finite_differences():
    r = RNG(9)
    for act in (ACT_GELU, ACT_SWIGLU):
        pre = r.standard_normal((3, 8)) * 2
        dH = r.standard_normal((3, 8 if act == ACT_GELU else 4))
        an = oracle.act_bwd(act, pre, dH)
        for idx in np.ndindex(*pre.shape):
            num = _fd(lambda: float((oracle.act_fwd(act, pre) * dH).sum()), pre, idx)
            assert abs(num - an[idx]) < 1e-7


# ---------------------------------------------------------------- routing
def _counting_sort(flat, E):
    buckets = [[] for _ in range(E)]
    for s, e in enumerate(flat):
        buckets[e].append(s)
    o = [s for b in buckets for s in b]
    se = [e for e, b in enumerate(buckets) for _ in b]
    off = [0]
    for b in buckets:
        off.append(off[-1] + len(b))
    return se, o, off


@pytest.mark.parametrize("T,E,k,seed", [(1, 1, 1, 0), (5, 3, 3, 1), (33, 8, 2, 2), (64, 64, 8, 3), (100, 7, 1, 4)])
def test_route_invariants_and_counting_sort(T, E, k, seed):
    logits = RNG(seed).standard_normal((T, E)).astype(np.float32)
    ei, g = oracle.topk_gate(logits, k)
    assert all(len(set(row)) == k for row in ei.tolist())           # k distinct experts per token
    np.testing.assert_allclose(g.sum(1), 1.0, atol=1e-12)
    assert (np.diff(g, axis=1) <= 1e-15).all()                      # slots by descending logit
    for t in range(T):                                              # kept logits dominate the rest
        rest = np.delete(logits[t], ei[t])
        assert rest.size == 0 or logits[t][ei[t]].min() >= rest.max()
    se, o, off = oracle.route(ei, E)
    flat = ei.reshape(-1)
    bse, bo, boff = _counting_sort(flat.tolist(), E)
    assert se.tolist() == bse and o.tolist() == bo and off.tolist() == boff
    assert sorted(o.tolist()) == list(range(T * k))
    assert (np.diff(se) >= 0).all()
    assert (flat[o] == se).all()
    assert off[0] == 0 and off[-1] == T * k
    assert (np.diff(off) == np.bincount(flat, minlength=E)).all()
    for e in range(E):
        assert (np.diff(o[off[e]:off[e + 1]]) > 0).all()            # stable: slots ascend in a segment


def test_topk_ties_go_to_lower_expert_id():
    logits = np.array([[1, 1, 1, 1], [0, 2, 2, 1], [3, 0, 3, 3]], dtype=np.float32)
    ei, g = oracle.topk_gate(logits, 2)
    assert ei.tolist() == [[0, 1], [1, 2], [0, 2]]
    np.testing.assert_allclose(g, 0.5)


def test_router_gradient_hand_example_and_closed_forms():
    # kept logits (ln 3, 0) give gates (3/4, 1/4); with dp = (1, 0) the softmax Jacobian gives
    # dlogit = g0 (1 - g0) = 3/16 on the first kept expert and -g0 g1 = -3/16 on the second
    logits = np.array([[-5.0, math.log(3.0), 0.0, -7.0]])
    ei, g = oracle.topk_gate(logits, 2)
    assert ei.tolist() == [[1, 2]]
    dl = oracle.topk_gate_bwd(ei, g, np.array([[1.0, 0.0]]), 4)
    np.testing.assert_allclose(dl, [[0.0, 3 / 16, -3 / 16, 0.0]], atol=1e-15)
    # k = 1: the only gate is the constant 1, no gradient reaches the router
    r = RNG(0)
    lg = r.standard_normal((6, 5))
    ei, g = oracle.topk_gate(lg, 1)
    assert np.abs(oracle.topk_gate_bwd(ei, g, r.standard_normal((6, 1)), 5)).max() == 0
    # softmax is shift invariant: every row of the gradient sums to zero; experts not kept get zero
    ei, g = oracle.topk_gate(lg, 3)
    dl = oracle.topk_gate_bwd(ei, g, r.standard_normal((6, 3)), 5)
    np.testing.assert_allclose(dl.sum(axis=1), 0, atol=1e-15)
    mask = np.ones_like(dl, dtype=bool)
    np.put_along_axis(mask, ei.astype(np.int64), False, axis=1)
    assert np.abs(dl[mask]).max() == 0 and np.abs(dl[~mask]).min() > 0


def test_router_gradient_vs_finite_differences():
    r = RNG(3)
    T, E, k = 5, 6, 3
    lg = r.permuted(np.tile(np.arange(E, dtype=np.float64), (T, 1)), axis=1) * 0.7 + r.uniform(-0.1, 0.1, (T, E))
    dp = r.standard_normal((T, k))
    ei, g = oracle.topk_gate(lg, k)
    dl = oracle.topk_gate_bwd(ei, g, dp, E)

    def loss(l):
        ei2, g2 = oracle.topk_gate(l, k)
        assert np.array_equal(ei2, ei)          # logits are 0.5 apart at least: the selection does not move
        return float((g2 * dp).sum())

    h = 1e-6
    for t in range(T):
        for e in range(E):
            lp, lm = lg.copy(), lg.copy()
            lp[t, e] += h
            lm[t, e] -= h
            assert abs((loss(lp) - loss(lm)) / (2 * h) - dl[t, e]) < 1e-8


def test_route_with_empty_experts_and_single_expert():
    se, o, off = oracle.route(np.array([[3, 3], [3, 3]]), 5)
    assert off.tolist() == [0, 0, 0, 0, 4, 4] and o.tolist() == [0, 1, 2, 3]
    with pytest.raises(ValueError):
        oracle.route(np.array([[5]]), 5)


# ---------------------------------------------------------------- flag combos (Fig. 2)
def test_grouped_and_scattered_variants_agree():
    r = RNG(10)
    T, k, E, d_in, d_out = 9, 2, 4, 5, 3
    ei, g = oracle.topk_gate(r.standard_normal((T, E)).astype(np.float32), k)
    se, o, off = oracle.route(ei, E)
    X = r.standard_normal((T, d_in))
    W = r.standard_normal((E, d_in, d_out))
    y_ss, _ = oracle.plinear_fwd(X, W, se, o, k, None, False, False)
    y_sg, _ = oracle.plinear_fwd(X, W, se, o, k, None, False, True)
    Xg = X[o // k]                                                  # the copy the method avoids
    y_gg, _ = oracle.plinear_fwd(Xg, W, se, o, 1, None, True, True)
    y_gs, _ = oracle.plinear_fwd(Xg, W, se, o, 1, None, True, False)
    np.testing.assert_allclose(y_sg, y_ss[o], atol=1e-14)
    np.testing.assert_allclose(y_gg, y_sg, atol=1e-14)
    np.testing.assert_allclose(y_gs, y_ss, atol=1e-14)
    # each scattered row is its token times its own expert's matrix
    flat = ei.reshape(-1)
    for s in range(T * k):
        np.testing.assert_allclose(y_ss[s], X[s // k] @ W[flat[s]], atol=1e-14)


@pytest.mark.parametrize("act", [ACT_GELU, ACT_SWIGLU])
def test_mlp_equals_two_plinears(act):
    """Alg. 3 (scatter->grouped, sigma, grouped->scatter with p) equals the per-token definition."""
    X, W1, W2, ei, g, dY = _rand_problem(11, T=10, E=4, k=2, act=act)
    se, o, off = oracle.route(ei, 4)
    Hpre, _ = oracle.plinear_fwd(X, W1, se, o, 2, None, False, True)
    H = oracle.act_fwd(act, Hpre)
    Y, Yhat = oracle.plinear_fwd(H, W2, se, o, 1, g, True, False)
    ref = oracle.mlp_fwd(X, W1, W2, ei, g, act)
    np.testing.assert_allclose(Y, ref["Y"], atol=1e-12)
    np.testing.assert_allclose(Yhat, ref["Yhat"], atol=1e-12)
    np.testing.assert_allclose(Hpre, ref["Hpre"][o], atol=1e-12)
    np.testing.assert_allclose(H, ref["H"][o], atol=1e-12)
    # backward through the same composition (Alg. 2 applied twice)
    dH, dW2, dg = oracle.plinear_bwd(dY, H, W2, se, o, 1, g, True, False)
    dHpre = oracle.act_bwd(act, Hpre, dH)
    dX, dW1, _ = oracle.plinear_bwd(dHpre, X, W1, se, o, 2, None, False, True)
    refg = oracle.mlp_bwd(dY, X, W1, W2, ei, g, act)
    np.testing.assert_allclose(dX, refg["dX"], atol=1e-12)
    np.testing.assert_allclose(dW1, refg["dW1"], atol=1e-12)
    np.testing.assert_allclose(dW2, refg["dW2"], atol=1e-12)
    np.testing.assert_allclose(dg, refg["dgates"], atol=1e-12)


# ---------------------------------------------------------------- Alg. 2 step by step
def _alg2_steps(dY, Yhat, X, W, se, o, off, k, p, grouped_in):
    """Alg. 2 as printed (group, groupXTY, scatter2scatter with W^T), matrix ops per expert."""
    Tk = len(o)
    E = W.shape[0]
    if p is not None:
        T, kp = p.shape
        dp = np.einsum("td,tjd->tj", dY, Yhat.reshape(T, kp, -1))              # bmm(dY, Yhat)
        dYbar = p.reshape(-1)[o][:, None] * dY[o // kp]                        # group(dY, o, p)
    else:
        dp = None
        dYbar = dY[o]                                                          # group(dY, o)
    Xbar = X if grouped_in else X[o // k]                                      # group(X, o)
    dW = np.zeros_like(W)
    dXbar = np.zeros((Tk, W.shape[1]))
    for e in range(E):
        lo, hi = off[e], off[e + 1]
        dW[e] = Xbar[lo:hi].T @ dYbar[lo:hi]                                   # groupXTY
        dXbar[lo:hi] = dYbar[lo:hi] @ W[e].T                                   # s2s with W^T
    if grouped_in:
        return dXbar, dW, dp
    scattered = np.zeros_like(dXbar)
    scattered[o] = dXbar
    return scattered.reshape(-1, k, W.shape[1]).sum(1), dW, dp


@pytest.mark.parametrize("gin,with_p", [(False, False), (False, True), (True, True), (True, False)])
def test_alg2_steps_equal_per_slot_gradients(gin, with_p):
    r = RNG(12)
    T, k, E, d_in, d_out = 8, 2, 3, 4, 5
    ei, g = oracle.topk_gate(r.standard_normal((T, E)).astype(np.float32), k)
    se, o, off = oracle.route(ei, E)
    X = r.standard_normal((T * k if gin else T, d_in))
    W = r.standard_normal((E, d_in, d_out))
    p = g if with_p else None
    fan = 1 if gin else k
    Y, Yhat = oracle.plinear_fwd(X, W, se, o, fan, p, gin, False)
    dY = r.standard_normal(Y.shape)
    dX, dW, dp = oracle.plinear_bwd(dY, X, W, se, o, fan, p, gin, False)
    sX, sW, sp = _alg2_steps(dY, Yhat, X, W, se, o, off, fan, p, gin)
    np.testing.assert_allclose(sX, dX, atol=1e-12)
    np.testing.assert_allclose(sW, dW, atol=1e-12)
    if with_p:
        np.testing.assert_allclose(sp, dp, atol=1e-12)


# ---------------------------------------------------------------- sampled dW entries
@pytest.mark.parametrize("act", [ACT_GELU, ACT_SWIGLU])
def test_sampled_weight_gradient_entries_match_full_pass(act):
    X, W1, W2, ei, g, dY = _rand_problem(13, T=12, d_model=5, d_expert=4, E=3, k=2, act=act)
    full = oracle.mlp_bwd(dY, X, W1, W2, ei, g, act)
    for e in range(3):
        rows = [0, 3]
        np.testing.assert_allclose(oracle.mlp_dW2_rows(dY, X, W1, W2, ei, g, act, e, rows),
                                   full["dW2"][e][rows], atol=1e-12)
        cols = oracle.mlp_dW1_cols(dY, X, W1, W2, ei, g, act, e, rows)
        for q, c in enumerate(rows):
            np.testing.assert_allclose(cols[q, 0], full["dW1"][e][:, c], atol=1e-12)
            if act == ACT_SWIGLU:
                np.testing.assert_allclose(cols[q, 1], full["dW1"][e][:, c + 4], atol=1e-12)


# ---------------------------------------------------------------- planted mistakes
def test_pins_catch_planted_mistakes(golden_dir, monkeypatch):
    """Typical slips (dropped gate, transposed weight, wrong slot->token map, unstable sort)
    must fail at least one pin; run on patched copies of the oracle, on the CPU."""
    import oracle.smoe_oracle as so
    G = _load(golden_dir, "smoe_mlp_hand_examples.json")
    c = G["k2"]
    ei, g = np.array(c["expert_idxs"]), np.array(c["gates"])

    def golden_fwd_ok():
        out = so.mlp_fwd(c["X"], G["W1"], G["W2"], ei, g, ACT_NONE)
        return np.allclose(out["Y"], c["Y"], atol=1e-12)

    def golden_bwd_ok():
        gr = so.mlp_bwd(c["dY"], c["X"], G["W1"], G["W2"], ei, g, ACT_NONE)
        return all(np.allclose(gr[n], c[n], atol=1e-12) for n in ("dX", "dW1", "dW2", "dgates"))

    assert golden_fwd_ok() and golden_bwd_ok()
    real_act_fwd = so.act_fwd
    # (1) activation off by a factor
    monkeypatch.setattr(so, "act_fwd", lambda act, h: 1.5 * real_act_fwd(act, h))
    assert not golden_fwd_ok()
    monkeypatch.setattr(so, "act_fwd", real_act_fwd)
    W1t = np.transpose(np.array(G["W1"], dtype=float), (0, 2, 1))
    out = so.mlp_fwd(c["X"], W1t, G["W2"], ei, g, ACT_NONE)              # (2) transposed W1
    assert not np.allclose(out["Y"], c["Y"])
    # (3) gate dropped in the backward
    gr = so.mlp_bwd(c["dY"], c["X"], G["W1"], G["W2"], ei, np.ones_like(g), ACT_NONE)
    assert not np.allclose(gr["dX"], c["dX"])
    # (4) unstable / descending sort would break the hand-sorted routing example
    R = _load(golden_dir, "routing_hand_examples.json")["sort"]
    flat = np.array(R["expert_idxs"]).reshape(-1)
    bad_o = np.argsort(-flat, kind="stable")[::-1]
    assert bad_o.tolist() != R["sorted_scattered_idxs"]
    # (5) slot->token map with the wrong fan-out is caught by the per-row check
    r = RNG(14)
    X = r.standard_normal((4, 3)); W = r.standard_normal((2, 3, 2))
    ei2 = np.array([[0, 1], [1, 0], [0, 1], [1, 0]])
    se, o, off = so.route(ei2, 2)
    good, _ = so.plinear_fwd(X, W, se, o, 2)
    bad, _ = so.plinear_fwd(np.repeat(X, 2, 0)[::-1].copy(), W, se, o, 1)
    assert not np.allclose(good, bad)


# ---------------------------------------------------------------- non-finite router logits (reading, Sec. 3.1 step 1)
NONFINITE_LOGITS = np.array([[np.nan, 1.0, -np.inf, 2.0],       # 2, 1, then the NaN (as -inf) before the real -inf: lower id
                             [np.nan, np.nan, np.nan, np.nan],  # nothing to choose from: ids in order, equal weights
                             [-np.inf, np.nan, 0.0, -np.inf],   # one number, then -inf ties by id
                             [3.0, np.nan, 3.0, 1.0]], dtype=np.float32)
NONFINITE_IDX = [[3, 1, 0], [0, 1, 2], [2, 0, 1], [0, 2, 3]]
E1 = float(np.e)
NONFINITE_GATES = [[E1 / (1 + E1), 1 / (1 + E1), 0.0], [1 / 3, 1 / 3, 1 / 3], [1.0, 0.0, 0.0],
                   [1 / (2 + np.exp(-2.0)), 1 / (2 + np.exp(-2.0)), np.exp(-2.0) / (2 + np.exp(-2.0))]]


def test_topk_gate_with_nan_and_infinite_logits():
    """The paper does not say what a NaN logit means.  Reading: NaN counts as -inf; kept logits that are all
    -inf share the weight equally.  Expected values worked out by hand (softmax of 2, 1, -inf is e/(1+e), 1/(1+e), 0)."""
    ei, g = oracle.topk_gate(NONFINITE_LOGITS, 3)
    assert ei.tolist() == NONFINITE_IDX
    np.testing.assert_allclose(g, NONFINITE_GATES, atol=1e-15)
    assert np.isfinite(g).all() and np.allclose(g.sum(1), 1.0)
