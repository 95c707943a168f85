"""Pins for the attention / SMoE multi-head attention oracle (Alg. 4); CPU only.

The oracle is checked against things other than itself: a library attention routine on the
special case it reduces to, closed forms (one position, zero queries, one key head of
constants), causality, central finite differences of every gradient, and the reduction of the
whole layer to a dense multi-head attention block when there is a single expert.
"""
import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng


def _qkv(seed, B=2, T=7, G=3, h=2, d=4):
    r = RNG(seed)
    return r.standard_normal((B, T, G, h, d)), r.standard_normal((B, T, h, d)), r.standard_normal((B, T, h, d))


def test_attention_matches_library_causal_attention():
    Q, K, V = _qkv(0)
    O, L = oracle.attention_fwd(Q, K, V)
    B, T, G, h, d = Q.shape
    for g in range(G):     # every query group is an ordinary causal multi-head attention over the shared keys
        q = torch.from_numpy(Q[:, :, g]).permute(0, 2, 1, 3)
        k = torch.from_numpy(K).permute(0, 2, 1, 3)
        v = torch.from_numpy(V).permute(0, 2, 1, 3)
        ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True).permute(0, 2, 1, 3).numpy()
        np.testing.assert_allclose(O[:, :, g], ref, atol=1e-12)


def test_attention_closed_forms():
    Q, K, V = _qkv(1)
    O, L = oracle.attention_fwd(Q, K, V)
    # the first position sees only itself
    np.testing.assert_allclose(O[:, 0], np.broadcast_to(V[:, 0][:, None], O[:, 0].shape), atol=1e-14)
    np.testing.assert_allclose(L[:, 0], np.einsum("bghd,bhd->bgh", Q[:, 0], K[:, 0]) / np.sqrt(Q.shape[-1]), atol=1e-13)
    # zero queries: uniform weights, O[t] is the running mean of V and the log-sum-exp is log(t+1)
    O0, L0 = oracle.attention_fwd(np.zeros_like(Q), K, V)
    T = Q.shape[1]
    run = np.cumsum(V, axis=1) / np.arange(1, T + 1)[None, :, None, None]
    np.testing.assert_allclose(O0, np.broadcast_to(run[:, :, None], O0.shape), atol=1e-13)
    np.testing.assert_allclose(L0, np.broadcast_to(np.log(np.arange(1, T + 1))[None, :, None, None], L0.shape), atol=1e-13)
    # constant values pass through whatever the weights are
    Vc = np.broadcast_to(np.arange(V.shape[-1], dtype=np.float64), V.shape)
    Oc, _ = oracle.attention_fwd(Q, K, Vc)
    np.testing.assert_allclose(Oc, np.broadcast_to(np.arange(V.shape[-1], dtype=np.float64), Oc.shape), atol=1e-13)


def test_attention_is_causal_and_sequences_are_independent():
    Q, K, V = _qkv(2)
    O, _ = oracle.attention_fwd(Q, K, V)
    K2, V2 = K.copy(), V.copy()
    K2[:, 4:] += 3.0
    V2[:, 4:] -= 2.0
    O2, _ = oracle.attention_fwd(Q, K2, V2)
    np.testing.assert_array_equal(O[:, :4], O2[:, :4])          # later keys never reach earlier queries
    assert np.abs(O[:, 4:] - O2[:, 4:]).max() > 1e-3
    K3 = K.copy()
    K3[1] += 1.0
    O3, _ = oracle.attention_fwd(Q, K3, V)
    np.testing.assert_array_equal(O[0], O3[0])                  # the other sequence is untouched


def test_attention_gradients_vs_finite_differences():
    Q, K, V = _qkv(3, B=1, T=5, G=2, h=2, d=3)
    dO = RNG(4).standard_normal(Q.shape)
    dQ, dK, dV = oracle.attention_bwd(dO, Q, K, V)
    loss = lambda q, k, v: float((oracle.attention_fwd(q, k, v)[0] * dO).sum())
    h = 1e-6
    for name, arr, grad in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        r = RNG(5)
        for _ in range(25):
            idx = tuple(r.integers(0, s) for s in arr.shape)
            ap, am = arr.copy(), arr.copy()
            ap[idx] += h
            am[idx] -= h
            args = {"Q": (ap, K, V), "K": (Q, ap, V), "V": (Q, K, ap)}[name], {"Q": (am, K, V), "K": (Q, am, V), "V": (Q, K, am)}[name]
            fd = (loss(*args[0]) - loss(*args[1])) / (2 * h)
            assert abs(fd - grad[idx]) < 1e-7, (name, idx, fd, grad[idx])


def _layer(seed, B=2, T=5, d_model=6, E=3, k=2, h=2, d=4):
    r = RNG(seed)
    N, d_out = B * T, h * d
    X = r.standard_normal((N, d_model))
    W_K, W_V = r.standard_normal((d_model, d_out)) * 0.4, r.standard_normal((d_model, d_out)) * 0.4
    W_Q, W_O = r.standard_normal((E, d_model, d_out)) * 0.4, r.standard_normal((E, d_out, d_model)) * 0.4
    ei, g = oracle.topk_gate(r.standard_normal((N, E)), k)
    return dict(X=X, W_K=W_K, W_V=W_V, W_Q=W_Q, W_O=W_O, expert_idxs=ei, gates=g, B=B, T=T, h_expert=h, d_head=d)


def test_single_expert_layer_is_dense_causal_attention_block():
    p = _layer(6, E=1, k=1)
    out = oracle.momha_fwd(**p)
    B, T, h, d = p["B"], p["T"], p["h_expert"], p["d_head"]
    to_heads = lambda a: torch.from_numpy(a).reshape(B, T, h, d).permute(0, 2, 1, 3)
    q, kk, v = to_heads(p["X"] @ p["W_Q"][0]), to_heads(p["X"] @ p["W_K"]), to_heads(p["X"] @ p["W_V"])
    att = torch.nn.functional.scaled_dot_product_attention(q, kk, v, is_causal=True).permute(0, 2, 1, 3).reshape(B * T, h * d)
    np.testing.assert_allclose(out["O"], att.numpy() @ p["W_O"][0], atol=1e-12)    # the only gate is 1


def test_layer_is_weighted_sum_over_slots_of_per_expert_attention():
    # identical experts and gates summing to one: the routing drops out
    p = _layer(7)
    p["W_Q"][:] = p["W_Q"][0]
    p["W_O"][:] = p["W_O"][0]
    out = oracle.momha_fwd(**p)
    q = dict(p, W_Q=p["W_Q"][:1], W_O=p["W_O"][:1], expert_idxs=np.zeros((p["X"].shape[0], 1), dtype=np.int32),
             gates=np.ones((p["X"].shape[0], 1)))
    np.testing.assert_allclose(out["O"], oracle.momha_fwd(**q)["O"], atol=1e-12)


def test_layer_gradients_vs_finite_differences():
    p = _layer(8)
    dO = RNG(9).standard_normal((p["X"].shape[0], p["X"].shape[1]))
    g = oracle.momha_bwd(dO, **p)
    loss = lambda q: float((oracle.momha_fwd(**q)["O"] * dO).sum())
    h = 1e-6
    r = RNG(10)
    for name, gname in (("X", "dX"), ("W_K", "dW_K"), ("W_V", "dW_V"), ("W_Q", "dW_Q"), ("W_O", "dW_O"), ("gates", "dgates")):
        for _ in range(12):
            idx = tuple(r.integers(0, s) for s in p[name].shape)
            qp, qm = dict(p), dict(p)
            qp[name], qm[name] = p[name].copy(), p[name].copy()
            qp[name][idx] += h
            qm[name][idx] -= h
            fd = (loss(qp) - loss(qm)) / (2 * h)
            assert abs(fd - g[gname][idx]) < 2e-7, (name, idx, fd, g[gname][idx])


def test_pins_catch_planted_attention_mistakes(monkeypatch):
    """A dropped scale, a missing mask and a transposed product each fail one of the pins above."""
    import oracle.momha_oracle as mo
    Q, K, V = _qkv(11)

    def lib(Q, K, V, g=0):
        q = torch.from_numpy(Q[:, :, g]).permute(0, 2, 1, 3)
        k, v = torch.from_numpy(K).permute(0, 2, 1, 3), torch.from_numpy(V).permute(0, 2, 1, 3)
        return torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True).permute(0, 2, 1, 3).numpy()

    good = mo._causal_scores
    for bad in (lambda q, k: good(q, k) * np.sqrt(q.shape[1]),                  # forgot 1/sqrt(d)
                lambda q, k: (q @ k.T) / np.sqrt(q.shape[1]),                   # forgot the mask
                lambda q, k: good(k, q)):                                       # swapped operands
        monkeypatch.setattr(mo, "_causal_scores", bad)
        O, _ = mo.attention_fwd(Q, K, V)
        assert np.abs(O[:, :, 0] - lib(Q, K, V)).max() > 1e-3
    monkeypatch.setattr(mo, "_causal_scores", good)
    O, _ = mo.attention_fwd(Q, K, V)
    assert np.abs(O[:, :, 0] - lib(Q, K, V)).max() < 1e-12


# ---------------------------------------------------------------- Alg. 4's slot -> expert and slot -> weight maps
# The reductions above (one expert, identical experts) cannot see which expert or which routing
# weight a slot uses.  The pins below can: a hand-derived example with three distinct experts and
# unequal weights, and the whole layer rebuilt from the separately pinned pieces (ParallelLinear of
# Alg. 1 / Alg. 2 and the attention) on distinct experts.  Each pin is a function of the pair
# (forward, backward) so that it can also be run on deliberately broken copies of the oracle.
LN3 = float(np.log(3.0))


def _ln3(v):
    """Golden entries written as [c, l] stand for c + l * ln 3."""
    a = np.asarray(v, dtype=np.float64)
    return a[..., 0] + a[..., 1] * LN3


def _hand_case(golden_dir):
    import json, os
    with open(os.path.join(golden_dir, "momha_hand_example.json")) as f:
        G = json.load(f)
    W_Q = (np.asarray(G["W_Q_ln3_halves"]) * LN3 / 2).reshape(3, 1, 1)
    args = dict(X=np.asarray(G["X"]), W_K=np.asarray(G["W_K"]), W_V=np.asarray(G["W_V"]), W_Q=W_Q,
                W_O=np.asarray(G["W_O"]), expert_idxs=np.asarray(G["expert_idxs"], dtype=np.int32),
                gates=np.asarray(G["gates"]), B=G["B"], T=G["T"], h_expert=G["h_expert"], d_head=G["d_head"])
    return G, args


def _hand_example_errors(golden_dir, fwd, bwd):
    """Largest deviation of (fwd, bwd) from the hand-derived numbers, forward and backward."""
    G, a = _hand_case(golden_dir)
    out = fwd(**a)
    ef = max(np.abs(out["O"] - np.asarray(G["O"])).max(), np.abs(out["Ohat"] - np.asarray(G["Ohat"])).max(),
             np.abs(out["Yhat"] - np.asarray(G["Yhat"])).max(), np.abs(out["K"] - np.asarray(G["K"])).max(),
             np.abs(out["V"] - np.asarray(G["V"])).max(), np.abs(out["Q"][:, 0] - _ln3(G["Q"])).max())
    g = bwd(np.asarray(G["dO"]), **a)
    eb = max(np.abs(g["dgates"] - np.asarray(G["dgates"])).max(), np.abs(g["dW_O"] - np.asarray(G["dW_O"])).max(),
             np.abs(g["dW_Q"] - np.asarray(G["dW_Q"])).max(), np.abs(g["dW_V"] - np.asarray(G["dW_V"])).max(),
             np.abs(g["dW_K"][0, 0] - _ln3(G["dW_K"])).max(), np.abs(g["dX"][:, 0] - _ln3(G["dX"])).max(),
             np.abs(g["dOhat"] - np.asarray(G["dOhat"])).max(), np.abs(g["dQ"] - np.asarray(G["dQ"])).max(),
             np.abs(g["dV"] - np.asarray(G["dV"])).max(), np.abs(g["dK"][:, 0] - _ln3(G["dK"])).max())
    return float(ef), float(eb)


def _distinct_layer(seed):
    """A layer whose tokens all pick two different experts out of five, with clearly unequal weights."""
    p = _layer(seed, B=2, T=6, d_model=5, E=5, k=2, h=2, d=3)
    assert (p["expert_idxs"][:, 0] != p["expert_idxs"][:, 1]).all()
    assert np.abs(p["gates"][:, 0] - p["gates"][:, 1]).min() > 1e-3
    assert len(np.unique(p["expert_idxs"])) == 5
    return p


def _composition_errors(fwd, bwd, seed=21):
    """Alg. 4 assembled from the pieces pinned elsewhere: Q = ParallelLinear(X, W_Q, o, no p, scattered ->
    scattered, fan-out k), Ohat = Attention(Q, K, V), O = ParallelLinear(Ohat, W_O, o, p, scattered ->
    scattered); backward through the same pieces with Alg. 2."""
    p = _distinct_layer(seed)
    B, T, h, d, k = p["B"], p["T"], p["h_expert"], p["d_head"], p["expert_idxs"].shape[1]
    N, E = B * T, p["W_Q"].shape[0]
    se, o, off = oracle.route(p["expert_idxs"], E)
    K, V = p["X"] @ p["W_K"], p["X"] @ p["W_V"]
    Q, _ = oracle.plinear_fwd(p["X"], p["W_Q"], se, o, k, None, False, False)
    sq, skv = (B, T, k, h, d), (B, T, h, d)
    Ohat = oracle.attention_fwd(Q.reshape(sq), K.reshape(skv), V.reshape(skv))[0].reshape(N * k, h * d)
    O, Yhat = oracle.plinear_fwd(Ohat, p["W_O"], se, o, 1, p["gates"], False, False)
    out = fwd(**p)
    ef = max(np.abs(out[n] - r).max() for n, r in (("O", O), ("Q", Q), ("Ohat", Ohat), ("Yhat", Yhat), ("K", K), ("V", V)))
    dO = RNG(seed + 1).standard_normal(O.shape)
    dOhat, dW_O, dg = oracle.plinear_bwd(dO, Ohat, p["W_O"], se, o, 1, p["gates"], False, False)
    dQ, dK, dV = oracle.attention_bwd(dOhat.reshape(sq), Q.reshape(sq), K.reshape(skv), V.reshape(skv))
    dQ, dK, dV = dQ.reshape(N * k, h * d), dK.reshape(N, h * d), dV.reshape(N, h * d)
    dXq, dW_Q, _ = oracle.plinear_bwd(dQ, p["X"], p["W_Q"], se, o, k, None, False, False)
    ref = dict(dX=dXq + dK @ p["W_K"].T + dV @ p["W_V"].T, dW_K=p["X"].T @ dK, dW_V=p["X"].T @ dV, dW_Q=dW_Q,
               dW_O=dW_O, dgates=dg)
    g = bwd(dO, **p)
    eb = max(np.abs(g[n] - r).max() for n, r in ref.items())
    return float(ef), float(eb)


def test_layer_hand_example_with_distinct_experts(golden_dir):
    ef, eb = _hand_example_errors(golden_dir, oracle.momha_fwd, oracle.momha_bwd)
    assert ef < 1e-12 and eb < 1e-11, (ef, eb)


def test_layer_equals_composition_of_pinned_pieces_on_distinct_experts():
    ef, eb = _composition_errors(oracle.momha_fwd, oracle.momha_bwd)
    assert ef < 1e-12 and eb < 1e-11, (ef, eb)


def _broken_copy(replacements):
    """A copy of the Alg. 4 oracle with textual slips planted in momha_fwd / momha_bwd (CPU only)."""
    import inspect
    import oracle.momha_oracle as mo
    ns = dict(vars(mo))
    for name in ("momha_fwd", "momha_bwd"):
        src = inspect.getsource(getattr(mo, name))
        for old, new in replacements:
            src = src.replace(old, new)
        exec(compile(src, f"<broken {name}>", "exec"), ns)
    return ns["momha_fwd"], ns["momha_bwd"]


@pytest.mark.parametrize("slip,replacements", [
    ("every slot uses the token's first expert", [("expert_idxs[t, j]", "expert_idxs[t, 0]")]),
    ("routing weights swapped between the slots of a token", [("gates[t, j]", "gates[t, k - 1 - j]")]),
    ("every slot uses the first routing weight", [("gates[t, j]", "gates[t, 0]")]),
    ("output projection uses the query's expert of the other slot", [("@ W_O[expert_idxs[t, j]]", "@ W_O[expert_idxs[t, k - 1 - j]]"),
                                                                      ("s, e = t * k + j, expert_idxs[t, j]\n            dgates", "s, e = t * k + j, expert_idxs[t, k - 1 - j]\n            dgates")]),
])
def test_pins_catch_planted_slot_map_mistakes(golden_dir, slip, replacements):
    """A mistake made consistently in forward and backward (so that finite differences of the function
    against itself still pass) must fail both the hand example and the composition pin."""
    import inspect
    import oracle.momha_oracle as mo
    src = inspect.getsource(mo.momha_fwd) + inspect.getsource(mo.momha_bwd)
    assert all(old in src for old, _ in replacements), "the oracle's text changed: update the planted slips"
    fwd, bwd = _broken_copy(replacements)
    hf, hb = _hand_example_errors(golden_dir, fwd, bwd)
    cf, cb = _composition_errors(fwd, bwd)
    assert hf > 1e-3 and hb > 1e-3, (slip, hf, hb)
    assert cf > 1e-6 and cb > 1e-6, (slip, cf, cb)
    # ... while the broken copy is still self-consistent: its own finite differences agree with its gradients
    p = _distinct_layer(21)
    dO = RNG(3).standard_normal((p["X"].shape[0], p["X"].shape[1]))
    g = bwd(dO, **p)
    loss = lambda q: float((fwd(**q)["O"] * dO).sum())
    idx = (1, 2)
    qp, qm = dict(p), dict(p)
    qp["X"], qm["X"] = p["X"].copy(), p["X"].copy()
    qp["X"][idx] += 1e-6
    qm["X"][idx] -= 1e-6
    assert abs((loss(qp) - loss(qm)) / 2e-6 - g["dX"][idx]) < 1e-6
    # the untouched oracle passes the same pins
    fwd0, bwd0 = _broken_copy([])
    assert max(_hand_example_errors(golden_dir, fwd0, bwd0)) < 1e-11
