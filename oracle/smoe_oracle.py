"""Plain fp64 CPU oracle for the ScatterMoE hot path.  TEST INFRASTRUCTURE ONLY.

This file is the independent definition the HIP kernels are checked against.
It shares no code with the GPU path, imports nothing from the product package
and must never be imported by it.  Everything is numpy float64 and follows the
paper's plain definitions, not its kernels:

* SMoE output, Sec. 3.1 step 5:   Y_t = sum_{e in topk(g(X_t))} g_e(X_t) * f_e(X_t)
  with f_e a one-hidden-layer MLP (Sec. 3.1, last sentence) = act(x W1[e]) W2[e]
  (Alg. 3).  The paper calls the naive way "iterating over all tokens and
  evaluating the respective expert output" (Sec. 3.1); that loop is this oracle.
* ParallelLinear forward, Alg. 1: Yhat = scatter2scatter(X, W, o, k), then an
  optional weighted sum over the k slots of a token with routing weights p.
* ParallelLinear backward, Alg. 2 and the gradient identities of Sec. 3.2.1:
  dX = dY W^T, dW = X^T dY per expert, dp = <dY, Yhat>.
* Routing, Sec. 3.1 steps 1-2: top-k experts per token, then "sort the tokens
  according to the experts".

Readings taken where the paper is silent or inconsistent (all listed again in
the design notes of the repository):
  - o has length T*k; o[i] is the flattened slot id t*k+j of the i-th row in
    expert-sorted order, token = o[i] // k  (Alg. 2 declares it Tk long).
  - the sort is stable: inside an expert segment slots ascend.
  - top-k ties go to the lower expert id; slots are ordered by descending logit;
    gates are the softmax over the k selected logits.
  - p given  => S = T, j = k, output must be scattered, Y has T rows.
  - the else-branch of Alg. 2 ("dYbar <- Y") means dY; dY is grouped whenever
    the forward output was scattered, and scaled whenever p was given.
  - dX has the shape of X: if the input was scattered with fan-out k, the k
    slot gradients of a token are summed.
  - GELU is the exact erf form; SwiGLU packs W1 columns as [gate | up] and
    H = silu(gate) * up.

Pins (tests/test_oracle_pins.py, all CPU): hand-derived worked examples in
tests/golden/, scalar brute force on tiny inputs, E=1 and identical-expert
reductions to a dense MLP computed with a library matmul, token-permutation
invariance, central finite differences for every gradient, routing invariants
and a counting-sort brute force, grouped/scattered flag consistency, and
Alg. 2 evaluated step by step against the per-token analytic gradients.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf as _erf

__all__ = [
    "ACT_NONE", "ACT_GELU", "ACT_SWIGLU",
    "act_fwd", "act_bwd", "hidden_width",
    "topk_gate", "topk_gate_bwd", "route",
    "plinear_fwd", "plinear_bwd",
    "mlp_token_fwd", "mlp_fwd", "mlp_token_bwd", "mlp_bwd",
    "mlp_dW2_rows", "mlp_dW1_cols",
]

ACT_NONE, ACT_GELU, ACT_SWIGLU = 0, 1, 2


# --------------------------------------------------------------------------
# activation (Alg. 3: "sigma is any point-wise non-linearity")
# --------------------------------------------------------------------------
def hidden_width(act: int, d_expert: int) -> int:
    """Number of W1 columns: SwiGLU packs gate and up projections side by side."""
    return 2 * d_expert if act == ACT_SWIGLU else d_expert


def act_fwd(act: int, hpre: np.ndarray) -> np.ndarray:
    """H = sigma(Hpre) on the last axis (Alg. 3, second step)."""
    hpre = np.asarray(hpre, dtype=np.float64)
    if act == ACT_NONE:
        return hpre.copy()
    if act == ACT_GELU:
        return 0.5 * hpre * (1.0 + _erf(hpre / np.sqrt(2.0)))
    if act == ACT_SWIGLU:
        d = hpre.shape[-1] // 2
        gate, up = hpre[..., :d], hpre[..., d:]
        return gate / (1.0 + np.exp(-gate)) * up
    raise ValueError("unknown activation")


def act_bwd(act: int, hpre: np.ndarray, dH: np.ndarray) -> np.ndarray:
    """dHpre = sigma'(Hpre) applied to dH (chain rule through Alg. 3's sigma)."""
    hpre = np.asarray(hpre, dtype=np.float64)
    dH = np.asarray(dH, dtype=np.float64)
    if act == ACT_NONE:
        return dH.copy()
    if act == ACT_GELU:
        cdf = 0.5 * (1.0 + _erf(hpre / np.sqrt(2.0)))
        pdf = np.exp(-0.5 * hpre * hpre) / np.sqrt(2.0 * np.pi)
        return dH * (cdf + hpre * pdf)
    if act == ACT_SWIGLU:
        d = hpre.shape[-1] // 2
        gate, up = hpre[..., :d], hpre[..., d:]
        sig = 1.0 / (1.0 + np.exp(-gate))
        silu = gate * sig
        dgate = dH * up * (sig + silu * (1.0 - sig))
        dup = dH * silu
        return np.concatenate([dgate, dup], axis=-1)
    raise ValueError("unknown activation")


# --------------------------------------------------------------------------
# routing (Sec. 3.1 steps 1 and 2)
# --------------------------------------------------------------------------
def topk_gate(logits: np.ndarray, k: int):
    """Step 1 of Sec. 3.1: keep the top-k experts of each token's router logits.

    Returns (expert_idxs [T,k] int32, gates [T,k] float64).  Slots are ordered
    by descending logit, ties to the lower expert id; the gates are the softmax
    over the k kept logits.  The paper is silent on non-finite logits; reading:
    a NaN logit counts as -inf, and kept logits that are all -inf share the
    weight equally (the limit of equal logits).
    """
    logits = np.asarray(logits)
    T, E = logits.shape
    if not 1 <= k <= E:
        raise ValueError("need 1 <= k <= E")
    expert_idxs = np.empty((T, k), dtype=np.int32)
    gates = np.empty((T, k), dtype=np.float64)
    for t in range(T):
        row = logits[t].astype(np.float64)
        row[np.isnan(row)] = -np.inf
        order = np.argsort(-row, kind="stable")      # descending, ties keep lower id first
        top = order[:k]
        z = row[top] - row[top[0]] if row[top[0]] > -np.inf else np.zeros(k)
        w = np.exp(z)
        expert_idxs[t] = top
        gates[t] = w / w.sum()
    return expert_idxs, gates


def topk_gate_bwd(expert_idxs: np.ndarray, gates: np.ndarray, dgates: np.ndarray, E: int) -> np.ndarray:
    """Gradient of step 1 of Sec. 3.1 with respect to the router logits.

    The gates of a token are the softmax of its k kept logits, so with g = gates[t] the Jacobian
    on the kept experts is diag(g) - g g^T and every other expert has a zero gradient (the
    selection itself is piecewise constant).  Takes Alg. 2's dp (dgates [T,k]) and returns
    dlogits [T,E] float64.
    """
    expert_idxs = np.asarray(expert_idxs)
    T, k = expert_idxs.shape
    g = np.asarray(gates, dtype=np.float64).reshape(T, k)
    dg = np.asarray(dgates, dtype=np.float64).reshape(T, k)
    dlogits = np.zeros((T, E), dtype=np.float64)
    for t in range(T):
        jac = np.diag(g[t]) - np.outer(g[t], g[t])
        dlogits[t, expert_idxs[t]] = jac @ dg[t]
    return dlogits


def route(expert_idxs: np.ndarray, E: int):
    """Step 2 of Sec. 3.1 ("sort the tokens according to the experts").

    expert_idxs is [T,k] (or flat [Tk]); slot s = t*k+j.  Returns
      sorted_expert_idxs   [Tk] int32, non-decreasing,
      sorted_scattered_idxs[Tk] int32, the paper's o: slot id of the i-th sorted row,
      expert_offsets       [E+1] int32, exclusive prefix of the per-expert counts.
    The sort is stable, so slots ascend inside an expert's segment.
    """
    flat = np.asarray(expert_idxs).reshape(-1)
    if flat.size and (flat.min() < 0 or flat.max() >= E):
        raise ValueError("expert index out of range")
    o = np.argsort(flat, kind="stable").astype(np.int32)
    sorted_e = flat[o].astype(np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    for e in flat:
        offsets[int(e) + 1] += 1
    offsets = np.cumsum(offsets).astype(np.int32)
    return sorted_e, o, offsets


# --------------------------------------------------------------------------
# ParallelLinear (Alg. 1 and Alg. 2)
# --------------------------------------------------------------------------
def _slot_experts(sorted_expert_idxs, o):
    """Expert of every slot, recovered from the two sorted routing arrays."""
    slot_e = np.empty(len(o), dtype=np.int64)
    slot_e[np.asarray(o, dtype=np.int64)] = np.asarray(sorted_expert_idxs, dtype=np.int64)
    return slot_e


def plinear_fwd(X, W, sorted_expert_idxs, o, k, p=None, grouped_in=False, grouped_out=False):
    """Alg. 1.  Returns (Y, Yhat).

    X: [Tk/k, d_in] scattered with fan-out k (row of slot s is s // k), or
       [Tk, d_in] in expert-sorted order if grouped_in.
    W: [E, d_in, d_out].   o: [Tk] slot id of each sorted row.
    Yhat: [Tk, d_out]; row i (grouped_out) or row o[i] (scattered) holds the
    product of the i-th sorted input row with its expert's matrix.
    p: optional [T, kp] weights with T*kp = Tk; then Y[t] = sum_j p[t,j] Yhat[t*kp+j]
    (needs scattered output), else Y is Yhat.
    """
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    o = np.asarray(o, dtype=np.int64)
    Tk = len(o)
    d_out = W.shape[2]
    Yhat = np.zeros((Tk, d_out), dtype=np.float64)
    for i in range(Tk):                       # one routed row at a time
        s = o[i]
        e = int(sorted_expert_idxs[i])
        x = X[i] if grouped_in else X[s // k]
        y = x @ W[e]
        Yhat[i if grouped_out else s] = y
    if p is None:
        return Yhat, Yhat
    if grouped_out:
        raise ValueError("weighted sum needs scattered output")
    p = np.asarray(p, dtype=np.float64)
    T, kp = p.shape
    if T * kp != Tk:
        raise ValueError("p must have Tk entries")
    Y = np.zeros((T, d_out), dtype=np.float64)
    for t in range(T):
        for j in range(kp):
            Y[t] += p[t, j] * Yhat[t * kp + j]
    return Y, Yhat


def plinear_bwd(dY, X, W, sorted_expert_idxs, o, k, p=None, grouped_in=False, grouped_out=False):
    """Gradients of Alg. 1's output w.r.t. X, W and p, from the plain definition.

    Sec. 3.2.1: per expert dX = dY W^T and dW = X^T dY; with weights, the row
    that reaches slot s is p_s * dY[token(s)] and dp_s = <dY[token(s)], Yhat_s>.
    dY has the shape of Alg. 1's Y.  Returns (dX like X, dW like W, dp like p or None).
    """
    dY = np.asarray(dY, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    o = np.asarray(o, dtype=np.int64)
    Tk = len(o)
    dX = np.zeros_like(X)
    dW = np.zeros_like(W)
    dp = None
    if p is not None:
        p = np.asarray(p, dtype=np.float64)
        kp = p.shape[1]
        dp = np.zeros_like(p)
    for i in range(Tk):
        s = o[i]
        e = int(sorted_expert_idxs[i])
        xi = i if grouped_in else s // k
        x = X[xi]
        if p is not None:
            t, j = divmod(int(s), kp)
            yhat = x @ W[e]
            dp[t, j] = dY[t] @ yhat
            g = p[t, j] * dY[t]
        else:
            g = dY[i if grouped_out else s]
        dX[xi] += g @ W[e].T
        dW[e] += np.outer(x, g)
    return dX, dW, dp


# --------------------------------------------------------------------------
# SMoE MLP (Alg. 3) -- the per-token definition
# --------------------------------------------------------------------------
def mlp_token_fwd(x, experts, gates, W1, W2, act):
    """One token of Sec. 3.1 step 5 with MLP experts (Alg. 3).

    Returns (y [d_model], hpre [k,d_h], h [k,d_expert], yhat [k,d_model]).
    W1/W2 may be any array type whose [e] slice converts to float64.
    """
    x = np.asarray(x, dtype=np.float64)
    k = len(experts)
    y = np.zeros(np.shape(W2)[2], dtype=np.float64)
    hpre_l, h_l, yhat_l = [], [], []
    for j in range(k):
        e = int(experts[j])
        hpre = x @ np.asarray(W1[e], dtype=np.float64)
        h = act_fwd(act, hpre)
        yhat = h @ np.asarray(W2[e], dtype=np.float64)
        y += float(gates[j]) * yhat
        hpre_l.append(hpre); h_l.append(h); yhat_l.append(yhat)
    return y, np.stack(hpre_l), np.stack(h_l), np.stack(yhat_l)


def mlp_fwd(X, W1, W2, expert_idxs, gates, act):
    """Naive SMoE MLP: loop over tokens, evaluate each selected expert (Sec. 3.1).

    Returns dict with Y [T,d_model] and, per slot s = t*k+j in scattered order,
    Hpre [Tk,d_h], H [Tk,d_expert], Yhat [Tk,d_model].
    """
    X = np.asarray(X, dtype=np.float64)
    T = X.shape[0]
    k = np.shape(expert_idxs)[1]
    d_h, d_model = np.shape(W1)[2], np.shape(W2)[2]
    d_expert = np.shape(W2)[1]
    out = dict(Y=np.zeros((T, d_model)), Hpre=np.zeros((T * k, d_h)),
               H=np.zeros((T * k, d_expert)), Yhat=np.zeros((T * k, d_model)))
    for t in range(T):
        y, hpre, h, yhat = mlp_token_fwd(X[t], expert_idxs[t], gates[t], W1, W2, act)
        out["Y"][t] = y
        out["Hpre"][t * k:(t + 1) * k] = hpre
        out["H"][t * k:(t + 1) * k] = h
        out["Yhat"][t * k:(t + 1) * k] = yhat
    return out


def mlp_token_bwd(x, dy, experts, gates, W1, W2, act):
    """Analytic gradient of one token's contribution (chain rule on Alg. 3).

    Returns (dx [d_model], dgates [k], dhpre [k,d_h], h [k,d_expert]); the
    weight gradients of this token are dW1[e_j] += outer(x, dhpre[j]) and
    dW2[e_j] += outer(h[j], gates[j]*dy).
    """
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    k = len(experts)
    dx = np.zeros_like(x)
    dg = np.zeros(k)
    dhpre_l, h_l = [], []
    for j in range(k):
        e = int(experts[j])
        w1 = np.asarray(W1[e], dtype=np.float64)
        w2 = np.asarray(W2[e], dtype=np.float64)
        hpre = x @ w1
        h = act_fwd(act, hpre)
        yhat = h @ w2
        dg[j] = dy @ yhat
        dh = float(gates[j]) * (w2 @ dy)
        dhpre = act_bwd(act, hpre, dh)
        dx += w1 @ dhpre
        dhpre_l.append(dhpre); h_l.append(h)
    return dx, dg, np.stack(dhpre_l), np.stack(h_l)


def mlp_bwd(dY, X, W1, W2, expert_idxs, gates, act):
    """Gradients of sum(Y * dY) for the naive SMoE MLP, token by token.

    Returns dict dX [T,d_model], dW1 like W1, dW2 like W2, dgates [T,k].
    """
    X = np.asarray(X, dtype=np.float64)
    dY = np.asarray(dY, dtype=np.float64)
    T = X.shape[0]
    k = np.shape(expert_idxs)[1]
    out = dict(dX=np.zeros_like(X), dW1=np.zeros(np.shape(W1)), dW2=np.zeros(np.shape(W2)),
               dgates=np.zeros((T, k)))
    for t in range(T):
        dx, dg, dhpre, h = mlp_token_bwd(X[t], dY[t], expert_idxs[t], gates[t], W1, W2, act)
        out["dX"][t] = dx
        out["dgates"][t] = dg
        for j in range(k):
            e = int(expert_idxs[t][j])
            out["dW1"][e] += np.outer(X[t], dhpre[j])
            out["dW2"][e] += np.outer(h[j], float(gates[t][j]) * dY[t])
    return out


# --------------------------------------------------------------------------
# single rows / columns of the weight gradients, for shapes where the full
# per-token pass does not finish in seconds.  Same definition, restricted to
# the entries asked for: every token routed to expert e contributes.
# --------------------------------------------------------------------------
def _expert_slots(expert_idxs, e):
    ei = np.asarray(expert_idxs)
    t_idx, j_idx = np.nonzero(ei == e)
    return t_idx, j_idx


def _hidden_cols(act, d_expert, c):
    """Columns of W1 that feed hidden unit c."""
    return [c, c + d_expert] if act == ACT_SWIGLU else [c]


def mlp_dW2_rows(dY, X, W1, W2, expert_idxs, gates, act, e, rows):
    """dW2[e][c, :] for each hidden unit c in rows: sum_t H_t[c] * g_t * dY_t."""
    X = np.asarray(X); dY = np.asarray(dY)
    d_expert = np.shape(W2)[1]
    t_idx, j_idx = _expert_slots(expert_idxs, e)
    out = np.zeros((len(rows), np.shape(W2)[2]))
    w1 = W1[e]
    for r, c in enumerate(rows):
        cols = _hidden_cols(act, d_expert, int(c))
        w1c = np.asarray(w1[:, cols], dtype=np.float64)          # [d_model, 1 or 2]
        for t, j in zip(t_idx, j_idx):
            hpre = np.asarray(X[t], dtype=np.float64) @ w1c
            h = act_fwd(act, hpre)[0]
            out[r] += h * float(gates[t][j]) * np.asarray(dY[t], dtype=np.float64)
    return out


def mlp_dW1_cols(dY, X, W1, W2, expert_idxs, gates, act, e, units):
    """Columns of dW1[e] feeding each hidden unit c in units.

    Returns [len(units), ncol, d_model] with ncol = 2 for SwiGLU (gate column c,
    up column c + d_expert) else 1:  sum_t X_t * dHpre_t[col].
    """
    X = np.asarray(X); dY = np.asarray(dY)
    d_expert = np.shape(W2)[1]
    t_idx, j_idx = _expert_slots(expert_idxs, e)
    ncol = 2 if act == ACT_SWIGLU else 1
    out = np.zeros((len(units), ncol, X.shape[1]))
    w1 = W1[e]; w2 = W2[e]
    for r, c in enumerate(units):
        cols = _hidden_cols(act, d_expert, int(c))
        w1c = np.asarray(w1[:, cols], dtype=np.float64)
        w2c = np.asarray(w2[int(c)], dtype=np.float64)             # [d_model]
        for t, j in zip(t_idx, j_idx):
            x = np.asarray(X[t], dtype=np.float64)
            hpre = x @ w1c
            dh = float(gates[t][j]) * (w2c @ np.asarray(dY[t], dtype=np.float64))
            dhpre = act_bwd(act, hpre, np.array([dh]))
            for q in range(ncol):
                out[r, q] += x * dhpre[q]
    return out
