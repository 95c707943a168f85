"""Plain fp64 CPU oracle for SMoE multi-head attention (Alg. 4).  TEST INFRASTRUCTURE ONLY.

Shares no code with the GPU path and must never be imported by the product package.

Alg. 4 in the paper's notation, for a flattened batch of B sequences of T tokens:
    V = X W_V,  K = X W_K                                   (dense, h_expert heads of d_head each)
    Q = ParallelLinear(X, W_Q, o, no p, scattered -> scattered)          one row per routed slot
    Ohat = Attention(Q, K, V)
    O = ParallelLinear(Ohat, W_O, o, p, scattered -> scattered)          weighted sum over the k slots
Sec. 3.3 describes the attention as the grouped-query kind: each of the h_expert key/value
heads serves the k * h_expert query heads a token selects (head h of every selected expert
attends key head h).  Both ParallelLinears keep the chronological (scattered) order.

Readings where the paper is silent: the attention is the standard scaled dot product
softmax(q k^T / sqrt(d_head)) v with a causal mask inside each sequence (position t sees
positions <= t of its own sequence), no bias, no positional rotation, no dropout.

Everything here is the definition written out: dense score matrices per (sequence, head),
a full softmax, and the analytic gradients of exactly those expressions.
"""
from __future__ import annotations

import numpy as np

__all__ = ["attention_fwd", "attention_bwd", "momha_fwd", "momha_bwd"]


def _causal_scores(q, k):
    """q [T, d], k [T, d] -> masked score matrix [T, T] (row = query position)."""
    T, d = q.shape
    s = (q @ k.T) / np.sqrt(d)
    s[np.triu_indices(T, 1)] = -np.inf
    return s


def _softmax_rows(s):
    m = s.max(axis=1, keepdims=True)
    w = np.exp(s - m)
    z = w.sum(axis=1, keepdims=True)
    return w / z, (m + np.log(z))[:, 0]


def attention_fwd(Q, K, V):
    """Causal grouped-query attention.

    Q [B, T, G, h, d] (G query groups per token: the k routed slots), K, V [B, T, h, d].
    Returns O [B, T, G, h, d] and the log-sum-exp of the scaled, masked scores [B, T, G, h].
    """
    Q, K, V = (np.asarray(a, dtype=np.float64) for a in (Q, K, V))
    B, T, G, h, d = Q.shape
    O = np.empty_like(Q)
    L = np.empty((B, T, G, h))
    for b in range(B):
        for hh in range(h):
            for g in range(G):
                p, lse = _softmax_rows(_causal_scores(Q[b, :, g, hh], K[b, :, hh]))
                O[b, :, g, hh] = p @ V[b, :, hh]
                L[b, :, g, hh] = lse
    return O, L


def attention_bwd(dO, Q, K, V):
    """Gradients of attention_fwd's O with respect to Q, K, V (same shapes)."""
    dO, Q, K, V = (np.asarray(a, dtype=np.float64) for a in (dO, Q, K, V))
    B, T, G, h, d = Q.shape
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    for b in range(B):
        for hh in range(h):
            for g in range(G):
                p, _ = _softmax_rows(_causal_scores(Q[b, :, g, hh], K[b, :, hh]))
                do = dO[b, :, g, hh]
                dV[b, :, hh] += p.T @ do
                dp = do @ V[b, :, hh].T
                ds = p * (dp - (p * dp).sum(axis=1, keepdims=True))      # softmax Jacobian, row by row
                dQ[b, :, g, hh] = ds @ K[b, :, hh] / np.sqrt(d)
                dK[b, :, hh] += ds.T @ Q[b, :, g, hh] / np.sqrt(d)
    return dQ, dK, dV


def momha_fwd(X, W_K, W_V, W_Q, W_O, expert_idxs, gates, B, T, h_expert, d_head):
    """Alg. 4.  X [B*T, d_model]; W_K, W_V [d_model, d_out]; W_Q [E, d_model, d_out];
    W_O [E, d_out, d_model] with d_out = h_expert * d_head; expert_idxs, gates [B*T, k].
    Returns a dict with O [B*T, d_model] and the intermediates K, V [B*T, d_out],
    Q, Ohat [B*T*k, d_out] and Yhat [B*T*k, d_model] in slot order (slot s = t*k + j)."""
    X, W_K, W_V, W_Q, W_O = (np.asarray(a, dtype=np.float64) for a in (X, W_K, W_V, W_Q, W_O))
    gates = np.asarray(gates, dtype=np.float64)
    N, k = expert_idxs.shape
    d_out = h_expert * d_head
    assert N == B * T and W_K.shape[1] == d_out
    K = X @ W_K
    V = X @ W_V
    Q = np.empty((N * k, d_out))
    for t in range(N):
        for j in range(k):
            Q[t * k + j] = X[t] @ W_Q[expert_idxs[t, j]]
    Ohat, _ = attention_fwd(Q.reshape(B, T, k, h_expert, d_head), K.reshape(B, T, h_expert, d_head),
                            V.reshape(B, T, h_expert, d_head))
    Ohat = Ohat.reshape(N * k, d_out)
    Yhat = np.empty((N * k, W_O.shape[2]))
    O = np.zeros((N, W_O.shape[2]))
    for t in range(N):
        for j in range(k):
            Yhat[t * k + j] = Ohat[t * k + j] @ W_O[expert_idxs[t, j]]
            O[t] += gates[t, j] * Yhat[t * k + j]
    return {"O": O, "K": K, "V": V, "Q": Q, "Ohat": Ohat, "Yhat": Yhat}


def momha_bwd(dO, X, W_K, W_V, W_Q, W_O, expert_idxs, gates, B, T, h_expert, d_head):
    """Gradients of momha_fwd's O: dict with dX, dW_K, dW_V, dW_Q, dW_O, dgates."""
    dO, X, W_K, W_V, W_Q, W_O = (np.asarray(a, dtype=np.float64) for a in (dO, X, W_K, W_V, W_Q, W_O))
    gates = np.asarray(gates, dtype=np.float64)
    N, k = expert_idxs.shape
    d_out = h_expert * d_head
    f = momha_fwd(X, W_K, W_V, W_Q, W_O, expert_idxs, gates, B, T, h_expert, d_head)
    dW_O, dW_Q = np.zeros_like(W_O), np.zeros_like(W_Q)
    dgates = np.empty((N, k))
    dOhat = np.empty((N * k, d_out))
    for t in range(N):
        for j in range(k):
            s, e = t * k + j, expert_idxs[t, j]
            dgates[t, j] = dO[t] @ f["Yhat"][s]
            dyh = gates[t, j] * dO[t]
            dW_O[e] += np.outer(f["Ohat"][s], dyh)
            dOhat[s] = W_O[e] @ dyh
    shp_q, shp_kv = (B, T, k, h_expert, d_head), (B, T, h_expert, d_head)
    dQ, dK, dV = attention_bwd(dOhat.reshape(shp_q), f["Q"].reshape(shp_q), f["K"].reshape(shp_kv),
                               f["V"].reshape(shp_kv))
    dQ, dK, dV = dQ.reshape(N * k, d_out), dK.reshape(N, d_out), dV.reshape(N, d_out)
    dX = dK @ W_K.T + dV @ W_V.T
    for t in range(N):
        for j in range(k):
            s, e = t * k + j, expert_idxs[t, j]
            dW_Q[e] += np.outer(X[t], dQ[s])
            dX[t] += W_Q[e] @ dQ[s]
    return {"dX": dX, "dW_K": X.T @ dK, "dW_V": X.T @ dV, "dW_Q": dW_Q, "dW_O": dW_O, "dgates": dgates,
            "dOhat": dOhat, "dQ": dQ, "dK": dK, "dV": dV}
