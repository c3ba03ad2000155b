"""Oracle for the backward pass of one MoE layer -- TEST INFRASTRUCTURE ONLY.

The paper trains the layer (Sec. 5: the runtime all-reduces the expert gradients over each
expert's replicas) but prints no backward formulas: what is computed is fixed by the forward
definition (Sec. 2.1) and the chain rule.  This module writes those derivatives out in fp64,
one forward step at a time in reverse order, with no blocking or fusion:

    forward                                         backward (upstream dy = dL/dy)
    y[t]   = sum_kk gates[t,kk] * yp[row(t,kk)]     dgates[t,kk] = <dy[t], yp[row]>,  dyp[row] = gates[t,kk] dy[t]
    yp     = H W2^T        (per slot)               dH = dyp W2,   dW2 = dyp^T H
    H      = act(Z)                                 dZ = dH * act'(Z)
    Z      = xp W1^T       (per slot)               dxp = dZ W1,   dW1 = dZ^T xp
    xp[row]= x[token(row)]                          dx[t] = sum_kk dxp[row(t,kk)]
    gates  = softmax(logits at the top-k ids)       dlogits[t, ids[t,j]] = g_j (dg_j - sum_i g_i dg_i)

Replicas of an expert hold equal weights, and the expert's gradient is the sum of its
replicas' gradients (the all-reduce over the replica set, Sec. 5).

Pins (tests/test_oracle_backward.py): central finite differences of the forward oracle
`moe_layer.layer_output` in every input, closed forms of the activation derivatives, and
reverse-mode differentiation of the forward written with a tensor library.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf as _erf

from .moe_layer import gelu, silu, widen


def gelu_grad(v: np.ndarray) -> np.ndarray:
    """d/dv [0.5 v (1 + erf(v / sqrt 2))] = Phi(v) + v phi(v)."""
    return 0.5 * (1.0 + _erf(v / np.sqrt(2.0))) + v * np.exp(-0.5 * v * v) / np.sqrt(2.0 * np.pi)


def silu_grad(v: np.ndarray) -> np.ndarray:
    """d/dv [v sigma(v)] = sigma(v) (1 + v (1 - sigma(v)))."""
    s = 1.0 / (1.0 + np.exp(-v))
    return s * (1.0 + v * (1.0 - s))


def combine_backward(dy, yp, pair_to_row, gates):
    """Backward of the gate-weighted combine.  Returns (dyp [P,d], dgates [T,k]); rows of
    dyp that no pair maps to are zero."""
    dY = widen(dy)
    Yp = widen(yp)
    gates = np.asarray(gates, dtype=np.float64)
    T, k = gates.shape
    p2r = np.asarray(pair_to_row).reshape(T, k)
    dyp = np.zeros_like(Yp)
    dgates = np.zeros((T, k), dtype=np.float64)
    for kk in range(k):
        rows = p2r[:, kk]
        dgates[:, kk] = np.sum(dY * Yp[rows], axis=1)
        dyp[rows] = gates[:, kk:kk + 1] * dY          # a row belongs to exactly one pair
    return dyp, dgates


def act_forward(Z: np.ndarray, act: str) -> np.ndarray:
    if act == "gelu":
        return gelu(Z)
    f = Z.shape[1] // 2
    return silu(Z[:, :f]) * Z[:, f:]


def act_backward(dH: np.ndarray, Z: np.ndarray, act: str) -> np.ndarray:
    """dZ from dH: gelu  dZ = dH gelu'(Z);  swiglu (Z = [G | U])  dG = dH U silu'(G), dU = dH silu(G)."""
    if act == "gelu":
        return dH * gelu_grad(Z)
    f = Z.shape[1] // 2
    G, U = Z[:, :f], Z[:, f:]
    return np.concatenate([dH * U * silu_grad(G), dH * silu(G)], axis=1)


def ffn_backward_slot(dYp, Xp, W1, W2, act):
    """Backward of one slot's FFN on its rows (all fp64): returns (dxp, dw1, dw2)."""
    Z = Xp @ W1.T
    H = act_forward(Z, act)
    dH = dYp @ W2
    dw2 = dYp.T @ H
    dZ = act_backward(dH, Z, act)
    dw1 = dZ.T @ Xp
    return dZ @ W1, dw1, dw2


def ffn_backward_rows(dyp, xp, slot_offsets, slot_expert, w1, w2, act):
    """Backward of the per-slot FFN.  w1 / w2 are indexed by expert.  Returns
    (dxp [P,d], dw1_slot [S,n1,d], dw2_slot [S,d,ffn]): every slot's own weight gradient
    (zero for a slot without rows), before the sum over an expert's replicas."""
    dYp = widen(dyp)
    Xp = widen(xp)
    S = len(slot_expert)
    n1, d = np.asarray(w1).shape[1:]
    f = np.asarray(w2).shape[2]
    dxp = np.zeros_like(Xp)
    dw1 = np.zeros((S, n1, d), dtype=np.float64)
    dw2 = np.zeros((S, d, f), dtype=np.float64)
    for s in range(S):
        a, b = int(slot_offsets[s]), int(slot_offsets[s + 1])
        if b <= a:
            continue
        e = int(slot_expert[s])
        dxp[a:b], dw1[s], dw2[s] = ffn_backward_slot(dYp[a:b], Xp[a:b], widen(w1[e]), widen(w2[e]), act)
    return dxp, dw1, dw2


def permute_backward(dxp, pair_to_row, k):
    """dx[t] = sum_kk dxp[pair_to_row[t*k+kk]], kk ascending."""
    dXp = widen(dxp)
    p2r = np.asarray(pair_to_row).reshape(-1, k)
    dx = np.zeros((p2r.shape[0], dXp.shape[1]), dtype=np.float64)
    for kk in range(k):
        dx = dx + dXp[p2r[:, kk]]
    return dx


def reduce_replica_grads(dw_slot, slot_expert, E):
    """Expert gradient = sum of its replicas' gradients, slots in ascending order (the
    all-reduce over the replica set, Sec. 5)."""
    dw_slot = np.asarray(dw_slot, dtype=np.float64)
    out = np.zeros((E,) + dw_slot.shape[1:], dtype=np.float64)
    for s, e in enumerate(slot_expert):
        out[int(e)] = out[int(e)] + dw_slot[s]
    return out


def route_backward(dgates, gates, ids, E):
    """Gradient of the top-k softmax gates with respect to the logits; experts a token
    did not select get zero (the selection itself is piecewise constant)."""
    dg = np.asarray(dgates, dtype=np.float64)
    g = np.asarray(gates, dtype=np.float64)
    ids = np.asarray(ids)
    T, k = g.shape
    inner = np.zeros(T, dtype=np.float64)
    for kk in range(k):
        inner = inner + g[:, kk] * dg[:, kk]
    dlogits = np.zeros((T, E), dtype=np.float64)
    rows = np.arange(T)
    for kk in range(k):
        dlogits[rows, ids[:, kk]] = g[:, kk] * (dg[:, kk] - inner)
    return dlogits


def layer_backward(dy, x, ids, gates, pair_to_row, row_to_pair, slot_offsets, slot_expert,
                   w1, w2, act):
    """The whole chain on the dispatch a plan produced.  Returns a dict with dx, dgates,
    dw1 / dw2 per expert (replica sums) and per slot."""
    from .moe_layer import expert_ffn_rows, permute
    ids = np.asarray(ids)
    T, k = ids.shape
    E = np.asarray(w1).shape[0]
    xp = widen(permute(x, row_to_pair, k))
    yp = expert_ffn_rows(xp, slot_offsets, slot_expert, w1, w2, act)
    dyp, dgates = combine_backward(dy, yp, pair_to_row, gates)
    dxp, dw1s, dw2s = ffn_backward_rows(dyp, xp, slot_offsets, slot_expert, w1, w2, act)
    return {
        "dx": permute_backward(dxp, pair_to_row, k),
        "dgates": dgates,
        "dyp": dyp,
        "dxp": dxp,
        "dw1_slot": dw1s,
        "dw2_slot": dw2s,
        "dw1": reduce_replica_grads(dw1s, slot_expert, E),
        "dw2": reduce_replica_grads(dw2s, slot_expert, E),
    }
