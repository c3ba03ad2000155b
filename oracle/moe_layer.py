"""Oracle for one MoE-layer pass under an asymmetric replica placement plan.

TEST INFRASTRUCTURE ONLY (see the package docstring).  fp64 for all floating point,
Python integers / int64 for all index work.  No blocking, fusion or reordering
beyond what the definitions state.

Notation (paper, Algorithm 1 and Sec. 4.1): T tokens, E experts, top-k, N ranks,
c slots per rank, slot id s = rank*c + local_slot, slot_expert[s] = the paper's
placement matrix entry for that slot, R[e,j] replicas of e on rank j, Tej[e,j]
tokens (pairs) routed to e whose token lives on rank j, D[e,i,j] pairs of expert e
that source rank i sends to rank j.  A "pair" is one (token, kk) routing decision,
pair index p = t*k + kk.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np
from scipy.special import erf as _erf


# ----------------------------------------------------------------------------- dtypes
def widen(a: np.ndarray) -> np.ndarray:
    """The fp64 values denoted by an input tensor: fp32/fp64 as is, uint16 = bf16 bits."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# ----------------------------------------------------------------------------- routing
def route(logits: np.ndarray, k: int):
    """Top-k gate routing (Sec. 2.1: the gate routes each token to the top-k experts).

    Reading (the paper does not fix order, ties or gate normalisation): ids are the k
    largest logits of the token in descending logit order, equal logits resolved
    towards the lower expert index; gates are the softmax over those k logits, so a
    token's gates sum to one.  Comparison is on the fp32 values as given (-0.0 == 0.0);
    gate arithmetic is fp64.  Returns (ids int32 [T,k], gates float64 [T,k]).
    """
    logits = np.asarray(logits)
    T, E = logits.shape
    assert 1 <= k <= E
    work = logits.astype(np.float64).copy()
    ids = np.empty((T, k), dtype=np.int32)
    sel = np.empty((T, k), dtype=np.float64)
    rows = np.arange(T)
    for kk in range(k):
        # np.argmax returns the first (lowest-index) occurrence of the maximum
        best = np.argmax(work, axis=1)
        ids[:, kk] = best
        sel[:, kk] = work[rows, best]
        work[rows, best] = -np.inf
    ex = np.exp(sel - sel[:, :1])          # sel[:,0] is the row maximum
    denom = np.zeros(T, dtype=np.float64)
    for kk in range(k):                    # summed in output order
        denom = denom + ex[:, kk]
    gates = ex / denom[:, None]
    return ids, gates


def source_rank(rank_tok_off: np.ndarray, T: int) -> np.ndarray:
    """src[t] = the rank i with rank_tok_off[i] <= t < rank_tok_off[i+1] (batch split, Sec. 2.1)."""
    off = np.asarray(rank_tok_off, dtype=np.int64)
    assert off[0] == 0 and off[-1] == T and np.all(np.diff(off) >= 0)
    src = np.empty(T, dtype=np.int64)
    for i in range(len(off) - 1):
        src[off[i]:off[i + 1]] = i
    return src


def histogram(ids: np.ndarray, rank_tok_off: np.ndarray, E: int) -> np.ndarray:
    """Tej[e,i] = number of pairs routed to expert e whose token is on rank i
    (Algorithm 1 input; in the paper it is a local count followed by an all-gather)."""
    T, k = ids.shape
    N = len(rank_tok_off) - 1
    src = source_rank(rank_tok_off, T)
    Tej = np.zeros((E, N), dtype=np.int64)
    for t in range(T):
        for kk in range(k):
            Tej[ids[t, kk], src[t]] += 1
    return Tej


def replicas_per_rank(slot_expert: np.ndarray, E: int, N: int, c: int) -> np.ndarray:
    """R[e,j] = number of slots of rank j that hold expert e (placement matrix, Appendix)."""
    slot_expert = np.asarray(slot_expert)
    assert slot_expert.shape == (N * c,)
    R = np.zeros((E, N), dtype=np.int64)
    for s in range(N * c):
        R[slot_expert[s], s // c] += 1
    return R


# ----------------------------------------------------------------------------- Algorithm 1
def schedule_real(Tej, R):
    """Algorithm 1's dispatch counts evaluated literally over the rationals.

    p_e = t_e / r_e; capacity P[e,j] = p_e * R[e,j]; each rank serves its own tokens
    first, residual P'[e,j] = P - min(P, T); the local share is D[e,i,i] = P[e,i] -
    P'[e,i]; the overflow T[e,i] - D[e,i,i] is spread over the other ranks in
    proportion to their residual capacity.  The printed denominator of the spreading
    line sums over k != j; it is read as the sum over the ranks other than the
    sender (k != i), which is what the prose describes and the only reading that
    conserves tokens.  Returns D as an E x N x N nested list of Fractions.
    """
    Tej = np.asarray(Tej)
    R = np.asarray(R)
    E, N = Tej.shape
    D = [[[Fraction(0)] * N for _ in range(N)] for _ in range(E)]
    for e in range(E):
        r_e = int(R[e].sum())
        t_e = int(Tej[e].sum())
        if t_e == 0:
            continue
        assert r_e >= 1, "expert has tokens but no replica"
        p_e = Fraction(t_e, r_e)
        cap = [p_e * int(R[e, j]) for j in range(N)]
        res = [cap[j] - min(cap[j], Fraction(int(Tej[e, j]))) for j in range(N)]
        for i in range(N):
            local = cap[i] - res[i]
            D[e][i][i] = local
            overflow = int(Tej[e, i]) - local
            if overflow == 0:
                continue
            others = sum(res[j] for j in range(N) if j != i)
            for j in range(N):
                if j != i:
                    D[e][i][j] = overflow * res[j] / others
    return D


def schedule(Tej, R) -> dict:
    """Algorithm 1's dispatch counts in exact integers (the reading used by the GPU path).

    The paper's per-replica share p_e = t_e / r_e is fractional and its rounding is
    not specified.  Reading: "contiguous balanced split".
      * capacity: order the r_e replicas by (rank, local slot) and cut t_e into r_e
        balanced consecutive parts; with lo_j = sum_{j'<j} R[e,j'], hi_j = lo_j + R[e,j]
            cap[e,j] = floor(hi_j*t_e/r_e) - floor(lo_j*t_e/r_e)      (sum_j cap = t_e)
      * local priority: L[e,j] = min(cap[e,j], Tej[e,j]); residual Pres = cap - L;
        overflow O[e,i] = Tej[e,i] - L[e,i]   (sum_i O = sum_j Pres =: tot)
      * spreading: the proportional formula is applied cumulatively with floors,
            D[e,i,j] = floor(O_i*(cum_j+Pres_j)/tot) - floor(O_i*cum_j/tot),  j != i,
            cum_j = sum_{j'<j, j'!=i} Pres[e,j'];   D[e,i,i] = L[e,i]
        so every row of D sums exactly to Tej[e,i].
    Returns dict with cap, L, Pres, O [E,N], D [E,N(src),N(dst)], recv [E,N] =
    sum_i D[e,i,j], send [N(src),N(dst)] = sum_e D[e,i,j] (the paper's s_j per source).
    """
    Tej = np.asarray(Tej, dtype=np.int64)
    R = np.asarray(R, dtype=np.int64)
    E, N = Tej.shape
    cap = np.zeros((E, N), dtype=np.int64)
    L = np.zeros((E, N), dtype=np.int64)
    Pres = np.zeros((E, N), dtype=np.int64)
    O = np.zeros((E, N), dtype=np.int64)
    D = np.zeros((E, N, N), dtype=np.int64)
    for e in range(E):
        r_e = int(R[e].sum())
        t_e = int(Tej[e].sum())
        if t_e == 0:
            continue
        if r_e < 1:
            raise ValueError(f"expert {e} has tokens but no replica in the plan")
        lo = 0
        for j in range(N):
            hi = lo + int(R[e, j])
            cap[e, j] = (hi * t_e) // r_e - (lo * t_e) // r_e
            lo = hi
        for j in range(N):
            L[e, j] = min(int(cap[e, j]), int(Tej[e, j]))
            Pres[e, j] = cap[e, j] - L[e, j]
            O[e, j] = Tej[e, j] - L[e, j]
        tot = int(Pres[e].sum())
        assert tot == int(O[e].sum())
        for i in range(N):
            D[e, i, i] = L[e, i]
            o = int(O[e, i])
            if o == 0:
                continue
            cum = 0
            for j in range(N):
                if j == i:
                    continue
                nxt = cum + int(Pres[e, j])
                D[e, i, j] = (o * nxt) // tot - (o * cum) // tot
                cum = nxt
    recv = D.sum(axis=1)
    send = D.sum(axis=0)
    return {"cap": cap, "L": L, "Pres": Pres, "O": O, "D": D, "recv": recv, "send": send}


def order_rows(ids, rank_tok_off, slot_expert, E, N, c, D) -> dict:
    """Row maps of the per-slot contiguous buffers (Algorithm 1's reshuffle, extended
    to the receive side).

    Paper: source rank i sends rank j the (sum_{j'<j} D[e,i,j'])-th to
    (sum_{j'<=j} D[e,i,j'])-th of its tokens routed to e, tokens taken in order.  The
    paper stops at the send buffer; reading for the receive side: the (e,j) receive
    list is the concatenation of those runs over source ranks in ascending i, and it is
    cut over the R[e,j] slots of rank j that hold e (ascending slot id) by the same
    balanced rule, slot m getting list positions [floor(m*n/R), floor((m+1)*n/R)).
    Rows are numbered slot after slot in ascending slot id.

    Returns slot_counts [S], slot_offsets [S+1], pair_to_row [P], row_to_pair [P].
    """
    ids = np.asarray(ids)
    T, k = ids.shape
    S = N * c
    off = np.asarray(rank_tok_off, dtype=np.int64)
    flat = ids.reshape(-1)
    recv_list = [[[] for _ in range(N)] for _ in range(E)]
    for e in range(E):
        pairs_e = np.nonzero(flat == e)[0]            # ascending pair index = ascending token
        tok_e = pairs_e // k
        for i in range(N):
            a = np.searchsorted(tok_e, off[i], side="left")
            b = np.searchsorted(tok_e, off[i + 1], side="left")
            mine = pairs_e[a:b].tolist()               # the (e,i) pair list, token order
            assert len(mine) == int(np.sum(D[e, i]))
            start = 0
            for j in range(N):                         # destinations ascending, local one in place
                end = start + int(D[e, i, j])
                recv_list[e][j].extend(mine[start:end])
                start = end
    slot_rows = [[] for _ in range(S)]
    for j in range(N):
        for e in range(E):
            slots = [s for s in range(j * c, (j + 1) * c) if slot_expert[s] == e]
            lst = recv_list[e][j]
            n = len(lst)
            if not slots:
                assert n == 0, "tokens scheduled to a rank without a replica"
                continue
            Rj = len(slots)
            for m, s in enumerate(slots):
                slot_rows[s] = lst[(m * n) // Rj:((m + 1) * n) // Rj]
    slot_counts = np.array([len(r) for r in slot_rows], dtype=np.int32)
    slot_offsets = np.zeros(S + 1, dtype=np.int32)
    slot_offsets[1:] = np.cumsum(slot_counts)
    P = T * k
    row_to_pair = np.full(P, -1, dtype=np.int32)
    pair_to_row = np.full(P, -1, dtype=np.int32)
    row = 0
    for s in range(S):
        for p in slot_rows[s]:
            row_to_pair[row] = p
            pair_to_row[p] = row
            row += 1
    assert row == P
    return {"slot_counts": slot_counts, "slot_offsets": slot_offsets,
            "pair_to_row": pair_to_row, "row_to_pair": row_to_pair}


def plan_dispatch(ids, rank_tok_off, slot_expert, E, N, c) -> dict:
    """Histogram + Algorithm 1 schedule + row maps for one batch."""
    Tej = histogram(ids, rank_tok_off, E)
    R = replicas_per_rank(slot_expert, E, N, c)
    sch = schedule(Tej, R)
    out = order_rows(ids, rank_tok_off, slot_expert, E, N, c, sch["D"])
    out.update({"Tej": Tej, "R": R, **sch})
    return out


# ----------------------------------------------------------------------------- data movement
def permute(x: np.ndarray, row_to_pair: np.ndarray, k: int) -> np.ndarray:
    """xp[row] = x[token of the pair in that row]  (the reshuffle h -> h', Algorithm 1)."""
    return np.asarray(x)[np.asarray(row_to_pair) // k]


# ----------------------------------------------------------------------------- expert FFN
def gelu(v: np.ndarray) -> np.ndarray:
    """Exact GELU, 0.5*v*(1+erf(v/sqrt 2)).  (The paper names no activation; the exact
    form is the reading taken, not the tanh approximation.)"""
    return 0.5 * v * (1.0 + _erf(v / np.sqrt(2.0)))


def silu(v: np.ndarray) -> np.ndarray:
    return v / (1.0 + np.exp(-v))


def ffn(X: np.ndarray, w1: np.ndarray, w2: np.ndarray, act: str) -> np.ndarray:
    """One expert's FFN on rows X [n,d] in fp64 (Sec. 2.1: experts are parallel FFNs).

    gelu:   Y = gelu(X W1^T) W2^T,                 w1 [ffn,d],   w2 [d,ffn]
    swiglu: Y = (silu(X Wg^T) * (X Wu^T)) Wd^T,    w1 [2ffn,d] = [Wg; Wu], w2 = Wd [d,ffn]
    """
    W1 = widen(w1)
    W2 = widen(w2)
    if act == "gelu":
        H = gelu(X @ W1.T)
    elif act == "swiglu":
        f = W1.shape[0] // 2
        H = silu(X @ W1[:f].T) * (X @ W1[f:].T)
    else:
        raise ValueError(act)
    return H @ W2.T


def expert_ffn_rows(xp, slot_offsets, slot_expert, w1, w2, act) -> np.ndarray:
    """The FFN applied slot by slot to the permuted buffer: rows [off_s, off_{s+1}) go
    through the weights of expert slot_expert[s].  w1/w2 are indexed by expert."""
    Xp = widen(xp)
    yp = np.zeros((Xp.shape[0], np.asarray(w2).shape[1]), dtype=np.float64)
    for s in range(len(slot_expert)):
        a, b = int(slot_offsets[s]), int(slot_offsets[s + 1])
        if b > a:
            e = int(slot_expert[s])
            yp[a:b] = ffn(Xp[a:b], w1[e], w2[e], act)
    return yp


def unpermute_combine(yp, pair_to_row, gates) -> np.ndarray:
    """y[t] = sum_kk gates[t,kk] * yp[pair_to_row[t*k+kk]], kk ascending (the combine
    after the second all-to-all, Sec. 2.1)."""
    gates = np.asarray(gates, dtype=np.float64)
    T, k = gates.shape
    Yp = widen(yp)
    y = np.zeros((T, Yp.shape[1]), dtype=np.float64)
    p2r = np.asarray(pair_to_row).reshape(T, k)
    for kk in range(k):
        y = y + gates[:, kk:kk + 1] * Yp[p2r[:, kk]]
    return y


def layer_output(x, ids, gates, w1, w2, act, tokens=None) -> np.ndarray:
    """The layer's plain definition, independent of any placement or dispatch:

        y[t] = sum_{kk<k} gates[t,kk] * FFN_{ids[t,kk]}(x[t])          (Sec. 2.1)

    All replicas of an expert hold the same weights, so which replica serves a pair
    cannot change y.  fp64 throughout, kk ascending.  `tokens` restricts the evaluation
    to a subset of token indices (rows of the result follow that order).
    """
    ids = np.asarray(ids)
    gates = np.asarray(gates, dtype=np.float64)
    T, k = ids.shape
    tokens = np.arange(T) if tokens is None else np.asarray(tokens, dtype=np.int64)
    X = widen(np.asarray(x)[tokens])
    sub_ids = ids[tokens]
    E = np.asarray(w1).shape[0]
    dout = np.asarray(w2).shape[1]
    F = np.zeros((len(tokens), k, dout), dtype=np.float64)
    for e in range(E):
        rr, kk = np.nonzero(sub_ids == e)
        if len(rr):
            F[rr, kk] = ffn(X[rr], w1[e], w2[e], act)
    y = np.zeros((len(tokens), dout), dtype=np.float64)
    for kk in range(k):
        y = y + gates[tokens, kk:kk + 1] * F[:, kk]
    return y
