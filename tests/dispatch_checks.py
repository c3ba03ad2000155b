"""Property checks for dispatch results, written as predicates rather than as a second
copy of the algorithm.  They hold at any size and are used against both the oracle
(pins) and the GPU path (full-size parity)."""
import numpy as np


def check_schedule_invariants(Tej, R, sch):
    """Invariants of Algorithm 1's counts (Sec. 4.2): tokens conserved, local capacity
    used first, every replica gets about t_e / r_e."""
    Tej = np.asarray(Tej, dtype=np.int64)
    R = np.asarray(R, dtype=np.int64)
    D, cap, recv = sch["D"], sch["cap"], sch["recv"]
    E, N = Tej.shape
    assert np.all(D >= 0)
    # every pair of every source rank is sent somewhere: row sums
    assert np.array_equal(D.sum(axis=2), Tej)
    # all tokens of an expert are received
    assert np.array_equal(recv.sum(axis=1), Tej.sum(axis=1))
    assert np.array_equal(cap.sum(axis=1), Tej.sum(axis=1))
    for e in range(E):
        r_e, t_e = int(R[e].sum()), int(Tej[e].sum())
        if t_e == 0:
            continue
        n_over = 0
        for i in range(N):
            # local first: the rank keeps min(capacity, own tokens)
            assert D[e, i, i] == min(cap[e, i], Tej[e, i])
            # capacity within one token of p_e * R[e,i]
            assert abs(cap[e, i] * r_e - t_e * R[e, i]) < r_e
            if Tej[e, i] <= cap[e, i]:
                # nothing leaves a rank that is within its capacity
                assert D[e, i].sum() == D[e, i, i]
            else:
                n_over += 1
            # nothing is sent to a rank without a replica
            if R[e, i] == 0:
                assert recv[e, i] == 0
        for j in range(N):
            # each overflowing source contributes a rounding error below one token
            assert abs(int(recv[e, j]) - int(cap[e, j])) <= max(n_over - 1, 0)
            # only ranks with residual capacity receive foreign tokens
            foreign = int(recv[e, j]) - int(D[e, j, j])
            if foreign > 0:
                assert cap[e, j] > Tej[e, j]


def check_row_maps(ids, rank_tok_off, slot_expert, E, N, c, D, maps):
    """The row maps are the unique ones that satisfy, given the counts D:
    a bijection pairs<->rows; each row lies in a slot of its pair's expert; along each
    (expert, source rank) list in token order the destination ranks are non-decreasing
    with D[e,i,j] pairs each; inside an (expert, rank) the rows are in ascending token
    order across its slots; and its slots share the received pairs by the balanced cut."""
    ids = np.asarray(ids)
    T, k = ids.shape
    P = T * k
    S = N * c
    slot_expert = np.asarray(slot_expert)
    cnt = np.asarray(maps["slot_counts"], dtype=np.int64)
    off = np.asarray(maps["slot_offsets"], dtype=np.int64)
    p2r = np.asarray(maps["pair_to_row"], dtype=np.int64)
    r2p = np.asarray(maps["row_to_pair"], dtype=np.int64)
    assert cnt.shape == (S,) and off.shape == (S + 1,)
    assert off[0] == 0 and np.array_equal(np.diff(off), cnt) and off[-1] == P
    assert np.array_equal(np.sort(r2p), np.arange(P))
    assert np.array_equal(p2r[r2p], np.arange(P))
    row_slot = np.searchsorted(off, np.arange(P), side="right") - 1
    pair_slot = row_slot[p2r]
    flat = ids.reshape(-1)
    assert np.array_equal(slot_expert[pair_slot], flat)
    pair_dst = pair_slot // c
    tok = np.arange(P) // k
    src = np.searchsorted(np.asarray(rank_tok_off, dtype=np.int64), tok, side="right") - 1
    for e in range(E):
        pe = np.nonzero(flat == e)[0]
        for i in range(N):
            mine = pe[src[pe] == i]
            dst = pair_dst[mine]
            assert np.all(np.diff(dst) >= 0)
            assert np.array_equal(np.bincount(dst, minlength=N), np.asarray(D[e, i]))
        for j in range(N):
            slots = [s for s in range(j * c, (j + 1) * c) if slot_expert[s] == e]
            if not slots:
                continue
            here = pe[pair_dst[pe] == j]
            rows = p2r[here]
            order = np.argsort(rows)
            assert np.all(np.diff(tok[here][order]) > 0)
            n, Rj = len(here), len(slots)
            for m, s in enumerate(slots):
                assert cnt[s] == ((m + 1) * n) // Rj - (m * n) // Rj
