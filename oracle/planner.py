"""Oracle for the host-side planning: allocation, placement, recovery probability, replan.

TEST INFRASTRUCTURE ONLY (see the package docstring).  Pure Python integers.

A plan is the flat array slot_expert[N*c], slot id = rank*c + local slot: the
paper's placement matrix T (Appendix, proof of Theorem 1) read column by column.
"""
from __future__ import annotations

from fractions import Fraction
from itertools import combinations


class Infeasible(ValueError):
    """Fewer slots than experts: no plan can cover every expert."""


class Unrecoverable(ValueError):
    """Some expert has no replica on any surviving rank (Sec. 4.3: recovery needs one)."""


def load_order(t_e):
    """Experts in ascending load, equal loads by ascending id (Eq. 1 assumes this order;
    the tie rule is a reading, the paper gives none)."""
    return sorted(range(len(t_e)), key=lambda e: (int(t_e[e]), e))


def allocate_replicas(t_e, N: int, c: int, f: int):
    """Replica counts r_e by Eq. 1 (Sec. 4.1).

    Experts are visited in ascending load; the e-th gets
        r_e = max( floor( t_e / sum_{e'>=e} t_e' * (N*c - sum_{e'<e} r_e') ), f ).
    Readings where the paper is silent: the floor is taken on the exact integer
    quotient; if the remaining loads are all zero the remaining slots are split evenly;
    if N*c < E*f the threshold is relaxed to floor(N*c/E) (the paper drops the
    f-replica minimum when slots run short, Sec. 6.2), and fewer slots than experts is
    infeasible.  Returns r indexed by original expert id.
    """
    E = len(t_e)
    slots = N * c
    f_eff = min(int(f), slots // E)
    if f_eff < 1:
        raise Infeasible(f"{slots} slots cannot hold {E} experts")
    order = load_order(t_e)
    r = [0] * E
    rem = slots
    for pos, e in enumerate(order):
        tail = sum(int(t_e[x]) for x in order[pos:])
        if tail == 0:
            share = rem // (E - pos)
        else:
            share = (int(t_e[e]) * rem) // tail
        r[e] = max(share, f_eff)
        rem -= r[e]
    assert rem == 0, "Eq. 1 must use every slot"
    return r


def placement_order(r_e, t_e):
    """Expert order used by the placement: ascending replica count, then load, then id
    (Theorem 1 assumes r sorted ascending; for Eq.-1 allocations this is the load order)."""
    return sorted(range(len(r_e)), key=lambda e: (int(r_e[e]), int(t_e[e]), e))


def place_mro(r_e, t_e, N: int, c: int):
    """Maximum-rank-overlap placement (Sec. 4.1; definition in Theorem 1).

    With experts in sorted order and G = ceil(E/c) groups of c consecutive experts,
    node group g takes the next r_{first expert of g} nodes (the last group: at most
    what is left), and every node of group g holds one replica of every expert of
    group g.  When all experts fit one group (E <= c), expert e is additionally placed
    once on each of the first min(r_e, N) nodes.  The paper fills vacant slots
    "uniformly"; reading: walk vacant slots by (node, local slot) and deal the
    remaining replicas round-robin over the experts in sorted order, skipping the
    exhausted ones.  Returns slot_expert[N*c] in original expert ids.
    """
    E = len(r_e)
    if sum(int(v) for v in r_e) != N * c:
        raise ValueError("replica counts must fill exactly N*c slots")
    if any(int(v) < 1 for v in r_e):
        raise ValueError("every expert needs at least one replica")
    order = placement_order(r_e, t_e)
    r = [int(r_e[e]) for e in order]              # sorted numbering 0..E-1
    left = list(r)
    node_slots = [[] for _ in range(N)]
    G = -(-E // c)
    if G == 1:
        for q in range(E):
            for j in range(min(r[q], N)):
                node_slots[j].append(q)
                left[q] -= 1
    else:
        node0 = 0
        for g in range(G):
            first = g * c
            members = list(range(first, min(first + c, E)))
            size = r[first] if g < G - 1 else min(N - node0, r[first])
            assert size >= 1 and node0 + size <= N
            for j in range(node0, node0 + size):
                for q in members:
                    node_slots[j].append(q)
                    left[q] -= 1
            node0 += size
    assert all(v >= 0 for v in left) and all(len(s) <= c for s in node_slots)
    cursor = 0
    for j in range(N):
        while len(node_slots[j]) < c:
            while left[cursor % E] == 0:
                cursor += 1
            q = cursor % E
            node_slots[j].append(q)
            left[q] -= 1
            cursor += 1
    assert all(v == 0 for v in left)
    return [order[q] for j in range(N) for q in node_slots[j]]


def place_spread(r_e, N: int, c: int):
    """Spread baseline (Sec. 6.3): replicas listed expert after expert in id order,
    the q-th replica goes to rank q mod N, local slot q div N."""
    if sum(int(v) for v in r_e) != N * c:
        raise ValueError("replica counts must fill exactly N*c slots")
    slot_expert = [-1] * (N * c)
    q = 0
    for e, cnt in enumerate(r_e):
        for _ in range(int(cnt)):
            slot_expert[(q % N) * c + q // N] = e
            q += 1
    return slot_expert


def place_compact(r_e, N: int, c: int):
    """Compact baseline (Sec. 6.3): an expert's replicas sit on as few ranks as possible.
    Replicas listed expert after expert in id order fill rank after rank: the q-th replica
    goes to rank q div c, local slot q mod c."""
    if sum(int(v) for v in r_e) != N * c:
        raise ValueError("replica counts must fill exactly N*c slots")
    slot_expert = []
    for e, cnt in enumerate(r_e):
        slot_expert += [e] * int(cnt)
    return slot_expert


def recoverable(slot_expert, E: int, c: int, alive_ranks) -> bool:
    """Recovery needs every expert to keep a replica on some alive rank (Sec. 4.3)."""
    seen = set()
    for j in alive_ranks:
        seen.update(slot_expert[j * c:(j + 1) * c])
    return len(seen) == E and all(0 <= e < E for e in seen)


def recovery_probability(slot_expert, E: int, N: int, c: int, n_alive: int) -> Fraction:
    """Pr(the union of the alive ranks' experts is all of [E]) over a uniformly drawn
    set of n_alive alive ranks, by enumerating every set (Sec. 6.3; objective of Theorem 1)."""
    good = total = 0
    for alive in combinations(range(N), n_alive):
        total += 1
        good += recoverable(slot_expert, E, c, alive)
    return Fraction(good, total)


def replan(old_slot_expert, N_old: int, c_old: int, alive, t_e, c_new: int, f: int) -> dict:
    """New plan on the surviving ranks and the state transfers that realise it (Sec. 4.3).

    1. survivors = alive ranks, ascending; unrecoverable if an expert lost every replica.
    2. Eq. 1 on len(survivors)*c_new slots, then MRO placement (plan nodes 0..N_new-1).
    3. Greedy node mapping.  The paper maps physical nodes to plan nodes so that few
       experts are newly assigned, without fixing the order; reading: physical
       survivors in ascending id each take the unused plan node with the fewest experts
       (as a set) that the physical node does not already hold, lowest plan node on ties.
    4. Transfers.  A new slot whose expert the node already held is filled locally from
       the node's lowest old slot of that expert.  Otherwise the node fetches the expert
       once, from one of its surviving owners; the requests for one expert are dealt
       round-robin over its owners in ascending rank (the paper: spread over all owners).

    Returns new_slot_expert (rank m = m-th survivor), plan2phys[plan node] = old rank id,
    transfers = [(dst_slot in the new numbering, src_slot in the old numbering, expert,
    remote 0/1)], one per new slot in ascending dst_slot.
    """
    E = len(t_e)
    survivors = [j for j in range(N_old) if alive[j]]
    N_new = len(survivors)
    held = {p: set(old_slot_expert[p * c_old:(p + 1) * c_old]) for p in survivors}
    if N_new == 0 or not recoverable(old_slot_expert, E, c_old, survivors):
        raise Unrecoverable("an expert has no surviving replica")
    r = allocate_replicas(t_e, N_new, c_new, f)
    plan = place_mro(r, t_e, N_new, c_new)
    plan_sets = [set(plan[q * c_new:(q + 1) * c_new]) for q in range(N_new)]
    used = [False] * N_new
    plan2phys = [-1] * N_new
    phys2plan = {}
    for p in survivors:
        best, best_cost = -1, None
        for q in range(N_new):
            if used[q]:
                continue
            cost = len(plan_sets[q] - held[p])
            if best_cost is None or cost < best_cost:
                best, best_cost = q, cost
        used[best] = True
        plan2phys[best] = p
        phys2plan[p] = best
    new_slot_expert = []
    for p in survivors:
        q = phys2plan[p]
        new_slot_expert.extend(plan[q * c_new:(q + 1) * c_new])
    owners = {e: [p for p in survivors if e in held[p]] for e in range(E)}
    next_owner = [0] * E
    fetched = {}
    transfers = []
    for m, p in enumerate(survivors):
        for l in range(c_new):
            e = new_slot_expert[m * c_new + l]
            if e in held[p]:
                src_rank, remote = p, 0
            else:
                if (p, e) not in fetched:
                    fetched[(p, e)] = owners[e][next_owner[e] % len(owners[e])]
                    next_owner[e] += 1
                src_rank, remote = fetched[(p, e)], 1
            src_slot = next(s for s in range(src_rank * c_old, (src_rank + 1) * c_old)
                            if old_slot_expert[s] == e)
            transfers.append((m * c_new + l, src_slot, e, remote))
    return {"r": r, "plan": plan, "new_slot_expert": new_slot_expert, "plan2phys": plan2phys,
            "transfers": transfers, "survivors": survivors}
