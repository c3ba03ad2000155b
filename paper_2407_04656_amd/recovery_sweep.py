"""Recovery probability of MRO placement against the spread and compact baselines (Sec. 6.3,
the multi-node-failure figure): for a Zipf expert-load profile, allocate replicas with Eq. 1,
place them three ways and enumerate every set of failed nodes.  Host-only; uses the library's
planner (lz_allocate_replicas, lz_place_*, lz_recovery_probability).

    python -m paper_2407_04656_amd.recovery_sweep --experts 16 --nodes 10 --slots 6 --zipf 1.0
"""
from __future__ import annotations

import argparse

import numpy as np

from . import binding as lz


def zipf_loads(E: int, s: float, total: int = 1_000_000) -> np.ndarray:
    """Expected tokens per expert when expert i is drawn with probability ~ (i+1)^-s."""
    p = np.array([(i + 1.0) ** -s for i in range(E)])
    return np.round(p / p.sum() * total).astype(np.int64)


def sweep(E: int, N: int, c: int, s: float, f: int = 1) -> dict:
    """{"r": replica counts, "rows": [(failed, p_mro, p_spread, p_compact), ...]}"""
    t_e = zipf_loads(E, s)
    r = lz.lz_allocate_replicas(t_e, N, c, f)
    plans = (lz.lz_place_mro(r, t_e, N, c), lz.lz_place_spread(r, N, c), lz.lz_place_compact(r, N, c))
    rows = []
    for failed in range(1, N):
        probs = []
        for plan in plans:
            good, total = lz.lz_recovery_probability(plan, E, N, c, N - failed)
            probs.append(good / total)
        rows.append((failed, *probs))
    return {"r": r.tolist(), "rows": rows}


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--experts", type=int, default=16)
    ap.add_argument("--nodes", type=int, default=10)
    ap.add_argument("--slots", type=int, default=6, help="replica slots per node (c)")
    ap.add_argument("--zipf", type=float, nargs="+", default=[0.5, 1.0, 1.5])
    a = ap.parse_args()
    for s in a.zipf:
        out = sweep(a.experts, a.nodes, a.slots, s)
        print(f"E={a.experts} N={a.nodes} c={a.slots} Zipf s={s}: replicas {out['r']}")
        print("  failed nodes |    MRO | spread | compact")
        for failed, mro, spread, compact in out["rows"]:
            print(f"  {failed:12d} | {mro:6.3f} | {spread:6.3f} | {compact:6.3f}")


if __name__ == "__main__":
    main()
