"""The synthetic workloads themselves: what the configs promise about their inputs (CPU only)."""
import numpy as np

from oracle import moe_layer as om
from oracle import planner as op
from workloads import CONFIGS, step_inputs
from workloads.synth import popularity_bias


def _ranking(bias):
    return np.argsort(-bias, kind="stable").tolist()


def test_post_failure_traffic_keeps_the_ranking_the_replan_was_proportioned_for():
    """Config 5 re-plans config 3's step-0 plan (Sec. 4.3: replica counts re-proportioned to the
    loads) and then serves traffic with the same popularity ranking; only the Zipf exponent is
    redrawn per step."""
    c5, c3 = CONFIGS["c5_postfailure"], CONFIGS["c3_gptmoe"]
    want = _ranking(popularity_bias(c3, 0))
    exps = set()
    for step in (0, 1, 57, 99):
        b = popularity_bias(c5, step)
        assert _ranking(b) == want
        exps.add(round(float(-b[want[1]] / np.log(2.0)), 4))      # b = -s ln(rank + 1): rank 1 gives s
    assert len(exps) == 4 and all(0.8 <= s <= 1.5 for s in exps)
    # config 3 itself still reshuffles its ranking every 5 steps
    assert _ranking(popularity_bias(c3, 5)) != want and _ranking(popularity_bias(c3, 4)) == want


def test_post_failure_plan_fits_its_traffic():
    """Under the re-planned layout the popular experts of config 5's traffic are the ones that got
    the replicas: the fullest slot holds about t_e / r_e rows of its expert (the dispatcher
    balances an expert's replicas), and that stays within 4x the mean slot size.  (Eq. 1 floors
    in ascending load order with a minimum of one replica, so the 28 small experts of this
    Zipf profile take 28 of the 48 slots and a mid-sized expert is left with one replica: 3.5x.
    With the ranking drawn from another seed the fullest slot held 16x the mean.)"""
    c5, c3 = CONFIGS["c5_postfailure"], CONFIGS["c3_gptmoe"]
    ids0, _ = om.route(step_inputs(c3, 0, with_x=False)["logits"], c3.k)
    t_e = np.bincount(ids0.reshape(-1), minlength=c3.E)
    old = op.place_mro(op.allocate_replicas(t_e, c3.N, c3.c, c3.f), t_e, c3.N, c3.c)
    alive = np.ones(c5.base_N, dtype=np.uint8)
    alive[list(c5.drop_ranks)] = 0
    new = np.array(op.replan(old, c5.base_N, c5.base_c, alive, t_e, c5.c, c5.f)["new_slot_expert"])
    for step in (0, 57):
        inp = step_inputs(c5, step, with_x=False)
        ids, _ = om.route(inp["logits"], c5.k)
        disp = om.plan_dispatch(ids, inp["rank_tok_off"], new, c5.E, c5.N, c5.c)
        counts = disp["slot_counts"]
        t_step = np.bincount(ids.reshape(-1), minlength=c5.E)
        r = np.bincount(new, minlength=c5.E)
        per_replica = int(np.max(-(-t_step // r)))
        assert counts.max() <= per_replica + c5.N
        assert counts.max() <= 4 * counts.mean(), (step, int(counts.max()), float(counts.mean()))
