#!/usr/bin/env python3
"""MoE-layer throughput of the Lazarus hot path on one MI355X.

A step is one pass of the whole path (route -> plan_dispatch -> permute -> expert FFN ->
unpermute_combine) over one batch of synthetic input that is already resident in HBM.
Prints ONE JSON line: whole-path tokens/s of the headline workload (config 2) plus a roofline
record for the dominant kernel (the first grouped GEMM), timed live with events on the launch
stream; a `workloads` object with the same figures for the other four configs (config 3 both
with the plan rebalanced at every popularity reshuffle and with the step-0 plan kept); and the
CPU oracle timed on a bounded sample of the headline workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3     # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM-side bytes per launch of the dominant kernel, from the rocprofv3 FETCH_SIZE / WRITE_SIZE passes
# summarised in profiles/<workload>_hbm_traffic.md (counters cannot be read from inside this
# process, so the figure is carried here and re-measured whenever the kernel changes).
# c2_mixtral GEMM-1: FETCH_SIZE x 2.00 (what the counter reads for a plain copy of known size) +
# WRITE_SIZE 459 402 KiB, from profiles/c2_mixtral_hbm_traffic.md.
MEASURED_TRAFFIC_BYTES = {"c2_mixtral": 16.06e9}

NAMES = ["route", "plan", "permute", "ffn_up", "ffn_down", "combine"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2_mixtral")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="0 = pick per workload")
    ap.add_argument("--copy-calib-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB (counter calibration for profiling)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the achievable-peak probes, the cold-cache bandwidth runs, the training pass, "
                         "the replan timing and the other workloads")
    ap.add_argument("--fused-gather", action="store_true",
                    help="headline step with the reshuffle fused into the first GEMM's activation loads "
                         "(lz_ffn_up_gather) instead of the permute kernel")
    return ap.parse_args()


def achievable_peaks(torch, dev):
    """What this machine reaches on a plain 1 GiB device copy and on a large square bf16 GEMM of the
    vendor library: context for the fractions of the nominal peaks, not part of the path."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(2):
        dst.copy_(src)
    a.record()
    for _ in range(10):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * n / (a.elapsed_time(b) / 10 * 1e-3) / 1e9
    del src, dst
    m = 8192
    p = torch.randn((m, m), device=dev, dtype=torch.float32).to(torch.bfloat16)
    q = torch.randn((m, m), device=dev, dtype=torch.float32).to(torch.bfloat16)
    for _ in range(3):
        torch.matmul(p, q.t())
    a.record()
    for _ in range(10):
        torch.matmul(p, q.t())
    b.record()
    torch.cuda.synchronize()
    tf = 2.0 * m ** 3 / (a.elapsed_time(b) / 10 * 1e-3) / 1e12
    return {"device_copy_GBps": copy_gbs, "vendor_bf16_gemm_8192_TFLOPs": tf,
            "note": "1 GiB torch copy (read + write bytes) and torch.matmul 8192^3 bf16 on this box"}


class Workload:
    """One config resident on the device: inputs, layer object, plan, and the step function."""

    def __init__(self, torch, lz, cfg, n_logit_draws, weights=None):
        from workloads import CONFIGS, expert_weights, step_inputs
        self.torch, self.lz, self.cfg = torch, lz, cfg
        self.dev = "cuda:0"
        self.shape = lz.Shape.from_config(cfg)
        self.bf16 = cfg.dtype == "bf16"
        t0 = time.perf_counter()
        self.inp = step_inputs(cfg, 0)
        self.w = weights if weights is not None else expert_weights(CONFIGS[cfg.base] if cfg.base else cfg, threads=16)
        n = max(1, n_logit_draws)
        self.logits_host = [self.inp["logits"]] + [step_inputs(cfg, i, with_x=False)["logits"] for i in range(1, n)]
        self.gen_s = time.perf_counter() - t0
        self.logits_all = [self.to_dev(l) for l in self.logits_host]
        self.x = self.to_dev(self.inp["x"], self.bf16)
        self.layer = lz.MoELayer(self.shape, self.dev)
        self.layer.set_plan(np.zeros(self.shape.S, dtype=np.int32), self.inp["rank_tok_off"])
        self.expert_w = None     # per-expert weights on the device, library layout (filled on demand)
        self.plan = None
        self.plan_note = ""

    def to_dev(self, a, as_bf16=False):
        t = self.torch.from_numpy(np.ascontiguousarray(a))
        if as_bf16:
            t = t.view(self.torch.bfloat16)
        return t.to(self.dev)

    # ---- plans, all computed by the library
    def routed_loads(self, cfg, logits_dev):
        lz = self.lz
        probe = self.layer if cfg is self.cfg else lz.MoELayer(lz.Shape.from_config(cfg), self.dev)
        if probe is not self.layer:
            probe.set_plan(np.zeros(cfg.N * cfg.c, dtype=np.int32),
                           np.array([(i * cfg.T) // cfg.N for i in range(cfg.N + 1)], dtype=np.int32))
        probe.route(logits_dev)
        self.torch.cuda.synchronize()
        return np.bincount(probe.topk_ids.cpu().numpy().reshape(-1), minlength=cfg.E)

    def lib_plan(self, cfg, t_e):
        lz = self.lz
        if cfg.replica_counts is not None:
            r = np.array(cfg.replica_counts, dtype=np.int32)
        else:
            r = lz.lz_allocate_replicas(t_e, cfg.N, cfg.c, cfg.f)
        if cfg.placement == "spread":
            return lz.lz_place_spread(r, cfg.N, cfg.c)
        return lz.lz_place_mro(r, t_e, cfg.N, cfg.c)

    def initial_plan(self):
        from workloads import CONFIGS, step_inputs
        cfg, lz = self.cfg, self.lz
        if cfg.base is None:
            # plan from the realised step-0 routing (the paper's routing history): Eq. 1 + MRO, or
            # the fixed allocation + spread placement of the tiny config
            self.plan = self.lib_plan(cfg, self.routed_loads(cfg, self.logits_all[0]))
            self.plan_note = "Eq.1 + MRO on step-0 loads" if cfg.replica_counts is None else "fixed counts, spread"
        else:
            # post-failure workload: the base config's step-0 plan loses ranks, lz_replan gives the new one
            base = CONFIGS[cfg.base]
            t_e = self.routed_loads(base, self.to_dev(step_inputs(base, 0, with_x=False)["logits"]))
            alive = np.ones(cfg.base_N, dtype=np.uint8)
            alive[list(cfg.drop_ranks)] = 0
            self.plan = lz.lz_replan(self.lib_plan(base, t_e), cfg.base_N, cfg.base_c, alive, t_e, cfg.c,
                                     cfg.f)["new_slot_expert"]
            self.plan_note = f"lz_replan of {cfg.base}'s step-0 plan after losing ranks {list(cfg.drop_ranks)}"
        self.torch.cuda.empty_cache()
        self.layer.set_plan(self.plan, self.inp["rank_tok_off"])
        self.layer.load_expert_weights(self.w["w1"], self.w["w2"], self.plan)
        self.torch.cuda.synchronize()

    def rebalance(self, logits_dev):
        """Periodic rebalance (Sec. 5): new Eq. 1 + MRO plan from this step's routing with every rank
        alive, weights moved between slot buffers by the transfer list.  Returns host ms, device ms."""
        torch, lz, s = self.torch, self.lz, self.shape
        t_e = self.routed_loads(self.cfg, logits_dev)
        alive = np.ones(s.N, dtype=np.uint8)
        t0 = time.perf_counter()
        re = lz.lz_replan(self.plan, s.N, s.c, alive, t_e, s.c, self.cfg.f)
        host_ms = (time.perf_counter() - t0) * 1e3
        lay = self.layer
        if getattr(self, "w1_alt", None) is None:
            self.w1_alt, self.w2_alt = torch.empty_like(lay.w1), torch.empty_like(lay.w2)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        lz.lz_apply_transfers(re["transfers"], lay.w1, lay.w2, s.S, self.w1_alt, self.w2_alt, s.S, s)
        b.record()
        torch.cuda.synchronize()
        lay.w1, self.w1_alt = self.w1_alt, lay.w1
        lay.w2, self.w2_alt = self.w2_alt, lay.w2
        self.plan = re["new_slot_expert"]
        lay.set_plan(self.plan, self.inp["rank_tok_off"])
        return host_ms, a.elapsed_time(b), int(sum(t[3] for t in re["transfers"]))

    # ---- one pass of the path
    def step(self, logits, marks=None, fused_gather=False):
        lz, s, shape = self.lz, self.layer, self.shape
        stream = self.torch.cuda.current_stream()
        rec = (lambda i: marks[i].record(stream)) if marks is not None else (lambda i: None)
        rec(0)
        s.route(logits)
        rec(1)
        s.plan_dispatch()
        lz.lz_ffn_tiles(s.slot_offsets, shape, s.ffn_ws, s.ffn_ws_bytes)   # row-tile table: dispatch bookkeeping
        rec(2)
        if not fused_gather:
            s.permute(self.x)
        rec(3)
        if fused_gather:
            lz.lz_ffn_up_gather(self.x, s.row_to_pair, s.w1, shape, s.ffn_ws, s.ffn_ws_bytes)
        else:
            lz.lz_ffn_up(s.xp, s.w1, shape, s.ffn_ws, s.ffn_ws_bytes)
        rec(4)
        lz.lz_ffn_down(s.w2, shape, s.yp, s.ffn_ws, s.ffn_ws_bytes)
        rec(5)
        s.unpermute_combine()
        rec(6)

    def burst(self, fn, n=20):
        torch = self.torch
        stream = torch.cuda.current_stream()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        a.record(stream)
        for _ in range(n):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    def cold(self, fn, n=8):
        torch = self.torch
        stream = torch.cuda.current_stream()
        scratch = torch.empty(1 << 30, dtype=torch.uint8, device=self.dev)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ts = []
        for i in range(n):
            scratch.fill_(i)
            a.record(stream)
            fn()
            b.record(stream)
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        del scratch
        return float(np.median(ts))


def measure(wl, steps, warmup, rebalance_every=0, fused_gather=False, cold=False):
    """warmup untimed steps, then exactly `steps` timed ones between two synchronisations.  With
    rebalance_every > 0 the plan is recomputed (outside the event-timed steps) whenever the step
    index is a multiple of it; the wall clock then contains those pauses, so tokens/s comes from
    the per-step event times."""
    torch, cfg, shape, layer = wl.torch, wl.cfg, wl.shape, wl.layer
    n_logits = len(wl.logits_all)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    rebal = []
    for i in range(warmup):
        wl.step(wl.logits_all[i % n_logits], fused_gather=fused_gather)
    torch.cuda.synchronize()
    assert int(layer.status.item()) == 0, "plan_dispatch flagged the plan"
    marks = [[ev() for _ in range(7)] for _ in range(steps)]
    slot_max, slot_mean = [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        idx = (warmup + i) % n_logits
        if rebalance_every and idx % rebalance_every == 0:
            torch.cuda.synchronize()
            rebal.append(wl.rebalance(wl.logits_all[idx]))
        wl.step(wl.logits_all[idx], marks[i], fused_gather=fused_gather)
        if rebalance_every or n_logits > 1:
            slot_max.append(layer.slot_counts.max())
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert int(layer.status.item()) == 0, "plan_dispatch flagged the plan"

    samples = {n: np.array([m[i].elapsed_time(m[i + 1]) for m in marks]) for i, n in enumerate(NAMES)}
    per = {n: float(np.mean(v)) for n, v in samples.items()}
    step_ms = np.array([m[0].elapsed_time(m[6]) for m in marks])
    eb = 4 if cfg.dtype == "f32" else 2
    P, T, d, ffn, k = shape.P, shape.T, shape.d, shape.ffn, shape.k
    mult = 2 if cfg.act == "swiglu" else 1
    flops_up = 2.0 * P * d * ffn * mult           # real rows only, no padding credit
    flops_down = 2.0 * P * ffn * d
    permute_bytes = (1 + k) * T * d * eb + 4 * P   # compulsory: read x once, write xp, read the map
    combine_bytes = (1 + k) * T * d * eb + 8 * P
    peak = PEAK_BF16_TFLOPS if wl.bf16 else PEAK_F32_TFLOPS
    burst_ms = {"permute": wl.burst(lambda: layer.permute(wl.x)), "combine": wl.burst(layer.unpermute_combine)}
    out = {
        "ms_per_step_wall": wall * 1e3 / steps,
        "step_ms_by_events": {"mean": float(np.mean(step_ms)), "median": float(np.median(step_ms)),
                              "min": float(np.min(step_ms))},
        "kernels_ms": per,
        "kernels_ms_median": {n: float(np.median(v)) for n, v in samples.items()},
        "kernels_ms_min": {n: float(np.min(v)) for n, v in samples.items()},
        "flops_up": flops_up, "flops_down": flops_down,
        "ffn_up_TFLOPs": flops_up / (per["ffn_up"] * 1e-3) / 1e12,
        "ffn_down_TFLOPs": flops_down / (per["ffn_down"] * 1e-3) / 1e12,
        "ffn_TFLOPs": (flops_up + flops_down) / ((per["ffn_up"] + per["ffn_down"]) * 1e-3) / 1e12,
        "permute_GBps": permute_bytes / (burst_ms["permute"] * 1e-3) / 1e9,
        "combine_GBps": combine_bytes / (burst_ms["combine"] * 1e-3) / 1e9,
        "combine_GBps_in_step": combine_bytes / (per["combine"] * 1e-3) / 1e9,
        "slot_rows_max": int(max(slot_max).item()) if slot_max else int(layer.slot_counts.max().item()),
        "slot_rows_mean": P / shape.S,
        "peak_TFLOPs": peak,
    }
    if not fused_gather:
        out["permute_GBps_in_step"] = permute_bytes / (per["permute"] * 1e-3) / 1e9
    if cold:
        c = {"permute": wl.cold(lambda: layer.permute(wl.x)), "combine": wl.cold(layer.unpermute_combine)}
        out["permute_GBps_cold"] = permute_bytes / (c["permute"] * 1e-3) / 1e9
        out["combine_GBps_cold"] = combine_bytes / (c["combine"] * 1e-3) / 1e9
    if rebal:
        out["rebalance"] = {"count": len(rebal), "host_ms_median": float(np.median([r[0] for r in rebal])),
                            "copy_ms_median": float(np.median([r[1] for r in rebal])),
                            "remote_copies_median": float(np.median([r[2] for r in rebal])),
                            "note": "lz_replan with every rank alive on that step's routing (host), "
                                    "lz_apply_transfers into the second weight buffer (device); not in the step times"}
    return out


def graph_replay_ms(wl, n=100):
    """The same step captured once in a HIP graph and replayed: what a launch-bound shape gains when
    the caller records the library's calls (they neither allocate nor synchronise) instead of
    issuing them one by one."""
    torch = wl.torch
    wl.step(wl.logits_all[0])
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=stream):
        wl.step(wl.logits_all[0])
    torch.cuda.synchronize()
    for _ in range(5):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / n


def compare_fused_gather(wl, rounds=4, steps=8):
    """The step with the permute kernel against the step whose first GEMM reads x through the row map
    (lz_ffn_up_gather), in the same process and interleaved (boxes and minutes differ by more than
    the two paths do): `rounds` alternating blocks of `steps` event-timed steps each."""
    torch = wl.torch
    ev = lambda: torch.cuda.Event(enable_timing=True)
    acc = {False: [], True: []}
    for fused in (False, True):
        for _ in range(3):
            wl.step(wl.logits_all[0], fused_gather=fused)
    torch.cuda.synchronize()
    for _ in range(rounds):
        for fused in (False, True):
            marks = [[ev() for _ in range(7)] for _ in range(steps)]
            wl.step(wl.logits_all[0], fused_gather=fused)        # untimed: the switch itself
            for m in marks:
                wl.step(wl.logits_all[0], m, fused_gather=fused)
            torch.cuda.synchronize()
            acc[fused] += [[m[i].elapsed_time(m[i + 1]) for i in range(6)] + [m[0].elapsed_time(m[6])] for m in marks]
    mean = {f: np.mean(np.array(v), axis=0) for f, v in acc.items()}
    col = {n: i for i, n in enumerate(NAMES + ["step"])}
    return {"ms_per_step": float(mean[True][col["step"]]), "ms_per_step_unfused": float(mean[False][col["step"]]),
            "ffn_up_ms": float(mean[True][col["ffn_up"]]), "ffn_up_ms_unfused": float(mean[False][col["ffn_up"]]),
            "ffn_down_ms": float(mean[True][col["ffn_down"]]), "ffn_down_ms_unfused": float(mean[False][col["ffn_down"]]),
            "permute_ms_unfused": float(mean[False][col["permute"]]),
            "steps_each": rounds * steps,
            "note": "same step with the reshuffle done by the first GEMM's activation loads (lz_ffn_up_gather reads x "
                    "through row_to_pair; no permute kernel, no xp buffer); the two paths measured in alternating "
                    "blocks of the same process"}


def compact(cfg, m, plan_note):
    """The figures of one workload for the `workloads` object."""
    T = cfg.T
    ms = m["step_ms_by_events"]["mean"]
    out = {
        "tokens_per_s": T / (ms * 1e-3), "ms_per_step": ms, "dtype": cfg.dtype, "plan": plan_note,
        "kernels_ms": {k: round(v, 5) for k, v in m["kernels_ms"].items()},
        "ffn_up_TFLOPs": m["ffn_up_TFLOPs"], "ffn_up_frac_peak": m["ffn_up_TFLOPs"] / m["peak_TFLOPs"],
        "ffn_down_TFLOPs": m["ffn_down_TFLOPs"], "ffn_down_frac_peak": m["ffn_down_TFLOPs"] / m["peak_TFLOPs"],
        "permute_GBps": m["permute_GBps"], "permute_frac_hbm": m["permute_GBps"] / PEAK_HBM_GBS,
        "combine_GBps": m["combine_GBps"], "combine_frac_hbm": m["combine_GBps"] / PEAK_HBM_GBS,
        "slot_rows_max": m["slot_rows_max"], "slot_rows_mean": m["slot_rows_mean"],
    }
    if "rebalance" in m:
        out["rebalance"] = m["rebalance"]
    return out


def other_workloads(torch, lz, skip):
    """Configs 1, 3, 4 and 5 through the same step function (fewer extras).  Config 3 twice: the plan
    rebalanced at every popularity reshuffle (Sec. 5's periodic rebalance; primary) and the step-0
    plan kept for all 20 steps (what the dispatcher does between rebalances)."""
    from workloads import CONFIGS, expert_weights
    res = {}
    shared_w = {}
    for name, steps, warmup in (("c1_tiny", 50, 5), ("c3_gptmoe", 20, 20), ("c4_finegrained", 20, 3),
                                ("c5_postfailure", 100, 5)):
        if name == skip:
            continue
        cfg = CONFIGS[name]
        wkey = cfg.base or name
        if wkey not in shared_w:
            shared_w.clear()
            shared_w[wkey] = expert_weights(CONFIGS[wkey], threads=16)
        wl = Workload(torch, lz, cfg, cfg.steps, weights=shared_w[wkey])
        wl.initial_plan()
        if name == "c3_gptmoe":
            # warm-up = one full cycle of the 20 draws, so the timed steps start at draw 0 again
            kept = measure(wl, steps, warmup)
            res[name + "_plan_kept"] = compact(cfg, kept, wl.plan_note + "; fresh logits each step, plan kept (stale after step 4)")
            reb = measure(wl, steps, warmup, rebalance_every=cfg.reshuffle_every)
            res[name] = compact(cfg, reb, "Eq.1 + MRO recomputed from the step's routing at steps 0, 5, 10, 15 "
                                          "(lz_replan + lz_apply_transfers, untimed); fresh logits each step")
        else:
            m = measure(wl, steps, warmup)
            note = wl.plan_note + ("; fresh logits each step, plan kept" if cfg.steps > 1 else "")
            res[name] = compact(cfg, m, note)
            if name == "c4_finegrained":                # top-6: the reshuffle moves the most bytes per flop here
                res[name]["fused_gather"] = compare_fused_gather(wl)
            if name in ("c1_tiny", "c4_finegrained"):   # the shapes with the most launches per unit of work
                g = graph_replay_ms(wl)
                res[name]["hip_graph_replay"] = {"ms_per_step": g, "tokens_per_s": cfg.T / (g * 1e-3),
                                                 "note": "the step's launches captured once and replayed (wall clock over 100 replays)"}
        del wl
        torch.cuda.empty_cache()
    return res


def replan_latency(torch, lz, dev):
    """Row a8 measured: config 5's scenario.  Config 3's step-0 plan loses two ranks; host time of
    lz_replan (Eq. 1, MRO, greedy mapping, transfer list) and device time of lz_apply_transfers."""
    from workloads import CONFIGS, expert_weights, step_inputs
    cfg = CONFIGS["c5_postfailure"]
    base = CONFIGS[cfg.base]
    w = expert_weights(base, threads=16)
    inp = step_inputs(base, 0, with_x=False)
    shape_old, shape_new = lz.Shape.from_config(base), lz.Shape.from_config(cfg)
    old = lz.MoELayer(shape_old, dev)
    old.set_plan(np.zeros(shape_old.S, dtype=np.int32), inp["rank_tok_off"])
    old.route(torch.from_numpy(inp["logits"]).to(dev))
    torch.cuda.synchronize()
    t_e = np.bincount(old.topk_ids.cpu().numpy().reshape(-1), minlength=base.E)
    r = lz.lz_allocate_replicas(t_e, base.N, base.c, base.f)
    old_plan = lz.lz_place_mro(r, t_e, base.N, base.c)
    old.load_expert_weights(w["w1"], w["w2"], old_plan)
    alive = np.ones(cfg.base_N, dtype=np.uint8)
    alive[list(cfg.drop_ranks)] = 0
    host = []
    for _ in range(20):
        t0 = time.perf_counter()
        re = lz.lz_replan(old_plan, cfg.base_N, cfg.base_c, alive, t_e, cfg.c, cfg.f)
        host.append((time.perf_counter() - t0) * 1e3)
    n1 = w["w1"].shape[1]
    w1n = torch.empty((shape_new.S, cfg.d, n1), dtype=torch.bfloat16, device=dev)
    w2n = torch.empty((shape_new.S, cfg.ffn, cfg.d), dtype=torch.bfloat16, device=dev)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    copy = []
    for _ in range(5):
        a.record()
        lz.lz_apply_transfers(re["transfers"], old.w1, old.w2, shape_old.S, w1n, w2n, shape_new.S, shape_new)
        b.record()
        torch.cuda.synchronize()
        copy.append(a.elapsed_time(b))
    slot_bytes = (n1 * cfg.d + cfg.d * cfg.ffn) * 2
    moved = len(re["transfers"]) * slot_bytes
    out = {"scenario": f"{cfg.base} plan ({cfg.base_N}x{cfg.base_c} slots) loses ranks {list(cfg.drop_ranks)} "
                       f"-> {cfg.N}x{cfg.c} slots",
           "host_ms_median": float(np.median(host)), "host_ms_min": float(np.min(host)),
           "copy_ms_median": float(np.median(copy)), "copy_ms_min": float(np.min(copy)),
           "slots_copied": len(re["transfers"]), "remote_copies": int(sum(t[3] for t in re["transfers"])),
           "copy_GBps": 2.0 * moved / (float(np.median(copy)) * 1e-3) / 1e9}
    del old, w1n, w2n
    torch.cuda.empty_cache()
    return out


def training_pass(torch, lz, layer, cfg, logits, x, iters=5):
    """Forward that keeps its intermediates plus the backward chain on the same layer object,
    every call timed by an event pair (median of `iters`); reported beside the headline, not in it."""
    s = layer.shape
    if lz.lz_train_workspace_bytes(s) == 0:
        return None
    layer.enable_training()
    gen = torch.Generator(device=layer.device)
    gen.manual_seed(1000 + cfg.seed)        # upstream gradient: seeded N(0, 1), rounded to bf16
    dy = torch.randn((s.T, s.d), device=layer.device, generator=gen).to(torch.bfloat16)
    n1 = layer.w1.shape[2]
    P, S = s.P, s.S

    def reduce():
        lz.lz_reduce_replica_grads(layer.dw1_slot, layer.slot_expert, S, s.E, layer.dw1_slot[0].numel(), layer.dw1)
        lz.lz_reduce_replica_grads(layer.dw2_slot, layer.slot_expert, S, s.E, layer.dw2_slot[0].numel(), layer.dw2)

    calls = [
        ("forward_train", lambda: layer.forward_train(logits, x)),
        ("combine_backward", lambda: lz.lz_combine_backward(dy, layer.yp, layer.pair_to_row, layer.topk_gates, s,
                                                            layer.dyp, layer.dgates)),
        ("ffn_backward", lambda: lz.lz_ffn_backward(layer.dyp, layer.xp, layer.z, layer.h, layer.slot_offsets,
                                                    layer.w1, layer.w2, s, layer.dxp, layer.dw1_slot,
                                                    layer.dw2_slot, layer.train_ws, layer.train_ws_bytes)),
        ("permute_backward", lambda: lz.lz_permute_backward(layer.dxp, layer.pair_to_row, s, layer.dx)),
        ("route_backward", lambda: lz.lz_route_backward(layer.dgates, layer.topk_gates, layer.topk_ids, s,
                                                        layer.dlogits)),
        ("reduce_replica_grads", reduce),
    ]
    ms = {}
    for name, fn in calls:
        fn()
        torch.cuda.synchronize()
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        for a, b in pairs:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        ms[name] = float(np.median([a.elapsed_time(b) for a, b in pairs]))
    flops_fwd = 2.0 * P * s.d * (n1 + s.ffn)
    backward_ms = sum(v for k, v in ms.items() if k != "forward_train")
    return {
        "ms": ms,
        "backward_ms": backward_ms,
        "forward_plus_backward_ms": ms["forward_train"] + backward_ms,
        "tokens_per_s_forward_plus_backward": s.T / ((ms["forward_train"] + backward_ms) * 1e-3),
        "ffn_backward_TFLOPs": 2 * flops_fwd / (ms["ffn_backward"] * 1e-3) / 1e12,
        "ffn_backward_frac_mfma_peak": 2 * flops_fwd / (ms["ffn_backward"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "forward_train_TFLOPs": flops_fwd / (ms["forward_train"] * 1e-3) / 1e12,
        "combine_backward_GBps": 2.0 * (s.T + 2 * P) * s.d / (ms["combine_backward"] * 1e-3) / 1e9,
        "reduce_replica_grads_GBps": 2.0 * (S + s.E) * (n1 + s.ffn) * s.d / (ms["reduce_replica_grads"] * 1e-3) / 1e9,
        "note": "ffn_backward = two dgrad and two wgrad grouped GEMMs (4 * P * d * (n1 + ffn) flops on real rows) "
                "and the activation backward",
    }


def cpu_baseline(cfg, inp, w, n_tokens):
    """The oracle, as it stands, over the first n_tokens tokens of the batch, in two legs:
    dispatch (route -> histogram -> Algorithm 1 -> row maps; NumPy and Python loops, so it runs on
    one core however many are allowed: timed with the BLAS pool limited to one thread and
    unlimited) and FFN + combine (fp64 matmuls on all BLAS threads).  The plan is computed outside
    both timed spans."""
    from threadpoolctl import threadpool_info, threadpool_limits
    from oracle import moe_layer as om
    from oracle import planner as op
    from workloads import CONFIGS, step_inputs
    n = min(n_tokens, cfg.T)
    logits = inp["logits"][:n]
    x = inp["x"][:n]
    off = np.array([(i * n) // cfg.N for i in range(cfg.N + 1)])

    def eq1_placement(c, loads):
        r = list(c.replica_counts) if c.replica_counts is not None else op.allocate_replicas(loads, c.N, c.c, c.f)
        if c.placement == "spread":
            return np.array(op.place_spread(r, c.N, c.c))
        return np.array(op.place_mro(r, loads, c.N, c.c))

    ids0, _ = om.route(logits, cfg.k)
    if cfg.base is None:
        plan = eq1_placement(cfg, np.bincount(ids0.reshape(-1), minlength=cfg.E))
    else:
        base = CONFIGS[cfg.base]
        idsb, _ = om.route(step_inputs(base, 0, with_x=False)["logits"], base.k)
        loads0 = np.bincount(idsb.reshape(-1), minlength=base.E)
        alive = np.ones(cfg.base_N, dtype=np.uint8)
        alive[list(cfg.drop_ranks)] = 0
        plan = np.array(op.replan(eq1_placement(base, loads0).tolist(), cfg.base_N, cfg.base_c, alive, loads0,
                                  cfg.c, cfg.f)["new_slot_expert"])

    def dispatch():
        t0 = time.perf_counter()
        ids, gates = om.route(logits, cfg.k)
        disp = om.plan_dispatch(ids, off, plan, cfg.E, cfg.N, cfg.c)
        return time.perf_counter() - t0, ids, gates, disp

    with threadpool_limits(limits=1):
        t_disp_1, _, _, _ = dispatch()
    t_disp_all, ids, gates, disp = dispatch()
    t0 = time.perf_counter()
    xp = om.permute(x, disp["row_to_pair"], cfg.k)
    yp = om.expert_ffn_rows(xp, disp["slot_offsets"], plan, w["w1"], w["w2"], cfg.act)
    y = om.unpermute_combine(yp, disp["pair_to_row"], gates)
    t_ffn = time.perf_counter() - t0
    assert np.isfinite(y).all()
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": n / (t_disp_all + t_ffn), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n} of {cfg.T} tokens, whole path in fp64 (numpy), {t_disp_all + t_ffn:.1f} s; "
                      f"plan computed outside the timed spans",
            "dispatch": {"tokens_per_s_1_thread": n / t_disp_1, "tokens_per_s_all_threads": n / t_disp_all,
                         "seconds_1_thread": t_disp_1, "seconds_all_threads": t_disp_all,
                         "note": "route + histogram + Algorithm 1 + row maps; NumPy/Python, effectively one core"},
            "ffn_combine": {"tokens_per_s": n / t_ffn, "seconds": t_ffn, "cores": int(threads),
                            "note": "permute + per-slot fp64 FFN (BLAS) + combine"}}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share only; run with --gpus 1 "
              "(the logical ranks of the plan are emulated in one GPU's memory)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2407_04656_amd as lz
    from workloads import CONFIGS

    cfg = CONFIGS[args.workload]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    # multi-step workloads: fresh logits (a new popularity draw) every step, resident before timing
    n_logits = min(cfg.steps, args.steps + args.warmup) if cfg.steps > 1 else 1
    wl = Workload(torch, lz, cfg, n_logits)
    wl.initial_plan()
    plan_note = wl.plan_note
    rebalance_every = cfg.reshuffle_every if cfg.steps > 1 else 0
    if rebalance_every:
        plan_note = (f"Eq.1 + MRO recomputed from the step's routing at every popularity reshuffle (every "
                     f"{rebalance_every} steps; lz_replan + lz_apply_transfers, untimed); fresh logits each step "
                     f"({n_logits} draws)")
    elif cfg.steps > 1:
        plan_note += f"; fresh logits each step ({n_logits} draws), plan kept"
    shape, layer = wl.shape, wl.layer
    bf16 = wl.bf16

    if args.copy_calib_mib:
        src = torch.empty(args.copy_calib_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    m = measure(wl, args.steps, args.warmup, rebalance_every=rebalance_every, fused_gather=args.fused_gather,
                cold=not args.no_extras)
    # with re-plans between steps the wall clock holds their pauses: the step time is the event-timed mean
    ms_per_step = m["step_ms_by_events"]["mean"] if rebalance_every else m["ms_per_step_wall"]
    per = m["kernels_ms"]
    T, d, ffn, k = shape.T, shape.d, shape.ffn, shape.k
    tf_up = m["ffn_up_TFLOPs"]
    if bf16:
        roofline = {"bound": "mfma", "kernel": "gemm_mfma_kernel (first grouped GEMM, fused activation)",
                    "achieved": tf_up, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": tf_up / PEAK_BF16_TFLOPS, "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name),
                    "flops_per_launch": m["flops_up"], "avg_ms": per["ffn_up"]}
    else:
        roofline = {"bound": "alu", "kernel": "gemm_generic_kernel (fp32 FMA)", "achieved": tf_up,
                    "peak": PEAK_F32_TFLOPS, "unit": "TFLOP/s", "frac": tf_up / PEAK_F32_TFLOPS, "traffic": None,
                    "flops_per_launch": m["flops_up"], "avg_ms": per["ffn_up"]}

    out = {
        "metric": "MoE-layer tokens/s (1 GPU)",
        "value": T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": cfg.name, "T": T, "d": d, "ffn": ffn, "E": shape.E, "k": k,
                   "N": shape.N, "c": shape.c, "act": cfg.act, "plan": plan_note,
                   "reshuffle": "fused into the first GEMM's loads" if args.fused_gather else "permute kernel"},
        "roofline": roofline,
        "kernels_ms": per,
        "kernels_ms_median": m["kernels_ms_median"],
        "kernels_ms_min": m["kernels_ms_min"],
        "step_ms_by_events": m["step_ms_by_events"],
        "derived": {
            "permute_GBps": m["permute_GBps"], "permute_frac_hbm": m["permute_GBps"] / PEAK_HBM_GBS,
            "combine_GBps": m["combine_GBps"], "combine_frac_hbm": m["combine_GBps"] / PEAK_HBM_GBS,
            "permute_GBps_in_step": m.get("permute_GBps_in_step"), "combine_GBps_in_step": m["combine_GBps_in_step"],
            "bandwidth_note": "GB/s on compulsory bytes; *_GBps from 20 back-to-back launches, *_in_step from the event pair inside the timed step",
            "ffn_up_TFLOPs": tf_up, "ffn_down_TFLOPs": m["ffn_down_TFLOPs"], "ffn_TFLOPs": m["ffn_TFLOPs"],
            "ffn_frac_mfma_peak": m["ffn_TFLOPs"] / PEAK_BF16_TFLOPS if bf16 else None,
            "slot_rows_max": m["slot_rows_max"],
            "slot_rows_min": int(layer.slot_counts.min().item()),
            "input_gen_s": wl.gen_s,
        },
    }
    if "rebalance" in m:
        out["rebalance"] = m["rebalance"]
    if "permute_GBps_cold" in m:
        out["derived"]["permute_GBps_cold"] = m["permute_GBps_cold"]
        out["derived"]["combine_GBps_cold"] = m["combine_GBps_cold"]
    if not args.no_extras:
        if bf16 and not args.fused_gather:
            out["fused_gather"] = compare_fused_gather(wl)
        g_ms = graph_replay_ms(wl, 50)
        out["hip_graph_replay"] = {"ms_per_step": g_ms, "tokens_per_s": T / (g_ms * 1e-3),
                                   "note": "the step's launches captured once in a HIP graph and replayed, no event "
                                           "records between the kernels (wall clock over 50 replays); not `value`"}
        if bf16:
            out["training"] = training_pass(torch, lz, layer, cfg, wl.logits_all[0], wl.x)
    host_inp, host_w = wl.inp, wl.w
    del layer, wl
    torch.cuda.empty_cache()
    if not args.no_extras:
        out["achievable"] = achievable_peaks(torch, dev)
        if bf16:
            out["roofline"]["frac_of_vendor_gemm"] = tf_up / out["achievable"]["vendor_bf16_gemm_8192_TFLOPs"]
        out["replan"] = replan_latency(torch, lz, dev)
        if cfg.name == "c2_mixtral":
            host_w_keep = host_w
            out["workloads"] = other_workloads(torch, lz, cfg.name)
            host_w = host_w_keep
    if not args.no_cpu_baseline:
        n_cpu = args.cpu_sample_tokens or {"c1_tiny": 256, "c2_mixtral": 8192, "c3_gptmoe": 16384,
                                           "c4_finegrained": 4096, "c5_postfailure": 16384}.get(cfg.name, 256)
        out["cpu_baseline"] = cpu_baseline(cfg, host_inp, host_w, n_cpu)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
