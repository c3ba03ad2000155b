#!/usr/bin/env python3
"""MoE-layer throughput of the Lazarus hot path on one MI355X.

A step is one pass of the whole path (route -> plan_dispatch -> permute -> expert FFN ->
unpermute_combine) over one batch of synthetic input that is already resident in HBM.
Prints ONE JSON line: whole-path tokens/s plus a roofline record for the dominant kernel
(the first grouped GEMM), timed live with events on the launch stream, and the CPU oracle
timed on a bounded sample of the same workload.
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
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM bytes per launch of the dominant kernel, from the rocprofv3 FETCH_SIZE / WRITE_SIZE passes
# summarised in profiles/<workload>_hbm_traffic.md (counters cannot be read from inside this
# process, so the figure is carried here and re-measured whenever the kernel changes).
MEASURED_TRAFFIC_BYTES = {"c2_mixtral": 14.39e9}


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
                    help="skip the achievable-peak probes, the cold-cache bandwidth runs and the replan timing")
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


def cpu_baseline(cfg, inp, w, plan_fn, n_tokens):
    """The oracle, as it stands, over the first n_tokens tokens of the batch: routing,
    dispatch schedule + row maps, permute, per-slot fp64 FFN, combine."""
    from threadpoolctl import threadpool_info
    from oracle import moe_layer as om
    from oracle import planner as op
    n = min(n_tokens, cfg.T)
    logits = inp["logits"][:n]
    x = inp["x"][:n]
    off = np.array([(i * n) // cfg.N for i in range(cfg.N + 1)])
    t0 = time.perf_counter()
    ids, gates = om.route(logits, cfg.k)
    t_e = np.bincount(ids.reshape(-1), minlength=cfg.E)
    plan = plan_fn(op, t_e)
    disp = om.plan_dispatch(ids, off, plan, cfg.E, cfg.N, cfg.c)
    xp = om.permute(x, disp["row_to_pair"], cfg.k)
    yp = om.expert_ffn_rows(xp, disp["slot_offsets"], plan, w["w1"], w["w2"], cfg.act)
    y = om.unpermute_combine(yp, disp["pair_to_row"], gates)
    dt = time.perf_counter() - t0
    assert np.isfinite(y).all()
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": n / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n} of {cfg.T} tokens, whole path in fp64 (numpy), {dt:.1f} s"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share only; run with --gpus 1 "
              "(the logical ranks of the plan are emulated in one GPU's memory)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2407_04656_amd as lz
    from workloads import CONFIGS, expert_weights, step_inputs

    cfg = CONFIGS[args.workload]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    shape = lz.Shape.from_config(cfg)
    bf16 = cfg.dtype == "bf16"

    t_gen = time.perf_counter()
    inp = step_inputs(cfg, 0)
    w = expert_weights(CONFIGS[cfg.base] if cfg.base else cfg, threads=16)
    # multi-step workloads: fresh logits (a new popularity draw) every step, resident before timing
    n_logits = min(cfg.steps, args.steps + args.warmup) if cfg.steps > 1 else 1
    logits_host = [inp["logits"]] + [step_inputs(cfg, i, with_x=False)["logits"] for i in range(1, n_logits)]
    t_gen = time.perf_counter() - t_gen

    def to_dev(a, as_bf16=False):
        t = torch.from_numpy(np.ascontiguousarray(a))
        if as_bf16:
            t = t.view(torch.bfloat16)
        return t.to(dev)

    logits_all = [to_dev(l) for l in logits_host]
    logits = logits_all[0]
    x = to_dev(inp["x"], bf16)
    layer = lz.MoELayer(shape, dev)

    def lib_plan(c, t_e):
        if c.replica_counts is not None:
            r = np.array(c.replica_counts, dtype=np.int32)
        else:
            r = lz.lz_allocate_replicas(t_e, c.N, c.c, c.f)
        if c.placement == "spread":
            return lz.lz_place_spread(r, c.N, c.c)
        return lz.lz_place_mro(r, t_e, c.N, c.c)

    def routed_loads(c, logit_array):
        probe = lz.MoELayer(lz.Shape.from_config(c), dev) if c is not cfg else layer
        probe.set_plan(np.zeros(c.N * c.c, dtype=np.int32), rank_offsets(c))
        probe.route(to_dev(logit_array))
        torch.cuda.synchronize()
        return np.bincount(probe.topk_ids.cpu().numpy().reshape(-1), minlength=c.E)

    def rank_offsets(c):
        return np.array([(i * c.T) // c.N for i in range(c.N + 1)], dtype=np.int32)

    if cfg.base is None:
        # plan from the realised step-0 routing (the paper's routing history): Eq. 1 + MRO, or
        # the fixed allocation + spread placement of the tiny config -- all in the library
        plan = lib_plan(cfg, routed_loads(cfg, inp["logits"]))
        plan_note = "Eq.1 + MRO on step-0 loads" if cfg.replica_counts is None else "fixed counts, spread"
    else:
        # post-failure workload: the base config's step-0 plan loses ranks, lz_replan gives the new one
        base = CONFIGS[cfg.base]
        t_e = routed_loads(base, step_inputs(base, 0, with_x=False)["logits"])
        alive = np.ones(cfg.base_N, dtype=np.uint8)
        alive[list(cfg.drop_ranks)] = 0
        plan = lz.lz_replan(lib_plan(base, t_e), cfg.base_N, cfg.base_c, alive, t_e, cfg.c, cfg.f)["new_slot_expert"]
        plan_note = f"lz_replan of {cfg.base}'s plan after losing ranks {list(cfg.drop_ranks)}"
    if cfg.steps > 1:
        plan_note += f"; fresh logits each step ({n_logits} draws), plan kept"
    torch.cuda.empty_cache()
    layer.set_plan(plan, inp["rank_tok_off"])
    layer.load_expert_weights(w["w1"], w["w2"], plan)
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    ev = lambda: torch.cuda.Event(enable_timing=True)
    names = ["route", "plan", "permute", "ffn_up", "ffn_down", "combine"]

    def step(marks=None, logits=logits):
        s = layer
        if marks is not None:
            marks[0].record(stream)
        s.route(logits)
        if marks is not None:
            marks[1].record(stream)
        s.plan_dispatch()
        lz.lz_ffn_tiles(s.slot_offsets, shape, s.ffn_ws, s.ffn_ws_bytes)   # row-tile table: dispatch bookkeeping
        if marks is not None:
            marks[2].record(stream)
        s.permute(x)
        if marks is not None:
            marks[3].record(stream)
        lz.lz_ffn_up(s.xp, s.w1, shape, s.ffn_ws, s.ffn_ws_bytes)
        if marks is not None:
            marks[4].record(stream)
        lz.lz_ffn_down(s.w2, shape, s.yp, s.ffn_ws, s.ffn_ws_bytes)
        if marks is not None:
            marks[5].record(stream)
        s.unpermute_combine()
        if marks is not None:
            marks[6].record(stream)

    if args.copy_calib_mib:
        src = torch.empty(args.copy_calib_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(logits=logits_all[i % n_logits])
    torch.cuda.synchronize()
    assert int(layer.status.item()) == 0, "plan_dispatch flagged the plan"

    marks = [[ev() for _ in range(7)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(marks[i], logits_all[(args.warmup + i) % n_logits])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # the two bandwidth kernels once more, back to back, so that launch gaps and event overhead
    # (several microseconds against ~40) do not dilute their GB/s
    def burst(fn, n=20):
        a, b = ev(), ev()
        fn()
        a.record(stream)
        for _ in range(n):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    burst_ms = {"permute": burst(lambda: layer.permute(x)), "combine": burst(layer.unpermute_combine)}

    # ... and cold: a 1 GiB fill between launches pushes x / yp out of L2 and the 256 MB memory-side cache
    def cold(fn, n=8):
        scratch = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        a, b = ev(), ev()
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

    cold_ms = None
    if not args.no_extras:
        cold_ms = {"permute": cold(lambda: layer.permute(x)), "combine": cold(layer.unpermute_combine)}

    ms_per_step = wall * 1e3 / args.steps
    samples = {n: np.array([m[i].elapsed_time(m[i + 1]) for m in marks]) for i, n in enumerate(names)}
    per = {n: float(np.mean(v)) for n, v in samples.items()}
    step_ms = np.array([m[0].elapsed_time(m[6]) for m in marks])
    eb = 4 if cfg.dtype == "f32" else 2
    P, T, d, ffn, k = shape.P, shape.T, shape.d, shape.ffn, shape.k
    mult = 2 if cfg.act == "swiglu" else 1
    flops_up = 2.0 * P * d * ffn * mult           # real rows only, no padding credit
    flops_down = 2.0 * P * ffn * d
    permute_bytes = (1 + k) * T * d * eb + 4 * P   # compulsory: read x once, write xp, read the map
    combine_bytes = (1 + k) * T * d * eb + 8 * P
    tf_up = flops_up / (per["ffn_up"] * 1e-3) / 1e12
    tf_down = flops_down / (per["ffn_down"] * 1e-3) / 1e12
    tf_ffn = (flops_up + flops_down) / ((per["ffn_up"] + per["ffn_down"]) * 1e-3) / 1e12
    gb_perm = permute_bytes / (burst_ms["permute"] * 1e-3) / 1e9
    gb_comb = combine_bytes / (burst_ms["combine"] * 1e-3) / 1e9
    gb_perm_step = permute_bytes / (per["permute"] * 1e-3) / 1e9
    gb_comb_step = combine_bytes / (per["combine"] * 1e-3) / 1e9

    if cfg.dtype == "bf16":
        roofline = {"bound": "mfma", "kernel": "gemm_mfma_kernel (first grouped GEMM, fused activation)",
                    "achieved": tf_up, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": tf_up / PEAK_BF16_TFLOPS, "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name),
                    "flops_per_launch": flops_up, "avg_ms": per["ffn_up"]}
    else:
        roofline = {"bound": "alu", "kernel": "gemm_generic_kernel (fp32 FMA)", "achieved": tf_up,
                    "peak": 157.3, "unit": "TFLOP/s", "frac": tf_up / 157.3, "traffic": None,
                    "flops_per_launch": flops_up, "avg_ms": per["ffn_up"]}

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
                   "N": shape.N, "c": shape.c, "act": cfg.act,
                   "plan": plan_note},
        "roofline": roofline,
        "kernels_ms": per,
        "kernels_ms_median": {n: float(np.median(v)) for n, v in samples.items()},
        "kernels_ms_min": {n: float(np.min(v)) for n, v in samples.items()},
        "step_ms_by_events": {"median": float(np.median(step_ms)), "min": float(np.min(step_ms))},
        "derived": {
            "permute_GBps": gb_perm, "permute_frac_hbm": gb_perm / PEAK_HBM_GBS,
            "combine_GBps": gb_comb, "combine_frac_hbm": gb_comb / PEAK_HBM_GBS,
            "permute_GBps_in_step": gb_perm_step, "combine_GBps_in_step": gb_comb_step,
            "bandwidth_note": "GB/s on compulsory bytes; *_GBps from 20 back-to-back launches, *_in_step from the event pair inside the timed step",
            "ffn_up_TFLOPs": tf_up, "ffn_down_TFLOPs": tf_down, "ffn_TFLOPs": tf_ffn,
            "ffn_frac_mfma_peak": tf_ffn / PEAK_BF16_TFLOPS if bf16 else None,
            "slot_rows_max": int(layer.slot_counts.max().item()),
            "slot_rows_min": int(layer.slot_counts.min().item()),
            "input_gen_s": t_gen,
        },
    }
    if cold_ms is not None:
        out["derived"]["permute_GBps_cold"] = permute_bytes / (cold_ms["permute"] * 1e-3) / 1e9
        out["derived"]["combine_GBps_cold"] = combine_bytes / (cold_ms["combine"] * 1e-3) / 1e9
    if not args.no_extras:
        if bf16:
            out["training"] = training_pass(torch, lz, layer, cfg, logits, x)
        del layer, x
        torch.cuda.empty_cache()
        out["achievable"] = achievable_peaks(torch, dev)
        if bf16:
            out["roofline"]["frac_of_vendor_gemm"] = tf_up / out["achievable"]["vendor_bf16_gemm_8192_TFLOPs"]
        out["replan"] = replan_latency(torch, lz, dev)
    if not args.no_cpu_baseline:
        n_cpu = args.cpu_sample_tokens or {"c1_tiny": 256, "c2_mixtral": 8192, "c3_gptmoe": 16384,
                                           "c4_finegrained": 4096, "c5_postfailure": 16384}.get(cfg.name, 256)

        def oracle_plan(op, t_e):
            def eq1_placement(c, loads):
                r = list(c.replica_counts) if c.replica_counts is not None else op.allocate_replicas(loads, c.N, c.c, c.f)
                if c.placement == "spread":
                    return np.array(op.place_spread(r, c.N, c.c))
                return np.array(op.place_mro(r, loads, c.N, c.c))
            if cfg.base is None:
                return eq1_placement(cfg, t_e)
            from oracle import moe_layer as om
            base = CONFIGS[cfg.base]
            ids0, _ = om.route(step_inputs(base, 0, with_x=False)["logits"], base.k)
            loads0 = np.bincount(ids0.reshape(-1), minlength=base.E)
            alive = np.ones(cfg.base_N, dtype=np.uint8)
            alive[list(cfg.drop_ranks)] = 0
            return np.array(op.replan(eq1_placement(base, loads0).tolist(), cfg.base_N, cfg.base_c, alive, loads0,
                                      cfg.c, cfg.f)["new_slot_expert"])

        out["cpu_baseline"] = cpu_baseline(cfg, inp, w, oracle_plan, n_cpu)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
