"""The whole layer pass captured in a HIP graph: the five calls neither allocate nor synchronise
nor record memsets, so a caller may capture them once and replay.  Every replay is checked
bit for bit against the same pass run eagerly on the same inputs, with eager work and
synchronisations between the replays, and the first result against the oracle."""
import numpy as np
import pytest
import torch

import paper_2407_04656_amd as lz
from oracle import moe_layer as om
from workloads import CONFIGS, expert_weights, step_inputs
from workloads.configs import scaled

from gpu_util import DEV, oracle_plan, rel_err, to_dev, to_host, tolerance

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


@pytest.mark.parametrize("name,kw", [
    ("c1_tiny", {}),                                                                   # plain fp32 kernels
    ("c1_tiny", dict(dtype="bf16", act="swiglu", T=1500, d=256, ffn=384, steps=4)),    # MFMA kernels, ragged slots
])
def test_captured_layer_pass_replays_bit_identically(name, kw):
    cfg = scaled(CONFIGS[name], **kw)
    bf16 = cfg.dtype == "bf16"
    shape = lz.Shape.from_config(cfg)
    draws = [step_inputs(cfg, i) for i in range(4)]
    w = expert_weights(cfg, threads=2)
    ids0, _ = om.route(draws[0]["logits"], cfg.k)
    plan = oracle_plan(cfg, ids0)

    layer = lz.MoELayer(shape, DEV)
    layer.set_plan(plan, draws[0]["rank_tok_off"])
    layer.load_expert_weights(w["w1"], w["w2"], plan)
    logits = to_dev(draws[0]["logits"])
    x = to_dev(draws[0]["x"], bf16)

    # eager reference results for every draw (also the warm-up that sets the kernels' attributes)
    eager = []
    for dr in draws:
        logits.copy_(to_dev(dr["logits"]))
        x.copy_(to_dev(dr["x"], bf16))
        layer.forward(logits, x)
        torch.cuda.synchronize()
        assert int(layer.status.item()) == 0
        eager.append((_bits(layer.y).clone(), layer.pair_to_row.clone(), layer.slot_offsets.clone()))
    ref = om.layer_output(draws[0]["x"], *om.route(draws[0]["logits"], cfg.k), w["w1"], w["w2"], cfg.act)
    assert rel_err(to_host(eager[0][0].view(layer.y.dtype)), ref) <= tolerance(cfg)

    graph = torch.cuda.CUDAGraph()
    stream = torch.cuda.Stream()                       # default priority
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=stream):
        layer.forward(logits, x)
    torch.cuda.synchronize()

    scratch = torch.zeros(1 << 20, dtype=torch.float32, device=DEV)
    for rep in range(2):
        for i, dr in enumerate(draws):
            logits.copy_(to_dev(dr["logits"]))
            x.copy_(to_dev(dr["x"], bf16))
            layer.y.zero_()
            layer.pair_to_row.fill_(-1)
            scratch.add_(1.0)                          # the program's own eager work between replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert int(layer.status.item()) == 0
            assert torch.equal(layer.pair_to_row, eager[i][1]), (rep, i)
            assert torch.equal(layer.slot_offsets, eager[i][2]), (rep, i)
            assert torch.equal(_bits(layer.y), eager[i][0]), (rep, i)


def test_captured_noalloc_dispatch():
    """lz_plan_dispatch_noalloc is the entry point meant for capture: route + dispatch in a graph."""
    cfg = scaled(CONFIGS["c1_tiny"], T=3000, E=12, k=3, N=6, c=4, replica_counts=None, placement="mro")
    shape = lz.Shape.from_config(cfg)
    rng = np.random.default_rng(11)
    off = to_dev(np.array([(i * cfg.T) // cfg.N for i in range(cfg.N + 1)], dtype=np.int32))
    plan_h = rng.integers(0, cfg.E, size=cfg.N * cfg.c)
    plan_h[rng.permutation(cfg.N * cfg.c)[:cfg.E]] = np.arange(cfg.E)
    plan = to_dev(plan_h.astype(np.int32))
    logits_h = [rng.standard_normal((cfg.T, cfg.E)).astype(np.float32) for _ in range(3)]
    logits = to_dev(logits_h[0])
    i32 = torch.int32
    ids = torch.empty((cfg.T, cfg.k), dtype=i32, device=DEV)
    gates = torch.empty((cfg.T, cfg.k), dtype=torch.float32, device=DEV)
    out = {k: torch.empty(n, dtype=i32, device=DEV) for k, n in
           (("slot_counts", shape.S), ("slot_offsets", shape.S + 1), ("pair_to_row", shape.P),
            ("row_to_pair", shape.P), ("status", 1))}

    def run():
        lz.lz_route(logits, cfg.T, cfg.E, cfg.k, ids, gates)
        lz.lz_plan_dispatch_noalloc(ids, shape, off, plan, out["slot_counts"], out["slot_offsets"],
                                    out["pair_to_row"], out["row_to_pair"], None, None, out["status"])

    run()                                              # first call on the device: looks the array's address up
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=stream):
        run()
    torch.cuda.synchronize()
    for lh in logits_h + logits_h[:1]:
        logits.copy_(to_dev(lh))
        for t in out.values():
            t.fill_(-3)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ids_ref, _ = om.route(lh, cfg.k)
        ref = om.plan_dispatch(ids_ref, to_host(off), plan_h.astype(np.int32), cfg.E, cfg.N, cfg.c)
        assert int(out["status"].item()) == 0
        for k in ("slot_counts", "slot_offsets", "pair_to_row", "row_to_pair"):
            assert np.array_equal(to_host(out[k]), np.asarray(ref[k])), k
