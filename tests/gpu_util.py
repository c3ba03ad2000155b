"""Helpers for the GPU parity tests: host<->device marshalling and one full layer pass."""
import numpy as np
import torch

import paper_2407_04656_amd as lz
from oracle import moe_layer as om
from oracle import planner as op
from workloads import expert_weights, step_inputs

DEV = "cuda:0"


def to_dev(a, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if bf16:
        t = t.view(torch.bfloat16)
    return t.to(DEV)


def slot_weights(w, slot_expert, bf16):
    """Device copies of every slot's expert weights in the library's input-major layout:
    w1 [S, d, n1], w2 [S, ffn, d] (the host arrays are [out, in])."""
    w1 = np.ascontiguousarray(np.asarray(w["w1"])[slot_expert].transpose(0, 2, 1))
    w2 = np.ascontiguousarray(np.asarray(w["w2"])[slot_expert].transpose(0, 2, 1))
    return to_dev(w1, bf16), to_dev(w2, bf16)


def to_host(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.uint16).cpu().numpy()
    return t.cpu().numpy()


def rel_err(got, ref):
    """max |got - ref| / max |ref| (global normalisation; element-wise relative error is
    undefined near zeros)."""
    got = om.widen(got)
    return float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))


def tolerance(cfg):
    return 1e-5 if cfg.dtype == "f32" else 2e-2


def oracle_plan(cfg, ids):
    """The plan the config prescribes, computed by the oracle from the given routing."""
    if cfg.replica_counts is not None:
        r = list(cfg.replica_counts)
    else:
        t_e = np.bincount(ids.reshape(-1), minlength=cfg.E)
        r = op.allocate_replicas(t_e, cfg.N, cfg.c, cfg.f)
    t_e = np.bincount(ids.reshape(-1), minlength=cfg.E)
    if cfg.placement == "spread":
        return np.array(op.place_spread(r, cfg.N, cfg.c), dtype=np.int32)
    return np.array(op.place_mro(r, t_e, cfg.N, cfg.c), dtype=np.int32)


def run_layer(cfg, plan, inp, w, layer=None):
    """One pass of the five library calls.  Returns the layer object and host copies."""
    shape = lz.Shape.from_config(cfg)
    bf16 = cfg.dtype == "bf16"
    if layer is None:
        layer = lz.MoELayer(shape, DEV)
        layer.load_expert_weights(w["w1"], w["w2"], plan)
    layer.set_plan(plan, inp["rank_tok_off"])
    logits = to_dev(inp["logits"])
    x = to_dev(inp["x"], bf16)
    layer.forward(logits, x)
    torch.cuda.synchronize()
    return layer


def check_dispatch_exact(cfg, layer, ids_ref, ref):
    assert np.array_equal(to_host(layer.topk_ids), ids_ref)
    assert int(layer.status.item()) == 0
    assert np.array_equal(to_host(layer.Tej), ref["Tej"])
    assert np.array_equal(to_host(layer.D), ref["D"])
    assert np.array_equal(to_host(layer.slot_counts), ref["slot_counts"])
    assert np.array_equal(to_host(layer.slot_offsets), ref["slot_offsets"])
    assert np.array_equal(to_host(layer.pair_to_row), ref["pair_to_row"])
    assert np.array_equal(to_host(layer.row_to_pair), ref["row_to_pair"])
