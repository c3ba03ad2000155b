"""Pins for the expert FFN / combine oracle (Sec. 2.1) and the bf16 widening."""
import math

import numpy as np
import pytest

from oracle import moe_layer as om
from oracle import planner as op
from workloads import CONFIGS, expert_weights, f32_to_bf16_bits, step_inputs
from workloads.configs import scaled


def test_widen_known_bf16_patterns():
    bits = np.array([0x3F80, 0xC000, 0x0000, 0x8000, 0x3DCD, 0x7F7F], dtype=np.uint16)
    vals = om.widen(bits)
    assert vals[0] == 1.0 and vals[1] == -2.0 and vals[2] == 0.0
    assert vals[3] == 0.0 and math.copysign(1, vals[3]) == -1
    assert vals[4] == (0x4D / 128 + 1) * 2.0 ** (0x7B - 127)   # 0x3DCD: exponent 0x7B, mantissa 0x4D
    assert vals[5] == (2 - 2.0 ** -7) * 2.0 ** 127            # largest finite bf16


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is exactly half-way between bf16 neighbours 1.0 and 1+2^-7: ties to even -> 1.0
    a = np.array([1 + 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20, 1 + 3 * 2.0 ** -8], dtype=np.float32)
    b = f32_to_bf16_bits(a)
    assert list(b) == [0x3F80, 0x3F81, 0x3F82]


def _ffn_python(x, w1, w2, act):
    n1, d = len(w1), len(x)
    pre = [sum(w1[r][q] * x[q] for q in range(d)) for r in range(n1)]
    if act == "gelu":
        h = [0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in pre]
    else:
        f = n1 // 2
        h = [(pre[r] / (1.0 + math.exp(-pre[r]))) * pre[f + r] for r in range(f)]
    return [sum(w2[o][r] * h[r] for r in range(len(h))) for o in range(len(w2))]


@pytest.mark.parametrize("act", ["gelu", "swiglu"])
def test_ffn_matches_scalar_loops(act):
    rng = np.random.default_rng(5)
    d, f, n = 5, 4, 3
    n1 = f * (2 if act == "swiglu" else 1)
    X = rng.standard_normal((n, d))
    w1 = rng.standard_normal((n1, d))
    w2 = rng.standard_normal((d, f))
    Y = om.ffn(X, w1, w2, act)
    for r in range(n):
        ref = _ffn_python(X[r].tolist(), w1.tolist(), w2.tolist(), act)
        assert np.allclose(Y[r], ref, rtol=1e-13, atol=1e-14)


def test_gelu_silu_known_values():
    assert om.gelu(np.array([0.0]))[0] == 0.0
    assert om.gelu(np.array([1.0]))[0] == pytest.approx(0.8413447460685429, rel=1e-14)   # Phi(1)
    assert om.gelu(np.array([-1.0]))[0] == pytest.approx(-0.15865525393145707, rel=1e-13)
    assert om.silu(np.array([0.0]))[0] == 0.0
    assert om.silu(np.array([math.log(3.0)]))[0] == pytest.approx(math.log(3.0) * 0.75, rel=1e-14)
    big = om.gelu(np.array([10.0, -10.0]))
    assert big[0] == pytest.approx(10.0, rel=1e-12) and abs(big[1]) < 1e-20


def _tiny_layer(cfg, plan):
    inp = step_inputs(cfg)
    w = expert_weights(cfg, threads=2)
    ids, gates = om.route(inp["logits"], cfg.k)
    disp = om.plan_dispatch(ids, inp["rank_tok_off"], np.array(plan), cfg.E, cfg.N, cfg.c)
    return inp, w, ids, gates, disp


def test_identity_experts_return_gate_sum_times_input():
    """Skipping the FFN (yp := xp) the combine must give x[t] * sum of gates = x[t]; with
    all-ones gates k * x[t]."""
    cfg = CONFIGS["c1_tiny"]
    plan = op.place_spread(cfg.replica_counts, cfg.N, cfg.c)
    inp, _, ids, gates, disp = _tiny_layer(cfg, plan)
    xp = om.permute(inp["x"], disp["row_to_pair"], cfg.k)
    y = om.unpermute_combine(xp, disp["pair_to_row"], gates)
    assert np.allclose(y, inp["x"].astype(np.float64), rtol=1e-14, atol=1e-15)
    y1 = om.unpermute_combine(xp, disp["pair_to_row"], np.ones_like(gates))
    assert np.array_equal(y1, cfg.k * inp["x"].astype(np.float64))


@pytest.mark.parametrize("act,dtype", [("gelu", "f32"), ("swiglu", "bf16")])
def test_dispatch_path_equals_plain_definition_for_any_plan(act, dtype):
    """permute -> per-slot FFN -> combine equals sum_k gate * FFN_expert(x) whatever the
    placement (replicas of an expert carry the same weights)."""
    cfg = scaled(CONFIGS["c1_tiny"], act=act, dtype=dtype, T=96, d=32, ffn=48)
    inp = step_inputs(cfg)
    w = expert_weights(cfg, threads=2)
    ids, gates = om.route(inp["logits"], cfg.k)
    y_def = om.layer_output(inp["x"], ids, gates, w["w1"], w["w2"], act)
    t_e = np.bincount(ids.reshape(-1), minlength=cfg.E)
    plans = [op.place_spread(cfg.replica_counts, cfg.N, cfg.c),
             op.place_mro(op.allocate_replicas(t_e, cfg.N, cfg.c, 1), t_e, cfg.N, cfg.c),
             op.place_mro(op.allocate_replicas(t_e, 2, 8, 2), t_e, 2, 8)]
    shapes = [(cfg.N, cfg.c), (cfg.N, cfg.c), (2, 8)]
    for plan, (N, c) in zip(plans, shapes):
        off = np.array([(i * cfg.T) // N for i in range(N + 1)])
        disp = om.plan_dispatch(ids, off, np.array(plan), cfg.E, N, c)
        xp = om.permute(inp["x"], disp["row_to_pair"], cfg.k)
        yp = om.expert_ffn_rows(xp, disp["slot_offsets"], plan, w["w1"], w["w2"], act)
        y = om.unpermute_combine(yp, disp["pair_to_row"], gates)
        assert np.allclose(y, y_def, rtol=1e-12, atol=1e-15)
    sub = np.array([5, 0, 77])
    y_sub = om.layer_output(inp["x"], ids, gates, w["w1"], w["w2"], act, tokens=sub)
    assert np.allclose(y_sub, y_def[sub], rtol=1e-12, atol=1e-15)


def test_layer_output_single_expert_is_dense_matmul():
    """E = 1, k = 1: the gate is 1 and the layer is one dense FFN (library matmul)."""
    rng = np.random.default_rng(6)
    x = rng.standard_normal((7, 6)).astype(np.float32)
    w1 = rng.standard_normal((1, 10, 6)).astype(np.float32)
    w2 = rng.standard_normal((1, 6, 10)).astype(np.float32)
    ids, gates = om.route(np.zeros((7, 1), dtype=np.float32), 1)
    y = om.layer_output(x, ids, gates, w1, w2, "gelu")
    pre = x.astype(np.float64) @ w1[0].astype(np.float64).T
    ref = om.gelu(pre) @ w2[0].astype(np.float64).T
    assert np.allclose(y, ref, rtol=1e-14, atol=0)
