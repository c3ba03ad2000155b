"""GPU parity of the training entry points (forward that keeps its intermediates, backward
chain) against the fp64 backward oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2407_04656_amd as lz
from oracle import moe_backward as ob
from oracle import moe_layer as om
from workloads import CONFIGS, expert_weights, f32_to_bf16_bits, step_inputs
from workloads.configs import scaled

from gpu_util import DEV, oracle_plan, rel_err, slot_weights, to_dev, to_host

pytestmark = pytest.mark.gpu

TOL = 2e-2   # bf16 tensors, fp32 accumulation: max |err| / max |ref|


def _bf16(rng, shape, scale=1.0):
    return f32_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))


def _ffn_backward_case(cfg, counts, seed):
    S, P = cfg.N * cfg.c, cfg.T * cfg.k
    assert len(counts) == S and sum(counts) == P
    offsets = np.zeros(S + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    rng = np.random.default_rng(seed)
    slot_expert = rng.integers(0, cfg.E, size=S).astype(np.int32)
    w = expert_weights(cfg, threads=4)
    n1 = w["w1"].shape[1]
    xph = _bf16(rng, (P, cfg.d))
    dyph = _bf16(rng, (P, cfg.d), 0.5)
    shape = lz.Shape.from_config(cfg)
    bf = torch.bfloat16
    w1, w2 = slot_weights(w, slot_expert, True)
    nbytes = lz.lz_train_workspace_bytes(shape)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    xp, dyp, off = to_dev(xph, True), to_dev(dyph, True), to_dev(offsets)
    z = torch.zeros((P, n1), dtype=bf, device=DEV)
    h = torch.zeros((P, cfg.ffn), dtype=bf, device=DEV)
    yp = torch.zeros((P, cfg.d), dtype=bf, device=DEV)
    lz.lz_ffn_forward_train(xp, off, w1, w2, shape, z, h, yp, ws, nbytes)
    dxp = torch.zeros((P, cfg.d), dtype=bf, device=DEV)
    dw1 = torch.full((S, cfg.d, n1), 7.0, dtype=bf, device=DEV)       # gradients in the weights' layout
    dw2 = torch.full((S, cfg.ffn, cfg.d), 7.0, dtype=bf, device=DEV)
    lz.lz_ffn_backward(dyp, xp, z, h, off, w1, w2, shape, dxp, dw1, dw2, ws, nbytes)
    torch.cuda.synchronize()

    # forward intermediates
    Xp = om.widen(xph)
    Zref = np.zeros((P, n1))
    for s in range(S):
        a, b = offsets[s], offsets[s + 1]
        Zref[a:b] = Xp[a:b] @ om.widen(w["w1"][slot_expert[s]]).T
    assert rel_err(to_host(z), Zref) <= TOL
    assert rel_err(to_host(h), ob.act_forward(Zref, cfg.act)) <= TOL
    assert rel_err(to_host(yp), om.expert_ffn_rows(xph, offsets, slot_expert, w["w1"], w["w2"], cfg.act)) <= TOL
    # backward
    dxp_ref, dw1_ref, dw2_ref = ob.ffn_backward_rows(dyph, xph, offsets, slot_expert, w["w1"], w["w2"], cfg.act)
    dw1_ref, dw2_ref = dw1_ref.transpose(0, 2, 1), dw2_ref.transpose(0, 2, 1)   # oracle: [out, in]
    assert rel_err(to_host(dxp), dxp_ref) <= TOL
    assert rel_err(to_host(dw1), dw1_ref) <= TOL
    assert rel_err(to_host(dw2), dw2_ref) <= TOL
    # slot by slot as well: a small slot's gradient must not hide behind a large one's scale
    g1, g2 = om.widen(to_host(dw1)), om.widen(to_host(dw2))
    for s in range(S):
        if counts[s] == 0:
            assert not g1[s].any() and not g2[s].any()
        else:
            assert np.max(np.abs(g1[s] - dw1_ref[s])) <= TOL * np.max(np.abs(dw1_ref[s]))
            assert np.max(np.abs(g2[s] - dw2_ref[s])) <= TOL * np.max(np.abs(dw2_ref[s]))


def _round_bf16(a):
    return om.widen(f32_to_bf16_bits(np.asarray(a, dtype=np.float32)))


@pytest.mark.parametrize("act", ["gelu", "swiglu"])
def test_ffn_backward_against_the_oracle_rounded_where_the_device_rounds(act):
    """Tighter than the 2e-2 bar: the oracle's steps with every stored intermediate (z, h, dH, dZ)
    rounded to bf16 where the device stores it.  What is left is fp32-versus-fp64 accumulation and
    the fast activation forms, so every output element must be within two bf16 steps of its
    reference value plus 2^-9 of the tensor's rms (sums that cancel inherit the absolute rounding
    error of their terms)."""
    cfg = scaled(CONFIGS["c1_tiny"], act=act, dtype="bf16", T=320, k=2, d=256, ffn=256, N=2, c=2)
    counts = [300, 0, 339, 1]
    S, P = 4, cfg.T * cfg.k
    offsets = np.zeros(S + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    rng = np.random.default_rng(31)
    slot_expert = np.array([2, 0, 5, 7], dtype=np.int32)
    w = expert_weights(cfg, threads=2)
    n1 = w["w1"].shape[1]
    xph, dyph = _bf16(rng, (P, cfg.d)), _bf16(rng, (P, cfg.d), 0.5)
    shape = lz.Shape.from_config(cfg)
    bf = torch.bfloat16
    w1, w2 = slot_weights(w, slot_expert, True)
    nbytes = lz.lz_train_workspace_bytes(shape)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    xp, dyp, off = to_dev(xph, True), to_dev(dyph, True), to_dev(offsets)
    z = torch.zeros((P, n1), dtype=bf, device=DEV)
    h = torch.zeros((P, cfg.ffn), dtype=bf, device=DEV)
    yp = torch.zeros((P, cfg.d), dtype=bf, device=DEV)
    dxp = torch.zeros((P, cfg.d), dtype=bf, device=DEV)
    dw1 = torch.zeros((S, cfg.d, n1), dtype=bf, device=DEV)
    dw2 = torch.zeros((S, cfg.ffn, cfg.d), dtype=bf, device=DEV)
    lz.lz_ffn_forward_train(xp, off, w1, w2, shape, z, h, yp, ws, nbytes)
    lz.lz_ffn_backward(dyp, xp, z, h, off, w1, w2, shape, dxp, dw1, dw2, ws, nbytes)
    torch.cuda.synchronize()

    def close(got, ref, what):
        got = om.widen(got)
        bound = 2.0 ** -7 * np.abs(ref) + 2.0 ** -9 * np.sqrt(np.mean(ref * ref))
        bad = np.abs(got - ref) > bound
        assert not bad.any(), (what, int(bad.sum()), float(np.max(np.abs(got - ref) / bound)))

    Xp, dYp = om.widen(xph), om.widen(dyph)
    for s in range(S):
        a, b = offsets[s], offsets[s + 1]
        if b == a:
            continue
        W1, W2 = om.widen(w["w1"][slot_expert[s]]), om.widen(w["w2"][slot_expert[s]])
        Z = _round_bf16(Xp[a:b] @ W1.T)
        H = _round_bf16(ob.act_forward(Z, act))
        close(to_host(z[a:b]), Z, "z")
        close(to_host(h[a:b]), H, "h")
        close(to_host(yp[a:b]), H @ W2.T, "yp")
        dH = _round_bf16(dYp[a:b] @ W2)
        dZ = _round_bf16(ob.act_backward(dH, Z, act))
        close(to_host(dxp[a:b]), dZ @ W1, "dxp")
        close(to_host(dw2[s]), (dYp[a:b].T @ H).T, "dw2")       # device layout [ffn, d]
        close(to_host(dw1[s]), (dZ.T @ Xp[a:b]).T, "dw1")       # device layout [d, n1]


@pytest.mark.parametrize("act,d,ffn", [("gelu", 256, 256), ("swiglu", 256, 192), ("gelu", 512, 320),
                                       ("swiglu", 512, 384)])
def test_ffn_forward_train_and_backward_ragged(act, d, ffn):
    cfg = scaled(CONFIGS["c1_tiny"], act=act, dtype="bf16", T=700, k=2, d=d, ffn=ffn, N=4, c=2)
    # several row tiles, a tile boundary + 1, an empty slot, one-row slots, ragged tails: the weight
    # gradients contract over 257, 0, 1, 512, 300, 255, 74 and 1 rows (whole and partial K steps)
    _ffn_backward_case(cfg, [257, 0, 1, 512, 300, 255, 74, 1], 3)


def test_weight_gradients_over_every_k_step_count_of_the_unrolled_loop():
    """The K loop is unrolled six times with a remainder chain, and three weight stages are in flight
    when it ends: slots of 1 ... 13 K steps (whole and partial) reach every exit of that chain in
    the weight-gradient kernels, whose contraction length is the slot's row count."""
    counts = [64, 100, 192, 250, 300, 384, 420, 500, 576, 630, 690, 768, 800]
    assert [(c + 63) // 64 for c in counts] == list(range(1, 14))
    cfg = scaled(CONFIGS["c1_tiny"], act="swiglu", dtype="bf16", T=sum(counts) // 2, k=2, d=256, ffn=128, N=13, c=1)
    _ffn_backward_case(cfg, counts, 17)


def test_ffn_backward_many_slots_mostly_empty():
    cfg = scaled(CONFIGS["c1_tiny"], act="swiglu", dtype="bf16", T=600, k=2, d=256, ffn=128, N=4, c=5)
    counts = [0] * 20
    counts[3], counts[4], counts[11], counts[19] = 700, 64, 435, 1
    _ffn_backward_case(cfg, counts, 9)


def test_streaming_backward_kernels():
    cfg = scaled(CONFIGS["c4_finegrained"], T=777, d=264, ffn=128, E=16, k=3, N=4, c=6)
    inp = step_inputs(cfg)
    ids, gates = om.route(inp["logits"], cfg.k)
    plan = oracle_plan(cfg, ids)
    disp = om.plan_dispatch(ids, inp["rank_tok_off"], plan, cfg.E, cfg.N, cfg.c)
    rng = np.random.default_rng(4)
    P = cfg.T * cfg.k
    shape = lz.Shape.from_config(cfg)
    dy, ypb = _bf16(rng, (cfg.T, cfg.d)), _bf16(rng, (P, cfg.d))
    p2r = to_dev(disp["pair_to_row"])
    g32 = to_dev(gates.astype(np.float32))
    dyp = torch.zeros((P, cfg.d), dtype=torch.bfloat16, device=DEV)
    dgates = torch.zeros((cfg.T, cfg.k), dtype=torch.float32, device=DEV)
    lz.lz_combine_backward(to_dev(dy, True), to_dev(ypb, True), p2r, g32, shape, dyp, dgates)
    dyp_ref, dg_ref = ob.combine_backward(dy, ypb, disp["pair_to_row"], gates.astype(np.float32))
    got = om.widen(to_host(dyp))
    assert np.all(np.abs(got - dyp_ref) <= 0.006 * np.abs(dyp_ref))         # one bf16 rounding (2^-8) and fp32 noise
    assert np.allclose(to_host(dgates), dg_ref, rtol=1e-5, atol=1e-4)        # fp32 dot of d products
    # dx = sum of the pair rows: the combine with unit gates, bit for bit
    dx = torch.zeros((cfg.T, cfg.d), dtype=torch.bfloat16, device=DEV)
    y1 = torch.zeros_like(dx)
    lz.lz_permute_backward(dyp, p2r, shape, dx)
    lz.lz_unpermute_combine(dyp, p2r, torch.ones_like(g32), shape, y1)
    assert torch.equal(dx.view(torch.int16), y1.view(torch.int16))
    dx_ref = ob.permute_backward(to_host(dyp), disp["pair_to_row"], cfg.k)
    assert np.all(np.abs(om.widen(to_host(dx)) - dx_ref) <= 0.006 * np.abs(dx_ref) + 1e-6)
    # gate backward
    dlogits = torch.full((cfg.T, cfg.E), 3.0, dtype=torch.float32, device=DEV)
    lz.lz_route_backward(dgates, g32, to_dev(ids), shape, dlogits)
    dl_ref = ob.route_backward(to_host(dgates), gates.astype(np.float32), ids, cfg.E)
    assert np.allclose(to_host(dlogits), dl_ref, rtol=1e-5, atol=1e-5 * np.max(np.abs(dl_ref)))
    # replica sums
    S, n = cfg.N * cfg.c, 1000 * 8
    dws = _bf16(rng, (S, n))
    dw = torch.full((cfg.E, n), 5.0, dtype=torch.bfloat16, device=DEV)
    lz.lz_reduce_replica_grads(to_dev(dws, True), to_dev(plan), S, cfg.E, n, dw)
    ref = ob.reduce_replica_grads(om.widen(dws), plan, cfg.E)
    assert np.all(np.abs(om.widen(to_host(dw)) - ref) <= 0.006 * np.abs(ref) + 1e-6)


@pytest.mark.parametrize("act", ["gelu", "swiglu"])
def test_layer_backward_end_to_end(act):
    cfg = scaled(CONFIGS["c4_finegrained"], act=act, T=900, d=256, ffn=128, E=16, k=3, N=4, c=6)
    inp = step_inputs(cfg)
    w = expert_weights(cfg, threads=4)
    ids, gates = om.route(inp["logits"], cfg.k)
    plan = oracle_plan(cfg, ids)
    disp = om.plan_dispatch(ids, inp["rank_tok_off"], plan, cfg.E, cfg.N, cfg.c)
    shape = lz.Shape.from_config(cfg)
    layer = lz.MoELayer(shape, DEV)
    layer.load_expert_weights(w["w1"], w["w2"], plan)
    layer.set_plan(plan, inp["rank_tok_off"])
    layer.enable_training()
    rng = np.random.default_rng(12)
    dy = _bf16(rng, (cfg.T, cfg.d))
    y = layer.forward_train(to_dev(inp["logits"]), to_dev(inp["x"], True))
    layer.backward(to_dev(dy, True))
    torch.cuda.synchronize()
    assert np.array_equal(to_host(layer.pair_to_row), disp["pair_to_row"])
    assert rel_err(to_host(y), om.layer_output(inp["x"], ids, gates, w["w1"], w["w2"], act)) <= TOL
    ref = ob.layer_backward(dy, inp["x"], ids, gates, disp["pair_to_row"], disp["row_to_pair"],
                            disp["slot_offsets"], plan, w["w1"], w["w2"], act)
    assert rel_err(to_host(layer.dx), ref["dx"]) <= TOL
    assert rel_err(to_host(layer.dgates), ref["dgates"]) <= TOL
    assert rel_err(to_host(layer.dw1), ref["dw1"].transpose(0, 2, 1)) <= TOL     # oracle: [out, in]
    assert rel_err(to_host(layer.dw2), ref["dw2"].transpose(0, 2, 1)) <= TOL
    dl_ref = ob.route_backward(ref["dgates"], gates, ids, cfg.E)
    assert rel_err(to_host(layer.dlogits), dl_ref) <= TOL
    # a second pass on the same buffers gives the same bits (queues and scratch are reset)
    first = [t.clone() for t in (layer.dx, layer.dw1, layer.dw2)]
    layer.backward(to_dev(dy, True))
    torch.cuda.synchronize()
    for a, b in zip(first, (layer.dx, layer.dw1, layer.dw2)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("name", ["c2_mixtral", "c3_gptmoe", "c4_finegrained"])
def test_full_config_backward(name):
    """Full size, in the launch configuration the timing runs use: the largest, the smallest
    non-empty, a middle and an empty slot are checked completely (dxp rows, both weight
    gradients) against the fp64 oracle; the streaming steps on all rows from the device's own
    inputs."""
    cfg = CONFIGS[name]
    w = expert_weights(cfg, threads=16)
    inp = step_inputs(cfg, 0)
    ids, gates = om.route(inp["logits"], cfg.k)
    plan = oracle_plan(cfg, ids)
    disp = om.plan_dispatch(ids, inp["rank_tok_off"], plan, cfg.E, cfg.N, cfg.c)
    shape = lz.Shape.from_config(cfg)
    layer = lz.MoELayer(shape, DEV)
    layer.load_expert_weights(w["w1"], w["w2"], plan)
    layer.set_plan(plan, inp["rank_tok_off"])
    layer.enable_training()
    dy = _bf16(np.random.default_rng(21), (cfg.T, cfg.d))
    layer.forward_train(to_dev(inp["logits"]), to_dev(inp["x"], True))
    layer.backward(to_dev(dy, True))
    torch.cuda.synchronize()
    assert np.array_equal(to_host(layer.pair_to_row), disp["pair_to_row"])
    off, counts = disp["slot_offsets"], disp["slot_counts"]
    # combine backward on all rows, from the device's own yp
    yp_dev = to_host(layer.yp)
    dyp_ref, dg_ref = ob.combine_backward(dy, yp_dev, disp["pair_to_row"], to_host(layer.topk_gates))
    dyp_dev = to_host(layer.dyp)
    assert np.all(np.abs(om.widen(dyp_dev) - dyp_ref) <= 0.006 * np.abs(dyp_ref))
    assert np.allclose(to_host(layer.dgates), dg_ref, rtol=1e-4, atol=1e-4 * np.max(np.abs(dg_ref)))
    # slots checked completely
    nz = np.nonzero(counts)[0]
    order = nz[np.argsort(counts[nz])]
    chosen = [int(order[0]), int(order[len(order) // 2]), int(order[-1])]
    xp_dev, dxp_dev = to_host(layer.xp), to_host(layer.dxp)
    for s in chosen:
        a, b = off[s], off[s + 1]
        e = int(plan[s])
        dxp_ref, dw1_ref, dw2_ref = ob.ffn_backward_slot(om.widen(dyp_dev[a:b]), om.widen(xp_dev[a:b]),
                                                        om.widen(w["w1"][e]), om.widen(w["w2"][e]), cfg.act)
        assert rel_err(dxp_dev[a:b], dxp_ref) <= TOL, (s, "dxp")
        assert rel_err(to_host(layer.dw1_slot[s]), dw1_ref.T) <= TOL, (s, "dw1")
        assert rel_err(to_host(layer.dw2_slot[s]), dw2_ref.T) <= TOL, (s, "dw2")
    for s in np.nonzero(counts == 0)[0][:2]:
        assert not layer.dw1_slot[int(s)].any().item() and not layer.dw2_slot[int(s)].any().item()
    # permute backward on all tokens from the device's own dxp; replica sums for one expert
    dx_ref = ob.permute_backward(dxp_dev, disp["pair_to_row"], cfg.k)
    assert np.all(np.abs(om.widen(to_host(layer.dx)) - dx_ref) <= 0.006 * np.abs(dx_ref) + 1e-6)
    e = int(plan[chosen[-1]])
    slots = [s for s in range(cfg.N * cfg.c) if plan[s] == e]
    ref = sum(om.widen(to_host(layer.dw2_slot[s])) for s in slots)
    assert np.all(np.abs(om.widen(to_host(layer.dw2[e])) - ref) <= 0.006 * np.abs(ref) + 1e-6)
    dl_ref = ob.route_backward(to_host(layer.dgates), to_host(layer.topk_gates), ids, cfg.E)
    assert np.allclose(to_host(layer.dlogits), dl_ref, rtol=1e-4, atol=1e-5 * np.max(np.abs(dl_ref)))


def test_odd_number_of_k_steps_with_short_tail_tiles_is_reproducible():
    """Regression: with an odd number of 64-wide K steps the trailing (empty) direct-to-LDS loads of
    one wave land in the LDS stage that holds the other waves' epilogue patches; the kernel has to
    wait for every wave's loads before the first patch is written.  ffn = 320 gives the data
    gradient dxp = dZ W1^T five K steps, the slot sizes give the weight gradients 1, 3 and 5 K
    steps, and the <= 64-row tail tiles run the narrowest tile variant.  Every repetition must
    give the same bits, and those bits must match the oracle."""
    cfg = scaled(CONFIGS["c1_tiny"], act="gelu", dtype="bf16", T=361, k=2, d=256, ffn=320, N=3, c=2)
    counts = [60, 300, 33, 1, 64, 264]
    S, P = 6, cfg.T * cfg.k
    assert sum(counts) == P
    offsets = np.zeros(S + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    rng = np.random.default_rng(17)
    slot_expert = np.array([1, 0, 4, 7, 2, 5], dtype=np.int32)
    w = expert_weights(cfg, threads=2)
    xph, dyph = _bf16(rng, (P, cfg.d)), _bf16(rng, (P, cfg.d), 0.5)
    shape = lz.Shape.from_config(cfg)
    bf = torch.bfloat16
    w1, w2 = slot_weights(w, slot_expert, True)
    n = lz.lz_train_workspace_bytes(shape)
    ws = torch.empty(n, dtype=torch.uint8, device=DEV)
    xp, dyp, off = to_dev(xph, True), to_dev(dyph, True), to_dev(offsets)
    first = None
    for rep in range(6):
        z = torch.zeros((P, cfg.ffn), dtype=bf, device=DEV)
        h = torch.zeros((P, cfg.ffn), dtype=bf, device=DEV)
        yp = torch.zeros((P, cfg.d), dtype=bf, device=DEV)
        dxp = torch.zeros((P, cfg.d), dtype=bf, device=DEV)
        dw1 = torch.zeros((S, cfg.d, cfg.ffn), dtype=bf, device=DEV)
        dw2 = torch.zeros((S, cfg.ffn, cfg.d), dtype=bf, device=DEV)
        lz.lz_ffn_forward_train(xp, off, w1, w2, shape, z, h, yp, ws, n)
        lz.lz_ffn_backward(dyp, xp, z, h, off, w1, w2, shape, dxp, dw1, dw2, ws, n)
        torch.cuda.synchronize()
        outs = [t.view(torch.int16).clone() for t in (yp, dxp, dw1, dw2)]
        if first is None:
            first = outs
        else:
            for a_, b_ in zip(first, outs):
                assert torch.equal(a_, b_), rep
    dxp_ref, dw1_ref, dw2_ref = ob.ffn_backward_rows(dyph, xph, offsets, slot_expert, w["w1"], w["w2"], cfg.act)
    assert rel_err(first[1].view(torch.uint16).cpu().numpy(), dxp_ref) <= TOL
    assert rel_err(first[2].view(torch.uint16).cpu().numpy(), dw1_ref.transpose(0, 2, 1)) <= TOL
    assert rel_err(first[3].view(torch.uint16).cpu().numpy(), dw2_ref.transpose(0, 2, 1)) <= TOL
    # row by row: a zeroed output row would hide behind the tensor's maximum
    got = om.widen(first[1].view(torch.uint16).cpu().numpy())
    assert np.all(np.max(np.abs(got - dxp_ref), axis=1) <= TOL * np.max(np.abs(dxp_ref), axis=1) * 2 + 1e-6)


def test_backward_without_tokens_and_with_bad_offsets():
    """T = 0: every call succeeds and the weight gradients are exact zeros.  Offsets outside
    [0, P] or decreasing are clipped as in the forward: never an out-of-bounds access, and the
    slots that stay valid still get their gradients."""
    bf = torch.bfloat16
    cfg0 = scaled(CONFIGS["c1_tiny"], act="gelu", dtype="bf16", T=0, k=2, d=256, ffn=256, N=2, c=2)
    shape0 = lz.Shape.from_config(cfg0)
    n = lz.lz_train_workspace_bytes(shape0)
    assert n > 0
    ws = torch.empty(n, dtype=torch.uint8, device=DEV)
    S = 4
    w1 = torch.ones((S, 256, 256), dtype=bf, device=DEV)
    w2 = torch.ones((S, 256, 256), dtype=bf, device=DEV)
    dw1 = torch.full((S, 256, 256), 3.0, dtype=bf, device=DEV)
    dw2 = torch.full((S, 256, 256), 3.0, dtype=bf, device=DEV)
    empty = torch.zeros((0, 256), dtype=bf, device=DEV)
    off0 = torch.zeros(S + 1, dtype=torch.int32, device=DEV)
    lz.lz_ffn_forward_train(empty, off0, w1, w2, shape0, empty, empty, empty, ws, n)
    lz.lz_ffn_backward(empty, empty, empty, empty, off0, w1, w2, shape0, empty, dw1, dw2, ws, n)
    lz.lz_combine_backward(empty, empty, off0, torch.zeros(0, device=DEV), shape0, empty, torch.zeros(0, device=DEV))
    lz.lz_permute_backward(empty, off0, shape0, empty)
    torch.cuda.synchronize()
    assert not dw1.any().item() and not dw2.any().item()

    cfg = scaled(cfg0, T=300)
    shape = lz.Shape.from_config(cfg)
    P = cfg.T * cfg.k
    rng = np.random.default_rng(3)
    w = expert_weights(cfg, threads=2)
    slot_expert = np.array([0, 1, 2, 3], dtype=np.int32)
    w1, w2 = slot_weights(w, slot_expert, True)
    xph, dyph = _bf16(rng, (P, cfg.d)), _bf16(rng, (P, cfg.d), 0.5)
    bad = np.array([-7, 200, 200, 700, 650], dtype=np.int32)     # clipped: [0,200) [200,200) [200,600) [600,600)
    good = np.array([0, 200, 200, 600, 600], dtype=np.int32)
    n = lz.lz_train_workspace_bytes(shape)
    ws = torch.empty(n, dtype=torch.uint8, device=DEV)
    outs = []
    for off in (bad, good):
        z = torch.zeros((P, cfg.ffn), dtype=bf, device=DEV)
        h = torch.zeros((P, cfg.ffn), dtype=bf, device=DEV)
        yp = torch.zeros((P, cfg.d), dtype=bf, device=DEV)
        dxp = torch.zeros((P, cfg.d), dtype=bf, device=DEV)
        dw1 = torch.full((S, cfg.d, cfg.ffn), 3.0, dtype=bf, device=DEV)
        dw2 = torch.full((S, cfg.ffn, cfg.d), 3.0, dtype=bf, device=DEV)
        lz.lz_ffn_forward_train(to_dev(xph, True), to_dev(off), w1, w2, shape, z, h, yp, ws, n)
        lz.lz_ffn_backward(to_dev(dyph, True), to_dev(xph, True), z, h, to_dev(off), w1, w2, shape, dxp, dw1, dw2,
                           ws, n)
        torch.cuda.synchronize()
        outs.append((yp, dxp, dw1, dw2))
    for a_, b_ in zip(*outs):
        assert torch.equal(a_.view(torch.int16), b_.view(torch.int16))
    dxp_ref, dw1_ref, dw2_ref = ob.ffn_backward_rows(dyph, xph, good, slot_expert, w["w1"], w["w2"], cfg.act)
    assert rel_err(to_host(outs[0][1])[:600], dxp_ref[:600]) <= TOL
    assert rel_err(to_host(outs[0][2]), dw1_ref.transpose(0, 2, 1)) <= TOL
    assert not outs[0][2][1].any().item() and not outs[0][3][3].any().item()      # the empty slots


@pytest.mark.parametrize("dtype,d,ffn,act", [("bf16", 256, 320, "gelu"), ("bf16", 512, 128, "swiglu"),
                                             ("f32", 72, 200, "swiglu")])
def test_weight_gradients_accumulate_in_fp32_over_micro_batches(dtype, d, ffn, act):
    """Two micro-batches with different inputs and routing through backward_accumulate: the fp32
    accumulators hold the sum of the two batches' slot gradients (an empty slot adds nothing), and
    their per-expert reduction matches the fp64 oracle's sum of the two batches' expert gradients.
    MFMA shapes (ragged K, n_out not a multiple of 256) and a generic fp32 shape."""
    cfg = scaled(CONFIGS["c4_finegrained"], dtype=dtype, act=act, T=700, d=d, ffn=ffn, E=12, k=3, N=4, c=4)
    bf16 = dtype == "bf16"
    tol = 2e-2 if bf16 else 1e-5
    w = expert_weights(cfg, threads=4)
    shape = lz.Shape.from_config(cfg)
    ids0, _ = om.route(step_inputs(cfg, 0)["logits"], cfg.k)
    plan = oracle_plan(cfg, ids0)
    layer = lz.MoELayer(shape, DEV)
    layer.load_expert_weights(w["w1"], w["w2"], plan)
    layer.enable_training()
    layer.enable_accumulation()
    rng = np.random.default_rng(33)
    ref1 = ref2 = 0.0
    for step in range(2):
        inp = step_inputs(cfg, step)
        layer.set_plan(plan, inp["rank_tok_off"])
        ids, gates = om.route(inp["logits"], cfg.k)
        disp = om.plan_dispatch(ids, inp["rank_tok_off"], plan, cfg.E, cfg.N, cfg.c)
        dy = rng.standard_normal((cfg.T, cfg.d)).astype(np.float32)
        dy = f32_to_bf16_bits(dy) if bf16 else dy
        layer.forward_train(to_dev(inp["logits"]), to_dev(inp["x"], bf16))
        layer.backward_accumulate(to_dev(dy, bf16))
        torch.cuda.synchronize()
        ref = ob.layer_backward(dy, inp["x"], ids, gates, disp["pair_to_row"], disp["row_to_pair"],
                                disp["slot_offsets"], plan, w["w1"], w["w2"], act)
        assert rel_err(to_host(layer.dx), ref["dx"]) <= tol
        ref1 = ref1 + ref["dw1"].transpose(0, 2, 1)
        ref2 = ref2 + ref["dw2"].transpose(0, 2, 1)
    dw1, dw2 = layer.reduce_accumulated()
    torch.cuda.synchronize()
    assert rel_err(dw1.cpu().numpy(), ref1) <= tol
    assert rel_err(dw2.cpu().numpy(), ref2) <= tol
    # slot level: the accumulators of the slots of one expert add up to that expert's sum
    acc1 = layer.dw1_acc.cpu().numpy().astype(np.float64)
    for e in range(cfg.E):
        slots = np.nonzero(plan == e)[0]
        assert np.allclose(acc1[slots].sum(axis=0), dw1[e].cpu().numpy(), rtol=1e-5, atol=1e-6)


def test_ffn_backward_slot_beyond_4_gib():
    """Maximum sizes: one slot of 131 500 rows makes the k-major operands of the weight gradients
    (dZ with 16 384 columns, h with 8 192) span 4.3 GB and 2.2 GB inside that slot, beyond 32-bit
    byte offsets, and puts the slots after it more than 4 GiB into the buffers.  Checked on sampled
    hidden columns (weight gradients) and sampled rows (data gradient) of the big slot and on the
    small slot behind it, against the fp64 oracle."""
    cfg = scaled(CONFIGS["c1_tiny"], act="swiglu", dtype="bf16", T=70000, k=2, d=256, ffn=8192, N=2, c=2)
    counts = [3000, 131500, 0, 5500]
    S, P, d, ffn = 4, cfg.T * cfg.k, cfg.d, cfg.ffn
    n1 = 2 * ffn
    assert sum(counts) == P and counts[1] * n1 * 2 > 2 ** 32
    offsets = np.zeros(S + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    rng = np.random.default_rng(41)
    slot_expert = np.array([3, 6, 1, 4], dtype=np.int32)
    w = expert_weights(cfg, threads=8)
    xph, dyph = _bf16(rng, (P, d)), _bf16(rng, (P, d), 0.5)
    shape = lz.Shape.from_config(cfg)
    bf = torch.bfloat16
    w1, w2 = slot_weights(w, slot_expert, True)
    nbytes = lz.lz_train_workspace_bytes(shape)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    xp, dyp, off = to_dev(xph, True), to_dev(dyph, True), to_dev(offsets)
    z = torch.empty((P, n1), dtype=bf, device=DEV)
    h = torch.empty((P, ffn), dtype=bf, device=DEV)
    yp = torch.empty((P, d), dtype=bf, device=DEV)
    dxp = torch.empty((P, d), dtype=bf, device=DEV)
    dw1 = torch.full((S, d, n1), 7.0, dtype=bf, device=DEV)
    dw2 = torch.full((S, ffn, d), 7.0, dtype=bf, device=DEV)
    print("slot beyond 4 GiB: forward_train", flush=True)
    lz.lz_ffn_forward_train(xp, off, w1, w2, shape, z, h, yp, ws, nbytes)
    torch.cuda.synchronize()
    print("slot beyond 4 GiB: ffn_backward", flush=True)
    lz.lz_ffn_backward(dyp, xp, z, h, off, w1, w2, shape, dxp, dw1, dw2, ws, nbytes)
    torch.cuda.synchronize()
    assert not dw1[2].any().item() and not dw2[2].any().item()          # the empty slot
    Xp, dYp = om.widen(xph), om.widen(dyph)
    F = np.array([0, 1, 257, 4095, 4096, 5000, 8190, 8191])
    for s_ in (1, 3):
        a_, b_ = int(offsets[s_]), int(offsets[s_ + 1])
        e = int(slot_expert[s_])
        W1, W2 = om.widen(w["w1"][e]), om.widen(w["w2"][e])                # [n1, d], [d, ffn]
        X, dY = Xp[a_:b_], dYp[a_:b_]
        Zs = np.concatenate([X @ W1[F].T, X @ W1[ffn + F].T], axis=1)     # gate columns, then up columns
        dHs = dY @ W2[:, F]
        dZs = ob.act_backward(dHs, Zs, "swiglu")
        Hs = ob.act_forward(Zs, "swiglu")
        cols = np.concatenate([F, ffn + F])
        got1 = om.widen(to_host(dw1[s_][:, torch.from_numpy(cols).to(DEV)]))
        ref1 = X.T @ dZs
        assert np.max(np.abs(got1 - ref1)) <= TOL * np.max(np.abs(ref1)), s_
        got2 = om.widen(to_host(dw2[s_][torch.from_numpy(F).to(DEV)]))
        ref2 = Hs.T @ dY
        assert np.max(np.abs(got2 - ref2)) <= TOL * np.max(np.abs(ref2)), s_
        # stored intermediates at the sampled columns
        zc = om.widen(to_host(z[a_:b_][:, torch.from_numpy(cols).to(DEV)]))
        assert np.max(np.abs(zc - Zs)) <= TOL * np.max(np.abs(Zs)), s_
        # data gradient and forward output on sampled rows (need the whole hidden width of a row)
        rows = np.array([a_, a_ + 1, (a_ + b_) // 2, b_ - 2, b_ - 1])
        Zr = Xp[rows] @ W1.T
        dxp_ref = ob.act_backward(dYp[rows] @ W2, Zr, "swiglu") @ W1
        yp_ref = ob.act_forward(Zr, "swiglu") @ W2.T
        ridx = torch.from_numpy(rows).to(DEV)
        assert rel_err(to_host(dxp[ridx]), dxp_ref) <= TOL, s_
        assert rel_err(to_host(yp[ridx]), yp_ref) <= TOL, s_


def _layer_backward_generic(cfg, tol):
    """Whole layer forward + backward through MoELayer on a shape the MFMA kernels do not serve."""
    inp = step_inputs(cfg)
    w = expert_weights(cfg, threads=4)
    ids, gates = om.route(inp["logits"], cfg.k)
    plan = oracle_plan(cfg, ids)
    disp = om.plan_dispatch(ids, inp["rank_tok_off"], plan, cfg.E, cfg.N, cfg.c)
    shape = lz.Shape.from_config(cfg)
    bf16 = cfg.dtype == "bf16"
    layer = lz.MoELayer(shape, DEV)
    layer.load_expert_weights(w["w1"], w["w2"], plan)
    layer.set_plan(plan, inp["rank_tok_off"])
    layer.enable_training()
    rng = np.random.default_rng(21)
    dy = rng.standard_normal((cfg.T, cfg.d)).astype(np.float32)
    dy = f32_to_bf16_bits(dy) if bf16 else dy
    y = layer.forward_train(to_dev(inp["logits"]), to_dev(inp["x"], bf16))
    layer.backward(to_dev(dy, bf16))
    torch.cuda.synchronize()
    assert np.array_equal(to_host(layer.pair_to_row), disp["pair_to_row"])
    assert rel_err(to_host(y), om.layer_output(inp["x"], ids, gates, w["w1"], w["w2"], cfg.act)) <= tol
    ref = ob.layer_backward(dy, inp["x"], ids, gates, disp["pair_to_row"], disp["row_to_pair"],
                            disp["slot_offsets"], plan, w["w1"], w["w2"], cfg.act)
    assert rel_err(to_host(layer.dx), ref["dx"]) <= tol
    assert rel_err(to_host(layer.dgates), ref["dgates"]) <= tol
    assert rel_err(to_host(layer.dw1), ref["dw1"].transpose(0, 2, 1)) <= tol     # oracle: [out, in]
    assert rel_err(to_host(layer.dw2), ref["dw2"].transpose(0, 2, 1)) <= tol
    assert rel_err(to_host(layer.dlogits), ob.route_backward(ref["dgates"], gates, ids, cfg.E)) <= tol
    # the kept intermediates against the oracle's
    Xp = om.widen(om.permute(inp["x"], disp["row_to_pair"], cfg.k))
    off = disp["slot_offsets"]
    Zref = np.zeros((cfg.T * cfg.k, to_host(layer.z).shape[1]))
    for s_ in range(cfg.N * cfg.c):
        a_, b_ = off[s_], off[s_ + 1]
        Zref[a_:b_] = Xp[a_:b_] @ om.widen(w["w1"][plan[s_]]).T
    assert rel_err(to_host(layer.z), Zref) <= tol
    assert rel_err(to_host(layer.h), ob.act_forward(Zref, cfg.act)) <= tol
    # experts without a slot cannot occur; an expert's gradient is the sum over its replicas
    return layer


def test_layer_backward_fp32_config_1():
    """Config 1 (fp32, GELU, fixed replica counts, spread placement) in full through the training
    entry points: the plain tiled fp32 kernels meet the fp32 error bar of the forward."""
    _layer_backward_generic(CONFIGS["c1_tiny"], 1e-5)


@pytest.mark.parametrize("act,dtype,tol", [("swiglu", "f32", 1e-5), ("gelu", "bf16", 2e-2), ("swiglu", "bf16", 2e-2)])
def test_layer_backward_generic_shapes(act, dtype, tol):
    """Sizes the MFMA tiling does not divide (d = 72, ffn = 200, top-3, ragged ranks), both dtypes."""
    cfg = scaled(CONFIGS["c1_tiny"], act=act, dtype=dtype, T=333, d=72, ffn=200, E=8, k=3, N=3, c=4,
                 replica_counts=(2, 2, 2, 2, 1, 1, 1, 1))
    _layer_backward_generic(cfg, tol)


def test_training_entry_points_reject_what_they_do_not_serve():
    bad = lz.Shape(T=16, d=8, ffn=8, E=4, k=9, N=2, c=2, dtype=lz.LZ_F32, act=lz.LZ_GELU)
    assert lz.lz_train_workspace_bytes(bad) == 0
    f32 = lz.Shape.from_config(CONFIGS["c1_tiny"])
    assert lz.lz_train_workspace_bytes(f32) > 0          # generic kernels
    odd = lz.Shape.from_config(scaled(CONFIGS["c1_tiny"], dtype="bf16", d=264, ffn=128))
    assert lz.lz_train_workspace_bytes(odd) > 0
    huge = lz.Shape.from_config(scaled(CONFIGS["c1_tiny"], T=1 << 23, k=2, d=264, ffn=128))
    assert lz.lz_train_workspace_bytes(huge) == 0        # too many 64-row tiles for the generic path
    ok = lz.Shape.from_config(scaled(CONFIGS["c1_tiny"], dtype="bf16", d=256, ffn=128))
    n = lz.lz_train_workspace_bytes(ok)
    ws = torch.empty(n, dtype=torch.uint8, device=DEV)
    dummy = torch.zeros(16, dtype=torch.uint8, device=DEV)
    with pytest.raises(lz.LzError) as e:
        lz.lz_ffn_backward(dummy, dummy, dummy, dummy, dummy, dummy, dummy, ok, dummy, dummy, dummy, ws, n - 256)
    assert e.value.code == -3
    with pytest.raises(lz.LzError) as e:
        lz.lz_ffn_backward(dummy, dummy, dummy, dummy, dummy, dummy, dummy, bad, dummy, dummy, dummy, ws, n)
    assert e.value.code == -2
    with pytest.raises(lz.LzError) as e:
        lz.lz_ffn_backward(dummy, dummy, dummy, dummy, dummy, dummy, dummy, f32, dummy, dummy, dummy, ws, 256)
    assert e.value.code == -3
