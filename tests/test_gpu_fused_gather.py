"""The reshuffle fused into the first GEMM's activation loads (lz_ffn_up_gather,
lz_expert_ffn_gather) against the oracle and against the unfused calls, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2407_04656_amd as lz
from oracle import moe_layer as om
from workloads import CONFIGS, expert_weights, f32_to_bf16_bits, step_inputs
from workloads.configs import scaled

from gpu_util import DEV, oracle_plan, rel_err, slot_weights, to_dev, to_host, tolerance

pytestmark = pytest.mark.gpu


def _case(cfg, counts, seed):
    """A permuted buffer of sum(counts) rows over S slots whose rows point at random tokens of x:
    row r holds pair row_to_pair[r] (a permutation of the pairs), its token is pair // k."""
    S, P = cfg.N * cfg.c, cfg.T * cfg.k
    assert len(counts) == S and sum(counts) == P
    offsets = np.zeros(S + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    rng = np.random.default_rng(seed)
    slot_expert = rng.integers(0, cfg.E, size=S).astype(np.int32)
    row_to_pair = rng.permutation(P).astype(np.int32)
    w = expert_weights(cfg, threads=4)
    bf16 = cfg.dtype == "bf16"
    xh = rng.standard_normal((cfg.T, cfg.d)).astype(np.float32)
    xh = f32_to_bf16_bits(xh) if bf16 else xh
    shape = lz.Shape.from_config(cfg)
    w1, w2 = slot_weights(w, slot_expert, bf16)
    tdt = torch.bfloat16 if bf16 else torch.float32
    x, off, r2p = to_dev(xh, bf16), to_dev(offsets), to_dev(row_to_pair)
    nbytes = lz.lz_ffn_workspace_bytes(shape)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    # unfused: permute, then the FFN on xp
    xp = torch.zeros((P, cfg.d), dtype=tdt, device=DEV)
    lz.lz_permute(x, r2p, shape, xp)
    yp_a = torch.zeros((P, cfg.d), dtype=tdt, device=DEV)
    lz.lz_expert_ffn(xp, off, w1, w2, shape, yp_a, ws, nbytes)
    # fused, twice (the tile queues must be left reusable)
    outs = []
    for _ in range(2):
        yp_b = torch.zeros((P, cfg.d), dtype=tdt, device=DEV)
        lz.lz_expert_ffn_gather(x, r2p, off, w1, w2, shape, yp_b, ws, nbytes)
        torch.cuda.synchronize()
        outs.append(yp_b)
    view = torch.int16 if bf16 else torch.int32
    assert torch.equal(yp_a.view(view), outs[0].view(view))
    assert torch.equal(outs[0].view(view), outs[1].view(view))
    xph = om.permute(xh, row_to_pair, cfg.k)
    assert np.array_equal(to_host(xp), xph)
    ref = om.expert_ffn_rows(xph, offsets, slot_expert, w["w1"], w["w2"], cfg.act)
    return rel_err(to_host(outs[1]), ref)


@pytest.mark.parametrize("act,d,ffn", [("gelu", 256, 256), ("swiglu", 256, 128), ("swiglu", 512, 384)])
def test_fused_gather_mfma_ragged(act, d, ffn):
    cfg = scaled(CONFIGS["c1_tiny"], act=act, dtype="bf16", T=700, k=2, d=d, ffn=ffn, N=4, c=2)
    # several row tiles, a tile boundary + 1, an empty slot, one-row slots, every 64-row tail class
    assert _case(cfg, [257, 0, 1, 512, 300, 255, 74, 1], 3) <= 2e-2
    assert _case(cfg, [130, 190, 65, 128, 64, 193, 400, 230], 4) <= 2e-2


@pytest.mark.parametrize("act", ["gelu", "swiglu"])
def test_fused_gather_generic_paths(act):
    f32 = scaled(CONFIGS["c1_tiny"], act=act, T=300, k=3, d=72, ffn=200, N=3, c=2)
    assert _case(f32, [100, 0, 333, 1, 66, 400], 8) <= 1e-5
    odd = scaled(CONFIGS["c1_tiny"], act=act, dtype="bf16", T=300, k=2, d=264, ffn=200, N=2, c=2)
    assert _case(odd, [1, 300, 0, 299], 9) <= 2e-2


def test_fused_gather_rows_without_a_pair_read_as_zero():
    """A map entry outside [0, P) (only possible outside every slot) must not fault and reads as zeros."""
    cfg = scaled(CONFIGS["c1_tiny"], act="gelu", dtype="bf16", T=256, k=2, d=256, ffn=256, N=2, c=1)
    shape = lz.Shape.from_config(cfg)
    P = 512
    rng = np.random.default_rng(2)
    r2p = rng.permutation(P).astype(np.int32)
    r2p[[3, 200, 511]] = [-1, P, 2 ** 31 - 1]
    x = to_dev(f32_to_bf16_bits(rng.standard_normal((cfg.T, cfg.d)).astype(np.float32)), True)
    w = expert_weights(cfg, threads=2)
    w1, w2 = slot_weights(w, np.array([0, 1], dtype=np.int32), True)
    off = to_dev(np.array([0, 300, 512], dtype=np.int32))
    nbytes = lz.lz_ffn_workspace_bytes(shape)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    yp = torch.ones((P, cfg.d), dtype=torch.bfloat16, device=DEV)
    lz.lz_expert_ffn_gather(x, to_dev(r2p), off, w1, w2, shape, yp, ws, nbytes)
    torch.cuda.synchronize()
    got = yp.float()
    assert torch.isfinite(got).all()
    assert not got[[3, 200, 511]].any().item()          # FFN of a zero row (no biases) is zero
    assert got[[4, 201, 510]].abs().sum().item() > 0


@pytest.mark.parametrize("name", ["c2_mixtral", "c4_finegrained"])
def test_fused_gather_full_config(name):
    """Whole layer at full size: the fused pass gives the same bits as the five-call pass and
    matches the fp64 definition on sampled tokens."""
    cfg = CONFIGS[name]
    inp = step_inputs(cfg, 0)
    w = expert_weights(cfg, threads=16)
    ids, gates = om.route(inp["logits"], cfg.k)
    plan = oracle_plan(cfg, ids)
    shape = lz.Shape.from_config(cfg)
    layer = lz.MoELayer(shape, DEV)
    layer.set_plan(plan, inp["rank_tok_off"])
    layer.load_expert_weights(w["w1"], w["w2"], plan)
    logits, x = to_dev(inp["logits"]), to_dev(inp["x"], True)
    y_a = layer.forward(logits, x).clone()
    layer.xp.zero_()
    y_b = layer.forward_fused(logits, x).clone()
    torch.cuda.synchronize()
    assert torch.equal(y_a.view(torch.int16), y_b.view(torch.int16))
    toks = np.random.default_rng(1).choice(cfg.T, size=96, replace=False)
    y_ref = om.layer_output(inp["x"], ids, gates, w["w1"], w["w2"], cfg.act, tokens=toks)
    assert rel_err(to_host(y_b[torch.from_numpy(toks).to(DEV)]), y_ref) <= tolerance(cfg)
