"""Pins for oracle.moe_layer.route / histogram (Sec. 2.1; Algorithm 1 input)."""
import math

import numpy as np
import pytest
from scipy.special import softmax

from oracle import moe_layer as om
from workloads import CONFIGS, step_inputs


def _logits(T, E, seed, ties=False):
    rng = np.random.default_rng(seed)
    z = rng.standard_normal((T, E)).astype(np.float32)
    if ties:
        z = np.round(z * 2) / 2          # many equal values, including +0.0 and -0.0
        z = z.astype(np.float32)
    return z


@pytest.mark.parametrize("ties", [False, True])
@pytest.mark.parametrize("E,k", [(8, 2), (64, 6), (5, 5), (3, 1)])
def test_ids_equal_stable_argsort(E, k, ties):
    """Library routine: the first k entries of a stable arg-sort of -logits."""
    z = _logits(300, E, 7 + E + k, ties)
    ids, _ = om.route(z, k)
    ref = np.argsort(-z, axis=1, kind="stable")[:, :k]
    assert np.array_equal(ids, ref)


def test_ids_bruteforce_python():
    z = _logits(40, 6, 3, ties=True)
    z[0, :] = 0.0
    z[1, :3] = -0.0
    z[1, 3:] = 0.0
    ids, _ = om.route(z, 3)
    for t in range(z.shape[0]):
        remaining = list(range(6))
        for kk in range(3):
            best = remaining[0]
            for e in remaining:
                if float(z[t, e]) > float(z[t, best]):   # strict: ties keep the lower index
                    best = e
            assert ids[t, kk] == best
            remaining.remove(best)
    assert list(ids[0]) == [0, 1, 2] and list(ids[1]) == [0, 1, 2]


def test_ids_distinct_and_sorted():
    z = step_inputs(CONFIGS["c1_tiny"])["logits"]
    ids, gates = om.route(z, 2)
    assert np.all(ids[:, 0] != ids[:, 1])
    sel = np.take_along_axis(z, ids.astype(np.int64), axis=1)
    assert np.all(np.diff(sel, axis=1) <= 0)
    assert np.all(np.diff(gates, axis=1) <= 0)


def test_gates_sum_to_one_and_full_softmax():
    z = _logits(200, 7, 11)
    _, g = om.route(z, 3)
    assert np.allclose(g.sum(axis=1), 1.0, rtol=0, atol=1e-12)
    # k = E: the gates are the softmax over all experts, listed in routing order
    ids, gE = om.route(z, 7)
    full = softmax(z.astype(np.float64), axis=1)
    assert np.allclose(gE, np.take_along_axis(full, ids.astype(np.int64), axis=1), rtol=1e-12, atol=0)
    # k < E: softmax over all, renormalised over the chosen k
    ids3, g3 = om.route(z, 3)
    part = np.take_along_axis(full, ids3.astype(np.int64), axis=1)
    assert np.allclose(g3, part / part.sum(axis=1, keepdims=True), rtol=1e-12, atol=0)


def test_gates_closed_form_two_experts():
    z = np.array([[0.0, math.log(3.0)]], dtype=np.float32)
    ids, g = om.route(z, 2)
    assert list(ids[0]) == [1, 0]
    l1 = float(z[0, 1])
    assert g[0, 0] == pytest.approx(math.exp(l1) / (1 + math.exp(l1)), rel=1e-14)
    assert g[0, 1] == pytest.approx(1 / (1 + math.exp(l1)), rel=1e-14)


def test_histogram_equals_bincount():
    cfg = CONFIGS["c1_tiny"]
    inp = step_inputs(cfg)
    ids, _ = om.route(inp["logits"], cfg.k)
    off = np.array([0, 10, 10, 200, 256])            # ragged, one empty rank
    Tej = om.histogram(ids, off, cfg.E)
    src = np.searchsorted(off, np.arange(cfg.T), side="right") - 1
    key = ids.astype(np.int64) * 4 + src[:, None]
    assert np.array_equal(Tej.reshape(-1), np.bincount(key.reshape(-1), minlength=cfg.E * 4))
    assert Tej.sum() == cfg.T * cfg.k


def test_source_rank_default_split():
    off = inp_off = step_inputs(CONFIGS["c5_postfailure"], with_x=False)["rank_tok_off"]
    assert list(off) == [0, 2730, 5461, 8192, 10922, 13653, 16384]
    src = om.source_rank(inp_off, 16384)
    assert src[2729] == 0 and src[2730] == 1 and src[-1] == 5
