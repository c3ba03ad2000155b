"""Host planning functions of the C ABI against the oracle (bit-exact), no GPU needed."""
import re
import os

import numpy as np
import pytest

import paper_2407_04656_amd as lz
from oracle import planner as op


def test_library_exports_every_declared_symbol():
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    header = open(os.path.join(root, "include", "lazarus_moe.h")).read()
    declared = sorted(set(re.findall(r"\b(lz_[a-z_]+)\s*\(", header)))
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(lz.lib, name), f"{name} declared in the header but not exported"
    assert lz.lz_version() >= 100
    assert "workspace" in lz.lz_strerror(-3)


def test_allocate_and_place_match_oracle():
    rng = np.random.default_rng(0)
    n = 0
    for _ in range(400):
        E = int(rng.integers(1, 40))
        N = int(rng.integers(1, 17))
        c = int(rng.integers(1, 9))
        f = int(rng.integers(1, 4))
        t = rng.integers(0, 10000, size=E)
        if rng.random() < 0.3:
            t = rng.integers(0, 4, size=E)        # many ties and zeros
        if N * c < E:
            with pytest.raises(lz.LzError) as ei:
                lz.lz_allocate_replicas(t, N, c, f)
            assert ei.value.code == -5
            continue
        r = lz.lz_allocate_replicas(t, N, c, f)
        assert r.tolist() == op.allocate_replicas(t, N, c, f)
        assert lz.lz_place_mro(r, t, N, c).tolist() == op.place_mro(r, t, N, c)
        assert lz.lz_place_spread(r, N, c).tolist() == op.place_spread(r, N, c)
        assert lz.lz_place_compact(r, N, c).tolist() == op.place_compact(r, N, c)
        n += 1
    assert n > 200


def test_place_rejects_bad_counts():
    with pytest.raises(lz.LzError):
        lz.lz_place_mro([1, 2], [1, 2], 2, 2)
    with pytest.raises(lz.LzError):
        lz.lz_place_mro([0, 4], [0, 4], 2, 2)
    with pytest.raises(lz.LzError):
        lz.lz_place_spread([1, 1], 2, 2)


def test_recovery_probability_matches_oracle():
    rng = np.random.default_rng(1)
    for _ in range(60):
        E = int(rng.integers(1, 10))
        N = int(rng.integers(1, 9))
        c = int(rng.integers(1, 5))
        if N * c < E:
            continue
        t = rng.integers(1, 100, size=E)
        r = op.allocate_replicas(t, N, c, 1)
        for plan in (op.place_mro(r, t, N, c), op.place_spread(r, N, c)):
            for n_alive in range(0, N + 1):
                good, total = lz.lz_recovery_probability(plan, E, N, c, n_alive)
                frac = op.recovery_probability(plan, E, N, c, n_alive)
                assert good * frac.denominator == frac.numerator * total


def test_replan_matches_oracle():
    rng = np.random.default_rng(2)
    ok = unrec = 0
    for _ in range(400):
        E = int(rng.integers(2, 24))
        N = int(rng.integers(2, 10))
        c = int(rng.integers(1, 7))
        if N * c < E:
            continue
        f = int(rng.integers(1, 3))
        t = rng.integers(1, 500, size=E)
        old = op.place_mro(op.allocate_replicas(t, N, c, f), t, N, c)
        alive = np.ones(N, dtype=bool)
        alive[rng.choice(N, size=int(rng.integers(0, N)), replace=False)] = False
        c_new = max(1, c + int(rng.integers(-1, 3)))
        t2 = rng.integers(0, 500, size=E)
        try:
            ref = op.replan(old, N, c, alive, t2, c_new, f)
        except op.Unrecoverable:
            with pytest.raises(lz.LzError) as ei:
                lz.lz_replan(old, N, c, alive, t2, c_new, f)
            assert ei.value.code == -4
            unrec += 1
            continue
        except op.Infeasible:
            with pytest.raises(lz.LzError) as ei:
                lz.lz_replan(old, N, c, alive, t2, c_new, f)
            assert ei.value.code == -5
            continue
        got = lz.lz_replan(old, N, c, alive, t2, c_new, f)
        assert got["new_slot_expert"].tolist() == ref["new_slot_expert"]
        assert got["plan2phys"].tolist() == ref["plan2phys"]
        assert got["transfers"] == ref["transfers"]
        ok += 1
    assert ok > 100 and unrec > 10


def test_replan_handworked_cases_through_the_library(golden_dir):
    """The hand-worked Sec. 4.3 cases (tests/golden/replan_handworked.txt) through lz_replan."""
    from test_oracle_planner import load_replan_cases
    cases = load_replan_cases(golden_dir)
    assert len(cases) >= 6
    for cs in cases:
        got = lz.lz_replan(cs["old"], cs["N_old"], cs["c_old"], np.array(cs["alive"], dtype=np.uint8),
                           np.array(cs["t"]), cs["c_new"], 1)
        assert got["plan2phys"].tolist() == cs["plan2phys"], cs["name"]
        assert got["new_slot_expert"].tolist() == cs["new"], cs["name"]
        assert [tuple(x) for x in got["transfers"]] == cs["transfers"], cs["name"]


def test_device_calls_validate_arguments_without_a_gpu():
    bad = lz.Shape(T=16, d=8, ffn=8, E=4, k=9, N=2, c=2, dtype=lz.LZ_F32, act=lz.LZ_GELU)
    assert lz.lz_plan_workspace_bytes(bad) == 0 and lz.lz_ffn_workspace_bytes(bad) == 0
    good = lz.Shape(T=16, d=8, ffn=8, E=4, k=2, N=2, c=2, dtype=lz.LZ_F32, act=lz.LZ_GELU)
    assert lz.lz_plan_workspace_bytes(good) > 0 and lz.lz_ffn_workspace_bytes(good) >= 16 * 2 * 8 * 4
    with pytest.raises(lz.LzError) as ei:
        lz.lz_route(None, 4, 300, 2, None, None, stream=0)
    assert ei.value.code == -2
    with pytest.raises(lz.LzError) as ei:
        lz.lz_route(None, 4, 8, 2, None, None, stream=0)
    assert ei.value.code == -1
    with pytest.raises(lz.LzError) as ei:
        lz.lz_permute(None, None, bad, None, stream=0)
    assert ei.value.code == -2


def test_training_calls_validate_arguments_without_a_gpu():
    def shape(**kw):
        base = dict(T=512, d=256, ffn=128, E=8, k=2, N=2, c=4, dtype=lz.LZ_BF16, act=lz.LZ_SWIGLU)
        base.update(kw)
        return lz.Shape(**base)

    ok = shape()
    n = lz.lz_train_workspace_bytes(ok)
    # at least the two gradient intermediates dH [P, ffn] and dZ [P, 2 ffn]
    assert n >= ok.P * ok.ffn * 2 + ok.P * 2 * ok.ffn * 2
    # served by the plain tiled kernels: fp32, sizes the MFMA tiling does not divide
    for generic in (shape(dtype=lz.LZ_F32), shape(d=264), shape(ffn=100)):
        assert lz.lz_train_workspace_bytes(generic) > 0
        with pytest.raises(lz.LzError) as ei:                        # no workspace
            lz.lz_ffn_backward(None, None, None, None, None, None, None, generic, None, None, None, None, 0, stream=0)
        assert ei.value.code == -3
    # activation tensors beyond 32-bit byte offsets are served too (the workspace is what it is)
    assert lz.lz_train_workspace_bytes(shape(T=1 << 20, k=8, d=4096, ffn=14336)) > (1 << 36)
    # invalid, or beyond both paths (one slot's weights past 32-bit offsets on the MFMA path and too
    # many 64-row tiles for the plain one)
    for bad in (shape(k=9), shape(T=1 << 23, k=2, d=264, ffn=128)):
        assert lz.lz_train_workspace_bytes(bad) == 0
        with pytest.raises(lz.LzError) as ei:
            lz.lz_ffn_backward(None, None, None, None, None, None, None, bad, None, None, None, None, 0, stream=0)
        assert ei.value.code == -2
        with pytest.raises(lz.LzError) as ei:
            lz.lz_ffn_forward_train(None, None, None, None, bad, None, None, None, None, 0, stream=0)
        assert ei.value.code == -2
    with pytest.raises(lz.LzError) as ei:                            # no workspace
        lz.lz_ffn_backward(None, None, None, None, None, None, None, ok, None, None, None, None, n, stream=0)
    assert ei.value.code == -3
    with pytest.raises(lz.LzError) as ei:                            # null tensors
        lz.lz_combine_backward(None, None, None, None, ok, None, None, stream=0)
    assert ei.value.code == -1
    with pytest.raises(lz.LzError) as ei:
        lz.lz_combine_backward(None, None, None, None, shape(k=9), None, None, stream=0)
    assert ei.value.code == -2
    with pytest.raises(lz.LzError) as ei:
        lz.lz_route_backward(None, None, None, ok, None, stream=0)
    assert ei.value.code == -1
    with pytest.raises(lz.LzError) as ei:
        lz.lz_reduce_replica_grads(None, None, 4, 2, 12, None, stream=0)   # not a multiple of 8 elements
    assert ei.value.code == -2
    with pytest.raises(lz.LzError) as ei:
        lz.lz_permute_backward(None, None, ok, None, stream=0)
    assert ei.value.code == -1
    with pytest.raises(lz.LzError) as ei:
        lz.lz_pack_weights(None, 2, 64, 64, lz.LZ_BF16, None, stream=0)
    assert ei.value.code == -1
    with pytest.raises(lz.LzError) as ei:
        lz.lz_pack_weights(None, 2, 0, 64, lz.LZ_BF16, None, stream=0)
    assert ei.value.code == -2
