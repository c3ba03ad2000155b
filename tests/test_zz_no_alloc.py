"""lz_plan_dispatch_noalloc (tables in the library's fixed device array, no workspace argument)
against lz_plan_dispatch, through the C ABI: same bits on two calls in a row, the second smaller."""
import numpy as np
import pytest
import torch

import paper_2407_04656_amd as lz
from oracle import moe_layer as om

from gpu_util import DEV, to_dev, to_host

pytestmark = pytest.mark.gpu

KEYS = ("slot_counts", "slot_offsets", "pair_to_row", "row_to_pair", "Tej", "D", "status")


def _buffers(s):
    i32 = torch.int32
    return {
        "slot_counts": torch.full((s.S,), -7, dtype=i32, device=DEV),
        "slot_offsets": torch.full((s.S + 1,), -7, dtype=i32, device=DEV),
        "pair_to_row": torch.full((max(s.P, 1),), -7, dtype=i32, device=DEV),
        "row_to_pair": torch.full((max(s.P, 1),), -7, dtype=i32, device=DEV),
        "Tej": torch.full((s.E, s.N), -7, dtype=i32, device=DEV),
        "D": torch.full((s.E, s.N, s.N), -7, dtype=i32, device=DEV),
        "status": torch.full((1,), -7, dtype=i32, device=DEV),
    }


def _case(T, E, k, N, c, seed):
    rng = np.random.default_rng(seed)
    shape = lz.Shape(T, 64, 64, E, k, N, c, lz.LZ_BF16, lz.LZ_GELU)
    bias = -1.1 * np.log(rng.permutation(E) + 1.0)
    ids, _ = om.route((rng.standard_normal((T, E)) + bias).astype(np.float32), k)
    off = np.array([(i * T) // N for i in range(N + 1)], dtype=np.int32)
    plan = rng.integers(0, E, size=N * c)
    plan[rng.permutation(N * c)[:E]] = np.arange(E)
    return shape, ids, off, plan.astype(np.int32)


def _run_both(shape, ids, off, plan):
    d_ids, d_off, d_plan = to_dev(ids), to_dev(off), to_dev(plan)
    a, b = _buffers(shape), _buffers(shape)
    nbytes = lz.lz_plan_workspace_bytes(shape)
    assert 0 < nbytes <= lz.LZ_PLAN_NOALLOC_SCRATCH_BYTES
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    lz.lz_plan_dispatch(d_ids, shape, d_off, d_plan, a["slot_counts"], a["slot_offsets"], a["pair_to_row"],
                        a["row_to_pair"], a["Tej"], a["D"], a["status"], ws, nbytes)
    lz.lz_plan_dispatch_noalloc(d_ids, shape, d_off, d_plan, b["slot_counts"], b["slot_offsets"],
                                b["pair_to_row"], b["row_to_pair"], b["Tej"], b["D"], b["status"])
    torch.cuda.synchronize()
    return {k: to_host(v) for k, v in a.items()}, {k: to_host(v) for k, v in b.items()}


def test_noalloc_dispatch_equals_the_workspace_entry_point_on_two_calls_in_a_row():
    # config 4's dispatch shape first (the largest tables of the five configs), then a smaller
    # input with ragged sizes, so the second call finds the first call's tables in the array
    for T, E, k, N, c, seed in ((16384, 64, 6, 16, 8, 4), (3001, 12, 3, 6, 8, 9)):
        print(f"noalloc dispatch: T={T} E={E} k={k} N={N} c={c} seed={seed}", flush=True)
        shape, ids, off, plan = _case(T, E, k, N, c, seed)
        want, got = _run_both(shape, ids, off, plan)
        assert want["status"][0] == 0 and got["status"][0] == 0
        for key in KEYS:
            assert np.array_equal(got[key], want[key]), (T, key)
        ref = om.plan_dispatch(ids, off, plan, E, N, c)
        for key in ("Tej", "D", "slot_counts", "slot_offsets", "pair_to_row", "row_to_pair"):
            assert np.array_equal(got[key], ref[key]), (T, key)


def test_noalloc_dispatch_rejects_shapes_beyond_its_array():
    big = lz.Shape(1 << 16, 64, 64, 256, 8, 64, 8, lz.LZ_BF16, lz.LZ_GELU)
    assert lz.lz_plan_workspace_bytes(big) > lz.LZ_PLAN_NOALLOC_SCRATCH_BYTES
    dummy = torch.zeros(16, dtype=torch.int32, device=DEV)
    with pytest.raises(lz.LzError) as e:
        lz.lz_plan_dispatch_noalloc(dummy, big, dummy, dummy, dummy, dummy, dummy, dummy, None, None, None)
    assert e.value.code == -3
