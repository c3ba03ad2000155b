"""The grouped GEMM's home-queue assumption: workgroup b of a one-workgroup-per-CU launch runs on
the same XCD as every other workgroup with the same b % 8 (consecutive workgroups go to
consecutive XCDs).  Only cache locality depends on it; this test records what the machine does."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
import paper_2407_04656_amd as lz

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_workgroups_with_equal_index_mod_8_share_an_xcd():
    n = torch.cuda.get_device_properties(0).multi_processor_count // 8 * 8
    assert n >= 8
    out = torch.full((n,), -1, dtype=torch.int32, device=DEV)
    torch.cuda.synchronize()                      # an idle GPU: the hand-out starts from a fresh launch
    lz.lz_debug_xcc_ids(out, n)
    torch.cuda.synchronize()
    xcc = out.cpu().numpy()
    print("xcc ids of the first 16 workgroups:", xcc[:16].tolist())
    assert xcc.min() >= 0 and xcc.max() <= 7
    home = xcc[:8]
    assert sorted(home.tolist()) == list(range(8)), "8 consecutive workgroups cover the 8 XCDs"
    assert np.array_equal(xcc, np.tile(home, n // 8)), "b % 8 decides the XCD"


def test_xcc_ids_validates_arguments():
    with pytest.raises(lz.LzError) as ei:
        lz.lz_debug_xcc_ids(None, 8)
    assert ei.value.code == -1
    with pytest.raises(lz.LzError) as ei:
        lz.lz_debug_xcc_ids(None, -1)
    assert ei.value.code == -1
    lz.lz_debug_xcc_ids(None, 0)
