"""The allocation-free entry point (tm_gemm_w4a16_static: split-K scratch in a fixed array inside the library's device
image) against tm_gemm_w4a16 on the same inputs.  Same kernels and the same plan, so the outputs must agree bit for bit
(which also puts them inside the oracle tolerance the other tests establish for tm_gemm_w4a16).  Two calls in a row,
the second on a smaller input, then a shape that needs no scratch, then one beyond the array's size."""
import ctypes
import sys

import numpy as np
import pytest

from workloads import w4a16 as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _both(tm, torch, packed, X):
    Xd = gu.to_dev(X)
    M = X.shape[0]
    Ya = torch.full((M, packed.N), float("nan"), dtype=torch.float16, device="cuda")
    Yb = torch.full((M, packed.N), float("nan"), dtype=torch.float16, device="cuda")
    tm.tm_gemm_w4a16(Xd, packed, Ya)
    tm.tm_gemm_w4a16_static(Xd, packed, Yb)
    torch.cuda.synchronize()
    return Ya.cpu().numpy(), Yb.cpu().numpy()


def test_static_scratch_entry_point_matches_the_allocating_one():
    import torch
    import paper_2508_15601_amd as tm
    tm.load_library()
    # deep and narrow layers: too few column strips to fill the chip, so the plan splits K across CTAs and the
    # partial sums and arrival counters go through the scratch array
    big = wl.make(wl.Case("static_big", 48, 8192, 1024, 128, seed=11))
    small = wl.make(wl.Case("static_small", 12, 12800, 512, 64, seed=12))
    pb, ps = gu.pack(big, 128), gu.pack(small, 64)
    for name, packed, d, M in (("first", pb, big, 48), ("second, smaller", ps, small, 12), ("first again", pb, big, 20)):
        plan = tm.tm_get_plan(packed, M)
        _say(f"static entry point, {name}: M={M} K={packed.K} N={packed.N} plan={plan}")
        assert plan["split_k"] > 1, "the case is meant to use the scratch array"
        Ya, Yb = _both(tm, torch, packed, d["X"][:M])
        assert not np.isnan(Yb).any()
        assert np.array_equal(Ya.view(np.uint16), Yb.view(np.uint16)), name
    # a plan without split-K goes through untouched
    wide = wl.make(wl.Case("static_wide", 3, 512, 8192, 128, seed=13))
    pw = gu.pack(wide, 128)
    _say(f"static entry point, no split: plan={tm.tm_get_plan(pw, 3)}")
    Ya, Yb = _both(tm, torch, pw, wide["X"])
    assert np.array_equal(Ya.view(np.uint16), Yb.view(np.uint16))
    # beyond the array: refused with a message, nothing launched
    deep = wl.make(wl.Case("static_deep", 32, 2048, 8192, 128, seed=14))
    pd = gu.pack(deep, 128)
    tm.tm_set_variant(4, 16)                   # 64-column strips, K split sixteen ways: 16 MiB of partial sums
    try:
        need = tm.tm_gemm_workspace_bytes(pd, 32)
        _say(f"static entry point, oversize: needs {need} bytes, plan={tm.tm_get_plan(pd, 32)}")
        assert need > (8 << 20) + 65536
        Y = torch.full((32, 8192), float("nan"), dtype=torch.float16, device="cuda")
        with pytest.raises(tm.TmError) as err:
            tm.tm_gemm_w4a16_static(gu.to_dev(deep["X"]), pd, Y)
        assert "static buffer" in str(err.value)
        torch.cuda.synchronize()
        assert torch.isnan(Y).all()
    finally:
        tm.tm_set_variant(-1, 0)
    lib = tm.load_library()
    assert lib.tm_gemm_w4a16_static(None, None, None, 1, None) == -1
    for p in (pb, ps, pw, pd):
        p.close()
