"""slicemoe_dispatch_noalloc (the dispatch with its scratch table in the library's own fixed device array, for callers
that cannot allocate) against slicemoe_dispatch, bit for bit, through the C ABI: two calls in a row, the second on a
smaller input, so that whatever the first call left in the shared array is there when the second runs."""
import ctypes

import numpy as np
import pytest

from paper_2510_04286_amd import workload as wl

pytestmark = pytest.mark.gpu

NAMES = ("counts_raw", "counts", "offsets", "perm", "inv")


def run(B, cfg, idx_dev, Na, no_alloc):
    import torch
    out = {n: torch.full((m,), -7, dtype=torch.int32, device="cuda:0")
           for n, m in [("counts_raw", cfg.E), ("counts", cfg.E), ("offsets", cfg.E + 1), ("perm", Na), ("inv", Na)]}
    if no_alloc:
        B.slicemoe_dispatch_noalloc(cfg, idx_dev, out["counts_raw"], out["counts"], out["offsets"], out["perm"], out["inv"])
    else:
        ws = torch.empty(B.slicemoe_dispatch_workspace_bytes(cfg), dtype=torch.uint8, device="cuda:0")
        B.slicemoe_dispatch(cfg, idx_dev, out["counts_raw"], out["counts"], out["offsets"], out["perm"], out["inv"], ws)
    torch.cuda.synchronize()
    return {n: t.cpu().numpy() for n, t in out.items()}


def test_dispatch_noalloc_matches_dispatch_on_two_calls_in_a_row():
    import torch
    assert torch.cuda.is_available(), "GPU tests need an MI355X"
    from paper_2510_04286_amd import binding as B
    B.lib()
    # a large call first (table scanned by its own kernel, capacity drop), then a smaller one (table summed by the
    # scatter blocks) that finds the first call's table in the array
    for T, S, k, E, cf, zipf in ((40000, 30, 2, 24, 1.2, 0.9), (3000, 16, 2, 32, 0.0, 0.4), (7, 3, 2, 5, 0.0, 0.0)):
        cfg = B.make_config(T, S * 64, S, k, E, 256, capacity_factor=cf)
        idx = wl.make_topk_idx(T * S, k, E, seed=5 + T, zipf_s=zipf)
        idx_dev = torch.from_numpy(np.ascontiguousarray(idx.reshape(-1))).to("cuda:0")
        got = run(B, cfg, idx_dev, T * S * k, True)
        ref = run(B, cfg, idx_dev, T * S * k, False)
        for n in NAMES:
            np.testing.assert_array_equal(got[n], ref[n], err_msg=f"{n} (T={T})")
        assert got["counts_raw"].sum() == T * S * k


def test_dispatch_noalloc_refuses_what_does_not_fit():
    import torch
    from paper_2510_04286_amd import binding as B
    L = B.lib()
    # 2^31 - 64 assignments with 64 experts would need a 32 MiB table: refused before anything is touched
    cfg = B.make_config((1 << 25) - 1, 64 * 32, 32, 2, 64, 256)
    dummy = ctypes.c_void_p(256)
    assert L.slicemoe_dispatch_noalloc(ctypes.byref(cfg), dummy, dummy, dummy, dummy, dummy, dummy, None) == B.SLICEMOE_ERR_WORKSPACE
    assert L.slicemoe_dispatch_noalloc(ctypes.byref(cfg), None, dummy, dummy, dummy, dummy, dummy, None) == B.SLICEMOE_ERR_INVALID_ARG
