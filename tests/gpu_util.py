"""Helpers of the GPU parity tests: run a workload through the C-ABI library
(via the thin binding) and compare decision tables with the CPU oracle."""
from __future__ import annotations

import numpy as np

REL_TOL = 1e-12     # bar for predicted times (binary64); ids and s must be equal


def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def stream_handle():
    torch = torch_cuda()
    return torch.cuda.current_stream().cuda_stream


def gpu_tune(wl, keep=None):
    """Decision table [n_tables, n_ops, n_m, n_P] of workload wl from the HIP library."""
    torch = torch_cuda()
    from paper_cs_0408034_amd import plogp
    tab = plogp.plogp_load_tables(wl.sizes, wl.gaps, wl.L)
    grid = plogp.plogp_grid_create(wl.m, wl.P, wl.s, wl.s_cap, wl.dtype_size, wl.strategy_mask)
    nbytes = plogp.plogp_decision_table_bytes(tab.count, grid)
    assert nbytes == wl.n_cells * 16
    out = torch.full((nbytes,), 0xAB, dtype=torch.uint8, device="cuda")
    plogp.plogp_tune_grid(tab, grid, out.data_ptr(), nbytes, stream_handle())
    torch.cuda.synchronize()
    arr = out.cpu().numpy().view(plogp.CELL_DTYPE).reshape(wl.n_tables, wl.n_ops, len(wl.m), len(wl.P))
    if keep is not None:
        keep.extend([tab, grid])
    else:
        grid.free()
        tab.free()
    return arr


def assert_tables_equal(got, want, what=""):
    """ids and segment sizes equal; times within REL_TOL (and report bit equality)."""
    assert got.shape == want.shape, (got.shape, want.shape)
    bad_id = got["strategy"] != want["strategy"]
    bad_s = got["s"] != want["s"]
    if bad_id.any() or bad_s.any():
        idx = np.argwhere(bad_id | bad_s)[:5]
        lines = ["%s: %d cells differ in strategy, %d in s" % (what, bad_id.sum(), bad_s.sum())]
        for ix in idx:
            ix = tuple(ix)
            lines.append("  cell %s: got %s want %s" % (ix, got[ix], want[ix]))
        raise AssertionError("\n".join(lines))
    gt, wt = got["time"], want["time"]
    both_inf = np.isinf(gt) & np.isinf(wt)
    with np.errstate(invalid="ignore"):
        err = np.where(both_inf, 0.0, np.abs(gt - wt) / np.maximum(np.abs(wt), 1e-300))
    assert (err <= REL_TOL).all(), "%s: max relative time error %g" % (what, err.max())
    return bool((gt.view(np.uint64) == wt.view(np.uint64)).all())
