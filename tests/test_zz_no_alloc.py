"""The allocation-free entry point, plogp_tune_grid_static, against plogp_tune_grid on the
same inputs through the C ABI: same decision table (ids and segment sizes equal, times
within 1e-12 relative; both run the same kernels, so the bytes are expected to be
identical), on calls in a row that share the one static scratch buffer, the later ones
with smaller inputs; a job that does not fit the buffer is refused before any launch."""
import numpy as np
import pytest

from plogp_workloads import ALL_STRATEGIES_MASK, Workload, make_workload
from tests.gpu_util import assert_tables_equal, stream_handle, torch_cuda

pytestmark = pytest.mark.gpu


def _both(wl):
    """(table by plogp_tune_grid, table by plogp_tune_grid_static) for one workload."""
    torch = torch_cuda()
    from paper_cs_0408034_amd import plogp
    tab = plogp.plogp_load_tables(wl.sizes, wl.gaps, wl.L)
    grid = plogp.plogp_grid_create(wl.m, wl.P, wl.s, wl.s_cap, wl.dtype_size, wl.strategy_mask)
    nbytes = plogp.plogp_decision_table_bytes(tab.count, grid)
    shape = (wl.n_tables, wl.n_ops, len(wl.m), len(wl.P))
    outs = []
    for fn in (plogp.plogp_tune_grid, plogp.plogp_tune_grid_static):
        out = torch.full((nbytes,), 0xCD, dtype=torch.uint8, device="cuda")
        fn(tab, grid, out.data_ptr(), nbytes, stream_handle())
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy().view(plogp.CELL_DTYPE).reshape(shape))
    grid.free()
    tab.free()
    return outs


def test_static_scratch_calls_in_a_row_match_the_allocating_entry_point():
    jobs = [
        # staged path, big table, long chain sums (prefix launch): 44 MB of scratch
        make_workload(5, m_slice=slice(0, 4096, 2), P_subset=None),
        # the same path on a much smaller input: stale contents of the larger call lie behind it
        make_workload(5, m_slice=slice(5, 4096, 37), P_subset=[2, 3, 64, 65, 66, 129, 4097, 40000, 65536]),
        # lanes over tables (batch scratch), then fewer tables
        make_workload(4, n_tables=300, table_offset=4000),
        make_workload(4, n_tables=70, table_offset=100, n_m=130),
        # many candidates: lanes over s, chain sums per row
        make_workload(3, m_slice=slice(0, 1024, 64)),
        # one workgroup per row (no scratch at all), and the smallest config
        make_workload(2, m_slice=slice(0, 1024, 4)),
        make_workload(1),
    ]
    for k, wl in enumerate(jobs):
        want, got = _both(wl)
        what = "job %d (%s: %d tables, %d m, %d P, %d s)" % (k, wl.name, wl.n_tables, len(wl.m), len(wl.P), len(wl.s))
        print(what, flush=True)
        assert assert_tables_equal(got, want, what), "times not bit-identical: " + what
        assert got.tobytes() == want.tobytes(), what


def test_static_scratch_refuses_a_job_that_does_not_fit():
    torch = torch_cuda()
    from paper_cs_0408034_amd import plogp
    base = make_workload(5)
    # 2200 process counts up to 65 536 x 3215 distinct sizes: the partial sums and the block
    # prefix alone are 113 MB, above the 64 MiB buffer
    P = np.concatenate([np.arange(2, 2201), [65536]]).astype(np.uint32)
    tab = plogp.plogp_load_tables(base.sizes, base.gaps, base.L)
    grid = plogp.plogp_grid_create(base.m, P, base.s, base.s_cap, base.dtype_size, ALL_STRATEGIES_MASK)
    nbytes = plogp.plogp_decision_table_bytes(1, grid)
    out = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(plogp.PlogpError) as e:
        plogp.plogp_tune_grid_static(tab, grid, out.data_ptr(), nbytes, stream_handle())
    assert e.value.status == plogp.ETOOBIG
    torch.cuda.synchronize()
    assert int(out.max().item()) == 0                   # nothing was launched
    # the argument checks of the allocating entry point hold here too
    with pytest.raises(plogp.PlogpError) as e:
        plogp.plogp_tune_grid_static(tab, grid, out.data_ptr() + 8, nbytes, stream_handle())
    assert e.value.status == plogp.EINVAL
    with pytest.raises(plogp.PlogpError) as e:
        plogp.plogp_tune_grid_static(tab, grid, out.data_ptr(), nbytes - 16, stream_handle())
    assert e.value.status == plogp.ENOSPC
    grid.free()
    tab.free()
    # and a small job right after the refusal runs
    wl = make_workload(1)
    want, got = _both(wl)
    assert got.tobytes() == want.tobytes()
