"""The tuning call under HIP graph capture: after a first (eager) call has sized the grid
handle's scratch, plogp_tune_grid and plogp_cutovers only launch kernels, so a caller can
capture them once and replay the graph.  Every replay must give the eager result."""
import numpy as np
import pytest

import oracle
from plogp_workloads import make_workload
from tests.gpu_util import assert_tables_equal, torch_cuda

pytestmark = pytest.mark.gpu


# (700 tables of config 4: the kernel whose lanes run over tables, and 33 600 rows for the
# one-pass extraction, whose workgroup counter and status words a small kernel clears)
@pytest.mark.parametrize("cfg,kw", [(1, {}), (2, dict(m_slice=slice(0, 1024, 9))), (4, dict(n_tables=700))])
def test_tune_and_cutovers_replayed_from_a_graph(cfg, kw):
    torch = torch_cuda()
    from paper_cs_0408034_amd import plogp
    wl = make_workload(cfg, **kw)
    want, _ = oracle.tune_workload(wl)
    tab = plogp.plogp_load_tables(wl.sizes, wl.gaps, wl.L)
    grid = plogp.plogp_grid_create(wl.m, wl.P, wl.s, wl.s_cap, wl.dtype_size, wl.strategy_mask)
    nbytes = plogp.plogp_decision_table_bytes(tab.count, grid)
    n_cells = nbytes // 16
    rows = plogp.plogp_cutover_rows(tab.count, grid)
    out = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    d_off = torch.zeros(rows + 1, dtype=torch.int64, device="cuda")
    d_runs = torch.zeros(n_cells * 16, dtype=torch.uint8, device="cuda")

    def step(stream_handle):
        plogp.plogp_tune_grid(tab, grid, out.data_ptr(), nbytes, stream_handle)
        plogp.plogp_cutovers(grid, tab.count, out.data_ptr(), plogp.KEY_STRATEGY_AND_SEGMENT,
                             d_off.data_ptr(), d_runs.data_ptr(), n_cells, stream_handle)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step(side.cuda_stream)                       # eager: sizes the scratch
    side.synchronize()
    eager_off = d_off.cpu().numpy().copy()
    eager_runs = d_runs.cpu().numpy().copy()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(torch.cuda.current_stream().cuda_stream)
    for k in range(3):
        out.fill_(0xCD)                              # the program's own eager work in between
        d_off.fill_(-1)
        d_runs.fill_(0xEE)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = out.cpu().numpy().view(plogp.CELL_DTYPE).reshape(want.shape)
        assert assert_tables_equal(got, want, "replay %d" % k)
        assert (d_off.cpu().numpy() == eager_off).all()
        total = int(eager_off[-1])
        assert (d_runs.cpu().numpy()[: total * 16] == eager_runs[: total * 16]).all()
    del graph
    grid.free()
    tab.free()
