"""GPU parity of the cut-over extraction: plogp_cutovers (through the C ABI)
against the CPU oracle's plain definition, record for record (integer and
index work: everything must be identical)."""
import numpy as np
import pytest

import oracle
from oracle import plogp_cutover as oc
from plogp_workloads import make_workload
from tests.gpu_util import stream_handle, torch_cuda

pytestmark = pytest.mark.gpu


def _plogp():
    from paper_cs_0408034_amd import plogp
    return plogp


def gpu_cutovers(cells, m, P, key_mode, capacity=None, d_cells=None):
    """Runs plogp_cutovers on a decision table given as a host array
    [tables][ops][m][P] (or already on the device); returns (offsets, runs, total)."""
    torch = torch_cuda()
    plogp = _plogp()
    nt, n_ops, n_m, n_P = cells.shape
    # the grid handle carries the sizes, the number of process counts and of planes
    mask = plogp.MASK_ALL if n_ops == 2 else plogp.MASK_BCAST
    grid = plogp.plogp_grid_create(m, P, [], plogp.NO_CAP, 1, mask)
    rows = plogp.plogp_cutover_rows(nt, grid)
    assert rows == nt * n_ops * n_P
    if d_cells is None:
        d_cells = torch.from_numpy(np.ascontiguousarray(cells).view(np.uint8).reshape(-1)).cuda()
    cap = cells.size if capacity is None else capacity
    d_off = torch.full((rows + 1,), -1, dtype=torch.int64, device="cuda")
    d_runs = torch.full((max(cap, 1) * 16,), 0xEE, dtype=torch.uint8, device="cuda")
    plogp.plogp_cutovers(grid, nt, d_cells.data_ptr(), key_mode, d_off.data_ptr(),
                         d_runs.data_ptr() if cap else 0, cap, stream_handle())
    torch.cuda.synchronize()
    off = d_off.cpu().numpy().view(np.uint64)
    runs = d_runs.cpu().numpy().view(plogp.RUN_DTYPE)[:cap]
    grid.free()
    return off, runs


def random_table(rng, nt, n_ops, n_m, n_P, p_change):
    """A decision table whose key changes along m with probability p_change per cell."""
    cells = np.zeros((nt, n_ops, n_m, n_P), dtype=oracle.CELL_DTYPE)
    ids = rng.integers(0, 10, size=cells.shape).astype(np.uint32)
    seg = (rng.integers(0, 3, size=cells.shape) * 8).astype(np.uint32)
    keep = rng.random(cells.shape) >= p_change
    for mi in range(1, n_m):
        ids[:, :, mi, :] = np.where(keep[:, :, mi, :], ids[:, :, mi - 1, :], ids[:, :, mi, :])
        seg[:, :, mi, :] = np.where(keep[:, :, mi, :], seg[:, :, mi - 1, :], seg[:, :, mi, :])
    cells["strategy"], cells["s"] = ids, seg
    cells["time"] = rng.random(cells.shape)
    return cells


def check(cells, m, P, key_mode):
    want_off, want_runs = oc.cutovers(cells, m, key_mode)
    off, runs = gpu_cutovers(cells, m, P, key_mode)
    assert (off == want_off).all()
    total = int(off[-1])
    assert total == len(want_runs)
    assert (runs[:total] == want_runs).all()
    # nothing is written past the last run
    assert (runs[total:].view(np.uint8) == 0xEE).all()


@pytest.mark.parametrize("key_mode", [0, 1])
@pytest.mark.parametrize("shape,p_change", [
    ((1, 1, 1, 1), 0.5),          # a single cell
    ((1, 2, 1, 7), 0.5),          # one size: every row is one run
    ((2, 2, 37, 5), 0.3),         # fewer than 64 process counts, ragged last tile of sizes
    ((1, 1, 16, 64), 1.0),        # every cell starts a run, exactly one tile
    ((1, 2, 17, 65), 0.0),        # no change at all; one process count past a wave
    ((3, 1, 100, 130), 0.1),
    ((1, 2, 1000, 3), 0.02),
    ((40, 2, 33, 24), 0.2),       # many tables, config 4's 24 process counts
])
def test_random_tables_match_the_definition(shape, p_change, key_mode):
    rng = np.random.default_rng(hash((shape, key_mode)) % (1 << 32))
    nt, n_ops, n_m, n_P = shape
    m = np.cumsum(rng.integers(1, 50, size=n_m)).astype(np.uint64)
    if n_m > 3:
        m[2] = m[1]               # a repeated size is still its own cell
    P = (np.arange(n_P) + 2).astype(np.uint32)
    check(random_table(rng, nt, n_ops, n_m, n_P, p_change), m, P, key_mode)


def test_scan_over_many_groups():
    # more than 2048 * 1024 (row, tile) pieces: the second level of the prefix loops
    rng = np.random.default_rng(7)
    nt, n_ops, n_m, n_P = 700, 2, 16 * 25, 64
    cells = random_table(rng, nt, n_ops, n_m, n_P, 0.01)
    m = (np.arange(n_m) * 8 + 8).astype(np.uint64)
    P = (np.arange(n_P) + 2).astype(np.uint32)
    assert nt * n_ops * n_P * (n_m // 16) > 2048 * 1024
    check(cells, m, P, 1)


@pytest.mark.parametrize("key_mode", [0, 1])
@pytest.mark.parametrize("shape,p_change", [
    ((700, 2, 37, 24), 0.2),      # 33 600 rows: one thread per row; sizes end inside a flag word
    ((1100, 2, 33, 15), 0.5),     # 33 000 rows: the last workgroup is ragged
    ((300, 2, 257, 64), 0.03),    # more than 256 sizes: sixteen flag words, one size into the ninth
    ((180, 1, 512, 200), 0.01),   # the most sizes this path takes
    ((40000, 1, 1, 1), 0.5),      # one cell per row
    ((600, 2, 64, 30), 1.0),      # every cell starts a run
    ((600, 2, 64, 30), 0.0),      # one run per row
])
def test_tables_of_many_rows_take_one_pass_and_match_the_definition(shape, p_change, key_mode):
    rng = np.random.default_rng(hash((shape, key_mode, "rows")) % (1 << 32))
    nt, n_ops, n_m, n_P = shape
    m = np.cumsum(rng.integers(1, 50, size=n_m)).astype(np.uint64)
    P = (np.arange(n_P) + 2).astype(np.uint32)
    check(random_table(rng, nt, n_ops, n_m, n_P, p_change), m, P, key_mode)


@pytest.mark.timeout(300)
def test_full_size_of_config_4_random_decisions():
    """The shape the benchmark times: 10 000 tables x 2 operations x 256 sizes x 24 process
    counts (480 000 rows, one pass), with a run start in about 2 % of the cells as in the tuned
    table; every offset and every run against the definition."""
    rng = np.random.default_rng(41)
    nt, n_ops, n_m, n_P = 10000, 2, 256, 24
    cells = random_table(rng, nt, n_ops, n_m, n_P, 0.019)
    m = (np.arange(n_m, dtype=np.uint64) + 1) * 8
    P = (np.arange(n_P) + 2).astype(np.uint32)
    check(cells, m, P, 1)


def test_one_grid_handle_many_rows_then_fewer_then_many_again():
    """The same handle serves a batch on the one-pass path, a smaller one on the tiled path and
    the first again: whatever a call leaves in the handle's scratch, the next one starts clean."""
    torch = torch_cuda()
    plogp = _plogp()
    rng = np.random.default_rng(23)
    n_ops, n_m, n_P = 2, 40, 24
    m = (np.arange(n_m) * 8 + 8).astype(np.uint64)
    P = (np.arange(n_P) + 2).astype(np.uint32)
    grid = plogp.plogp_grid_create(m, P, [], plogp.NO_CAP, 1, plogp.MASK_ALL)
    big = random_table(rng, 800, n_ops, n_m, n_P, 0.1)
    for nt in (800, 5, 800, 799):
        cells = big[:nt]
        want_off, want_runs = oc.cutovers(cells, m, 1)
        rows = nt * n_ops * n_P
        d_cells = torch.from_numpy(np.ascontiguousarray(cells).view(np.uint8).reshape(-1)).cuda()
        d_off = torch.full((rows + 1,), -1, dtype=torch.int64, device="cuda")
        d_runs = torch.full((cells.size * 16,), 0xEE, dtype=torch.uint8, device="cuda")
        plogp.plogp_cutovers(grid, nt, d_cells.data_ptr(), 1, d_off.data_ptr(), d_runs.data_ptr(),
                             cells.size, stream_handle())
        torch.cuda.synchronize()
        off = d_off.cpu().numpy().view(np.uint64)
        assert (off == want_off).all(), nt
        runs = d_runs.cpu().numpy().view(plogp.RUN_DTYPE)
        assert (runs[:len(want_runs)] == want_runs).all(), nt
        assert (runs[len(want_runs):].view(np.uint8) == 0xEE).all(), nt
    grid.free()


def test_capacity_smaller_than_the_number_of_runs_on_the_one_pass_path():
    rng = np.random.default_rng(29)
    cells = random_table(rng, 700, 2, 20, 24, 0.3)
    m = (np.arange(20) * 8 + 8).astype(np.uint64)
    P = (np.arange(24) + 2).astype(np.uint32)
    want_off, want_runs = oc.cutovers(cells, m, 0)
    cap = len(want_runs) // 3
    off, runs = gpu_cutovers(cells, m, P, 0, capacity=cap)
    assert (off == want_off).all() and int(off[-1]) > cap
    assert (runs == want_runs[:cap]).all()
    off, runs = gpu_cutovers(cells, m, P, 0, capacity=0)
    assert (off == want_off).all()


def test_capacity_smaller_than_the_number_of_runs_and_count_only():
    rng = np.random.default_rng(11)
    cells = random_table(rng, 2, 2, 50, 9, 0.5)
    m = (np.arange(50) * 8 + 8).astype(np.uint64)
    P = (np.arange(9) + 2).astype(np.uint32)
    want_off, want_runs = oc.cutovers(cells, m, 1)
    cap = len(want_runs) // 3
    off, runs = gpu_cutovers(cells, m, P, 1, capacity=cap)
    assert (off == want_off).all() and int(off[-1]) > cap
    assert (runs == want_runs[:cap]).all()
    off, runs = gpu_cutovers(cells, m, P, 1, capacity=0)
    assert (off == want_off).all()


@pytest.mark.parametrize("cfg,kw", [(1, {}), (2, dict(m_slice=slice(0, 1024, 4))),
                                    (4, dict(n_tables=7)), (5, dict(m_slice=slice(0, 4096, 16)))])
@pytest.mark.parametrize("key_mode", [0, 1])
def test_decision_tables_of_the_configs(cfg, kw, key_mode):
    """The oracle's decision table of a config, compressed on the GPU, equals the oracle's runs."""
    wl = make_workload(cfg, **kw)
    cells, _ = oracle.tune_workload(wl)
    check(cells, wl.m, wl.P, key_mode)


def test_tune_then_extract_on_the_device_full_config_2():
    """The headline configuration at full size: sweep and extraction chained on the device,
    checked against the oracle's runs of the oracle's table."""
    torch = torch_cuda()
    plogp = _plogp()
    wl = make_workload(2)
    tab = plogp.plogp_load_tables(wl.sizes, wl.gaps, wl.L)
    grid = plogp.plogp_grid_create(wl.m, wl.P, wl.s, wl.s_cap, wl.dtype_size, wl.strategy_mask)
    nbytes = plogp.plogp_decision_table_bytes(tab.count, grid)
    out = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    rows = plogp.plogp_cutover_rows(1, grid)
    d_off = torch.zeros(rows + 1, dtype=torch.int64, device="cuda")
    cap = nbytes // 16
    d_runs = torch.zeros(cap * 16, dtype=torch.uint8, device="cuda")
    sh = stream_handle()
    plogp.plogp_tune_grid(tab, grid, out.data_ptr(), nbytes, sh)
    plogp.plogp_cutovers(grid, 1, out.data_ptr(), 1, d_off.data_ptr(), d_runs.data_ptr(), cap, sh)
    torch.cuda.synchronize()
    want_cells, _ = oracle.tune_workload(wl)
    want_off, want_runs = oc.cutovers(want_cells, wl.m, 1)
    off = d_off.cpu().numpy().view(np.uint64)
    assert (off == want_off).all()
    runs = d_runs.cpu().numpy().view(plogp.RUN_DTYPE)[:int(off[-1])]
    assert (runs == want_runs).all()
    grid.free()
    tab.free()


def test_bad_arguments_are_refused():
    torch = torch_cuda()
    plogp = _plogp()
    grid = plogp.plogp_grid_create([8, 16], [2, 3], [], plogp.NO_CAP, 1, plogp.MASK_BCAST)
    buf = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()
    lib = plogp._lib
    assert lib.plogp_cutovers(grid._h, 1, p, 2, p, p, 4, None) == plogp.EINVAL        # key mode
    assert lib.plogp_cutovers(grid._h, 0, p, 0, p, p, 4, None) == plogp.EINVAL        # no table
    assert lib.plogp_cutovers(grid._h, 1, p + 8, 0, p, p, 4, None) == plogp.EINVAL    # misaligned
    assert lib.plogp_cutovers(grid._h, 1, p, 0, p, None, 4, None) == plogp.EINVAL     # no room
    assert lib.plogp_cutovers(None, 1, p, 0, p, p, 4, None) == plogp.EINVAL
    grid.free()
