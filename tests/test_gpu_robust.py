"""GPU parity of the robustness summary: plogp_robustness (through the C ABI) against
the CPU oracle's plain definition.  Counts are integers and the largest deviation is a
maximum of correctly rounded quotients, so everything must be identical."""
import numpy as np
import pytest

import oracle
from oracle import plogp_robust as orb
from plogp_workloads import make_perturbed, make_workload
from tests.gpu_util import gpu_tune, stream_handle, torch_cuda

pytestmark = pytest.mark.gpu


def _plogp():
    from paper_cs_0408034_amd import plogp
    return plogp


def gpu_robustness(cells, key_mode, with_dev=True, with_tables=True, d_cells=None):
    """plogp_robustness on decision tables given as a host array [tables][ops][m][P]."""
    torch = torch_cuda()
    plogp = _plogp()
    nt, n_ops, n_m, n_P = cells.shape
    mask = plogp.MASK_ALL if n_ops == 2 else plogp.MASK_BCAST
    grid = plogp.plogp_grid_create(np.arange(1, n_m + 1, dtype=np.uint64) * 8,
                                   np.arange(2, n_P + 2, dtype=np.uint32), [], plogp.NO_CAP, 1, mask)
    if d_cells is None:
        d_cells = torch.from_numpy(np.ascontiguousarray(cells).view(np.uint8).reshape(-1)).cuda()
    n = n_ops * n_m * n_P
    d_agree = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    d_dev = torch.full((n,), float("nan"), dtype=torch.float64, device="cuda")
    d_tab = torch.full((nt,), -7, dtype=torch.int32, device="cuda")
    plogp.plogp_robustness(grid, nt, d_cells.data_ptr(), key_mode, d_agree.data_ptr(),
                           d_dev.data_ptr() if with_dev else 0, d_tab.data_ptr() if with_tables else 0,
                           stream_handle())
    torch.cuda.synchronize()
    grid.free()
    agree = d_agree.cpu().numpy().view(np.uint32).reshape(n_ops, n_m, n_P)
    dev = d_dev.cpu().numpy().reshape(n_ops, n_m, n_P)
    tab = d_tab.cpu().numpy().view(np.uint32)
    return agree, dev, tab


def random_cells(rng, nt, n_ops, n_m, n_P, p_same):
    cells = np.zeros((nt, n_ops, n_m, n_P), dtype=oracle.CELL_DTYPE)
    cells["strategy"] = rng.integers(0, 13, size=cells.shape)
    cells["s"] = rng.integers(0, 3, size=cells.shape) * 8
    cells["time"] = rng.random(cells.shape) * 100 + 1
    keep = rng.random(cells.shape) < p_same
    for name in ("strategy", "s"):
        cells[name] = np.where(keep, cells[name][:1], cells[name])
    return cells


def check(cells, key_mode):
    want_a, want_d, want_t = orb.robustness(cells, key_mode)
    agree, dev, tab = gpu_robustness(cells, key_mode)
    assert (agree == want_a).all()
    assert (tab == want_t).all()
    assert (dev.view(np.uint64) == want_d.view(np.uint64)).all()


@pytest.mark.parametrize("key_mode", [0, 1])
@pytest.mark.parametrize("shape,p_same", [
    ((1, 1, 1, 1), 0.5),           # the reference alone: nothing to compare with
    ((2, 1, 1, 1), 0.5),
    ((5, 2, 3, 7), 0.5),           # fewer cells than a wave, a ragged slice of tables
    ((6, 2, 37, 5), 0.0),          # nobody agrees
    ((9, 1, 16, 64), 1.0),         # everybody agrees
    ((131, 2, 9, 31), 0.7),        # many tables over a small grid: slices of tables meet in atomics
    ((3, 2, 100, 130), 0.8),       # many cells, few tables
    ((40, 2, 33, 24), 0.6),
])
def test_random_tables(shape, p_same, key_mode):
    check(random_cells(np.random.default_rng(sum(shape) + key_mode), *shape, p_same=p_same), key_mode)


def test_optional_outputs_are_left_alone():
    cells = random_cells(np.random.default_rng(3), 7, 2, 11, 13, 0.5)
    want_a, _, _ = orb.robustness(cells, 1)
    agree, dev, tab = gpu_robustness(cells, 1, with_dev=False, with_tables=False)
    assert (agree == want_a).all()
    assert np.isnan(dev).all() and (tab.view(np.int32) == -7).all()


def test_degenerate_times():
    cells = np.zeros((3, 1, 1, 2), dtype=oracle.CELL_DTYPE)
    cells["time"][:, 0, 0, 0] = [0.0, 0.0, 0.0]
    cells["time"][:, 0, 0, 1] = [0.0, 1.0, 2.0]
    check(cells, 0)


def test_perturbed_parameters_end_to_end():
    """Config 1's table and 200 perturbed copies (10 % on every gap and on L): the oracle's
    tuning goes through both summaries; the library's own tuning of the same batch (the
    table-lane path) followed by its summary gives the same answer."""
    torch = torch_cuda()
    wl = make_perturbed(make_workload(1), 200, 0.1, seed=2)
    cells, _ = oracle.tune_workload(wl)
    check(cells, 0)
    check(cells, 1)
    want_a, want_d, want_t = orb.robustness(cells, 1)
    mine = gpu_tune(wl)
    d_cells = torch.from_numpy(np.ascontiguousarray(mine).view(np.uint8).reshape(-1)).cuda()
    agree, dev, tab = gpu_robustness(mine, 1, d_cells=d_cells)
    assert (agree == want_a).all() and (tab == want_t).all()
    assert (np.abs(dev - want_d) <= 1e-11).all()
    frac = agree / 200.0
    assert 0.5 < frac.mean() < 1.0


def test_bad_arguments_are_refused():
    torch = torch_cuda()
    plogp = _plogp()
    grid = plogp.plogp_grid_create([8, 16], [2, 3], [], plogp.NO_CAP, 1, plogp.MASK_ALL)
    buf = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()
    lib = plogp._lib
    assert lib.plogp_robustness(grid._h, 0, p, 0, p, None, None, None) == plogp.EINVAL
    assert lib.plogp_robustness(grid._h, 2, p, 2, p, None, None, None) == plogp.EINVAL
    assert lib.plogp_robustness(grid._h, 2, p + 8, 0, p, None, None, None) == plogp.EINVAL
    assert lib.plogp_robustness(grid._h, 2, p, 0, None, None, None, None) == plogp.EINVAL
    assert lib.plogp_robustness(grid._h, 2, p, 0, p, p + 4, None, None) == plogp.EINVAL
    grid.free()
