"""GPU parity of the rows beyond Tables 1 and 2 - Gather (ids 13..15) and Barrier (16, 17) -
through the C ABI against the CPU oracle: each row alone at random points, the planes of the
tuned table on slices of the five configs and on random jobs with random 18-bit masks, and the
steps that consume a decision table (cut-over extraction, robustness) on a table of four planes."""
import numpy as np
import pytest

import oracle
from oracle import plogp_cutover as oc
from plogp_workloads import NO_CAP, Workload, make_workload
from tests.gpu_util import REL_TOL, assert_tables_equal, gpu_tune, stream_handle, torch_cuda
from tests.test_gpu_parity import _dev, _random_problem

pytestmark = pytest.mark.gpu
EVERY = 0x3FFFF


def _plogp():
    from paper_cs_0408034_amd import plogp
    return plogp


@pytest.mark.parametrize("cfg", [2, 5])
def test_gather_and_barrier_rows_at_random_points(cfg):
    torch = torch_cuda()
    plogp = _plogp()
    wl = make_workload(cfg)
    x, y, L = wl.sizes[0], wl.gaps[0], float(wl.L[0])
    tab = plogp.plogp_load_table(x, y, L)
    rng = np.random.default_rng(80 + cfg)
    n = 500
    m = rng.choice(wl.m, size=n)
    P = rng.choice(wl.P[wl.P <= 3000], size=n).astype(np.uint32)
    P[:8] = [2, 3, 64, 65, 66, 128, 129, 2049]
    dm, dP = _dev(m, np.uint64), _dev(P, np.uint32)
    out = torch.empty(n, dtype=torch.float64, device="cuda")
    for sid in range(13, 18):
        plogp.plogp_eval_strategy(tab, 0, sid, dm.data_ptr(), dP.data_ptr(), 0, n, out.data_ptr(), stream_handle())
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        want = np.array([oracle.eval_strategy(x, y, L, sid, int(m[i]), int(P[i])) for i in range(n)])
        assert (np.abs(got - want) <= REL_TOL * np.abs(want)).all(), sid
        assert (got.view(np.uint64) == want.view(np.uint64)).all(), "strategy %d not bit-exact" % sid
    tab.free()


def _with_mask(wl, mask):
    return Workload(wl.name, wl.sizes, wl.gaps, wl.L, wl.m, wl.P, wl.s, wl.s_cap, mask)


@pytest.mark.parametrize("cfg,kw", [
    (1, {}),
    (2, dict(m_slice=slice(0, 1024, 16))),
    (3, dict(m_slice=slice(5, 1024, 128))),
    (4, dict(n_tables=70, table_offset=3000)),
    (5, dict(m_slice=slice(3, 4096, 64))),
])
def test_four_planes_on_slices_of_the_configs(cfg, kw):
    wl = _with_mask(make_workload(cfg, **kw), EVERY if cfg != 1 else 0xA9 | 0x3E000)
    assert wl.n_ops == (4 if cfg != 1 else 3)
    want, _ = oracle.tune_workload(wl)
    got = gpu_tune(wl)
    assert assert_tables_equal(got, want, "cfg%d with Gather and Barrier" % cfg), "times not bit-identical"
    # the planes of Tables 1 and 2 are what they are without the other rows
    base = _with_mask(wl, wl.strategy_mask & 0x1FFF)
    assert got[:, :base.n_ops].tobytes() == gpu_tune(base).tobytes()


@pytest.mark.parametrize("mask", [0xE000, 0x30000, 1 << 14, (1 << 15) | (1 << 16), (1 << 14) | 0x1400, 0x3E000,
                                  (1 << 13) | (1 << 17) | 0x3FF])
def test_subsets_of_the_new_rows(mask):
    # a Gather chain row without the Scatter chain row still needs the chain sums; a plane exists
    # only if one of its rows is enabled
    for base in (make_workload(2, m_slice=slice(3, 1024, 53), P_subset=[2, 3, 5, 64, 65, 66, 127, 129, 700, 1024]),
                 make_workload(5, m_slice=slice(9, 4096, 301), P_subset=[2, 65, 4097, 40000, 65536])):
        wl = _with_mask(base, mask)
        want, _ = oracle.tune_workload(wl)
        assert assert_tables_equal(gpu_tune(wl), want, "mask %#x" % mask)


@pytest.mark.parametrize("mask", [
    EVERY,                                           # four planes, the Gather rows as the Scatter rows
    0x3FF | 0xE000,                                  # Broadcast and Gather, no Scatter plane
    (1 << 10) | (1 << 12) | (1 << 13) | (1 << 15),   # two Scatter rows and their two Gather twins
    0x1C00 | 0x30000,                                # Scatter and Barrier
    0x3FF | (1 << 16),                               # Broadcast and the flat Barrier alone
    (1 << 14) | (1 << 17),                           # the Gather chain row and the binomial Barrier, nothing else
    0x30000,                                         # a Barrier plane alone
    0x1FFF | (1 << 14),                              # Gather rows unlike the Scatter rows: the staged path
])
def test_batches_of_tables_that_share_their_sizes(mask):
    """100 tables of config 4 (a full group of 64 lanes and a ragged one of 36): the kernel whose
    lanes run over tables writes the Gather and Barrier planes itself."""
    wl = _with_mask(make_workload(4, n_tables=100, table_offset=500), mask)
    want, _ = oracle.tune_workload(wl)
    got = gpu_tune(wl)
    assert assert_tables_equal(got, want, "100 tables, mask %#x" % mask), "times not bit-identical"


def test_batch_with_process_counts_that_do_not_fill_a_group_of_eight():
    # 21 process counts: the last store of a row covers five cells; 200 sizes: a ragged chunk
    base = make_workload(4, n_tables=70, n_m=200)
    wl = Workload(base.name, base.sizes, base.gaps, base.L, base.m, base.P[:21], base.s, base.s_cap, EVERY)
    want, _ = oracle.tune_workload(wl)
    assert assert_tables_equal(gpu_tune(wl), want, "70 tables, 21 process counts"), "times not bit-identical"


@pytest.mark.parametrize("seed", range(6))
def test_random_problems_with_random_masks(seed):
    rng = np.random.default_rng(9000 + seed)
    for k in range(6):
        wl = _random_problem(rng)
        wl.strategy_mask = int(rng.choice([EVERY, EVERY, 0x3E000 | (wl.strategy_mask & 0x1FFF), int(rng.integers(1, 1 << 18))]))
        want, _ = oracle.tune_workload(wl)
        what = "random %d/%d: n=%d tables=%d m=%d P=%d s=%d mask=%#x" % (
            seed, k, wl.sizes.shape[1], wl.n_tables, len(wl.m), len(wl.P), len(wl.s), wl.strategy_mask)
        print(what, flush=True)
        assert_tables_equal(gpu_tune(wl), want, what)


def test_cutovers_and_robustness_of_a_table_of_four_planes():
    torch = torch_cuda()
    plogp = _plogp()
    from oracle import plogp_robust as orb
    wl = _with_mask(make_workload(4, n_tables=9, table_offset=40, n_m=90), EVERY)
    keep = []
    cells = gpu_tune(wl, keep=keep)
    tab, grid = keep
    assert grid.ops == 4
    d_cells = torch.from_numpy(cells.view(np.uint8).reshape(-1)).cuda()
    rows = plogp.plogp_cutover_rows(tab.count, grid)
    assert rows == wl.n_tables * 4 * len(wl.P)
    d_off = torch.empty(rows + 1, dtype=torch.int64, device="cuda")
    d_runs = torch.empty(cells.size * 16, dtype=torch.uint8, device="cuda")
    plogp.plogp_cutovers(grid, tab.count, d_cells.data_ptr(), plogp.KEY_STRATEGY_AND_SEGMENT, d_off.data_ptr(),
                         d_runs.data_ptr(), cells.size, stream_handle())
    torch.cuda.synchronize()
    want_off, want_runs = oc.cutovers(cells, wl.m, 1)
    off = d_off.cpu().numpy().astype(np.uint64)
    assert (off == want_off).all()
    runs = d_runs.cpu().numpy().view(plogp.RUN_DTYPE)[: int(off[-1])]
    assert runs.tobytes() == want_runs.tobytes()
    per_table = cells[0].size
    d_agree = torch.empty(per_table, dtype=torch.int32, device="cuda")
    plogp.plogp_robustness(grid, tab.count, d_cells.data_ptr(), plogp.KEY_STRATEGY, d_agree.data_ptr(), 0, 0,
                           stream_handle())
    torch.cuda.synchronize()
    want_agree = orb.robustness(cells, 0)[0]
    assert (d_agree.cpu().numpy().astype(np.uint32).reshape(want_agree.shape) == want_agree).all()
    grid.free(); tab.free()
