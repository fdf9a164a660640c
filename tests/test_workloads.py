"""Host logic of the seeded input generators (no GPU): block boundaries, schedules, the partition by relation."""
import numpy as np

from paper_2002_00655_amd import workloads as wl


def test_bounds_cover_the_range_and_balanced_ones_balance():
    w = wl.make_mf("tiny", scale=0.5, seed=4, col=1.0)
    d = 7
    for ids, size in ((w.rows, w.m), (w.cols, w.n)):
        eq, bal = wl.equal_bounds(size, d), wl.balanced_bounds(ids, size, d)
        for b in (eq, bal):
            assert b[0] == 0 and b[-1] == size and b.size == d + 1 and np.all(np.diff(b) >= 0)
        assert np.array_equal(eq, np.arange(d + 1) * size // d)
        per_range = np.add.reduceat(np.bincount(ids, minlength=size), bal[:-1])
        heaviest = np.bincount(ids, minlength=size).max()
        assert per_range.max() - per_range.min() <= 2 * heaviest          # no range is off by more than a couple of ids
        # with a weight per id on top of its entries, the ranges have equal weight instead
        per_id = 25.0
        wb = wl.balanced_bounds(ids, size, d, per_id=per_id)
        assert wb[0] == 0 and wb[-1] == size and wb.size == d + 1 and np.all(np.diff(wb) >= 0)
        weight = np.add.reduceat(np.bincount(ids, minlength=size) + per_id, wb[:-1])
        assert weight.max() - weight.min() <= 2 * (heaviest + per_id)
        # and a very large weight per id makes them ranges of equal length
        assert np.abs(wl.balanced_bounds(ids, size, d, per_id=1e9) - eq).max() <= 1


def test_balanced_bounds_set_heavy_indices_apart():
    """An index with more entries than an average range has gets a range of its own; every range is non-empty and the
    others share what is left evenly; with too few ranges for that the plain cut by weight is used."""
    rng = np.random.default_rng(0)
    size, d = 1000, 16
    deg = rng.integers(1, 50, size=size)
    heavy = [0, 1, 500, 999]
    deg[heavy] = [5000, 4000, 9000, 7000]
    ids = np.repeat(np.arange(size), deg)
    for per_id in (0.0, 3.0):
        b = wl.balanced_bounds(ids, size, d, per_id=per_id)
        assert b[0] == 0 and b[-1] == size and b.size == d + 1 and np.all(np.diff(b) > 0)
        for h in heavy:
            assert h in b and h + 1 in b
        per_range = np.add.reduceat(deg, b[:-1])
        rest = np.array([x for x, lo in zip(per_range, b[:-1]) if lo not in heavy])
        # the stretches between the heavy indices get whole numbers of ranges: alike within a few per cent
        assert rest.max() <= 1.15 * rest.min()
    # three indices with all the entries and four ranges: no way to set them all apart
    ids3 = np.repeat([0, 5, 9], [100, 100, 100])
    b = wl.balanced_bounds(ids3, 10, 4)
    assert b[0] == 0 and b[-1] == 10 and b.size == 5 and np.all(np.diff(b) >= 0)
    # ... with eight there is: each alone, the stretches between them cut further
    b = wl.balanced_bounds(ids3, 10, 8)
    assert b.size == 9 and all(x in b for x in (0, 1, 5, 6, 9, 10)) and np.all(np.diff(b) >= 0)


def test_schedules_are_strata():
    rng = np.random.default_rng(0)
    for sched in (wl.cyclic_schedule(6), wl.random_schedule(6, rng)):
        seen = set()
        for stratum in sched:
            workers, rbs, cbs = stratum[:, 0], stratum[:, 1], stratum[:, 2]
            for x in (workers, rbs, cbs):
                assert sorted(x.tolist()) == list(range(6))                # no worker, row block or column block twice
            seen |= {(int(r), int(c)) for r, c in zip(rbs, cbs)}
        assert len(seen) == 36                                             # every block once per epoch


def test_workloads_are_reproducible_and_shaped_as_stated():
    a, b = wl.make_mf("tiny", seed=3), wl.make_mf("tiny", seed=3)
    assert np.array_equal(a.rows, b.rows) and np.array_equal(a.vals, b.vals) and np.array_equal(a.W0, b.W0)
    assert a.nnz == 100_000 and a.rank == 16 and (a.m, a.n) == (1000, 1000)
    cells = a.rows.astype(np.int64) * a.n + a.cols
    assert np.unique(cells).size == a.nnz and np.all(np.diff(cells) > 0)   # distinct cells, sorted by (row, column)
    k = wl.make_kge(num_entities=300, num_relations=5, triples=400, dim=8, n_neg_s=2, n_neg_o=3, seed=1)
    assert k.neg_subj.shape == (400, 2) and k.neg_obj.shape == (400, 3) and k.E0.shape == (300, 16) and k.R0.shape == (5, 16)
    assert k.subj.max() < 300 and k.rel.max() < 5
    kp, part_ptr = wl.partition_by_relation(k, 3)
    assert part_ptr[0] == 0 and part_ptr[-1] == 400 and sorted(kp.subj.tolist()) == sorted(k.subj.tolist())
    sizes = np.diff(part_ptr)
    assert sizes.max() - sizes.min() <= np.bincount(k.rel).max()           # relations are dealt to the least loaded worker
