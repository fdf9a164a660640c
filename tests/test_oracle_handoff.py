"""An epoch in which column blocks pass from worker to worker without barriers (the asynchronous form of the
blocked schedule, Sec. 2.2.2) is replayed on the oracle as strata of mf_sgd_epoch.  What pins the replay: blocks
that share neither a row block nor a column block touch disjoint parameters, so every sequence that keeps each
worker's order and each column block's order must give the same state bit for bit - and a sequence that breaks one
of the two orders must not."""
import numpy as np
import pytest

from paper_2002_00655_amd import workloads as wl
from _util import oracle_epochs, check_handoff_order, replay_schedule, simulate_handoff


def _setup(d_row, d_col, seed=3):
    from oracle.oracle import mf_block_ratings
    w = wl.make_mf("tiny", scale=0.6, seed=seed)
    rb, cb = wl.balanced_bounds(w.rows, w.m, d_row), wl.equal_bounds(w.n, d_col)
    return w, rb, cb, mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)


def _state(orc):
    return orc.pull(np.arange(orc.K)), orc.owner(), orc.stats()


@pytest.mark.parametrize("d_row,d_col", [(4, 4), (3, 7), (5, 2)])
def test_simulated_orders_are_valid_and_replays_agree(d_row, d_col):
    w, rb, cb, blocked = _setup(d_row, d_col)
    rng = np.random.default_rng(d_row * 10 + d_col)
    order = simulate_handoff(d_row, d_col, rng)
    check_handoff_order(order)
    levels = replay_schedule(order)
    assert sum(len(s) for s in levels) == d_row * d_col
    for prec in ("f32", "f64"):
        ref = _state(oracle_epochs(prec, w, rb, cb, blocked, levels))
        for _ in range(3):
            serial = replay_schedule(order, rng)
            assert len(serial) == d_row * d_col
            got = _state(oracle_epochs(prec, w, rb, cb, blocked, serial))
            assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1]) and got[2] == ref[2]


def test_rotation_is_one_of_the_orders():
    """The rotating schedule with barriers is the order 'worker w has column block (w + s) mod d at step s'."""
    d = 4
    w, rb, cb, blocked = _setup(d, d)
    order = np.empty((d, d, 2), dtype=np.int32)
    for b in range(d):
        for s in range(d):
            c = (b + s) % d
            order[b, s] = (c, s)                  # stratum s is every column block's visit number s
    check_handoff_order(order)
    ref = _state(oracle_epochs("f32", w, rb, cb, blocked, wl.cyclic_schedule(d)))
    got = _state(oracle_epochs("f32", w, rb, cb, blocked, replay_schedule(order, np.random.default_rng(0))))
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1]) and got[2] == ref[2]


def test_breaking_a_column_blocks_order_changes_the_result():
    d = 3
    w, rb, cb, blocked = _setup(d, d, seed=5)
    rng = np.random.default_rng(1)
    order = simulate_handoff(d, d, rng)
    good = replay_schedule(order, rng)
    ref = _state(oracle_epochs("f64", w, rb, cb, blocked, good))
    # swap two tasks on the same column block
    c = int(good[0][0, 2])
    idx = [i for i, s in enumerate(good) if s[0, 2] == c]
    bad = list(good)
    bad[idx[0]], bad[idx[1]] = bad[idx[1]], bad[idx[0]]
    got = _state(oracle_epochs("f64", w, rb, cb, blocked, bad))
    assert not np.array_equal(got[0], ref[0])
