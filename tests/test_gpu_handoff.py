"""GPU parity: an epoch in which column blocks are handed from worker to worker without barriers
(mf_sgd_epoch_handoff) against the CPU oracle.  The order of the blocks depends on timing, so the library reports
it; the test checks that the reported order is a valid one and replays it on the oracle as strata of one epoch
(see test_oracle_handoff.py for what pins the replay).  Bars as for mf_sgd_epoch: owner map and counters
bit-exact, factors within 1e-4, training RMSE within 1e-5 relative."""
import numpy as np
import pytest

from paper_2002_00655_amd import workloads as wl
from _util import oracle_epochs, compare_state, check_handoff_order, replay_schedule

pytestmark = pytest.mark.gpu


def _server(w, rb, cb, blocked, workers):
    import torch
    from paper_2002_00655_amd import ps as P
    br, bc, bv, bp = blocked
    srv = P.ParameterServer(w.m + w.n, w.rank, workers)
    dev = torch.device("cuda")
    srv.push(torch.arange(w.m, device=dev), torch.from_numpy(w.W0).to(dev))
    srv.push(w.m + torch.arange(w.n, device=dev), torch.from_numpy(w.H0).to(dev))
    srv.mf_load_ratings(w.m, w.n, torch.from_numpy(br).to(dev), torch.from_numpy(bc).to(dev), torch.from_numpy(bv).to(dev),
                        rb, cb, bp)
    return srv


def _oracle(w, rb, cb, blocked, workers, orders, prec="f64"):
    from oracle.oracle import Oracle
    br, bc, bv, bp = blocked
    orc = Oracle(prec, w.m + w.n, w.rank, workers)
    orc.push(np.arange(w.m), w.W0)
    orc.push(w.m + np.arange(w.n), w.H0)
    for order in orders:
        orc.mf_sgd_epoch(w.m, w.n, br, bc, bv, rb, cb, bp, replay_schedule(order), w.lr, w.lam)
    return orc


@pytest.mark.parametrize("name,scale,d_row,d_col,workers,epochs", [
    ("tiny", 1.0, 4, 4, 4, 2),
    ("tiny", 1.0, 3, 7, 5, 1),          # more column blocks than workers, a worker without a row block
    ("tiny", 0.3, 5, 2, 5, 1),          # fewer column blocks than workers: most of them wait
    ("medium", 0.05, 16, 16, 16, 2),
    ("medium", 0.05, 12, 40, 12, 1),
    ("large", 0.002, 32, 64, 32, 1),    # rank 100
])
def test_epoch_with_handoff_matches_replay(name, scale, d_row, d_col, workers, epochs):
    from oracle.oracle import mf_block_ratings
    w = wl.make_mf(name, scale=scale, seed=21)
    print(f"case {name}@{scale} {d_row}x{d_col} workers={workers} nnz={w.nnz} rank={w.rank}", flush=True)
    rb, cb = wl.balanced_bounds(w.rows, w.m, d_row), wl.balanced_bounds(w.cols, w.n, d_col)
    blocked = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)
    srv = _server(w, rb, cb, blocked, workers)
    orders = []
    for _ in range(epochs):
        order = srv.mf_sgd_epoch_handoff(w.lr, w.lam)
        check_handoff_order(order)
        orders.append(order)
    srv.status()
    orc = _oracle(w, rb, cb, blocked, workers, orders)
    compare_state(orc, srv, exact=False)
    sse_gpu = srv.mf_train_sse()
    want = orc.pull(np.arange(orc.K)).astype(np.float64)
    pred = np.einsum("ij,ij->i", want[w.rows], want[w.m + w.cols])
    sse = float(((w.vals - pred) ** 2).sum())
    assert abs(np.sqrt(sse_gpu / w.nnz) - np.sqrt(sse / w.nnz)) <= 1e-5 * np.sqrt(sse / w.nnz)


def test_empty_and_one_wide_blocks():
    """Block boundaries that leave some row blocks and column blocks empty or one index wide: an empty block is
    still taken, localized (nothing to relocate) and given back."""
    from oracle.oracle import mf_block_ratings
    w = wl.make_mf("tiny", scale=0.5, seed=8)
    d_row, d_col = 6, 9
    rb = np.sort(np.concatenate([[0, w.m], np.random.default_rng(1).integers(0, w.m, d_row - 1)])).astype(np.int64)
    rb[2] = rb[1]                                                      # an empty row block
    cb = np.sort(np.concatenate([[0, w.n], np.random.default_rng(2).integers(0, 3, d_col - 1)])).astype(np.int64)
    print(f"case ragged rows {rb.tolist()} columns {cb.tolist()}", flush=True)
    blocked = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)
    srv = _server(w, rb, cb, blocked, d_row)
    orders = [srv.mf_sgd_epoch_handoff(w.lr, w.lam) for _ in range(2)]
    srv.status()
    for order in orders:
        check_handoff_order(order)
    compare_state(_oracle(w, rb, cb, blocked, d_row, orders), srv, exact=False)


def test_single_worker_and_single_column_block():
    from oracle.oracle import mf_block_ratings
    w = wl.make_mf("tiny", scale=0.2, seed=3)
    for d_row, d_col in ((1, 5), (4, 1), (1, 1)):
        rb, cb = wl.equal_bounds(w.m, d_row), wl.equal_bounds(w.n, d_col)
        blocked = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)
        srv = _server(w, rb, cb, blocked, d_row)
        order = srv.mf_sgd_epoch_handoff(w.lr, w.lam)
        srv.status()
        check_handoff_order(order)
        if d_row == 1:
            assert order[0, :, 0].tolist() == list(range(d_col))      # alone, a worker takes the column blocks in cyclic order
        compare_state(_oracle(w, rb, cb, blocked, d_row, [order]), srv, exact=False)


def test_very_long_runs_in_column_blocks_of_their_own():
    """Columns with half of all rows, 4 row blocks and 256 column ranges cut by `balanced_bounds`: the heaviest columns
    get ranges of their own, their runs have over a hundred groups (the kernel's variant for very long runs), and
    there are 64 times more column blocks than workers."""
    from oracle.oracle import mf_block_ratings
    w = wl.make_mf("wide", scale=0.002)
    d_row, d_col = 4, 256
    rb, cb = wl.balanced_bounds(w.rows, w.m, d_row), wl.balanced_bounds(w.cols, w.n, d_col, per_id=8.0 * d_row)
    counts = np.bincount(w.cols, minlength=w.n)
    alone = [int(c) for c in np.flatnonzero(counts > w.nnz / d_col) if c in cb and c + 1 in cb]
    print(f"case wide@0.002 {d_row}x{d_col}: {len(alone)} columns in ranges of their own, longest run {counts.max() // d_row} entries",
          flush=True)
    assert len(alone) >= 10 and counts.max() // d_row >= 64 * 15
    blocked = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)
    srv = _server(w, rb, cb, blocked, d_row)
    orders = [srv.mf_sgd_epoch_handoff(w.lr, w.lam) for _ in range(2)]
    srv.status()
    for order in orders:
        check_handoff_order(order)
    compare_state(_oracle(w, rb, cb, blocked, d_row, orders), srv, exact=False)


def test_many_more_workers_than_column_blocks():
    """300 workers and 3 column blocks: nearly everybody waits nearly all the time, and a column block's 300 visits
    are one long chain of hand-overs."""
    from oracle.oracle import mf_block_ratings
    w = wl.make_mf("tiny", scale=0.5, seed=12)
    d_row, d_col = 300, 3
    rb, cb = wl.equal_bounds(w.m, d_row), wl.equal_bounds(w.n, d_col)
    blocked = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)
    srv = _server(w, rb, cb, blocked, d_row)
    order = srv.mf_sgd_epoch_handoff(w.lr, w.lam)
    srv.status()
    check_handoff_order(order)
    compare_state(_oracle(w, rb, cb, blocked, d_row, [order]), srv, exact=False)


def test_uncached_columns_and_rank_not_multiple_of_four():
    """Column factors that do not fit in LDS are handed over through memory inside a block as well; rank 50 is
    read in 4-byte pieces."""
    from oracle.oracle import mf_block_ratings
    from paper_2002_00655_amd import ps as P
    w = wl.make_mf("medium", scale=0.03, seed=5)
    assert w.rank % 4 != 0
    d = 8
    rb, cb = wl.equal_bounds(w.m, d), wl.equal_bounds(w.n, d)
    blocked = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)
    srv = _server(w, rb, cb, blocked, d)
    srv.set_option(P.OPT_MF_CACHE_ROWS, 3)
    order = srv.mf_sgd_epoch_handoff(w.lr, w.lam)
    check_handoff_order(order)
    srv.status()
    compare_state(_oracle(w, rb, cb, blocked, d, [order]), srv, exact=False)


def test_limits():
    from oracle.oracle import mf_block_ratings
    from paper_2002_00655_amd import ps as P
    w = wl.make_mf("tiny", scale=0.3, seed=2)
    rb, cb = wl.equal_bounds(w.m, 4), wl.equal_bounds(w.n, 4)
    blocked = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)
    srv = _server(w, rb, cb, blocked, 3)                   # four row blocks, three workers
    with pytest.raises(P.PSError) as e:
        srv.mf_sgd_epoch_handoff(w.lr, w.lam)
    assert e.value.code == P.PS_EWORKER
    srv = _server(w, rb, cb, blocked, 4)
    srv.set_option(P.OPT_MF_EXACT, 1)
    with pytest.raises(P.PSError) as e:
        srv.mf_sgd_epoch_handoff(w.lr, w.lam)
    assert e.value.code == P.PS_ELIMIT
    srv.set_option(P.OPT_MF_EXACT, 0)
    assert srv.mf_sgd_epoch_handoff(w.lr, w.lam, want_order=False) is None
    srv.status()


def test_large_config_full_size_with_handoff():
    """The large configuration (100M entries, rank 100, 256 x 256 blocks, bench.py's block boundaries) in the launch
    shape that bench.py --handoff times: one epoch, the reported order replayed on the fp32 oracle (about a minute
    of host work), every key compared."""
    import time
    from oracle.oracle import Oracle, mf_block_ratings
    w = wl.make_mf("large")
    d = 256
    print(f"case large with hand-over nnz={w.nnz}", flush=True)
    rb, cb = wl.balanced_bounds(w.rows, w.m, d), wl.balanced_bounds(w.cols, w.n, d, per_id=8.0 * d)
    t0 = time.time()
    blocked = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)
    print(f"  oracle layout {time.time() - t0:.0f} s", flush=True)
    srv = _server(w, rb, cb, blocked, d)
    order = srv.mf_sgd_epoch_handoff(w.lr, w.lam)
    srv.status()
    check_handoff_order(order)
    strata = replay_schedule(order)
    print(f"  reported order: {len(strata)} strata when every block runs as early as the order allows", flush=True)
    br, bc, bv, bp = blocked
    orc = Oracle("f32", w.m + w.n, w.rank, d)
    orc.push(np.arange(w.m), w.W0)
    orc.push(w.m + np.arange(w.n), w.H0)
    quarter = (len(strata) + 3) // 4
    for q in range(4):
        t0 = time.time()
        part = strata[q * quarter:(q + 1) * quarter]
        if part:
            orc.mf_sgd_epoch(w.m, w.n, br, bc, bv, rb, cb, bp, part, w.lr, w.lam)
        print(f"  oracle quarter {q + 1} of the replay {time.time() - t0:.0f} s", flush=True)
    compare_state(orc, srv, exact=False)
    sse_gpu, sse_orc = srv.mf_train_sse(), orc.mf_train_sse(w.m, br, bc, bv)
    assert abs(np.sqrt(sse_gpu / w.nnz) - np.sqrt(sse_orc / w.nnz)) <= 1e-5 * np.sqrt(sse_orc / w.nnz)
