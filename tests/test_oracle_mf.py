"""Pins of the CPU oracle's blocked matrix-factorization epoch (no GPU).

Pinned against: a step worked out by hand in exact fractions
(tests/golden/mf_step_3x3.txt), the gradient of the per-entry loss by finite
differences, monotone decrease of the loss at a small step size, recovery of a
planted low-rank matrix, the independence of the workers of a subepoch (Sec.
2.2.2), the closed-form relocation counts of the rotating block assignment,
and "within a subepoch all parameter access is local" (Sec. 4.1).
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle.oracle import Oracle, OracleError, mf_block_ratings, ECONFLICT
from paper_2002_00655_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "mf_step_3x3.txt")


def test_golden_file_is_what_its_generator_writes():
    """The expected values of the hand-computed example come from exact fractions (tests/golden/make_mf_step_3x3.py,
    which imports nothing of the oracle or the library)."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_mf_step_3x3", os.path.join(os.path.dirname(GOLDEN), "make_mf_step_3x3.py"))
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    stored = [l.strip() for l in open(GOLDEN)]
    for line in gen.lines():
        assert line in stored, line


def _install(orc, W0, H0):
    """Initial factors go in through push onto the zeroed store (0 + x = x exactly)."""
    m, n = W0.shape[0], H0.shape[0]
    orc.push(np.arange(m), W0)
    orc.push(m + np.arange(n), H0)


def _factors(orc, m, n):
    v = orc.pull(np.arange(m + n))
    return v[:m], v[m:]


def _one_block(m, n):
    return np.array([0, m], np.int64), np.array([0, n], np.int64), [np.array([[0, 0, 0]], np.int32)]


def _parse_golden():
    d = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, rest = line.split(None, 1)
        d[key] = [[Fraction(x) for x in row.split()] for row in rest.split(";")]
    return d


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_hand_computed_3x3(prec):
    g = _parse_golden()
    lr, lam = float(g["lr"][0][0]), float(g["lambda"][0][0])
    W0 = np.array([[float(x) for x in r] for r in g["W0"]])
    H0 = np.array([[float(x) for x in r] for r in g["H0"]])
    ent = g["entries"]
    rows = np.array([int(e[0]) for e in ent], np.int32)
    cols = np.array([int(e[1]) for e in ent], np.int32)
    vals = np.array([float(e[2]) for e in ent], np.float32)
    rb, cb, sched = _one_block(3, 3)
    bp = np.array([0, len(ent)], np.int64)

    # first entry alone: exact in both precisions
    orc = Oracle(prec, 6, 2, 1)
    _install(orc, W0, H0)
    orc.mf_sgd_epoch(3, 3, rows[:1], cols[:1], vals[:1], rb, cb, np.array([0, 1], np.int64), sched, lr, lam)
    W, H = _factors(orc, 3, 3)
    assert [Fraction(float(x)) for x in W[0]] == g["after1_W0"][0]
    assert [Fraction(float(x)) for x in H[0]] == g["after1_H0"][0]
    assert np.array_equal(W[1:], W0[1:].astype(orc.dtype)) and np.array_equal(H[1:], H0[1:].astype(orc.dtype))

    # all five entries in order
    orc = Oracle(prec, 6, 2, 1)
    _install(orc, W0, H0)
    orc.mf_sgd_epoch(3, 3, rows, cols, vals, rb, cb, bp, sched, lr, lam)
    W, H = _factors(orc, 3, 3)
    want_W = np.array([[float(x) for x in r] for r in g["W"]])
    want_H = np.array([[float(x) for x in r] for r in g["H"]])
    if prec == "f64":   # every intermediate is a dyadic rational short enough for a double
        assert [[Fraction(float(x)) for x in r] for r in W] == g["W"]
        assert [[Fraction(float(x)) for x in r] for r in H] == g["H"]
    else:
        assert np.abs(W - want_W).max() < 1e-6 and np.abs(H - want_H).max() < 1e-6
        assert np.array_equal(W[:2], want_W[:2].astype(np.float32))   # these need < 24 bits: exact
    st = orc.stats()
    assert st["pull_local"] == 10 and st["push_local"] == 10 and st["pull_remote"] == st["push_remote"] == 0


def _loss(W, H, rows, cols, vals, lam):
    """sum over revealed entries of 1/2 e^2 + lam/2 (|w_i|^2 + |h_j|^2), in fp64."""
    W, H = W.astype(np.float64), H.astype(np.float64)
    e = vals.astype(np.float64) - np.einsum("ij,ij->i", W[rows], H[cols])
    return 0.5 * np.sum(e * e) + 0.5 * lam * (np.sum(W[rows] ** 2) + np.sum(H[cols] ** 2))


@pytest.mark.parametrize("lam", [0.0, 0.3])
def test_step_is_minus_lr_times_gradient(lam):
    """A single entry: the change of (w_i, h_j) equals -lr * d loss / d (w_i, h_j),
    the gradient taken by central differences of the loss written out above."""
    rng = np.random.default_rng(11)
    m, n, r, lr = 4, 5, 6, 0.125
    W0, H0 = rng.standard_normal((m, r)), rng.standard_normal((n, r))
    rows, cols, vals = np.array([2], np.int32), np.array([3], np.int32), np.array([0.7], np.float32)
    orc = Oracle("f64", m + n, r, 1)
    _install(orc, W0, H0)
    rb, cb, sched = _one_block(m, n)
    orc.mf_sgd_epoch(m, n, rows, cols, vals, rb, cb, np.array([0, 1], np.int64), sched, lr, lam)
    W1, H1 = _factors(orc, m, n)
    lam32 = float(np.float32(lam))
    gW, gH = np.zeros_like(W0), np.zeros_like(H0)
    eps = 1e-6
    for A, G in ((W0, gW), (H0, gH)):
        for idx in np.ndindex(*A.shape):
            old = A[idx]
            A[idx] = old + eps; up = _loss(W0, H0, rows, cols, vals, lam32)
            A[idx] = old - eps; dn = _loss(W0, H0, rows, cols, vals, lam32)
            A[idx] = old
            G[idx] = (up - dn) / (2 * eps)
    assert np.allclose(W1 - W0, -lr * gW, atol=1e-8)
    assert np.allclose(H1 - H0, -lr * gH, atol=1e-8)
    assert np.abs(W1 - W0)[2].min() > 1e-3 and np.abs(H1 - H0)[3].min() > 1e-3     # the step is not trivial
    untouched = np.ones(m, bool); untouched[2] = False
    assert np.array_equal(W1[untouched], W0[untouched])


def _small_problem(seed, m=40, n=30, planted=3, density=0.5, noise=0.0):
    rng = np.random.default_rng(seed)
    U = rng.standard_normal((m, planted)) / planted ** 0.25
    V = rng.standard_normal((n, planted)) / planted ** 0.25
    mask = rng.random((m, n)) < density
    rows, cols = np.nonzero(mask)
    vals = (np.einsum("ij,ij->i", U[rows], V[cols]) + noise * rng.standard_normal(rows.size)).astype(np.float32)
    return rows.astype(np.int32), cols.astype(np.int32), vals


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_loss_decreases_monotonically_at_small_lr(prec):
    m, n, r, d = 40, 30, 4, 2
    rows, cols, vals = _small_problem(5, m, n)
    rng = np.random.default_rng(6)
    W0 = (rng.random((m, r)) - 0.5).astype(np.float32)
    H0 = (rng.random((n, r)) - 0.5).astype(np.float32)
    rb, cb = wl.equal_bounds(m, d), wl.equal_bounds(n, d)
    br, bc, bv, bp = mf_block_ratings(m, n, rows, cols, vals, rb, cb)
    orc = Oracle(prec, m + n, r, d)
    _install(orc, W0, H0)
    lam = 0.02
    losses = [_loss(*_factors(orc, m, n), rows, cols, vals, lam)]
    for _ in range(30):
        orc.mf_sgd_epoch(m, n, br, bc, bv, rb, cb, bp, wl.cyclic_schedule(d), 0.005, lam)
        losses.append(_loss(*_factors(orc, m, n), rows, cols, vals, lam))
    assert all(b < a for a, b in zip(losses, losses[1:])), losses
    assert losses[-1] < 0.9 * losses[0]


def test_recovers_planted_matrix():
    """Noiseless rank-3 data, rank-3 model, no regularisation: training RMSE goes to ~0;
    with noise of std 0.1 it goes to about the noise level."""
    m, n, r, d = 60, 50, 3, 2
    rb, cb = wl.equal_bounds(m, d), wl.equal_bounds(n, d)
    for noise, lo, hi in ((0.0, 0.0, 0.01), (0.1, 0.07, 0.115)):
        rows, cols, vals = _small_problem(8, m, n, planted=3, density=0.6, noise=noise)
        rng = np.random.default_rng(9)
        W0 = ((rng.random((m, r)) - 0.5)).astype(np.float32)
        H0 = ((rng.random((n, r)) - 0.5)).astype(np.float32)
        br, bc, bv, bp = mf_block_ratings(m, n, rows, cols, vals, rb, cb)
        orc = Oracle("f64", m + n, r, d)
        _install(orc, W0, H0)
        rmse0 = np.sqrt(orc.mf_train_sse(m, br, bc, bv) / rows.size)
        for _ in range(400):
            orc.mf_sgd_epoch(m, n, br, bc, bv, rb, cb, bp, wl.cyclic_schedule(d), 0.05, 0.0)
        rmse = np.sqrt(orc.mf_train_sse(m, br, bc, bv) / rows.size)
        assert lo <= rmse <= hi, (noise, rmse0, rmse)
        assert rmse < 0.2 * rmse0


def _plain_sgd_f32(W, H, rows, cols, vals, lr, lam):
    """Textbook sequential SGD over the entries in the given order, fp32, one
    IEEE operation at a time (special case d = 1 of the blocked algorithm)."""
    f = np.float32
    W, H = W.astype(f).copy(), H.astype(f).copy()
    lr, lam = f(lr), f(lam)
    for i, j, v in zip(rows, cols, vals):
        w, h = W[i].copy(), H[j].copy()
        dot = f(0)
        for k in range(w.size):
            dot = f(dot + f(w[k] * h[k]))
        e = f(f(v) - dot)
        for k in range(w.size):
            W[i, k] = f(w[k] + f(lr * f(f(e * h[k]) - f(lam * w[k]))))
            H[j, k] = f(h[k] + f(lr * f(f(e * w[k]) - f(lam * h[k]))))
    return W, H


def test_single_block_is_plain_sequential_sgd():
    m, n, r = 25, 20, 5
    rows, cols, vals = _small_problem(12, m, n, density=0.3, noise=0.05)
    rng = np.random.default_rng(13)
    W0 = (rng.random((m, r)) - 0.5).astype(np.float32)
    H0 = (rng.random((n, r)) - 0.5).astype(np.float32)
    rb, cb, sched = _one_block(m, n)
    br, bc, bv, bp = mf_block_ratings(m, n, rows, cols, vals, rb, cb)
    orc = Oracle("f32", m + n, r, 1)
    _install(orc, W0, H0)
    orc.mf_sgd_epoch(m, n, br, bc, bv, rb, cb, bp, sched, 0.05, 0.1)
    W, H = _factors(orc, m, n)
    Wp, Hp = _plain_sgd_f32(W0, H0, br, bc, bv, 0.05, 0.1)
    assert np.array_equal(W, Wp) and np.array_equal(H, Hp)


def test_block_ratings_layout():
    """Entries are stored block by block; inside a block, busiest column first,
    then by column, then by row.  Checked against numpy's lexsort and histogram."""
    w = wl.make_mf("tiny", scale=0.2, seed=3)
    d = 4
    rb, cb = wl.equal_bounds(w.m, d), wl.equal_bounds(w.n, d)
    perm = np.random.default_rng(0).permutation(w.nnz)          # input order must not matter
    br, bc, bv, bp = mf_block_ratings(w.m, w.n, w.rows[perm], w.cols[perm], w.vals[perm], rb, cb)
    rblk = np.searchsorted(rb, w.rows, side="right") - 1
    cblk = np.searchsorted(cb, w.cols, side="right") - 1
    blk = rblk * d + cblk
    cnt = np.zeros(w.nnz, np.int64)
    key = rblk.astype(np.int64) * w.n + w.cols
    uniq, inv, c = np.unique(key, return_inverse=True, return_counts=True)
    cnt = c[inv]
    order = np.lexsort((w.rows, w.cols, -cnt, blk))
    assert np.array_equal(br, w.rows[order]) and np.array_equal(bc, w.cols[order]) and np.array_equal(bv, w.vals[order])
    hist = np.bincount(blk, minlength=d * d)
    assert np.array_equal(np.diff(bp), hist) and bp[0] == 0 and bp[-1] == w.nnz
    # uneven, explicitly given boundaries
    rb2 = np.array([0, 10, 10, 150, w.m], np.int64)
    cb2 = np.array([0, 1, w.n], np.int64)
    br, bc, bv, bp = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb2, cb2)
    for b in range(8):
        seg = slice(bp[b], bp[b + 1])
        r_, c_ = b // 2, b % 2
        assert np.all((br[seg] >= rb2[r_]) & (br[seg] < rb2[r_ + 1]))
        assert np.all((bc[seg] >= cb2[c_]) & (bc[seg] < cb2[c_ + 1]))
    assert bp[3] == bp[2] == bp[4]  # the empty row block


def _run_tiny(prec, schedule, w=None, d=4):
    w = w or wl.make_mf("tiny", scale=0.3, seed=1)
    rb, cb = wl.equal_bounds(w.m, d), wl.equal_bounds(w.n, d)
    br, bc, bv, bp = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)
    orc = Oracle(prec, w.m + w.n, w.rank, d)
    _install(orc, w.W0, w.H0)
    orc.mf_sgd_epoch(w.m, w.n, br, bc, bv, rb, cb, bp, schedule, w.lr, w.lam)
    return orc, w, (br, bc, bv, bp)


def test_workers_of_a_subepoch_are_independent():
    """Sec. 2.2.2: within a subepoch each worker is restricted to its own block,
    so the order in which the tasks of a stratum run cannot matter - bit for bit."""
    d = 4
    sched = wl.cyclic_schedule(d)
    a, w, _ = _run_tiny("f32", sched)
    rng = np.random.default_rng(2)
    shuffled = np.stack([s[rng.permutation(d)] for s in sched])
    b, _, _ = _run_tiny("f32", shuffled)
    assert np.array_equal(a.pull(np.arange(w.m + w.n)), b.pull(np.arange(w.m + w.n)))
    # but the order of the strata does matter (they share blocks)
    c, _, _ = _run_tiny("f32", sched[::-1])
    assert not np.array_equal(a.pull(np.arange(w.m + w.n)), c.pull(np.arange(w.m + w.n)))


@pytest.mark.parametrize("prec", ["f32", "f64"])
@pytest.mark.parametrize("threads", [1, 3, 0])
def test_workers_on_all_cores_equal_the_sequential_epoch(prec, threads):
    """The timing baseline that runs the workers of a subepoch side by side (Sec. 2.2.2: their blocks share no
    parameters) leaves the server exactly as the sequential epoch does: values bit for bit, owner map, every
    counter - over two epochs, with ragged blocks, an idle worker and a permuted schedule."""
    d = 5
    w = wl.make_mf("tiny", scale=0.4, seed=3)
    rng = np.random.default_rng(7)
    rb = np.concatenate([[0], np.sort(rng.choice(np.arange(1, w.m), d - 1, replace=False)), [w.m]])
    cb = np.concatenate([[0], np.sort(rng.choice(np.arange(1, w.n), d - 1, replace=False)), [w.n]])
    br, bc, bv, bp = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)
    sched = [s[rng.permutation(d)][: d - (i % 2)] for i, s in enumerate(wl.cyclic_schedule(d)[rng.permutation(d)])]
    a, b = Oracle(prec, w.m + w.n, w.rank, d + 1), Oracle(prec, w.m + w.n, w.rank, d + 1)
    for o in (a, b):
        _install(o, w.W0, w.H0)
    for _ in range(2):
        a.mf_sgd_epoch(w.m, w.n, br, bc, bv, rb, cb, bp, sched, w.lr, w.lam)
        used = b.mf_sgd_epoch_workers(w.m, w.n, br, bc, bv, rb, cb, bp, sched, w.lr, w.lam, threads=threads)
        assert used >= 1 and (threads == 0 or used == threads)
    keys = np.arange(w.m + w.n)
    assert np.array_equal(a.pull(keys), b.pull(keys))
    assert np.array_equal(a.owner(), b.owner())
    assert a.stats() == b.stats()
    # a conflicting stratum is rejected by it as well, and changes nothing
    bad = [np.array([[0, 0, 0], [1, 0, 1]], np.int32)]
    with pytest.raises(OracleError) as e:
        b.mf_sgd_epoch_workers(w.m, w.n, br, bc, bv, rb, cb, bp, bad, w.lr, w.lam)
    assert e.value.code == ECONFLICT
    assert np.array_equal(a.pull(keys), b.pull(keys)) and a.stats() == b.stats()


def test_relocation_counts_of_the_rotating_assignment():
    """With worker b keeping row block b and taking column block (b+s) mod d:
    every stratum after the first relocates all n column keys and no row key;
    the first relocates every key not already at its worker; all accesses inside
    the subepochs are local (Sec. 4.1, Sec. 4.6 "Location caching")."""
    d = 4
    w = wl.make_mf("tiny", scale=0.3, seed=1)
    rb, cb = wl.equal_bounds(w.m, d), wl.equal_bounds(w.n, d)
    br, bc, bv, bp = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)
    orc = Oracle("f32", w.m + w.n, w.rank, d)
    _install(orc, w.W0, w.H0)
    sched = wl.cyclic_schedule(d)
    home = orc.home()
    target = np.empty(w.m + w.n, np.int32)
    for b in range(d):
        target[rb[b]:rb[b + 1]] = b
        target[w.m + cb[b]:w.m + cb[b + 1]] = b          # stratum 0: column block b -> worker b
    first = int(np.sum(home != target))
    reloc = []
    for s in range(d):
        before = orc.stats()["relocated"]
        orc.mf_sgd_epoch(w.m, w.n, br, bc, bv, rb, cb, bp, sched[s:s + 1], w.lr, w.lam)
        reloc.append(orc.stats()["relocated"] - before)
    assert reloc[0] == first and reloc[1:] == [w.n] * (d - 1)
    st = orc.stats()
    assert st["pull_remote"] == st["push_remote"] == 0
    assert st["pull_local"] == st["push_local"] == 2 * w.nnz
    assert sum(st[k] for k in ("msg_acc_req", "msg_acc_fwd", "msg_acc_reply")) == 0
    # the second epoch relocates n column keys in each of its d strata
    before = orc.stats()["relocated"]
    orc.mf_sgd_epoch(w.m, w.n, br, bc, bv, rb, cb, bp, sched, w.lr, w.lam)
    assert orc.stats()["relocated"] - before == d * w.n


def test_conflicting_stratum_is_rejected():
    d = 4
    bad = wl.cyclic_schedule(d)[:1].copy()
    bad[0, 1, 2] = bad[0, 0, 2]                           # two tasks share a column block
    with pytest.raises(OracleError) as e:
        _run_tiny("f32", bad)
    assert e.value.code == ECONFLICT
    bad = wl.cyclic_schedule(d)[:1].copy()
    bad[0, 1, 0] = bad[0, 0, 0]                           # two tasks share a worker
    with pytest.raises(OracleError) as e:
        _run_tiny("f32", bad)
    assert e.value.code == ECONFLICT


def test_train_sse_matches_numpy_and_precisions_agree():
    sched = wl.cyclic_schedule(4)
    a, w, (br, bc, bv, bp) = _run_tiny("f32", sched)
    b, _, _ = _run_tiny("f64", sched)
    for orc in (a, b):
        W, H = _factors(orc, w.m, w.n)
        e = bv.astype(np.float64) - np.einsum("ij,ij->i", W[br].astype(np.float64), H[bc].astype(np.float64))
        assert np.isclose(orc.mf_train_sse(w.m, br, bc, bv), np.sum(e * e), rtol=1e-12)
    fa, fb = a.pull(np.arange(w.m + w.n)), b.pull(np.arange(w.m + w.n))
    assert np.abs(fa - fb).max() < 1e-5                     # fp32 rounding only
    assert np.abs(fa - fb).max() > 0
