"""Pins of the CPU oracle's epoch on a classic parameter server (no relocation; Sec. 2.1, Sec. 4.2, Sec. 4.6 of the
paper): the values against the epoch with relocation (location transparency, Sec. 2.3), the access and message
counts against a count written out in Python from the paper's rules.  No GPU."""
import numpy as np

from oracle.oracle import Oracle, mf_block_ratings
from paper_2002_00655_amd import workloads as wl


def _setup(d, num_workers, seed=1, scale=0.3):
    w = wl.make_mf("tiny", scale=scale, seed=seed)
    rb, cb = wl.equal_bounds(w.m, d), wl.equal_bounds(w.n, d)
    blocked = mf_block_ratings(w.m, w.n, w.rows, w.cols, w.vals, rb, cb)
    orc = Oracle("f32", w.m + w.n, w.rank, num_workers)
    orc.push(np.arange(w.m), w.W0)
    orc.push(w.m + np.arange(w.n), w.H0)
    return w, rb, cb, blocked, orc


def _expected_counts(w, rb, cb, blocked, sched, owner, home):
    """Every entry is one pull and one push of its two keys.  A key is local if the worker owns it.  A remote key
    costs a request to its home unless the worker is the home, a forward unless home and owner coincide, a reply
    unless the worker is the owner (Sec. 3.3); messages of one call to the same destination are grouped (Sec. 3.7)."""
    br, bc, bv, bp = blocked
    d_col = cb.size - 1
    c = dict(local=0, remote=0, req=0, fwd=0, reply=0)
    for stratum in sched:
        for worker, rblk, cblk in stratum:
            b = rblk * d_col + cblk
            for p in range(bp[b], bp[b + 1]):
                keys = (int(br[p]), w.m + int(bc[p]))
                req, fwd, rep = set(), set(), set()
                for k in keys:
                    o, h = int(owner[k]), int(home[k])
                    if o == worker:
                        c["local"] += 1
                        continue
                    c["remote"] += 1
                    if h != worker:
                        req.add(h)
                    if h != o:
                        fwd.add((h, o))
                    rep.add(o)
                c["req"] += len(req); c["fwd"] += len(fwd); c["reply"] += len(rep)
    return c


def test_values_are_those_of_the_epoch_with_relocation():
    d = 4
    sched = wl.cyclic_schedule(d)
    w, rb, cb, blocked, a = _setup(d, d)
    _, _, _, _, b = _setup(d, d)
    a.mf_sgd_epoch(w.m, w.n, *blocked[:3], rb, cb, blocked[3], sched, w.lr, w.lam)
    b.mf_sgd_epoch(w.m, w.n, *blocked[:3], rb, cb, blocked[3], sched, w.lr, w.lam, classic=True)
    assert np.array_equal(a.pull(np.arange(w.m + w.n)), b.pull(np.arange(w.m + w.n)))
    assert b.stats()["relocated"] == 0 and np.array_equal(b.owner(), b.home())
    assert a.stats()["relocated"] > 0


def test_counts_with_every_key_at_its_home():
    d = 4
    sched = wl.cyclic_schedule(d)
    w, rb, cb, blocked, orc = _setup(d, d)
    home = orc.home()
    orc.mf_sgd_epoch(w.m, w.n, *blocked[:3], rb, cb, blocked[3], sched, w.lr, w.lam, classic=True)
    want = _expected_counts(w, rb, cb, blocked, sched, home, home)
    st = orc.stats()
    assert st["pull_local"] == st["push_local"] == want["local"]
    assert st["pull_remote"] == st["push_remote"] == want["remote"]
    assert want["remote"] > want["local"] > 0                      # most accesses are remote without relocation
    assert st["msg_acc_req"] == 2 * want["req"] and st["msg_acc_reply"] == 2 * want["reply"] and st["msg_acc_fwd"] == 0
    assert st["pull_local"] + st["pull_remote"] == 2 * w.nnz


def test_counts_with_keys_that_live_away_from_home():
    """Some keys were relocated before (by an explicit localize): their accesses are forwarded by the home node."""
    d = 4
    sched = wl.cyclic_schedule(d)
    w, rb, cb, blocked, orc = _setup(d, d, seed=2)
    rng = np.random.default_rng(0)
    moved = rng.choice(w.m + w.n, size=(w.m + w.n) // 3, replace=False)
    for part, worker in zip(np.array_split(moved, 3), (0, 2, 3)):
        orc.localize(part, worker)
    owner, home = orc.owner(), orc.home()
    st0 = orc.stats()
    orc.mf_sgd_epoch(w.m, w.n, *blocked[:3], rb, cb, blocked[3], sched, w.lr, w.lam, classic=True)
    want = _expected_counts(w, rb, cb, blocked, sched, owner, home)
    st = orc.stats()
    assert st["pull_local"] - st0["pull_local"] == want["local"] and st["pull_remote"] - st0["pull_remote"] == want["remote"]
    assert st["msg_acc_req"] - st0["msg_acc_req"] == 2 * want["req"]
    assert st["msg_acc_fwd"] - st0["msg_acc_fwd"] == 2 * want["fwd"] > 0
    assert st["msg_acc_reply"] - st0["msg_acc_reply"] == 2 * want["reply"]
    assert np.array_equal(orc.owner(), owner)


def test_one_node_has_only_local_accesses():
    d = 3
    w, rb, cb, blocked, orc = _setup(d, 1)
    sched = [np.array([[0, s % d, (s * 2) % d]], np.int32) for s in range(d)]
    orc.mf_sgd_epoch(w.m, w.n, *blocked[:3], rb, cb, blocked[3], sched, w.lr, w.lam, classic=True)
    st = orc.stats()
    assert st["pull_remote"] == st["push_remote"] == 0
    assert sum(st[k] for k in ("msg_acc_req", "msg_acc_fwd", "msg_acc_reply")) == 0
