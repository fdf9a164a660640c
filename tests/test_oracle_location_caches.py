"""Pins of the oracle's location caches (Sec. 3.3 "Location caching", Fig. "routing" (c), (d); no GPU): the message
counts the paper states - 3 without an entry, 2 with a correct one, 4 with a stale one -, the rule that entries
change only with the replies to pull and push and with relocations, and random operation sequences against an
independent model that keeps, per call, the set of messages as (kind, from, to) tuples."""
import numpy as np
import pytest

from oracle.oracle import Oracle


def _acc(st):
    return st["msg_acc_req"], st["msg_acc_fwd"], st["msg_acc_reply"]


def _delta(orc, fn):
    before = orc.stats()
    fn()
    after = orc.stats()
    return {k: after[k] - before[k] for k in after}


def test_counts_of_the_routing_figure():
    # 40 keys on 4 nodes: key 15 has home 1
    orc = Oracle("f32", 40, 1, 4)
    orc.location_caches(True)
    orc.localize([15], 3)                                   # owner 3
    d = _delta(orc, lambda: orc.pull([15], worker=0))       # no entry: request -> home, forward -> owner, reply
    assert _acc(d) == (1, 1, 1) and d["cache_hit"] == 0 and d["cache_stale"] == 0
    d = _delta(orc, lambda: orc.pull([15], worker=0))       # the reply told node 0 the owner: 2 messages
    assert _acc(d) == (1, 0, 1) and d["cache_hit"] == 1
    d = _delta(orc, lambda: orc.push([15], np.ones((1, 1), np.float32), worker=0))
    assert _acc(d) == (1, 0, 1) and d["cache_hit"] == 1     # push is routed like pull
    orc.localize([15], 2)                                   # the key moves on; node 0 is not told
    d = _delta(orc, lambda: orc.pull([15], worker=0))       # stale: request -> 3, forward -> home 1, forward -> 2, reply
    assert _acc(d) == (1, 2, 1) and d["cache_stale"] == 1 and d["cache_hit"] == 0
    d = _delta(orc, lambda: orc.pull([15], worker=0))       # ... and that reply corrected the entry
    assert _acc(d) == (1, 0, 1) and d["cache_hit"] == 1
    # the old owner took part in the relocation: node 3 knows that the key went to node 2
    d = _delta(orc, lambda: orc.pull([15], worker=3))
    assert _acc(d) == (1, 0, 1) and d["cache_hit"] == 1
    # a local access needs no cache and no message
    d = _delta(orc, lambda: orc.pull([15], worker=2))
    assert _acc(d) == (0, 0, 0) and d["pull_local"] == 1


def test_entries_change_only_with_replies_and_relocations():
    orc = Oracle("f32", 40, 1, 4)
    orc.location_caches(True)
    orc.localize([5], 2)                                    # home 0, owner 2
    orc.pull([5], worker=1)                                 # node 1 learns "2"
    orc.localize([5], 3)                                    # 2 -> 3: nodes 2 (old owner) learns, node 1 does not
    orc.localize([5], 0)                                    # 3 -> 0 (home): node 3 learns
    # node 1's entry still says 2: request -> 2, forward -> home 0 = owner: 1 forward, then the reply
    d = _delta(orc, lambda: orc.pull([5], worker=1))
    assert d["cache_stale"] == 1 and _acc(d) == (1, 1, 1)
    # node 2's entry says 3 (stale as well): request -> 3, forward -> 0, reply
    d = _delta(orc, lambda: orc.pull([5], worker=2))
    assert d["cache_stale"] == 1 and _acc(d) == (1, 1, 1)
    # an outside client (worker -1) neither uses nor fills a cache
    orc.localize([25], 1)
    d = _delta(orc, lambda: orc.pull([25], worker=-1))
    assert _acc(d) == (0, 0, 0)
    d = _delta(orc, lambda: orc.pull([25], worker=0))
    assert d["cache_hit"] == 0 and d["cache_stale"] == 0


def test_a_call_routes_with_the_caches_as_it_finds_them_and_groups_by_destination():
    orc = Oracle("f32", 40, 1, 4)
    orc.location_caches(True)
    orc.localize([10, 11, 20], 3)                           # homes 1, 1, 2; owner 3
    # the same key twice in one call: both mentions find no entry; one request, one forward, one reply
    d = _delta(orc, lambda: orc.pull([10, 10], worker=0))
    assert _acc(d) == (1, 1, 1) and d["cache_hit"] == 0 and d["pull_remote"] == 2
    # now 10 is cached (correct), 11 and 20 are not: requests to node 3 (cached), home 1, home 2; forwards 1->3, 2->3;
    # one reply from node 3
    d = _delta(orc, lambda: orc.pull([10, 11, 20], worker=0))
    assert _acc(d) == (3, 2, 1) and d["cache_hit"] == 1


def test_off_by_default_and_switching_off_forgets():
    orc = Oracle("f32", 40, 1, 4)
    orc.localize([15], 3)
    for _ in range(2):
        d = _delta(orc, lambda: orc.pull([15], worker=0))
        assert _acc(d) == (1, 1, 1) and d["cache_hit"] == 0
    orc.location_caches(True)
    orc.pull([15], worker=0)
    orc.location_caches(False)
    d = _delta(orc, lambda: orc.pull([15], worker=0))
    assert _acc(d) == (1, 1, 1) and d["cache_hit"] == 0
    orc.location_caches(True)                               # switched on again: empty
    d = _delta(orc, lambda: orc.pull([15], worker=0))
    assert _acc(d) == (1, 1, 1) and d["cache_hit"] == 0


class CachedModel:
    """Home / owner / per-node caches as dicts; the messages of one call as a set of tuples."""
    def __init__(self, K, W):
        per = -(-K // W)
        self.home = {k: k // per for k in range(K)}
        self.owner = dict(self.home)
        self.cache = {n: {} for n in range(W)}
        self.msgs = dict(req=0, fwd=0, reply=0, lreq=0, instr=0, transfer=0, hit=0, stale=0, local=0, remote=0)

    def access(self, worker, keys):
        sent = set()
        for k in keys:
            if worker < 0:
                continue
            o, h = self.owner[k], self.home[k]
            if o == worker:
                self.msgs["local"] += 1
                continue
            self.msgs["remote"] += 1
            c = self.cache[worker].get(k)
            if c is None:
                path = [("req", worker, h), ("fwd", h, o), ("reply", o, worker)]
            elif c == o:
                self.msgs["hit"] += 1
                path = [("req", worker, o), ("reply", o, worker)]
            else:
                self.msgs["stale"] += 1
                path = [("req", worker, c), ("fwd", c, h), ("fwd", h, o), ("reply", o, worker)]
            sent.update(m for m in path if m[1] != m[2])
        for kind in ("req", "fwd", "reply"):
            self.msgs[kind] += sum(1 for m in sent if m[0] == kind)
        if worker >= 0:
            for k in keys:
                if self.owner[k] != worker:
                    self.cache[worker][k] = self.owner[k]

    def localize(self, worker, keys):
        sent = set()
        for k in keys:
            o, h = self.owner[k], self.home[k]
            if o == worker:
                continue
            sent.update(m for m in [("lreq", worker, h), ("instr", h, o), ("transfer", o, worker)] if m[1] != m[2])
            self.cache[o][k] = worker
            self.owner[k] = worker
        for kind in ("lreq", "instr", "transfer"):
            self.msgs[kind] += sum(1 for m in sent if m[0] == kind)


@pytest.mark.parametrize("seed", range(8))
def test_random_sequences_match_the_model(seed):
    rng = np.random.default_rng(100 + seed)
    K, W = int(rng.integers(4, 40)), int(rng.integers(2, 6))
    orc = Oracle("f64", K, 1, W)
    orc.location_caches(True)
    model = CachedModel(K, W)
    for _ in range(400):
        op = int(rng.integers(0, 3))
        keys = rng.integers(0, K, size=int(rng.integers(0, 9)))
        if op == 0:
            worker = int(rng.integers(-1, W))
            orc.pull(keys, worker)
            model.access(worker, [int(k) for k in keys])
        elif op == 1:
            worker = int(rng.integers(-1, W))
            orc.push(keys, np.zeros((keys.size, 1)), worker)
            model.access(worker, [int(k) for k in keys])
        else:
            worker = int(rng.integers(0, W))
            orc.localize(keys, worker)
            model.localize(worker, [int(k) for k in keys])
        st = orc.stats()
        got = (st["msg_acc_req"], st["msg_acc_fwd"], st["msg_acc_reply"], st["msg_loc_req"], st["msg_loc_instruct"],
               st["msg_loc_transfer"], st["cache_hit"], st["cache_stale"], st["pull_local"] + st["push_local"],
               st["pull_remote"] + st["push_remote"])
        m = model.msgs
        want = (m["req"], m["fwd"], m["reply"], m["lreq"], m["instr"], m["transfer"], m["hit"], m["stale"], m["local"], m["remote"])
        assert got == want, (op, keys)
    assert list(orc.owner()) == [model.owner[k] for k in range(K)]
    assert model.msgs["hit"] > 0
    # (with two nodes an entry cannot go stale: a key leaves the other node only to come here, and its way back
    # is a relocation that this node takes part in)
    assert (model.msgs["stale"] > 0) == (W > 2)
