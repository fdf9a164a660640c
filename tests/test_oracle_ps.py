"""Pins of the CPU oracle's parameter-server primitives (no GPU).

The oracle is checked against things other than itself: an independent
dictionary model driven by random operation sequences, the message counts the
paper states (Table "Location management strategies", Sec. 3.2, Sec. 3.3, Sec.
3.7, Table "reloc-stats" caption), and invariants of dynamic allocation (one
owner per key, values untouched by relocation, cumulative pushes).
"""
import numpy as np
import pytest

from oracle.oracle import Oracle, OracleError, EKEY, EWORKER, EINVAL


# ----------------------------------------------------------------------------
# an independent model: dict of lists + python sets
# ----------------------------------------------------------------------------
class DictPS:
    def __init__(self, K, L, W, dtype):
        self.K, self.L, self.W, self.dtype = K, L, W, dtype
        self.val = {k: [dtype(0)] * L for k in range(K)}
        per = -(-K // W)
        self.home = {k: k // per for k in range(K)}
        self.owner = dict(self.home)
        self.st = dict(pull_local=0, pull_remote=0, push_local=0, push_remote=0, relocated=0, localize_keys=0,
                       msg_acc=0, msg_loc=0)

    @staticmethod
    def _msgs(worker, travelling):
        """travelling: list of (home, owner) of keys that need the network."""
        to_home = {h for h, _ in travelling if h != worker}
        fwd = {(h, o) for h, o in travelling if h != o}
        back = {o for _, o in travelling if o != worker}
        return len(to_home) + len(fwd) + len(back)

    def pull(self, worker, keys):
        out, trav = [], []
        for k in keys:
            out.append(list(self.val[k]))
            if worker >= 0:
                if self.owner[k] == worker:
                    self.st["pull_local"] += 1
                else:
                    self.st["pull_remote"] += 1
                    trav.append((self.home[k], self.owner[k]))
        self.st["msg_acc"] += self._msgs(worker, trav)
        return out

    def push(self, worker, keys, deltas):
        trav = []
        for k, d in zip(keys, deltas):
            self.val[k] = [self.dtype(a + self.dtype(b)) for a, b in zip(self.val[k], d)]
            if worker >= 0:
                if self.owner[k] == worker:
                    self.st["push_local"] += 1
                else:
                    self.st["push_remote"] += 1
                    trav.append((self.home[k], self.owner[k]))
        self.st["msg_acc"] += self._msgs(worker, trav)

    def localize(self, worker, keys):
        trav = []
        for k in keys:
            self.st["localize_keys"] += 1
            if self.owner[k] != worker:
                trav.append((self.home[k], self.owner[k]))
                self.owner[k] = worker
                self.st["relocated"] += 1
        self.st["msg_loc"] += self._msgs(worker, trav)


def _check_same(orc, model):
    st = orc.stats()
    for name in ("pull_local", "pull_remote", "push_local", "push_remote", "relocated", "localize_keys"):
        assert st[name] == model.st[name], name
    assert st["msg_acc_req"] + st["msg_acc_fwd"] + st["msg_acc_reply"] == model.st["msg_acc"]
    assert st["msg_loc_req"] + st["msg_loc_instruct"] + st["msg_loc_transfer"] == model.st["msg_loc"]
    assert list(orc.owner()) == [model.owner[k] for k in range(model.K)]
    got = orc.pull(np.arange(model.K))
    want = np.array([model.val[k] for k in range(model.K)], dtype=orc.dtype)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("prec", ["f32", "f64"])
@pytest.mark.parametrize("seed", range(6))
def test_random_sequences_match_dict_model(prec, seed):
    rng = np.random.default_rng(seed)
    K, L, W = int(rng.integers(1, 17)), int(rng.integers(1, 4)), int(rng.integers(1, 5))
    orc = Oracle(prec, K, L, W)
    model = DictPS(K, L, W, orc.dtype)
    for _ in range(300):
        op = rng.integers(0, 3)
        n = int(rng.integers(0, 7))
        keys = rng.integers(0, K, size=n)
        if op == 0:
            worker = int(rng.integers(-1, W))
            got = orc.pull(keys, worker)
            want = model.pull(worker, list(keys))
            assert np.array_equal(got, np.array(want, dtype=orc.dtype).reshape(n, L))
        elif op == 1:
            worker = int(rng.integers(-1, W))
            d = rng.standard_normal((n, L)).astype(orc.dtype)
            orc.push(keys, d, worker)
            model.push(worker, list(keys), d)
        else:
            worker = int(rng.integers(0, W))
            orc.localize(keys, worker)
            model.localize(worker, list(keys))
    _check_same(orc, model)


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_push_is_cumulative_and_ordered(prec):
    """Sec. 2.1: the update term is added to the value; no update is lost.
    Duplicates in one call are applied in argument order (fp addition does not
    commute in rounding, so the order is observable)."""
    orc = Oracle(prec, 4, 1, 2)
    t = orc.dtype
    big, small = t(1.0), t(2.0 ** -24 if prec == "f32" else 2.0 ** -53)
    # (1 + s) + s rounds to 1 twice (ties to even); (s + s) + 1 does not.
    orc.push([0, 0, 0], np.array([[big], [small], [small]], dtype=t))
    orc.push([1, 1, 1], np.array([[small], [small], [big]], dtype=t))
    v = orc.pull([0, 1])
    assert v[0, 0] == t(1.0)
    assert v[1, 0] == t(1.0) + t(2) * small and v[1, 0] != v[0, 0]
    # sum of many pushes equals the running sum in call order
    rng = np.random.default_rng(1)
    acc = t(0)
    for _ in range(50):
        d = t(rng.standard_normal())
        orc.push([3], np.array([[d]], dtype=t))
        acc = t(acc + d)
    assert orc.pull([3])[0, 0] == acc


@pytest.mark.parametrize("prec", ["f32", "f64"])
def test_location_transparency(prec):
    """Sec. 2.3: pull and push are oblivious of a parameter's location - the
    same operations with relocations sprinkled in give the same values."""
    rng = np.random.default_rng(7)
    K, L, W = 40, 3, 4
    a, b = Oracle(prec, K, L, W), Oracle(prec, K, L, W)
    for _ in range(200):
        keys = rng.integers(0, K, size=int(rng.integers(1, 9)))
        d = rng.standard_normal((keys.size, L)).astype(a.dtype)
        w = int(rng.integers(0, W))
        a.push(keys, d, w)
        b.localize(rng.integers(0, K, size=5), int(rng.integers(0, W)))
        b.push(keys, d, w)
        assert np.array_equal(a.pull(keys, w), b.pull(keys, w))
    assert np.array_equal(a.pull(np.arange(K)), b.pull(np.arange(K)))
    assert a.stats()["relocated"] == 0 and b.stats()["relocated"] > 0


def test_one_owner_per_key_and_last_localize_wins():
    """Sec. 3.2: without replicas a parameter resides at one node at a time; on
    a conflict it goes to each requester once, in request order."""
    K, W = 30, 5
    orc = Oracle("f32", K, 2, W)
    assert np.array_equal(orc.owner(), orc.home())                      # classic allocation to start with
    assert np.array_equal(orc.home(), np.arange(K) // 6)                # range partition, ceil(30/5) = 6
    orc.localize([3, 4, 5], 2)
    orc.localize([4], 0)
    orc.localize([4, 4], 3)                                             # second mention is a no-op
    own = orc.owner()
    assert own[3] == 2 and own[5] == 2 and own[4] == 3
    assert np.bincount(own, minlength=W).sum() == K and own.min() >= 0 and own.max() < W
    st = orc.stats()
    assert st["relocated"] == 3 + 1 + 1                                 # key 4 moved three times, 3 and 5 once
    assert st["localize_keys"] == 6
    orc.localize([3, 5], 2)                                             # already there: nothing travels
    assert orc.stats()["relocated"] == 5
    assert orc.stats()["msg_loc_req"] + orc.stats()["msg_loc_instruct"] + orc.stats()["msg_loc_transfer"] == \
        st["msg_loc_req"] + st["msg_loc_instruct"] + st["msg_loc_transfer"]


def _msgs(st, kind):
    names = {"acc": ("msg_acc_req", "msg_acc_fwd", "msg_acc_reply"),
             "loc": ("msg_loc_req", "msg_loc_instruct", "msg_loc_transfer")}[kind]
    return tuple(st[x] for x in names)


def test_message_counts_stated_in_the_paper():
    # K = 40 keys on W = 4 nodes: homes 0..9 -> 0, 10..19 -> 1, 20..29 -> 2, 30..39 -> 3
    orc = Oracle("f32", 40, 1, 4)
    # Static partition (owner == home): a remote access takes 2 messages (Table "Location management").
    orc.pull([15], worker=0)
    assert _msgs(orc.stats(), "acc") == (1, 0, 1)
    # Relocation with three distinct parties: 3 messages (Sec. 3.2, Fig. "localize-messages").
    orc.localize([15], 2)          # requester 2, home 1, owner 1 -> home and owner coincide: 2 messages
    assert _msgs(orc.stats(), "loc") == (1, 0, 1)
    orc.localize([15], 3)          # requester 3, home 1, owner 2: all distinct -> 3 messages
    assert _msgs(orc.stats(), "loc") == (2, 1, 2)
    # Home-node strategy, remote access, uncached: 3 messages (Sec. 3.3 "forward").
    before = _msgs(orc.stats(), "acc")
    orc.push([15], np.ones((1, 1), np.float32), worker=0)     # worker 0, home 1, owner 3
    after = _msgs(orc.stats(), "acc")
    assert tuple(a - b for a, b in zip(after, before)) == (1, 1, 1)
    # Local access: no message at all.
    before = after
    orc.pull([15], worker=3)
    assert _msgs(orc.stats(), "acc") == before
    # Message grouping (Sec. 3.7): several keys with the same home and the same owner still cost 3.
    orc.localize([20, 21, 22, 23], 3)                          # home 2, owner 2 -> (1,0,1)
    before = _msgs(orc.stats(), "loc")
    orc.localize([20, 21, 22, 23], 0)                          # requester 0, home 2, owner 3
    after = _msgs(orc.stats(), "loc")
    assert tuple(a - b for a, b in zip(after, before)) == (1, 1, 1)
    # ... and keys of two homes held by one owner: 2 requests, 2 instructions, 1 transfer.
    orc.localize([30, 31], 0)                                  # (h=3,o=3) -> requester 0
    before = _msgs(orc.stats(), "loc")
    orc.localize([20, 30, 21, 31], 1)                          # homes 2 and 3, owner 0 for all
    after = _msgs(orc.stats(), "loc")
    assert tuple(a - b for a, b in zip(after, before)) == (2, 2, 1)


def test_two_nodes_every_relocation_is_two_messages():
    """Caption of Table "reloc-stats": on 2 nodes every relocation involves only 2 nodes."""
    rng = np.random.default_rng(3)
    orc = Oracle("f32", 64, 1, 2)
    for _ in range(200):
        k = int(rng.integers(0, 64))
        w = int(rng.integers(0, 2))
        b_rel, b_msg = orc.stats()["relocated"], sum(_msgs(orc.stats(), "loc"))
        orc.localize([k], w)
        d_rel, d_msg = orc.stats()["relocated"] - b_rel, sum(_msgs(orc.stats(), "loc")) - b_msg
        assert d_msg == 2 * d_rel


def test_single_node_everything_is_local():
    """Table "reloc-stats", first line: one node, no non-local reads, no relocations."""
    rng = np.random.default_rng(4)
    orc = Oracle("f64", 50, 2, 1)
    for _ in range(50):
        keys = rng.integers(0, 50, size=6)
        orc.localize(keys, 0)
        orc.push(keys, rng.standard_normal((6, 2)), 0)
        orc.pull(keys, 0)
    st = orc.stats()
    assert st["pull_remote"] == st["push_remote"] == st["relocated"] == 0
    assert sum(_msgs(st, "acc")) == sum(_msgs(st, "loc")) == 0
    assert st["pull_local"] == st["push_local"] == 300


def test_error_codes():
    orc = Oracle("f32", 10, 2, 3)
    with pytest.raises(OracleError) as e:
        orc.pull([10])
    assert e.value.code == EKEY
    with pytest.raises(OracleError) as e:
        orc.push([-1], np.zeros((1, 2), np.float32))
    assert e.value.code == EKEY
    with pytest.raises(OracleError) as e:
        orc.localize([1], 3)
    assert e.value.code == EWORKER
    with pytest.raises(OracleError) as e:
        orc.localize([1], -1)
    assert e.value.code == EWORKER
    with pytest.raises(OracleError) as e:
        orc.pull([1], worker=5)
    assert e.value.code == EWORKER
    # a failed call changes nothing
    assert orc.stats()["localize_keys"] == 0 and np.array_equal(orc.owner(), orc.home())
    with pytest.raises(OracleError) as e:
        Oracle("f32", 0, 1, 1)
    assert e.value.code == EINVAL
