"""GPU parity of the knowledge-graph-embedding step (kge_sgd_step, through the C ABI) against the CPU oracle on the
same seeded inputs.  Two bars, both fixed:
  - exact mode (PS_OPT_KGE_EXACT with PS_OPT_PUSH_SEQUENTIAL): every value bit for bit equal to the fp32 oracle's,
    from zero accumulators (the benchmark's start) - this is what separates a mistake in scheduling or indexing
    from rounding;
  - the normal arithmetic (scores summed per lane and across lanes, hardware reciprocal square root, sums of a
    push range by range): max-abs difference to the fp32 oracle at most ATOL on servers whose accumulators start
    at G0 = 0.01, where values stay O(1) and AdaGrad's division passes a rounding difference dg of a gradient on as
    lr dg / sqrt(G0) = dg.  (From G = 0 the first step divides by sqrt(g^2 + eps): a component whose gradient
    nearly cancels, |g| < 1e-5, turns a rounding difference of 1e-8 into 1e-4 - no fixed bound holds there that
    would still catch anything, which is why that start is checked in exact mode.)
Owner map and counters are exact in both, the loss of every step within 1e-5 relative."""
import numpy as np
import pytest

from oracle.oracle import Oracle
from paper_2002_00655_amd import workloads as wl

pytestmark = pytest.mark.gpu

LR, EPS = 0.1, 1e-10
ATOL = 2e-5          # normal arithmetic against the fp32 oracle, accumulators from 0.01, a few steps, values O(1)


def _pair(w, num_workers=4, G0=0.0, exact=False):
    """An fp32 oracle and a GPU server, both holding the workload's initial embeddings, accumulators G0."""
    import torch
    from paper_2002_00655_amd import ps as P
    K, L = w.num_entities + w.num_relations, 4 * w.dim
    init = np.zeros((K, L), np.float32)
    init[:w.num_entities, :2 * w.dim] = w.E0
    init[w.num_entities:, :2 * w.dim] = w.R0
    init[:, 2 * w.dim:] = G0
    orc = Oracle("f32", K, L, num_workers)
    orc.push(np.arange(K), init)
    srv = P.ParameterServer(K, L, num_workers)
    dev = torch.device("cuda")
    srv.push(torch.arange(K, device=dev), torch.from_numpy(init).to(dev))
    if exact:
        srv.set_option(P.OPT_KGE_EXACT, 1)
        srv.set_option(P.OPT_PUSH_SEQUENTIAL, 1)
    return orc, srv


def _steps(w, orc, srv, batch, nsteps, worker=-1, first=0):
    import torch
    dev = torch.device("cuda")
    losses = []
    for i in range(nsteps):
        sl = slice(first + i * batch, first + (i + 1) * batch)
        lo = orc.kge_step(w.num_entities, w.dim, w.subj[sl], w.rel[sl], w.obj[sl], w.neg_subj[sl], w.neg_obj[sl], LR, EPS, worker)
        lg = srv.kge_sgd_step(w.num_entities, w.dim, *(torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in
                              (w.subj[sl], w.rel[sl], w.obj[sl], w.neg_subj[sl], w.neg_obj[sl])), LR, EPS, worker)
        assert abs(lg - lo) <= 1e-5 * max(1.0, abs(lo)), (i, lg, lo)
        losses.append(lg)
    return losses


def _compare(orc, srv, exact):
    import torch
    got = srv.pull(torch.arange(srv.K, device="cuda")).cpu().numpy()
    want = orc.pull(np.arange(orc.K))
    scale = float(np.abs(want).max())
    err = float(np.abs(got - want).max())
    print(f"  max abs difference GPU to fp32 oracle {err:.3e} (largest value {scale:.3g}, exact mode {exact})", flush=True)
    if exact:
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    else:
        assert scale < 20.0, "this bar is for values that stay O(1)"
        assert err <= ATOL
    assert np.array_equal(srv.owner().cpu().numpy(), orc.owner())
    assert srv.stats() == orc.stats()


CASES = [(100, 5, 5, 64), (100, 10, 10, 7), (1, 1, 0, 5), (64, 0, 0, 33), (65, 2, 3, 16), (200, 1, 1, 8), (256, 0, 2, 3)]


@pytest.mark.parametrize("dim,nns,nno,batch", CASES)
def test_steps_match_the_oracle_bit_for_bit_in_exact_mode(dim, nns, nno, batch):
    """A few steps on a small graph with heavily repeated entities (Zipf), from zero accumulators."""
    w = wl.make_kge(num_entities=300, num_relations=7, triples=4 * batch, dim=dim, n_neg_s=nns, n_neg_o=nno, seed=dim + batch)
    print(f"case dim={dim} negatives={nns}+{nno} batch={batch}", flush=True)
    orc, srv = _pair(w, exact=True)
    _steps(w, orc, srv, batch, 4, worker=2)
    _compare(orc, srv, True)


@pytest.mark.parametrize("dim,nns,nno,batch", CASES)
def test_steps_match_the_oracle_within_the_fixed_bound(dim, nns, nno, batch):
    w = wl.make_kge(num_entities=300, num_relations=7, triples=4 * batch, dim=dim, n_neg_s=nns, n_neg_o=nno, seed=dim + batch)
    print(f"case dim={dim} negatives={nns}+{nno} batch={batch}", flush=True)
    orc, srv = _pair(w, G0=0.01)
    _steps(w, orc, srv, batch, 4, worker=2)
    _compare(orc, srv, False)


@pytest.mark.parametrize("exact", [True, False])
def test_scaled_shape_of_the_complex_configuration(exact):
    """The configuration's shape at 1/100 of its size: 5,000 entities, 600 relations, dim 100, 5 + 5 negatives,
    batches of 1,024; 10 steps."""
    w = wl.make_kge(num_entities=5000, num_relations=600, triples=10 * 1024, dim=100, n_neg_s=5, n_neg_o=5, seed=11)
    orc, srv = _pair(w, G0=0.0 if exact else 0.01, exact=exact)
    _steps(w, orc, srv, 1024, 10, worker=0)
    _compare(orc, srv, exact)


def test_training_on_a_planted_graph_lowers_the_loss():
    """The planted graph of the oracle's own pin (the highest-scoring triples of random embeddings are the true ones),
    trained on the GPU in its normal arithmetic: the epoch's loss falls to less than half, and true triples end up
    scoring higher than the others."""
    import torch
    from paper_2002_00655_amd import ps as P
    D = 5
    rng = np.random.default_rng(5)
    ne, nr, n_tr = 30, 3, 200
    truth = rng.standard_normal((ne + nr, 2 * D))

    def cscore(es, wr, eo):
        a, b, c = (x[:D] + 1j * x[D:2 * D] for x in (es, wr, eo))
        return float(np.real(np.sum(a * b * np.conj(c))))
    cand = [(s, r, ob) for s in range(ne) for r in range(nr) for ob in range(ne)]
    sc = np.array([cscore(truth[s], truth[ne + r], truth[ob]) for s, r, ob in cand])
    pos = [cand[i] for i in np.argsort(-sc)[:n_tr]]
    subj, rel, obj = (np.array(x, np.int32) for x in zip(*pos))
    dev = torch.device("cuda")
    srv = P.ParameterServer(ne + nr, 4 * D, 2)
    init = np.zeros((ne + nr, 4 * D), np.float32)
    init[:, :2 * D] = rng.standard_normal((ne + nr, 2 * D)) * 0.1
    srv.push(torch.arange(ne + nr, device=dev), torch.from_numpy(init).to(dev))
    i32 = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(dev)
    losses = []
    for epoch in range(30):
        ns_, no_ = rng.integers(0, ne, (n_tr, 2)), rng.integers(0, ne, (n_tr, 2))
        tot = 0.0
        for b0 in range(0, n_tr, 20):
            sl = slice(b0, b0 + 20)
            tot += srv.kge_sgd_step(ne, D, i32(subj[sl]), i32(rel[sl]), i32(obj[sl]), i32(ns_[sl]), i32(no_[sl]), LR, EPS)
        losses.append(tot)
    print(f"  loss per epoch {losses[0]:.2f} -> {losses[-1]:.2f}", flush=True)
    assert losses[-1] < 0.5 * losses[0]
    theta = srv.pull(torch.arange(ne + nr, device=dev)).cpu().numpy()[:, :2 * D].astype(np.float64)
    learned = np.array([cscore(theta[s], theta[ne + r], theta[ob]) for s, r, ob in cand])
    true_set = set(pos)
    is_true = np.array([c in true_set for c in cand])
    assert learned[is_true].mean() > learned[~is_true].mean() + 1.0
    srv.status()


def test_edge_cases_and_errors():
    import torch
    from paper_2002_00655_amd import ps as P
    dev = torch.device("cuda")
    w = wl.make_kge(num_entities=50, num_relations=3, triples=8, dim=4, n_neg_s=1, n_neg_o=1, seed=1)
    orc, srv = _pair(w, exact=True)
    i32 = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(dev)
    # empty batch: nothing happens
    assert srv.kge_sgd_step(50, 4, i32([]), i32([]), i32([]), i32(np.zeros((0, 1))), i32(np.zeros((0, 1))), LR, EPS) == 0.0
    # subject == object == its own negative, all triples the same: every update lands on the same three keys in order
    s, r, o = [7] * 6, [1] * 6, [7] * 6
    ns_, no_ = np.full((6, 1), 7), np.full((6, 1), 7)
    orc.kge_step(50, 4, s, r, o, ns_, no_, LR, EPS, 1)
    srv.kge_sgd_step(50, 4, i32(s), i32(r), i32(o), i32(ns_), i32(no_), LR, EPS, worker=1)
    _compare(orc, srv, True)
    # value length must be 4 * dim
    with pytest.raises(P.PSError) as e:
        srv.kge_sgd_step(50, 5, i32([1]), i32([0]), i32([2]), i32([[3]]), i32([[4]]), LR, EPS)
    assert e.value.code == P.PS_EINVAL
    # an entity index outside the key space is found on the device and reported by the next status call
    srv.kge_sgd_step(50, 4, i32([1]), i32([0]), i32([99]), i32([[3]]), i32([[4]]), LR, EPS, want_loss=False)
    with pytest.raises(P.PSError) as e:
        srv.status()
    assert e.value.code == P.PS_EKEY


@pytest.mark.parametrize("exact", [True, False])
@pytest.mark.parametrize("parts,batch,lookahead", [(3, 8, 1), (3, 8, 0), (1, 16, 1), (4, 5, 1), (2, 1000, 1)])
def test_epoch_over_workers_with_pre_localization(parts, batch, lookahead, exact):
    """kge_sgd_epoch against the oracle's epoch: the same sequence of localize calls and steps, so owner map and every
    counter (relocations, local and remote accesses - the localization conflicts -, messages) are exact; values bit
    for bit in exact mode and within the fixed bound otherwise, the epoch's loss within 1e-6 relative."""
    import torch
    w = wl.make_kge(num_entities=400, num_relations=9, triples=150, dim=24, n_neg_s=2, n_neg_o=3, seed=parts * 10 + batch)
    wp, part_ptr = wl.partition_by_relation(w, parts)
    print(f"case parts={parts} batch={batch} lookahead={lookahead} exact={exact}", flush=True)
    orc, srv = _pair(wp, num_workers=4, G0=0.0 if exact else 0.01, exact=exact)
    dev = torch.device("cuda")
    lo = orc.kge_epoch(wp.num_entities, wp.dim, wp.subj, wp.rel, wp.obj, wp.neg_subj, wp.neg_obj, part_ptr, batch, lookahead, LR, EPS)
    lg = srv.kge_sgd_epoch(wp.num_entities, wp.dim, *(torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in
                           (wp.subj, wp.rel, wp.obj, wp.neg_subj, wp.neg_obj)), part_ptr, batch, lookahead, LR, EPS)
    assert abs(lg - lo) <= 1e-6 * abs(lo), (lg, lo)
    _compare(orc, srv, exact)
    st = srv.stats()
    if lookahead == 0:
        assert st["relocated"] == 0
    elif parts == 1:
        assert st["pull_remote"] == 0
    else:
        assert 0 < st["pull_remote"] < st["pull_local"]


def test_epoch_rejects_bad_indices_without_touching_anything():
    import torch
    from paper_2002_00655_amd import ps as P
    w = wl.make_kge(num_entities=50, num_relations=3, triples=20, dim=4, n_neg_s=1, n_neg_o=1, seed=1)
    wp, part_ptr = wl.partition_by_relation(w, 2)
    orc, srv = _pair(wp)
    dev = torch.device("cuda")
    before = srv.pull(torch.arange(srv.K, device=dev)).clone()
    bad_obj = wp.obj.copy()
    bad_obj[7] = 50                                         # a relation's key, not an entity
    srv.kge_sgd_epoch(wp.num_entities, wp.dim, *(torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in
                      (wp.subj, wp.rel, bad_obj, wp.neg_subj, wp.neg_obj)), part_ptr, 4, 1, LR, EPS, want_loss=False)
    with pytest.raises(P.PSError) as e:
        srv.status()
    assert e.value.code == P.PS_EKEY
    assert torch.equal(srv.pull(torch.arange(srv.K, device=dev)), before)
    with pytest.raises(P.PSError) as e:                    # more parts than workers
        srv.kge_sgd_epoch(wp.num_entities, wp.dim, *(torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in
                          (wp.subj, wp.rel, wp.obj, wp.neg_subj, wp.neg_obj)), np.arange(0, 21, 4), 4, 1, LR, EPS)
    assert e.value.code == P.PS_EWORKER


def test_limits_of_the_step():
    """63 negatives per triple (the most one wavefront's lanes can hold scores for) and dim 256 work; one more negative
    and a larger dim are refused without touching anything."""
    import torch
    from paper_2002_00655_amd import ps as P
    w = wl.make_kge(num_entities=120, num_relations=4, triples=6, dim=256, n_neg_s=40, n_neg_o=23, seed=2)
    orc, srv = _pair(w, num_workers=2, exact=True)
    _steps(w, orc, srv, 3, 2, worker=1)
    _compare(orc, srv, True)
    dev = torch.device("cuda")
    w2 = wl.make_kge(num_entities=120, num_relations=4, triples=2, dim=256, n_neg_s=40, n_neg_o=24, seed=2)
    with pytest.raises(P.PSError) as e:
        srv.kge_sgd_step(w2.num_entities, w2.dim, *(torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in
                         (w2.subj, w2.rel, w2.obj, w2.neg_subj, w2.neg_obj)), LR, EPS, 0)
    assert e.value.code == P.PS_ELIMIT
    _compare(orc, srv, True)


@pytest.mark.parametrize("exact", [False, True])
def test_full_configuration_steps(exact):
    """The configuration itself - 500,000 entities, 600 relations, dim 100, 5 + 5 negatives - and the launch shape
    bench.py times (batches of 8,192 data points): two steps against the fp32 oracle, every value of every key
    compared - in the normal arithmetic within the fixed bound (accumulators from 0.01), and in exact mode bit for
    bit from zero accumulators, the benchmark's start."""
    w = wl.make_kge(triples=2 * 8192)
    print(f"case complex entities={w.num_entities} relations={w.num_relations} dim={w.dim} exact={exact}", flush=True)
    orc, srv = _pair(w, G0=0.0 if exact else 0.01, exact=exact)
    _steps(w, orc, srv, 8192, 2, worker=0)
    _compare(orc, srv, exact)
