"""Pins of the CPU oracle's knowledge-graph-embedding step (oracle/kge_oracle.c) against things other than
itself: complex arithmetic in numpy, central differences of the loss, the AdaGrad formula written out for one
number, linearity of the cumulative push, and a small planted graph.  No GPU."""
import numpy as np
import pytest

from oracle.oracle import Oracle

D = 5


def _server(prec, ne, nr, rng, G0=0.0, scale=0.5):
    o = Oracle(prec, ne + nr, 4 * D, 2)
    emb = rng.standard_normal((ne + nr, 2 * D)) * scale
    acc = np.full((ne + nr, 2 * D), G0)
    o.push(np.arange(ne + nr), np.concatenate([emb, acc], axis=1))
    return o


def _cscore(es, wr, eo):
    a, b, c = (x[:D] + 1j * x[D:2 * D] for x in (es, wr, eo))
    return float(np.real(np.sum(a * b * np.conj(c))))


def _loss(theta, triples_with_labels):
    """Sum over scored triples of log(1 + exp(-label * score)), from a dense table of embeddings."""
    tot = 0.0
    for s, r, o, y in triples_with_labels:
        tot += np.logaddexp(0.0, -y * _cscore(theta[s], theta[r], theta[o]))
    return tot


def test_score_is_the_real_part_of_the_trilinear_product():
    rng = np.random.default_rng(1)
    o64, o32 = Oracle("f64", 3, 4 * D, 1), Oracle("f32", 3, 4 * D, 1)
    for _ in range(20):
        es, wr, eo = rng.standard_normal((3, 2 * D))
        want = _cscore(es, wr, eo)
        assert abs(o64.kge_score(D, es, wr, eo) - want) < 1e-13
        assert abs(o32.kge_score(D, es, wr, eo) - want) < 1e-5
    # conjugation is on the object: swapping subject and object changes the sign of the imaginary-relation part
    es, wr, eo = rng.standard_normal((3, 2 * D))
    wr_real, wr_imag = wr.copy(), wr.copy()
    wr_real[D:] = 0.0
    wr_imag[:D] = 0.0
    assert abs(o64.kge_score(D, es, wr_real, eo) - o64.kge_score(D, eo, wr_real, es)) < 1e-13
    assert abs(o64.kge_score(D, es, wr_imag, eo) + o64.kge_score(D, eo, wr_imag, es)) < 1e-13


@pytest.mark.parametrize("G0", [0.0, 0.3])
def test_one_triple_step_is_adagrad_on_the_gradient_of_the_logistic_loss(G0):
    rng = np.random.default_rng(2)
    ne, nr, lr, eps = 6, 2, 0.1, 1e-10
    o = _server("f64", ne, nr, rng, G0)
    before = o.pull(np.arange(ne + nr))
    s, r, ob = 1, 0, 4
    loss = o.kge_step(ne, D, [s], [r], [ob], np.zeros((1, 0)), np.zeros((1, 0)), lr, eps)
    after = o.pull(np.arange(ne + nr))
    theta = before[:, :2 * D]
    trip = [(s, ne + r, ob, +1.0)]
    assert abs(loss - _loss(theta, trip)) < 1e-12
    h = 1e-6
    for key in (s, ne + r, ob):
        for c in range(2 * D):
            tp, tm = theta.copy(), theta.copy()
            tp[key, c] += h
            tm[key, c] -= h
            g = (_loss(tp, trip) - _loss(tm, trip)) / (2 * h)               # central difference
            dG = after[key, 2 * D + c] - before[key, 2 * D + c]
            dth = after[key, c] - before[key, c]
            assert abs(dG - g * g) < 1e-8
            assert abs(dth - (-lr * g / np.sqrt(G0 + g * g + eps))) < 1e-7
    untouched = [k for k in range(ne + nr) if k not in (s, ne + r, ob)]
    assert np.array_equal(after[untouched], before[untouched])


def test_negatives_have_label_minus_one_and_every_occurrence_is_its_own_adagrad_term():
    rng = np.random.default_rng(3)
    ne, nr, lr, eps = 8, 1, 0.1, 1e-10
    o = _server("f64", ne, nr, rng)
    before = o.pull(np.arange(ne + nr))
    theta = before[:, :2 * D]
    s, r, ob, s_neg, o_neg = 0, 0, 1, 5, 6
    o.kge_step(ne, D, [s], [r], [ob], [[s_neg]], [[o_neg]], lr, eps)
    after = o.pull(np.arange(ne + nr))
    scored = [(s, ne + r, ob, +1.0), (s_neg, ne + r, ob, -1.0), (s, ne + r, o_neg, -1.0)]
    h = 1e-6

    def grad(trip, key, c):
        tp, tm = theta.copy(), theta.copy()
        tp[key, c] += h
        tm[key, c] -= h
        return (_loss(tp, [trip]) - _loss(tm, [trip])) / (2 * h)
    for c in range(2 * D):
        # the perturbed subject occurs once, with the negative label
        g = grad(scored[1], s_neg, c)
        assert abs(after[s_neg, 2 * D + c] - g * g) < 1e-8
        assert abs((after[s_neg, c] - before[s_neg, c]) + lr * g / np.sqrt(g * g + eps)) < 1e-7
        # the relation occurs in all three scored triples: three separate terms, all from the pulled accumulator (0)
        gs = [grad(t, ne + r, c) for t in scored]
        assert abs(after[ne + r, 2 * D + c] - sum(x * x for x in gs)) < 1e-8
        want = sum(-lr * x / np.sqrt(x * x + eps) for x in gs)
        assert abs((after[ne + r, c] - before[ne + r, c]) - want) < 1e-7


def test_a_batch_is_the_sum_of_its_triples_steps_from_the_same_state():
    """All values are pulled before anything is pushed, and push is cumulative: a batch changes every value by the
    sum of what its triples would change on their own (entities repeated across the batch included)."""
    ne, nr, lr, eps = 7, 2, 0.1, 1e-10
    subj, rel, obj = [0, 0, 3, 2], [0, 1, 0, 1], [1, 2, 0, 2]          # repeats, and a triple with subject == object
    negs, nego = [[4, 5], [0, 6], [1, 1], [3, 4]], [[2], [5], [6], [0]]
    seed = 4
    o = _server("f64", ne, nr, np.random.default_rng(seed), G0=0.01)
    before = o.pull(np.arange(ne + nr))
    o.kge_step(ne, D, subj, rel, obj, negs, nego, lr, eps)
    total = o.pull(np.arange(ne + nr)) - before
    acc = np.zeros_like(total)
    for b in range(4):
        ob = _server("f64", ne, nr, np.random.default_rng(seed), G0=0.01)
        ob.kge_step(ne, D, subj[b:b + 1], rel[b:b + 1], obj[b:b + 1], negs[b:b + 1], nego[b:b + 1], lr, eps)
        acc += ob.pull(np.arange(ne + nr)) - before
    assert np.allclose(total, acc, rtol=0, atol=1e-12)


def test_large_scores_do_not_overflow_and_counters_see_every_occurrence():
    ne, nr = 4, 1
    for prec in ("f32", "f64"):
        o = Oracle(prec, ne + nr, 4 * D, 2)
        big = np.zeros((ne + nr, 4 * D))
        big[:, :D] = 30.0                                              # score = 5 * 27000
        o.push(np.arange(ne + nr), big)
        st0 = o.stats()
        loss = o.kge_step(ne, D, [0], [0], [1], [[2]], [[3]], 0.1, 1e-10, worker=1)
        assert np.isfinite(loss) and loss > 1e5                         # two confidently wrong negatives
        assert np.isfinite(o.pull(np.arange(ne + nr))).all()
        st = o.stats()
        assert st["pull_local"] + st["pull_remote"] - st0["pull_local"] - st0["pull_remote"] == 9
        assert st["push_local"] + st["push_remote"] - st0["push_local"] - st0["push_remote"] == 9


def test_training_on_a_small_planted_graph_lowers_the_loss_and_ranks_true_triples_first():
    rng = np.random.default_rng(5)
    ne, nr, n_tr = 30, 3, 200
    truth = rng.standard_normal((ne + nr, 2 * D))
    cand = [(s, r, ob) for s in range(ne) for r in range(nr) for ob in range(ne)]
    sc = np.array([_cscore(truth[s], truth[ne + r], truth[ob]) for s, r, ob in cand])
    pos = [cand[i] for i in np.argsort(-sc)[:n_tr]]                      # the highest-scoring triples are "true"
    subj, rel, obj = (np.array(x, np.int32) for x in zip(*pos))
    o = _server("f32", ne, nr, rng, scale=0.1)
    losses = []
    for epoch in range(30):
        ns_ = rng.integers(0, ne, (n_tr, 2))
        no_ = rng.integers(0, ne, (n_tr, 2))
        tot = 0.0
        for b0 in range(0, n_tr, 20):
            sl = slice(b0, b0 + 20)
            tot += o.kge_step(ne, D, subj[sl], rel[sl], obj[sl], ns_[sl], no_[sl], 0.1, 1e-10)
        losses.append(tot)
    assert losses[-1] < 0.5 * losses[0]
    theta = o.pull(np.arange(ne + nr))[:, :2 * D]
    learned = np.array([_cscore(theta[s], theta[ne + r], theta[ob]) for s, r, ob in cand])
    true_set = set(pos)
    is_true = np.array([c in true_set for c in cand])
    assert learned[is_true].mean() > learned[~is_true].mean() + 1.0
