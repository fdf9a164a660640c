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


def test_negatives_have_label_minus_one_and_a_slot_takes_one_adagrad_step_on_its_summed_gradient():
    """Appendix A: SGD with AdaGrad per data point, the negatives derived from the data point.  The data point's
    loss is the sum over its scored triples; a key slot (subject, relation, object, each negative) gets the gradient
    of that loss - the sum of the terms of the triples it occurs in - and one AdaGrad step on it."""
    rng = np.random.default_rng(3)
    ne, nr, lr, eps = 8, 1, 0.1, 1e-10
    G0 = 0.2
    o = _server("f64", ne, nr, rng, G0)
    before = o.pull(np.arange(ne + nr))
    theta = before[:, :2 * D]
    s, r, ob, s_neg, o_neg = 0, 0, 1, 5, 6
    o.kge_step(ne, D, [s], [r], [ob], [[s_neg]], [[o_neg]], lr, eps)
    after = o.pull(np.arange(ne + nr))
    scored = [(s, ne + r, ob, +1.0), (s_neg, ne + r, ob, -1.0), (s, ne + r, o_neg, -1.0)]
    h = 1e-6

    def grad(key, c):                                                  # of the data point's whole loss
        tp, tm = theta.copy(), theta.copy()
        tp[key, c] += h
        tm[key, c] -= h
        return (_loss(tp, scored) - _loss(tm, scored)) / (2 * h)

    def grad_one(trip, key, c):
        tp, tm = theta.copy(), theta.copy()
        tp[key, c] += h
        tm[key, c] -= h
        return (_loss(tp, [trip]) - _loss(tm, [trip])) / (2 * h)
    for c in range(2 * D):
        # every key of the data point: one AdaGrad step on the gradient of the data point's loss
        for key in (s, ne + r, ob, s_neg, o_neg):
            g = grad(key, c)
            assert abs((after[key, 2 * D + c] - before[key, 2 * D + c]) - g * g) < 1e-8
            assert abs((after[key, c] - before[key, c]) + lr * g / np.sqrt(G0 + g * g + eps)) < 1e-7
        # the perturbed subject occurs once, with the negative label; the relation in all three scored triples,
        # the subject in the positive triple and the one with the replaced object
        assert abs(grad(s_neg, c) - grad_one(scored[1], s_neg, c)) < 1e-8
        assert abs(grad(ne + r, c) - sum(grad_one(t, ne + r, c) for t in scored)) < 1e-8
        assert abs(grad(s, c) - grad_one(scored[0], s, c) - grad_one(scored[2], s, c)) < 1e-8
    # not one step per occurrence: three steps of the relation from the same accumulator would have moved it further
    c = 0
    gs = [grad_one(t, ne + r, c) for t in scored]
    per_occurrence = sum(-lr * x / np.sqrt(G0 + x * x + eps) for x in gs)
    assert abs((after[ne + r, c] - before[ne + r, c]) - per_occurrence) > 1e-4


def test_a_key_in_two_slots_gets_one_term_per_slot_from_the_pulled_accumulator():
    """A negative that happens to be the positive triple's own subject fills a slot of its own: two terms for that key,
    both normalised with the accumulator as pulled, added by the cumulative push."""
    rng = np.random.default_rng(11)
    ne, nr, lr, eps = 6, 1, 0.1, 1e-10
    G0 = 0.05
    o = _server("f64", ne, nr, rng, G0)
    before = o.pull(np.arange(ne + nr))
    theta = before[:, :2 * D]
    s, r, ob = 2, 0, 4
    o.kge_step(ne, D, [s], [r], [ob], [[s]], np.zeros((1, 0)), lr, eps)     # the subject "replaced" by itself
    after = o.pull(np.arange(ne + nr))
    h = 1e-6
    pos, neg = (s, ne + r, ob, +1.0), (s, ne + r, ob, -1.0)

    def grad_one(trip, key, c):
        tp, tm = theta.copy(), theta.copy()
        tp[key, c] += h
        tm[key, c] -= h
        return (_loss(tp, [trip]) - _loss(tm, [trip])) / (2 * h)
    for c in range(2 * D):
        g1, g2 = grad_one(pos, s, c), grad_one(neg, s, c)              # subject slot, negative's slot
        want = -lr * g1 / np.sqrt(G0 + g1 * g1 + eps) - lr * g2 / np.sqrt(G0 + g2 * g2 + eps)
        assert abs((after[s, c] - before[s, c]) - want) < 1e-7
        assert abs((after[s, 2 * D + c] - before[s, 2 * D + c]) - (g1 * g1 + g2 * g2)) < 1e-8


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


def test_large_scores_do_not_overflow_and_counters_see_every_slot():
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
        assert st["pull_local"] + st["pull_remote"] - st0["pull_local"] - st0["pull_remote"] == 5      # s, r, o, two negatives
        assert st["push_local"] + st["push_remote"] - st0["push_local"] - st0["push_remote"] == 5


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


# ---- the epoch with relation partitioning and pre-localization (Appendix A) ------------------------------------
def _epoch_setup(P, seed=7, ne=60, nr=6, n_tr=90):
    from paper_2002_00655_amd import workloads as wl
    w = wl.make_kge(num_entities=ne, num_relations=nr, triples=n_tr, dim=D, n_neg_s=2, n_neg_o=1, seed=seed)
    wp, part_ptr = wl.partition_by_relation(w, P)
    K = ne + nr
    init = np.zeros((K, 4 * D))
    init[:ne, :2 * D] = w.E0
    init[ne:, :2 * D] = w.R0
    return wp, part_ptr, init


def _epoch(prec, wp, part_ptr, init, P, B, lookahead):
    o = Oracle(prec, init.shape[0], init.shape[1], P)
    o.push(np.arange(init.shape[0]), init)
    loss = o.kge_epoch(wp.num_entities, D, wp.subj, wp.rel, wp.obj, wp.neg_subj, wp.neg_obj, part_ptr, B, lookahead, 0.1, 1e-10)
    return o, loss


def test_partition_keeps_every_relation_with_one_worker():
    wp, part_ptr, _ = _epoch_setup(3)
    owners = {}
    for p in range(3):
        for r in set(wp.rel[part_ptr[p]:part_ptr[p + 1]].tolist()):
            assert owners.setdefault(r, p) == p
    assert part_ptr[-1] == wp.subj.size


def test_epoch_is_the_steps_in_turn_and_values_do_not_depend_on_where_parameters_live():
    P, B = 3, 8
    wp, part_ptr, init = _epoch_setup(P)
    a, loss_a = _epoch("f64", wp, part_ptr, init, P, B, 1)
    b, loss_b = _epoch("f64", wp, part_ptr, init, P, B, 0)
    # written out with the step alone: round r, workers in turn
    c = Oracle("f64", init.shape[0], init.shape[1], P)
    c.push(np.arange(init.shape[0]), init)
    loss_c, r = 0.0, 0
    while any(part_ptr[p] + r * B < part_ptr[p + 1] for p in range(P)):
        for p in range(P):
            t0, t1 = part_ptr[p] + r * B, min(part_ptr[p] + (r + 1) * B, part_ptr[p + 1])
            if t0 < t1:
                sl = slice(t0, t1)
                loss_c += c.kge_step(wp.num_entities, D, wp.subj[sl], wp.rel[sl], wp.obj[sl], wp.neg_subj[sl], wp.neg_obj[sl], 0.1, 1e-10, p)
        r += 1
    K = init.shape[0]
    assert np.array_equal(a.pull(np.arange(K)), c.pull(np.arange(K))) and np.array_equal(b.pull(np.arange(K)), c.pull(np.arange(K)))
    assert abs(loss_a - loss_c) < 1e-9 and abs(loss_b - loss_c) < 1e-9
    assert b.stats() == c.stats() and b.stats()["relocated"] == 0


def test_relations_are_always_local_and_entities_remote_only_after_a_conflict():
    """With pre-localization an access is remote only if another worker localized the key after this worker did
    (counted here from the sequence of localize calls written out in Python)."""
    P, B = 3, 8
    wp, part_ptr, init = _epoch_setup(P, seed=9)
    o, _ = _epoch("f64", wp, part_ptr, init, P, B, 1)
    ne, per = wp.num_entities, 1 + wp.neg_subj.shape[1] + wp.neg_obj.shape[1]
    owner = {}                                                         # key -> worker that localized it last
    def ents(t0, t1):
        out = []
        for t in range(t0, t1):
            out += [wp.subj[t], wp.obj[t], *wp.neg_subj[t], *wp.neg_obj[t]]
        return out
    for p in range(P):
        for t in range(part_ptr[p], part_ptr[p + 1]):
            owner[ne + wp.rel[t]] = p
    for p in range(P):
        for k in ents(part_ptr[p], min(part_ptr[p] + B, part_ptr[p + 1])):
            owner[k] = p
    local = remote = 0
    r = 0
    while any(part_ptr[p] + r * B < part_ptr[p + 1] for p in range(P)):
        for p in range(P):
            t0, end = part_ptr[p] + r * B, part_ptr[p + 1]
            if t0 >= end:
                continue
            t1 = min(t0 + B, end)
            for k in ents(t1, min(t1 + B, end)):
                owner[k] = p
            for t in range(t0, t1):                             # the slots of the data point
                for k in [wp.subj[t], ne + wp.rel[t], wp.obj[t], *wp.neg_subj[t], *wp.neg_obj[t]]:
                    if owner[k] == p:
                        local += 1
                    else:
                        remote += 1
        r += 1
    st = o.stats()
    assert st["pull_local"] == st["push_local"] == local and st["pull_remote"] == st["push_remote"] == remote
    assert local + remote == (2 + per) * wp.subj.size
    assert 0 < remote < local / 2                                       # conflicts exist (popular entities) but are the exception
    # one worker: never a conflict
    wp1, pp1, init1 = _epoch_setup(1, seed=9)
    o1, _ = _epoch("f64", wp1, pp1, init1, 1, B, 1)
    assert o1.stats()["pull_remote"] == 0 and o1.stats()["push_remote"] == 0
