/*
 * CPU oracle, part 2: one mini-batch step of knowledge-graph-embedding training
 * through the parameter server (Sec. 4.1 "Knowledge graph embeddings" and
 * Appendix A of the paper: SGD with AdaGrad and negative sampling, the AdaGrad
 * metadata stored in the parameter server; model ComplEx, which the paper cites
 * but does not restate - its score is the standard one, written out below).
 *
 * TEST INFRASTRUCTURE ONLY: plain, slow, single-threaded; used by tests/, by the
 * smoke test and by the benchmark's CPU baseline, never by the product path.
 * It shares no code with the HIP path.
 *
 * Key space: entity e is key e, relation r is key num_entities + r.  A value has
 * 4 D numbers: [0, D) real parts, [D, 2D) imaginary parts of the embedding,
 * [2D, 4D) the AdaGrad accumulators of those 2 D numbers.
 *
 * One step (a mini-batch of B data points; a data point is a positive triple (s, r, o) with ns negatives that
 * replace its subject and no negatives that replace its object - Appendix A: the negatives are derived from the
 * data point, and the parameters a worker needs for a data point include those of its negatives).  A data point
 * has 3 + ns + no key slots: subject, relation, object, each subject negative, each object negative.
 *   1. pull the keys of all slots of the batch (values as they are before the step);
 *   2. per data point, the loss is the sum over its scored triples (positive: label +1, negative: label -1) of
 *        loss  = log(1 + exp(-label * score)),   score = Re sum_k e_s[k] w_r[k] conj(e_o[k]),
 *        dloss/dscore = -label * sigmoid(-label * score);
 *      the gradient g of that loss for the 2 D numbers of a slot is the sum, in the order of the scored triples
 *      (positive, subject negatives, object negatives), of the terms of the triples the slot occurs in - the
 *      subject in the positive triple and every object negative, the relation in all, the object in the positive
 *      triple and every subject negative, a negative in its own triple;
 *      AdaGrad, once per slot:  dtheta = -lr * g / sqrt(G + g*g + eps),  dG = g*g,  G the pulled accumulator;
 *   3. push all slots as cumulative deltas, in the order (data point; subject, relation, object, subject
 *      negatives, object negatives).  A key that fills several slots of the batch (in one data point or in
 *      several) gets one term per slot, each from the accumulator as pulled.
 * Negatives are passed in (no random numbers are drawn here).
 *
 * Compiled twice: -DREAL=float and -DREAL=double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL float
#endif

typedef struct orc_ps orc_ps;
int orc_ps_pull(orc_ps *ps, int32_t worker, const int64_t *keys, int64_t n, REAL *out);
int orc_ps_push(orc_ps *ps, int32_t worker, const int64_t *keys, int64_t n, const REAL *deltas);
int orc_ps_localize(orc_ps *ps, const int64_t *keys, int64_t n, int32_t worker);

/* score of one triple; e_s, w_r, e_o point at 2 D numbers (real parts, then imaginary parts) */
REAL orc_kge_score(int32_t D, const REAL *es, const REAL *wr, const REAL *eo) {
    REAL acc = 0;
    for (int32_t k = 0; k < D; ++k) {
        const REAL sr = es[k], si = es[D + k], rr = wr[k], ri = wr[D + k], or_ = eo[k], oi = eo[D + k];
        /* Re((sr + i si)(rr + i ri)(or - i oi)) */
        acc += sr * rr * or_ + si * rr * oi + sr * ri * oi - si * ri * or_;
    }
    return acc;
}

/* number of keys a step pulls (and pushes): the slots of its data points */
int64_t orc_kge_occurrences(int64_t B, int32_t ns, int32_t no) { return B * (3 + ns + no); }

/* One step.  loss_out (may be NULL): sum of the losses of all scored triples.  Returns the push's status. */
int orc_kge_step(orc_ps *ps, int32_t worker, int64_t num_entities, int32_t D, int64_t B, const int32_t *subj, const int32_t *rel,
                 const int32_t *obj, int32_t ns, const int32_t *neg_subj, int32_t no, const int32_t *neg_obj, REAL lr, REAL eps,
                 double *loss_out) {
    const int32_t L = 4 * D, per = 1 + ns + no, slots = 3 + ns + no;
    const int64_t nkeys = B * slots;
    int64_t *keys = (int64_t *)calloc((size_t)(nkeys > 0 ? nkeys : 1), sizeof(int64_t));
    REAL *vals = (REAL *)malloc((size_t)(nkeys > 0 ? nkeys : 1) * L * sizeof(REAL));
    REAL *delta = (REAL *)calloc((size_t)(nkeys > 0 ? nkeys : 1) * L, sizeof(REAL));
    REAL *grad = (REAL *)malloc((size_t)slots * 2 * D * sizeof(REAL));
    if (!keys || !vals || !delta || !grad) { free(keys); free(vals); free(delta); free(grad); return -4; }
    /* the slots, in the stated order */
    for (int64_t b = 0; b < B; ++b) {
        int64_t *kb = keys + b * slots;
        kb[0] = subj[b]; kb[1] = num_entities + rel[b]; kb[2] = obj[b];
        for (int32_t j = 0; j < ns; ++j) kb[3 + j] = neg_subj[b * ns + j];
        for (int32_t j = 0; j < no; ++j) kb[3 + ns + j] = neg_obj[b * no + j];
    }
    int rc = orc_ps_pull(ps, worker, keys, nkeys, vals);
    double loss = 0.0;
    if (rc == 0) {
        for (int64_t b = 0; b < B; ++b) {
            const REAL *vb = vals + b * slots * L;
            for (int32_t i = 0; i < slots * 2 * D; ++i) grad[i] = 0;
            for (int32_t j = 0; j < per; ++j) {                      /* the scored triples of the data point */
                const int32_t slot_s = (j >= 1 && j <= ns) ? 3 + (j - 1) : 0;
                const int32_t slot_o = j > ns ? 3 + ns + (j - 1 - ns) : 2;
                const REAL label = j == 0 ? (REAL)1 : (REAL)-1;
                const REAL *es = vb + slot_s * L, *wr = vb + 1 * L, *eo = vb + slot_o * L;
                const REAL score = orc_kge_score(D, es, wr, eo);
                const REAL z = -label * score;
                /* log(1 + exp(z)) and sigmoid(z), written so that neither overflows */
                const REAL sig = z >= 0 ? (REAL)1 / ((REAL)1 + (REAL)exp((double)-z)) : (REAL)exp((double)z) / ((REAL)1 + (REAL)exp((double)z));
                loss += z >= 0 ? (double)z + log1p(exp((double)-z)) : log1p(exp((double)z));
                const REAL dl = -label * sig;                         /* dloss / dscore */
                REAL *gs = grad + slot_s * 2 * D, *gr = grad + 1 * 2 * D, *go = grad + slot_o * 2 * D;
                for (int32_t k = 0; k < D; ++k) {
                    const REAL sr = es[k], si = es[D + k], rr = wr[k], ri = wr[D + k], or_ = eo[k], oi = eo[D + k];
                    gs[k] = gs[k] + dl * (rr * or_ + ri * oi);  gs[D + k] = gs[D + k] + dl * (rr * oi - ri * or_);   /* d/d Re e_s, d/d Im e_s */
                    gr[k] = gr[k] + dl * (sr * or_ + si * oi);  gr[D + k] = gr[D + k] + dl * (sr * oi - si * or_);   /* d/d Re w_r, d/d Im w_r */
                    go[k] = go[k] + dl * (sr * rr - si * ri);   go[D + k] = go[D + k] + dl * (si * rr + sr * ri);    /* d/d Re e_o, d/d Im e_o */
                }
            }
            for (int32_t sl = 0; sl < slots; ++sl) {                  /* AdaGrad, once per slot */
                const REAL *v = vb + sl * L;
                REAL *d = delta + (b * slots + sl) * L;
                for (int32_t i = 0; i < 2 * D; ++i) {
                    const REAL gg = grad[sl * 2 * D + i], G = v[2 * D + i];
                    d[i] = -lr * gg / (REAL)sqrt((double)(G + gg * gg + eps));
                    d[2 * D + i] = gg * gg;
                }
            }
        }
        rc = orc_ps_push(ps, worker, keys, nkeys, delta);
    }
    if (loss_out) *loss_out = loss;
    free(keys); free(vals); free(delta); free(grad);
    return rc;
}

/* the entity keys a batch of triples [t0, t1) will access: per triple its subject, its object, its subject
 * negatives, its object negatives */
static int64_t entity_keys(int64_t t0, int64_t t1, const int32_t *subj, const int32_t *obj, int32_t ns, const int32_t *neg_subj,
                           int32_t no, const int32_t *neg_obj, int64_t *keys) {
    int64_t n = 0;
    for (int64_t t = t0; t < t1; ++t) {
        keys[n++] = subj[t]; keys[n++] = obj[t];
        for (int32_t j = 0; j < ns; ++j) keys[n++] = neg_subj[t * ns + j];
        for (int32_t j = 0; j < no; ++j) keys[n++] = neg_obj[t * no + j];
    }
    return n;
}

/*
 * One epoch as the paper sets knowledge-graph-embedding training up (Appendix A): the triples are partitioned
 * over P workers (by relation: worker w has the triples [part_ptr[w], part_ptr[w+1])), every worker goes through
 * its part in batches of B, the workers taking turns (worker 0's batch r, worker 1's batch r, ...).
 * With lookahead != 0 parameters are allocated where they are used: each worker first localizes the relation
 * keys of its part ("data clustering": all relation accesses local) and the entity keys of its first batch,
 * and before it works on a batch it localizes the entity keys of its next one ("latency hiding").  An entity
 * that another worker localizes in between is accessed remotely: a localization conflict.  With lookahead == 0
 * nothing is relocated (a classic parameter server).  The values do not depend on lookahead.
 * loss_out (may be NULL): summed loss of all scored triples of the epoch.
 */
int orc_kge_epoch(orc_ps *ps, int64_t num_entities, int32_t D, const int32_t *subj, const int32_t *rel, const int32_t *obj,
                  int32_t ns, const int32_t *neg_subj, int32_t no, const int32_t *neg_obj, const int64_t *part_ptr, int32_t P,
                  int64_t B, int32_t lookahead, REAL lr, REAL eps, double *loss_out) {
    if (P <= 0 || B <= 0) return -1;
    int64_t longest = 0;
    for (int32_t w = 0; w < P; ++w) if (part_ptr[w + 1] - part_ptr[w] > longest) longest = part_ptr[w + 1] - part_ptr[w];
    int64_t cap = (longest > B ? longest : B) * (2 + ns + no) + 1;
    int64_t *keys = (int64_t *)malloc((size_t)cap * sizeof(int64_t));
    if (!keys) return -4;
    int rc = 0;
    double loss = 0.0;
    if (lookahead) {
        for (int32_t w = 0; w < P && !rc; ++w) {                     /* relations go where their triples are */
            int64_t n = 0;
            for (int64_t t = part_ptr[w]; t < part_ptr[w + 1]; ++t) keys[n++] = num_entities + rel[t];
            rc = orc_ps_localize(ps, keys, n, w);
        }
        for (int32_t w = 0; w < P && !rc; ++w) {                     /* the first batch's entities */
            int64_t t0 = part_ptr[w], t1 = t0 + B < part_ptr[w + 1] ? t0 + B : part_ptr[w + 1];
            rc = orc_ps_localize(ps, keys, entity_keys(t0, t1, subj, obj, ns, neg_subj, no, neg_obj, keys), w);
        }
    }
    for (int64_t r = 0; r * B < longest && !rc; ++r) {
        for (int32_t w = 0; w < P && !rc; ++w) {
            int64_t t0 = part_ptr[w] + r * B, end = part_ptr[w + 1];
            if (t0 >= end) continue;
            int64_t t1 = t0 + B < end ? t0 + B : end;
            if (lookahead && t1 < end) {                              /* the batch after this one */
                int64_t u1 = t1 + B < end ? t1 + B : end;
                rc = orc_ps_localize(ps, keys, entity_keys(t1, u1, subj, obj, ns, neg_subj, no, neg_obj, keys), w);
                if (rc) break;
            }
            double l = 0.0;
            rc = orc_kge_step(ps, w, num_entities, D, t1 - t0, subj + t0, rel + t0, obj + t0, ns, neg_subj + t0 * ns, no,
                              neg_obj + t0 * no, lr, eps, &l);
            loss += l;
        }
    }
    if (loss_out) *loss_out = loss;
    free(keys);
    return rc;
}
