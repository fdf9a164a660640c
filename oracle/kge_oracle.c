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
 * One step (a mini-batch of B positive triples (s, r, o), each with ns negatives
 * that replace the subject and no negatives that replace the object):
 *   1. pull every key occurrence of the batch (values as they are before the step);
 *   2. for every scored triple (positive: label +1, negative: label -1):
 *        score = Re sum_k e_s[k] w_r[k] conj(e_o[k])
 *        loss  = log(1 + exp(-label * score)),  dloss/dscore = -label * sigmoid(-label * score)
 *        g     = dloss/dscore * dscore/dtheta   for the 2 D numbers of each of its three keys;
 *        the occurrence's update is  dtheta = -lr * g / sqrt(G + g*g + eps),  dG = g*g
 *        with G the pulled accumulator (AdaGrad with the occurrence's own gradient);
 *   3. push all occurrences as cumulative deltas, in the order (triple of the
 *      batch, positive then subject-negatives then object-negatives, role s, r, o).
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

/* number of key occurrences of a step */
int64_t orc_kge_occurrences(int64_t B, int32_t ns, int32_t no) { return B * (1 + ns + no) * 3; }

/* One step.  loss_out (may be NULL): sum of the losses of all scored triples.  Returns the push's status. */
int orc_kge_step(orc_ps *ps, int32_t worker, int64_t num_entities, int32_t D, int64_t B, const int32_t *subj, const int32_t *rel,
                 const int32_t *obj, int32_t ns, const int32_t *neg_subj, int32_t no, const int32_t *neg_obj, REAL lr, REAL eps,
                 double *loss_out) {
    const int32_t L = 4 * D, per = 1 + ns + no;
    const int64_t nocc = B * per * 3;
    int64_t *keys = (int64_t *)malloc((size_t)(nocc > 0 ? nocc : 1) * sizeof(int64_t));
    REAL *vals = (REAL *)malloc((size_t)(nocc > 0 ? nocc : 1) * L * sizeof(REAL));
    REAL *delta = (REAL *)calloc((size_t)(nocc > 0 ? nocc : 1) * L, sizeof(REAL));
    if (!keys || !vals || !delta) { free(keys); free(vals); free(delta); return -4; }
    /* the occurrences, in the stated order */
    for (int64_t b = 0; b < B; ++b) {
        for (int32_t j = 0; j < per; ++j) {
            int64_t s = subj[b], o = obj[b];
            if (j >= 1 && j <= ns) s = neg_subj[b * ns + (j - 1)];
            if (j > ns) o = neg_obj[b * no + (j - 1 - ns)];
            int64_t *k3 = keys + (b * per + j) * 3;
            k3[0] = s; k3[1] = num_entities + rel[b]; k3[2] = o;
        }
    }
    int rc = orc_ps_pull(ps, worker, keys, nocc, vals);
    double loss = 0.0;
    if (rc == 0) {
        for (int64_t t = 0; t < B * per; ++t) {
            const REAL label = (t % per) == 0 ? (REAL)1 : (REAL)-1;
            const REAL *es = vals + (t * 3 + 0) * L, *wr = vals + (t * 3 + 1) * L, *eo = vals + (t * 3 + 2) * L;
            const REAL score = orc_kge_score(D, es, wr, eo);
            const REAL z = -label * score;
            /* log(1 + exp(z)) and sigmoid(z), written so that neither overflows */
            const REAL sig = z >= 0 ? (REAL)1 / ((REAL)1 + (REAL)exp((double)-z)) : (REAL)exp((double)z) / ((REAL)1 + (REAL)exp((double)z));
            loss += z >= 0 ? (double)z + log1p(exp((double)-z)) : log1p(exp((double)z));
            const REAL dl = -label * sig;                         /* dloss / dscore */
            for (int32_t k = 0; k < D; ++k) {
                const REAL sr = es[k], si = es[D + k], rr = wr[k], ri = wr[D + k], or_ = eo[k], oi = eo[D + k];
                REAL g[3][2];
                g[0][0] = dl * (rr * or_ + ri * oi);  g[0][1] = dl * (rr * oi - ri * or_);      /* d/d Re e_s, d/d Im e_s */
                g[1][0] = dl * (sr * or_ + si * oi);  g[1][1] = dl * (sr * oi - si * or_);      /* d/d Re w_r, d/d Im w_r */
                g[2][0] = dl * (sr * rr - si * ri);   g[2][1] = dl * (si * rr + sr * ri);       /* d/d Re e_o, d/d Im e_o */
                for (int role = 0; role < 3; ++role) {
                    const REAL *v = vals + (t * 3 + role) * L;
                    REAL *d = delta + (t * 3 + role) * L;
                    for (int part = 0; part < 2; ++part) {
                        const REAL gg = g[role][part], G = v[2 * D + part * D + k];
                        d[part * D + k] = -lr * gg / (REAL)sqrt((double)(G + gg * gg + eps));
                        d[2 * D + part * D + k] = gg * gg;
                    }
                }
            }
        }
        rc = orc_ps_push(ps, worker, keys, nocc, delta);
    }
    if (loss_out) *loss_out = loss;
    free(keys); free(vals); free(delta);
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
