/*
 * TEST INFRASTRUCTURE - NOT PART OF THE PRODUCT.
 *
 * Plain, slow CPU statement of what the parameter-server path computes,
 * single-threaded except for orc_mf_sgd_epoch_workers (a timing baseline that
 * runs the independent workers of a subepoch on all cores).  Only tests, the smoke check and the benchmark's CPU-baseline leg
 * may load this file; the HIP library never does, and shares no code with it.
 *
 * Compiled twice: -DREAL=float (values and arithmetic in fp32, the precision
 * the device path stores) and -DREAL=double.  Build with
 *     gcc -O2 -ffp-contract=off -fno-fast-math
 * so that every statement below is one IEEE operation in the written order.
 *
 * What follows the paper and where:
 *   - pull / push / localize and their meaning ........ Table "Primitives" (Sec. 3.1),
 *     Sec. 2.1 (push is cumulative), Sec. 2.3 (location transparency)
 *   - home node (static) / owner node (dynamic) ....... Sec. 3.1 "Location management", Sec. 3.5
 *   - relocation protocol, three messages ............. Sec. 3.2, Fig. "localize-messages"
 *   - remote access, forward strategy, three messages . Sec. 3.3, Fig. "routing" (b)
 *   - location caches (optional): two messages with a correct entry, four with a
 *     stale one (double-forward); entries change only with the replies to pull and
 *     push and with relocations ....................... Sec. 3.3 "Location caching", Fig. "routing" (c), (d)
 *   - message grouping per destination node ........... Sec. 3.7 "Message grouping"
 *   - localization conflict = arrival order ........... Sec. 3.2 (last paragraph)
 *   - parameter blocking with subepochs and a barrier . Sec. 2.2.2, Sec. 4.1, Appendix A
 *
 * Readings where the paper is silent (each also listed in the design notes):
 *   - the SGD step: loss 1/2 (v - <w,h>)^2 + lambda/2 (|w|^2 + |h|^2) per revealed
 *     entry, both factor rows updated from their old values;
 *   - home(k) = k / ceil(K / W) (range partition), initial owner = home;
 *   - a hop whose two ends are the same node sends no message (this is what
 *     makes every relocation on two nodes a two-node affair, Table "reloc-stats");
 *   - duplicates of a key in one push are all applied, in argument order;
 *   - location caches: one per node, key -> node, empty at first.  A call routes all its keys with the caches as
 *     they are when it starts; its replies then set the requester's entries to the owners they came from.  A
 *     relocation tells the old owner where the key went (it hands the value over); the home node always knows, the
 *     new owner needs no entry.  A stale entry that names the home node costs what no entry costs.
 *
 * Parity pins for every function here live in tests/test_oracle_*.py.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef REAL
#define REAL float
#endif

enum {
    ST_PULL_LOCAL = 0, ST_PULL_REMOTE, ST_PUSH_LOCAL, ST_PUSH_REMOTE,
    ST_RELOCATED, ST_LOCALIZE_KEYS,
    ST_MSG_ACC_REQ, ST_MSG_ACC_FWD, ST_MSG_ACC_REPLY,
    ST_MSG_LOC_REQ, ST_MSG_LOC_INSTRUCT, ST_MSG_LOC_TRANSFER,
    ST_CACHE_HIT, ST_CACHE_STALE,     /* remote accesses routed by a correct / by a stale location cache entry */
    ST_COUNT
};

enum { ORC_OK = 0, ORC_EINVAL = -1, ORC_EKEY = -2, ORC_EWORKER = -3, ORC_ECONFLICT = -4,
       ORC_ENOMEM = -5, ORC_EREMOTE = -7 };

typedef struct orc_ps {
    int64_t K;          /* number of keys */
    int32_t L;          /* values per key */
    int32_t W;          /* number of workers (= nodes) */
    int64_t per_home;   /* ceil(K / W): keys per home node */
    REAL *val;          /* K x L, row-major */
    int32_t *owner;     /* K */
    int64_t stats[ST_COUNT];
    /* scratch for counting distinct message destinations of one call */
    uint8_t *seen_h, *seen_o, *seen_pair;
    int64_t *touched;   /* indices set in seen_pair during the call */
    int64_t n_touched;
    int32_t *loc;       /* location caches, W x K: loc[n * K + k] = where node n believes key k to be, -1 = no entry;
                           NULL = the server runs without location caches */
} orc_ps;

int32_t orc_real_bytes(void) { return (int32_t)sizeof(REAL); }
int32_t orc_stats_count(void) { return ST_COUNT; }

/* Sec. 3.5: the home node is assigned statically; here by range partitioning. */
static int32_t home_of(const orc_ps *ps, int64_t k) { return (int32_t)(k / ps->per_home); }

orc_ps *orc_ps_create(int64_t K, int32_t L, int32_t W) {
    if (K <= 0 || L <= 0 || W <= 0) return NULL;
    orc_ps *ps = (orc_ps *)calloc(1, sizeof(orc_ps));
    if (!ps) return NULL;
    ps->K = K; ps->L = L; ps->W = W;
    ps->per_home = (K + W - 1) / W;
    ps->val = (REAL *)calloc((size_t)K * (size_t)L, sizeof(REAL));
    ps->owner = (int32_t *)malloc((size_t)K * sizeof(int32_t));
    ps->seen_h = (uint8_t *)calloc((size_t)W, 1);
    ps->seen_o = (uint8_t *)calloc((size_t)W, 1);
    ps->seen_pair = (uint8_t *)calloc((size_t)W * (size_t)W, 1);
    ps->touched = (int64_t *)malloc((size_t)W * (size_t)W * sizeof(int64_t));
    if (!ps->val || !ps->owner || !ps->seen_h || !ps->seen_o || !ps->seen_pair || !ps->touched) return NULL;
    for (int64_t k = 0; k < K; ++k) ps->owner[k] = home_of(ps, k);   /* classic allocation */
    return ps;
}

void orc_ps_destroy(orc_ps *ps) {
    if (!ps) return;
    free(ps->val); free(ps->owner); free(ps->seen_h); free(ps->seen_o); free(ps->seen_pair); free(ps->touched);
    free(ps->loc);
    free(ps);
}

static int check_keys(const orc_ps *ps, const int64_t *keys, int64_t n) {
    for (int64_t p = 0; p < n; ++p) if (keys[p] < 0 || keys[p] >= ps->K) return ORC_EKEY;
    return ORC_OK;
}

/* One key that has to travel: requester `worker`, home h, current owner o.
 * Grouped per call: one message requester->h for each distinct h, one h->o for
 * each distinct (h,o), one o->requester for each distinct o (Sec. 3.7).  A hop
 * between a node and itself is free. */
static void route_key(orc_ps *ps, int32_t worker, int32_t h, int32_t o, int st_req, int st_fwd, int st_back) {
    if (h != worker && !ps->seen_h[h]) { ps->seen_h[h] = 1; ps->stats[st_req]++; }
    int64_t pi = (int64_t)h * ps->W + o;
    if (!ps->seen_pair[pi]) {
        ps->seen_pair[pi] = 1; ps->touched[ps->n_touched++] = pi;
        if (h != o) ps->stats[st_fwd]++;
    }
    if (o != worker && !ps->seen_o[o]) { ps->seen_o[o] = 1; ps->stats[st_back]++; }
}

static void route_reset(orc_ps *ps) {
    for (int64_t t = 0; t < ps->n_touched; ++t) {
        int64_t pi = ps->touched[t];
        ps->seen_pair[pi] = 0; ps->seen_h[pi / ps->W] = 0; ps->seen_o[pi % ps->W] = 0;
    }
    ps->n_touched = 0;
}

/* Sec. 3.3 "Location caching": switch the location caches on (all entries empty) or off. */
int orc_ps_location_caches(orc_ps *ps, int32_t on) {
    if (!ps) return ORC_EINVAL;
    free(ps->loc); ps->loc = NULL;
    if (on) {
        ps->loc = (int32_t *)malloc((size_t)ps->W * (size_t)ps->K * sizeof(int32_t));
        if (!ps->loc) return ORC_ENOMEM;
        for (int64_t i = 0; i < (int64_t)ps->W * ps->K; ++i) ps->loc[i] = -1;
    }
    return ORC_OK;
}

/* A remote pull or push of key k by `worker`.  Without an entry in the worker's node's location cache: the
 * forward strategy (route_key).  With a correct entry the request goes straight to the owner, which replies: two
 * messages.  With a stale entry it goes to the node named there, which forwards it to the home node, which
 * forwards it to the owner, which replies: four.  Grouping as in route_key: one request per distinct node
 * asked, one forward per distinct (from, to), one reply per distinct owner. */
static void route_access(orc_ps *ps, int32_t worker, int64_t k) {
    const int32_t h = home_of(ps, k), o = ps->owner[k];
    const int32_t c = ps->loc ? ps->loc[(int64_t)worker * ps->K + k] : -1;
    if (c < 0) { route_key(ps, worker, h, o, ST_MSG_ACC_REQ, ST_MSG_ACC_FWD, ST_MSG_ACC_REPLY); return; }
    if (c == o) {
        ps->stats[ST_CACHE_HIT]++;
        /* (the pair (o, o) is marked only so that route_reset finds the two node flags) */
        int64_t pi = (int64_t)o * ps->W + o;
        if (!ps->seen_pair[pi]) { ps->seen_pair[pi] = 1; ps->touched[ps->n_touched++] = pi; }
        if (!ps->seen_h[o]) { ps->seen_h[o] = 1; ps->stats[ST_MSG_ACC_REQ]++; }
        if (!ps->seen_o[o]) { ps->seen_o[o] = 1; ps->stats[ST_MSG_ACC_REPLY]++; }
        return;
    }
    ps->stats[ST_CACHE_STALE]++;
    if (c != worker && !ps->seen_h[c]) { ps->seen_h[c] = 1; ps->stats[ST_MSG_ACC_REQ]++; }
    int64_t p1 = (int64_t)c * ps->W + h, p2 = (int64_t)h * ps->W + o;
    if (!ps->seen_pair[p1]) { ps->seen_pair[p1] = 1; ps->touched[ps->n_touched++] = p1; if (c != h) ps->stats[ST_MSG_ACC_FWD]++; }
    if (!ps->seen_pair[p2]) { ps->seen_pair[p2] = 1; ps->touched[ps->n_touched++] = p2; if (h != o) ps->stats[ST_MSG_ACC_FWD]++; }
    if (!ps->seen_o[o]) { ps->seen_o[o] = 1; ps->stats[ST_MSG_ACC_REPLY]++; }
}

/* The replies of a call have arrived: the requester's node now knows the owner of every key it asked for. */
static void cache_replies(orc_ps *ps, int32_t worker, const int64_t *keys, int64_t n) {
    if (!ps->loc || worker < 0) return;
    for (int64_t p = 0; p < n; ++p)
        if (ps->owner[keys[p]] != worker) ps->loc[(int64_t)worker * ps->K + keys[p]] = ps->owner[keys[p]];
}

/* pull: the current value of each key, wherever it lives (Sec. 2.3). */
int orc_ps_pull(orc_ps *ps, int32_t worker, const int64_t *keys, int64_t n, REAL *out) {
    if (!ps || n < 0 || (n > 0 && (!keys || !out))) return ORC_EINVAL;
    if (worker < -1 || worker >= ps->W) return ORC_EWORKER;
    int rc = check_keys(ps, keys, n); if (rc) return rc;
    for (int64_t p = 0; p < n; ++p) {
        int64_t k = keys[p];
        for (int32_t c = 0; c < ps->L; ++c) out[p * ps->L + c] = ps->val[k * ps->L + c];
        if (worker >= 0) {
            if (ps->owner[k] == worker) ps->stats[ST_PULL_LOCAL]++;
            else { ps->stats[ST_PULL_REMOTE]++; route_access(ps, worker, k); }
        }
    }
    route_reset(ps);
    cache_replies(ps, worker, keys, n);
    return ORC_OK;
}

/* push: cumulative (Sec. 2.1) - the update term is added to the value; the
 * terms of one call are applied in argument order. */
int orc_ps_push(orc_ps *ps, int32_t worker, const int64_t *keys, int64_t n, const REAL *deltas) {
    if (!ps || n < 0 || (n > 0 && (!keys || !deltas))) return ORC_EINVAL;
    if (worker < -1 || worker >= ps->W) return ORC_EWORKER;
    int rc = check_keys(ps, keys, n); if (rc) return rc;
    for (int64_t p = 0; p < n; ++p) {
        int64_t k = keys[p];
        for (int32_t c = 0; c < ps->L; ++c) ps->val[k * ps->L + c] = ps->val[k * ps->L + c] + deltas[p * ps->L + c];
        if (worker >= 0) {
            if (ps->owner[k] == worker) ps->stats[ST_PUSH_LOCAL]++;
            else { ps->stats[ST_PUSH_REMOTE]++; route_access(ps, worker, k); }
        }
    }
    route_reset(ps);
    cache_replies(ps, worker, keys, n);
    return ORC_OK;
}

/* localize: the single copy of each key moves to the caller (Sec. 3.1, 3.2);
 * the value is not touched.  Requests are served in the order given. */
int orc_ps_localize(orc_ps *ps, const int64_t *keys, int64_t n, int32_t worker) {
    if (!ps || n < 0 || (n > 0 && !keys)) return ORC_EINVAL;
    if (worker < 0 || worker >= ps->W) return ORC_EWORKER;
    int rc = check_keys(ps, keys, n); if (rc) return rc;
    for (int64_t p = 0; p < n; ++p) {
        int64_t k = keys[p];
        ps->stats[ST_LOCALIZE_KEYS]++;
        if (ps->owner[k] == worker) continue;          /* already here: nothing travels */
        route_key(ps, worker, home_of(ps, k), ps->owner[k], ST_MSG_LOC_REQ, ST_MSG_LOC_INSTRUCT, ST_MSG_LOC_TRANSFER);
        if (ps->loc) ps->loc[(int64_t)ps->owner[k] * ps->K + k] = worker;   /* the old owner hands the value to `worker` */
        ps->owner[k] = worker;                          /* home updates the location at once */
        ps->stats[ST_RELOCATED]++;
    }
    route_reset(ps);
    return ORC_OK;
}

int orc_ps_owner(const orc_ps *ps, const int64_t *keys, int64_t n, int32_t *out) {
    if (!ps || n < 0 || (n > 0 && (!keys || !out))) return ORC_EINVAL;
    int rc = check_keys(ps, keys, n); if (rc) return rc;
    for (int64_t p = 0; p < n; ++p) out[p] = ps->owner[keys[p]];
    return ORC_OK;
}

int orc_ps_home(const orc_ps *ps, const int64_t *keys, int64_t n, int32_t *out) {
    if (!ps || n < 0 || (n > 0 && (!keys || !out))) return ORC_EINVAL;
    int rc = check_keys(ps, keys, n); if (rc) return rc;
    for (int64_t p = 0; p < n; ++p) out[p] = home_of(ps, keys[p]);
    return ORC_OK;
}

void orc_ps_stats(const orc_ps *ps, int64_t *out) { memcpy(out, ps->stats, sizeof(ps->stats)); }

/* ------------------------------------------------------------------------
 * Matrix factorization by parameter blocking (Sec. 2.2.2, Sec. 4.1).
 * Keys: row i -> key i, column j -> key m + j.
 * ---------------------------------------------------------------------- */

static int32_t block_of(const int64_t *bounds, int32_t d, int64_t id) {
    int32_t b = 0;
    while (b + 1 < d && id >= bounds[b + 1]) ++b;      /* linear scan: plain, not fast */
    return b;
}

typedef struct { int32_t row, col; float val; int64_t cnt; int64_t pos; } ent_t;

static int cmp_ent(const void *a, const void *b) {
    const ent_t *x = (const ent_t *)a, *y = (const ent_t *)b;
    if (x->cnt != y->cnt) return x->cnt > y->cnt ? -1 : 1;   /* busiest column first */
    if (x->col != y->col) return x->col < y->col ? -1 : 1;
    if (x->row != y->row) return x->row < y->row ? -1 : 1;
    return x->pos < y->pos ? -1 : (x->pos > y->pos);
}

/* Data layout for the subepochs: each worker "only processes the corresponding
 * part of its data" (Sec. 2.2.2), so the revealed entries are stored block by
 * block (row block major).  Inside a block the order is a convention of this
 * implementation: columns by decreasing number of entries in the block (ties:
 * smaller column first), and within a column by increasing row. */
int orc_mf_block_ratings(int64_t m, int64_t n, int64_t nnz, const int32_t *rows, const int32_t *cols,
                         const float *vals, int32_t d_row, int32_t d_col, const int64_t *row_bounds,
                         const int64_t *col_bounds, int32_t *rows_out, int32_t *cols_out, float *vals_out,
                         int64_t *block_ptr /* d_row*d_col+1 */) {
    if (m <= 0 || n <= 0 || nnz < 0 || d_row <= 0 || d_col <= 0) return ORC_EINVAL;
    int64_t nb = (int64_t)d_row * d_col;
    int32_t *rb_of = (int32_t *)malloc((size_t)m * sizeof(int32_t));
    int32_t *cb_of = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int64_t *fill = (int64_t *)calloc((size_t)nb + 1, sizeof(int64_t));
    ent_t *ent = (ent_t *)malloc((size_t)(nnz > 0 ? nnz : 1) * sizeof(ent_t));
    int64_t *ccount = (int64_t *)calloc((size_t)n, sizeof(int64_t));
    if (!rb_of || !cb_of || !fill || !ent || !ccount) return ORC_ENOMEM;
    for (int64_t i = 0; i < m; ++i) rb_of[i] = block_of(row_bounds, d_row, i);
    for (int64_t j = 0; j < n; ++j) cb_of[j] = block_of(col_bounds, d_col, j);
    for (int64_t p = 0; p < nnz; ++p) {
        if (rows[p] < 0 || rows[p] >= m || cols[p] < 0 || cols[p] >= n) return ORC_EKEY;
        fill[(int64_t)rb_of[rows[p]] * d_col + cb_of[cols[p]] + 1]++;
    }
    block_ptr[0] = 0;
    for (int64_t b = 0; b < nb; ++b) block_ptr[b + 1] = block_ptr[b] + fill[b + 1];
    for (int64_t b = 0; b <= nb; ++b) fill[b] = block_ptr[b];
    for (int64_t p = 0; p < nnz; ++p) {
        int64_t b = (int64_t)rb_of[rows[p]] * d_col + cb_of[cols[p]];
        ent_t *e = &ent[fill[b]++];
        e->row = rows[p]; e->col = cols[p]; e->val = vals[p]; e->pos = p; e->cnt = 0;
    }
    for (int64_t b = 0; b < nb; ++b) {
        int64_t a = block_ptr[b], z = block_ptr[b + 1];
        for (int64_t p = a; p < z; ++p) ccount[ent[p].col]++;
        for (int64_t p = a; p < z; ++p) ent[p].cnt = ccount[ent[p].col];
        for (int64_t p = a; p < z; ++p) ccount[ent[p].col] = 0;
        qsort(ent + a, (size_t)(z - a), sizeof(ent_t), cmp_ent);
    }
    for (int64_t p = 0; p < nnz; ++p) { rows_out[p] = ent[p].row; cols_out[p] = ent[p].col; vals_out[p] = ent[p].val; }
    free(rb_of); free(cb_of); free(fill); free(ent); free(ccount);
    return ORC_OK;
}

/* One epoch = the given strata in order (Sec. 2.2.2: subepochs; which worker
 * has which block changes from subepoch to subepoch).  tasks[t] = (worker, row
 * block, column block); stratum s holds tasks[stratum_ptr[s] .. stratum_ptr[s+1]).
 * Per subepoch: every task localizes the keys of its two factor blocks (Sec.
 * 2.3: the parameters of a block are relocated to the node that will work on the block), then
 * processes its entries one by one with pull / SGD step / push, then all
 * workers meet at a barrier (Appendix A).  Within a subepoch every access must
 * be local (Sec. 4.1); anything else is reported as ORC_EREMOTE. */
static int mf_epoch(orc_ps *ps, int64_t m, int64_t n, const int32_t *rows, const int32_t *cols, const float *vals,
                    int32_t d_row, int32_t d_col, const int64_t *row_bounds, const int64_t *col_bounds,
                    const int64_t *block_ptr, const int32_t *tasks, const int32_t *stratum_ptr,
                    int32_t num_strata, double lr_in, double lambda_in, int relocate) {
    if (!ps || m + n != ps->K || num_strata < 0) return ORC_EINVAL;
    const int32_t L = ps->L;
    const REAL lr = (REAL)lr_in, lambda = (REAL)lambda_in;
    REAL *buf = (REAL *)malloc((size_t)4 * L * sizeof(REAL));
    uint8_t *used = (uint8_t *)malloc((size_t)ps->W + d_row + d_col);
    if (!buf || !used) return ORC_ENOMEM;
    REAL *wh = buf, *dwh = buf + 2 * L;                 /* pulled [w;h] and the update terms [dw;dh] */
    int rc = ORC_OK;
    for (int32_t s = 0; s < num_strata && rc == ORC_OK; ++s) {
        int32_t t0 = stratum_ptr[s], t1 = stratum_ptr[s + 1];
        /* a stratum is a set of tasks that share no worker and no factor block */
        memset(used, 0, (size_t)ps->W + d_row + d_col);
        for (int32_t t = t0; t < t1; ++t) {
            int32_t w = tasks[3 * t], rb = tasks[3 * t + 1], cb = tasks[3 * t + 2];
            if (w < 0 || w >= ps->W) { rc = ORC_EWORKER; break; }
            if (rb < 0 || rb >= d_row || cb < 0 || cb >= d_col) { rc = ORC_EINVAL; break; }
            if (used[w] || used[ps->W + rb] || used[ps->W + d_row + cb]) { rc = ORC_ECONFLICT; break; }
            used[w] = used[ps->W + rb] = used[ps->W + d_row + cb] = 1;
        }
        if (rc) break;
        for (int32_t t = t0; relocate && t < t1; ++t) { /* relocate the blocks */
            int32_t w = tasks[3 * t], rb = tasks[3 * t + 1], cb = tasks[3 * t + 2];
            int64_t nr = row_bounds[rb + 1] - row_bounds[rb], nc = col_bounds[cb + 1] - col_bounds[cb];
            int64_t *keys = (int64_t *)malloc((size_t)(nr + nc + 1) * sizeof(int64_t));
            if (!keys) { rc = ORC_ENOMEM; break; }
            for (int64_t i = 0; i < nr; ++i) keys[i] = row_bounds[rb] + i;
            for (int64_t j = 0; j < nc; ++j) keys[nr + j] = m + col_bounds[cb] + j;
            rc = orc_ps_localize(ps, keys, nr + nc, w);
            free(keys);
            if (rc) break;
        }
        if (rc) break;
        int64_t remote_before = ps->stats[ST_PULL_REMOTE] + ps->stats[ST_PUSH_REMOTE];
        for (int32_t t = t0; t < t1 && rc == ORC_OK; ++t) {   /* the workers of a stratum are independent */
            int32_t w = tasks[3 * t], rb = tasks[3 * t + 1], cb = tasks[3 * t + 2];
            int64_t b = (int64_t)rb * d_col + cb;
            for (int64_t p = block_ptr[b]; p < block_ptr[b + 1]; ++p) {
                int64_t keys[2] = { rows[p], m + cols[p] };
                rc = orc_ps_pull(ps, w, keys, 2, wh); if (rc) break;
                const REAL *wv = wh, *hv = wh + L;
                REAL dot = 0;
                for (int32_t k = 0; k < L; ++k) dot = dot + wv[k] * hv[k];
                REAL e = (REAL)vals[p] - dot;
                for (int32_t k = 0; k < L; ++k) {
                    dwh[k]     = lr * (e * hv[k] - lambda * wv[k]);
                    dwh[L + k] = lr * (e * wv[k] - lambda * hv[k]);
                }
                rc = orc_ps_push(ps, w, keys, 2, dwh); if (rc) break;
            }
        }
        if (relocate && rc == ORC_OK && ps->stats[ST_PULL_REMOTE] + ps->stats[ST_PUSH_REMOTE] != remote_before) rc = ORC_EREMOTE;
        /* barrier: nothing to do in a sequential program */
    }
    free(buf); free(used);
    return rc;
}

int orc_mf_sgd_epoch(orc_ps *ps, int64_t m, int64_t n, const int32_t *rows, const int32_t *cols, const float *vals,
                     int32_t d_row, int32_t d_col, const int64_t *row_bounds, const int64_t *col_bounds,
                     const int64_t *block_ptr, const int32_t *tasks, const int32_t *stratum_ptr,
                     int32_t num_strata, double lr_in, double lambda_in) {
    return mf_epoch(ps, m, n, rows, cols, vals, d_row, d_col, row_bounds, col_bounds, block_ptr, tasks, stratum_ptr,
                    num_strata, lr_in, lambda_in, 1);
}

/* The same epoch with the workers of a subepoch running side by side on the host's cores, as the workers of the
 * paper do (Sec. 2.2.2: the blocks of a subepoch share no parameters, so their workers need not wait for each
 * other; Appendix A: a barrier after each subepoch).  A timing baseline, kept equal to orc_mf_sgd_epoch bit for
 * bit by tests: the relocation step is the same sequential code; a worker's entry loop is the loop above with
 * pull (copy the two rows out), step and push (one addition per term) written out on the store - every access
 * is checked to be local, which is all the routing there is to count - and its four access counters kept per
 * thread and added up at the barrier.  threads <= 0: as many as the runtime offers. */
int orc_mf_sgd_epoch_workers(orc_ps *ps, int64_t m, int64_t n, const int32_t *rows, const int32_t *cols, const float *vals,
                             int32_t d_row, int32_t d_col, const int64_t *row_bounds, const int64_t *col_bounds,
                             const int64_t *block_ptr, const int32_t *tasks, const int32_t *stratum_ptr,
                             int32_t num_strata, double lr_in, double lambda_in, int32_t threads, int32_t *threads_used) {
    if (!ps || m + n != ps->K || num_strata < 0) return ORC_EINVAL;
    const int32_t L = ps->L;
    const REAL lr = (REAL)lr_in, lambda = (REAL)lambda_in;
    int rc = ORC_OK;
    int used = 1;
    for (int32_t s = 0; s < num_strata && rc == ORC_OK; ++s) {
        int32_t t0 = stratum_ptr[s], t1 = stratum_ptr[s + 1];
        /* validation and relocation: the sequential epoch's, with no entries to process */
        {
            int32_t one[2] = { 0, t1 - t0 };
            int64_t *zero_ptr = (int64_t *)calloc((size_t)d_row * d_col + 1, sizeof(int64_t));
            if (!zero_ptr) return ORC_ENOMEM;
            rc = mf_epoch(ps, m, n, rows, cols, vals, d_row, d_col, row_bounds, col_bounds, zero_ptr, tasks + 3 * (int64_t)t0, one, 1,
                          lr_in, lambda_in, 1);
            free(zero_ptr);
            if (rc) break;
        }
        int64_t pulls = 0, pushes = 0;
        int bad = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(threads > 0 ? threads : omp_get_max_threads()) reduction(+ : pulls, pushes) reduction(| : bad)
#endif
        {
            REAL *wh = (REAL *)malloc((size_t)4 * L * sizeof(REAL));
            REAL *dwh = wh ? wh + 2 * L : NULL;
            if (!wh) bad |= 2;
#ifdef _OPENMP
#pragma omp single
            used = omp_get_num_threads();
#pragma omp for schedule(dynamic, 1)
#endif
            for (int32_t t = t0; t < t1; ++t) {
                if (!wh) continue;
                int32_t w = tasks[3 * t], rb = tasks[3 * t + 1], cb = tasks[3 * t + 2];
                int64_t b = (int64_t)rb * d_col + cb;
                for (int64_t p = block_ptr[b]; p < block_ptr[b + 1]; ++p) {
                    int64_t ki = rows[p], kj = m + cols[p];
                    if (ps->owner[ki] != w || ps->owner[kj] != w) { bad |= 1; break; }      /* Sec. 4.1: all access is local */
                    REAL *vw = ps->val + ki * L, *vh = ps->val + kj * L;
                    for (int32_t k = 0; k < L; ++k) { wh[k] = vw[k]; wh[L + k] = vh[k]; }   /* pull */
                    pulls += 2;
                    const REAL *wv = wh, *hv = wh + L;
                    REAL dot = 0;
                    for (int32_t k = 0; k < L; ++k) dot = dot + wv[k] * hv[k];
                    REAL e = (REAL)vals[p] - dot;
                    for (int32_t k = 0; k < L; ++k) {
                        dwh[k]     = lr * (e * hv[k] - lambda * wv[k]);
                        dwh[L + k] = lr * (e * wv[k] - lambda * hv[k]);
                    }
                    for (int32_t k = 0; k < L; ++k) { vw[k] = vw[k] + dwh[k]; vh[k] = vh[k] + dwh[L + k]; }   /* push */
                    pushes += 2;
                }
            }
            free(wh);
        }
        ps->stats[ST_PULL_LOCAL] += pulls;
        ps->stats[ST_PUSH_LOCAL] += pushes;
        if (bad & 2) rc = ORC_ENOMEM;
        else if (bad & 1) rc = ORC_EREMOTE;
    }
    if (threads_used) *threads_used = used;
    return rc;
}

/* The same epoch on a classic parameter server (Sec. 2.1 "Basic PS Architectures": parameters are allocated
 * statically; Sec. 4.2, Sec. 4.6): nothing is relocated, every entry's pull and push goes to wherever the two
 * keys live and is counted as local or remote, with its messages.  The values come out the same (Sec. 2.3:
 * location transparency). */
int orc_mf_sgd_epoch_classic(orc_ps *ps, int64_t m, int64_t n, const int32_t *rows, const int32_t *cols, const float *vals,
                             int32_t d_row, int32_t d_col, const int64_t *row_bounds, const int64_t *col_bounds,
                             const int64_t *block_ptr, const int32_t *tasks, const int32_t *stratum_ptr,
                             int32_t num_strata, double lr_in, double lambda_in) {
    return mf_epoch(ps, m, n, rows, cols, vals, d_row, d_col, row_bounds, col_bounds, block_ptr, tasks, stratum_ptr,
                    num_strata, lr_in, lambda_in, 0);
}

/* sum over the revealed entries of (v - <w_i, h_j>)^2, accumulated in double */
double orc_mf_train_sse(const orc_ps *ps, int64_t m, int64_t nnz, const int32_t *rows, const int32_t *cols,
                        const float *vals) {
    double sse = 0.0;
    for (int64_t p = 0; p < nnz; ++p) {
        const REAL *w = ps->val + (int64_t)rows[p] * ps->L, *h = ps->val + (m + cols[p]) * ps->L;
        double dot = 0.0;
        for (int32_t k = 0; k < ps->L; ++k) dot += (double)w[k] * (double)h[k];
        double e = (double)vals[p] - dot;
        sse += e * e;
    }
    return sse;
}
