/*
 * dpaps - a parameter server with dynamic parameter allocation, and the blocked
 * latent-factor SGD it drives, on one AMD MI355X (gfx950).
 *
 * C ABI.  Every function returns a status (0 = PS_OK, negative = error) and
 * never throws or prints.  Unless a parameter says "host", a pointer is a
 * device pointer valid on the device that was current at ps_create; the caller
 * owns every buffer it passes and may reuse it once the stream has passed the
 * call.  `stream` is a hipStream_t (NULL = the null stream).  Calls are
 * asynchronous on that stream and take effect in stream order, which is the
 * program order of one client (Sec. 3.4, "Asynchronous operations"); one
 * handle must not be driven from two streams at once.  Some calls put part of
 * their work (statistics, a sort) on a second stream that the library creates
 * at default priority; that work starts after what precedes the call on
 * `stream` and `stream` waits for it before the call's effects are complete, so
 * the order seen on `stream` is unchanged.
 *
 * Keys are 0 .. num_keys-1; each key holds a vector of value_len fp32 values
 * (Sec. 4.1 "Settings and measures": the experiments keep one vector of
 * parameter values under every key; dense storage, Sec. 3.7).  There are
 * num_workers workers, each its own node.  Every key has a static home node, home(k) = k / ceil(num_keys /
 * num_workers) (range partitioning, Sec. 3.5), and a dynamic owner node,
 * initially its home (Sec. 3.1 "Location management").
 *
 * Where a call waits.  "Asynchronous" holds for the steady state; these calls wait for
 * `stream` (hipStreamSynchronize) or for the device, and may allocate device memory:
 *   ps_create, ps_destroy, mf_load_ratings, mf_block_ratings   set-up calls: allocate, wait for the device;
 *   ps_status, ps_stats, mf_train_sse                          return a value to the host: wait for `stream`;
 *   ps_push, kge_sgd_step, kge_sgd_epoch, mf_train_sse         scratch of the library grows with the largest
 *       call so far: a call that outgrows it waits for the work that uses the old scratch, frees it and
 *       allocates (the push's scratch: waits for the device; the step's own: for `stream`); calls of a size
 *       seen before do not wait.  kge_sgd_step / kge_sgd_epoch with loss_host_out also wait for `stream` to hand back the loss;
 *   mf_sgd_epoch     the first epoch after mf_load_ratings allocates a small per-block plan; an epoch whose
 *       schedule differs from the previous call's waits for `stream` before it replaces the schedule on the
 *       device (and allocates if it is longer); repeated epochs with one schedule do neither;
 *   mf_sgd_epoch_handoff   allocates its state on first use, and always waits for `stream` at its end: it
 *       returns the order of the epoch to the host;
 *   ps_set_option(PS_OPT_LOCATION_CACHES)   waits for the device, frees and allocates the caches.
 * ps_pull, ps_localize, ps_owner and ps_push_noalloc neither wait nor allocate.
 *
 * Errors.  Host-visible mistakes (null pointers, sizes, worker ids, a bad
 * schedule) are reported by the call itself and nothing is changed.  A key
 * outside [0, num_keys) is found on the device: the offending call and every
 * later call on the handle then change nothing, and PS_EKEY is returned by the
 * next ps_status / ps_stats / mf_train_sse, which also re-arms the handle.
 */
#ifndef DPAPS_H
#define DPAPS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dpaps_ps *ps_handle;

enum {
    PS_OK = 0,
    PS_EINVAL = -1,     /* null pointer, negative size, value_len out of range, call out of sequence */
    PS_EKEY = -2,       /* a key, row or column index out of range (deferred, see above) */
    PS_EWORKER = -3,    /* worker id outside [-1, num_workers) (or [0, num_workers) where a worker is required) */
    PS_ECONFLICT = -4,  /* two tasks of one stratum share a worker, a row block or a column block */
    PS_ENOMEM = -5,     /* device or host allocation failed */
    PS_EHIP = -6,       /* a HIP runtime call failed; ps_last_error gives its text */
    PS_EREMOTE = -7,    /* an access inside a subepoch was not local (cannot happen through mf_sgd_epoch) */
    PS_ELAYOUT = -8,    /* entries are not stored block by block with each column's entries contiguous */
    PS_ELIMIT = -9,     /* a documented capacity limit was exceeded (see mf_load_ratings) */
    PS_ESTALL = -10     /* internal: a bounded wait inside the SGD kernel ran out (deferred like PS_EKEY) */
};

/* Integer statistics of a handle (ps_stats).  "Local" and "remote" are judged
 * against the owner map at the time of the access (Table "reloc-stats": local
 * / non-local reads).  Message counts follow the home-node strategy without
 * location caches: a remote access is request -> home, forward -> owner, reply
 * -> requester (Sec. 3.3 "forward"); a relocation is request -> home, instruct
 * -> old owner, transfer -> requester (Sec. 3.2).  Within one call, messages to
 * the same node are grouped into one (Sec. 3.7 "Message grouping"), and a hop
 * whose two ends are the same node sends nothing. */
enum {
    PS_STAT_PULL_LOCAL = 0, PS_STAT_PULL_REMOTE, PS_STAT_PUSH_LOCAL, PS_STAT_PUSH_REMOTE,
    PS_STAT_RELOCATED,          /* keys whose owner changed */
    PS_STAT_LOCALIZE_KEYS,      /* keys passed to localize, moved or not */
    PS_STAT_MSG_ACC_REQ, PS_STAT_MSG_ACC_FWD, PS_STAT_MSG_ACC_REPLY,
    PS_STAT_MSG_LOC_REQ, PS_STAT_MSG_LOC_INSTRUCT, PS_STAT_MSG_LOC_TRANSFER,
    PS_STAT_CACHE_HIT, PS_STAT_CACHE_STALE,   /* remote accesses routed by a correct / a stale location cache entry
                                                 (PS_OPT_LOCATION_CACHES) */
    PS_STAT_COUNT
};

/* Options for ps_set_option. */
enum {
    PS_OPT_MF_EXACT = 1,        /* 1: the SGD kernel sums each inner product in index order with separately
                                   rounded multiplies and adds (slow; for bit-for-bit checks).  default 0 */
    PS_OPT_MF_CACHE_ROWS = 2,   /* upper bound on row factors a workgroup keeps in LDS (-1 = as many as fit) */
    PS_OPT_MF_WAVES = 3,        /* wavefronts per workgroup in the SGD kernel: 1..16, or 0 (default): 16, but 12 for the
                                   grouped kernel on data with very long column runs or mostly one entry per row
                                   and block */
    PS_OPT_MF_PROFILE = 4,      /* 1: bracket every SGD kernel launch with a pair of events (see mf_profile_read) */
    PS_OPT_MF_GROUPED = 5,      /* 1 (default): where rank <= 128 and PS_OPT_MF_EXACT is off, process the long column
                                   runs of a block in groups of up to 15 entries with dense 16x16xr products and
                                   the other entries row by row; 0: every column run entry by entry */
    PS_OPT_MF_HEAVY_LEN = 6,    /* column runs with at least this many entries count as long (default 48; read by
                                   mf_load_ratings, so set it before) */
    PS_OPT_PUSH_SEQUENTIAL = 7, /* 1: ps_push adds the update terms of a key strictly one after the other in argument
                                   order, however many there are (one wavefront per key; for bit-for-bit checks
                                   against a sequential server).  0 (default): see ps_push */
    PS_OPT_MF_TEAM_MAX = 8,     /* grouped SGD kernel: the most wavefronts that take the groups of one long column run
                                   in turn, 1..14, or 0 (default): 4, one per vector unit of a compute unit - 8 on data
                                   with very long column runs, where the workgroup has 12 wavefronts */
    PS_OPT_MF_CLASSIC = 9,      /* mf_sgd_epoch as on a classic parameter server (Sec. 2.1, Sec. 4.2, Sec. 4.6): no
                                   relocation, no residency - every entry pulls its two keys from the store and
                                   pushes the update terms back, counted as local or remote by the owner map as it
                                   stands, with the messages.  1: the push reads the stored values again (values
                                   are copied out of and back into the server); 2: the rows are updated in place.
                                   0 (default): dynamic parameter allocation.  The values are the same in all
                                   three; honours PS_OPT_MF_EXACT.  A comparison mode: one wavefront per task */
    PS_OPT_KGE_EXACT = 11,      /* 1: kge_sgd_step / kge_sgd_epoch sum every score in index order and take the AdaGrad root in
                                   double with a correctly rounded division (slow; together with PS_OPT_PUSH_SEQUENTIAL
                                   the step then gives, bit for bit, what a sequential fp32 program gives).  default 0 */
    PS_OPT_LOCATION_CACHES = 10 /* 1: every node keeps a location cache, key -> node (Sec. 3.3 "Location caching", Fig.
                                   "routing" (c), (d)), for the message counts of remote pulls and pushes: with a
                                   correct entry the request goes straight to the owner (2 messages), with a stale
                                   one to the node named there, on to the home node and on to the owner (4); without
                                   an entry as without caches (3).  A call is routed with the caches as it finds
                                   them; afterwards its replies have set the requester's entries for the remote keys
                                   it mentioned to their owners.  A relocation tells the old owner where the key
                                   went.  Nothing else changes an entry.  Statistics only: values and owners are
                                   the same.  Two bytes per node and key (at most 16 GiB: PS_ELIMIT); switching on
                                   or off empties the caches and synchronizes the device.  While on, mf_sgd_epoch and
                                   mf_sgd_epoch_handoff return PS_EINVAL: their accesses are local, or go to keys
                                   at home (classic mode), where an entry changes nothing (Sec. 4.6).  0 (default) */
};

/* ---- the parameter server (Table "Primitives", Sec. 3.1) ---------------- */

/* Create a server of num_keys x value_len zeros, owner[k] = home(k).
 * 1 <= value_len <= 1024 (matrix factorization: rank <= 256), 1 <= num_workers <= 2048.  *out is owned by the
 * library until ps_destroy. */
int ps_create(int64_t num_keys, int32_t value_len, int32_t num_workers, ps_handle *out);
int ps_destroy(ps_handle ps);

/* pull: out[p*value_len + c] = value of keys[p], wherever the key lives (Sec.
 * 2.3: location transparency).  Duplicate keys are allowed.  worker = -1 is an
 * outside client: values only, no locality statistics. */
int ps_pull(ps_handle ps, int32_t worker, const int64_t *keys, int64_t n, float *out, void *stream);

/* push: cumulative (Sec. 2.1) - value[keys[p]] += deltas[p*value_len ..], one
 * fp32 addition per term.  All terms of a call are applied, in an order that
 * depends on the arguments only, never on how the device schedules the work (no
 * floating-point atomics): the (key, p) pairs are sorted by key, p ascending,
 * and cut into ranges of 64 pairs.  The terms of a key inside one range are
 * added one after the other in increasing p - onto the stored value where the
 * key's terms start in that range, onto zero otherwise - and the sums of a
 * key's ranges are then added in range order.  A key whose terms lie in one
 * range (every key mentioned once, most keys mentioned a few times) thus gets
 * exactly what a sequential server computes; with PS_OPT_PUSH_SEQUENTIAL every
 * key does, at the price of one wavefront per key. */
int ps_push(ps_handle ps, int32_t worker, const int64_t *keys, int64_t n, const float *deltas, void *stream);

/* ps_push for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Same arguments, same result bit for bit and same statistics as ps_push, but
 * the call makes no hipMalloc / hipFree and calls no allocating routine: its scratch (sorted pairs, the sort's
 * buffers, partial sums) is a fixed array of 16 MiB in device memory, one per device the library runs on, held
 * until the process ends.  Limits (PS_ELIMIT, nothing changed): n <= PS_PUSH_NOALLOC_MAX_KEYS and
 * ceil(n / 64) * value_len <= PS_PUSH_NOALLOC_MAX_PARTIAL.  The statistics run on `stream` itself (no second
 * stream).  All calls on one device share that device's array, whatever the handle: calls that overlap on one
 * device (two streams, two handles) race; the array keeps the last call's contents and every call overwrites
 * what it reads.  No memset nodes are issued, so the call may be captured into a graph. */
#define PS_PUSH_NOALLOC_MAX_KEYS 262144
#define PS_PUSH_NOALLOC_MAX_PARTIAL 1048576
int ps_push_noalloc(ps_handle ps, int32_t worker, const int64_t *keys, int64_t n, const float *deltas, void *stream);

/* localize: relocate the keys to `worker` (Sec. 3.1 "API", Sec. 3.2).  The
 * value is untouched, there is no replica, and the last localize of a key in
 * stream order decides its owner (Sec. 3.2, localization conflicts). */
int ps_localize(ps_handle ps, const int64_t *keys, int64_t n, int32_t worker, void *stream);

/* owner_out[p] = current owner of keys[p]. */
int ps_owner(ps_handle ps, const int64_t *keys, int64_t n, int32_t *owner_out, void *stream);

/* Copy the PS_STAT_COUNT counters to host memory.  Synchronizes the stream. */
int ps_stats(ps_handle ps, int64_t *host_out, void *stream);

/* Synchronize the stream and report (and clear) a deferred error. */
int ps_status(ps_handle ps, void *stream);

int ps_set_option(ps_handle ps, int32_t option, int64_t value);

/* Text of the last failure on this handle (host string owned by the library). */
const char *ps_last_error(ps_handle ps);

/* ---- matrix factorization by parameter blocking (Sec. 2.2.2, Sec. 4.1) --- */
/* Row i of the m x n matrix is key i, column j is key m + j (num_keys = m + n,
 * as in Table "ML tasks, models, and datasets"), value_len is the rank.       */

/* Store the revealed entries block by block for the subepochs: block (rb, cb)
 * holds the entries with row_bounds[rb] <= row < row_bounds[rb+1] and
 * col_bounds[cb] <= col < col_bounds[cb+1]; blocks are laid out row-block
 * major.  Inside a block: columns by decreasing number of entries in the block
 * (ties: smaller column first), a column's entries by increasing row, equal
 * cells in input order.  rows/cols/vals (nnz each, any order) are read,
 * rows_out/cols_out/vals_out (nnz each) and block_ptr_host_out (d_row*d_col+1,
 * host) are written.  Synchronizes the stream. */
int mf_block_ratings(int64_t m, int64_t n, int64_t nnz, const int32_t *rows, const int32_t *cols, const float *vals,
                     int32_t d_row, int32_t d_col, const int64_t *row_bounds_host, const int64_t *col_bounds_host,
                     int32_t *rows_out, int32_t *cols_out, float *vals_out, int64_t *block_ptr_host_out,
                     void *stream);

/* Hand the blocked entries (layout of mf_block_ratings: block by block, and in
 * a block the entries of one column contiguous; any order of the columns and
 * of the rows within a column is accepted and is the processing order) to the
 * server, which keeps its own copy.  ps must have m + n keys.  Limits
 * (PS_ELIMIT): nnz < 2^32; in one block at most 65534 rows with two or more
 * entries, at most 32767 entries of one row, and at most 32768 entries of one
 * column outside the block's 8 longest column runs.  Synchronizes the stream. */
int mf_load_ratings(ps_handle ps, int64_t m, int64_t n, int64_t nnz, const int32_t *rows, const int32_t *cols,
                    const float *vals, int32_t d_row, int32_t d_col, const int64_t *row_bounds_host,
                    const int64_t *col_bounds_host, const int64_t *block_ptr_host, void *stream);

/* One pass over the given strata, in order (Sec. 2.2.2).  tasks_host holds
 * (worker, row block, column block) triples; stratum s consists of tasks
 * stratum_ptr_host[s] .. stratum_ptr_host[s+1]-1.  For each stratum: every
 * task localizes the keys of its row block and of its column block (rows
 * ascending, then columns ascending); then each task visits the entries of its
 * block in stored order and for entry (i, j, v) pulls w = value(i), h =
 * value(m+j), forms e = v - <w,h> and pushes lr*(e*h - lambda*w) to key i and
 * lr*(e*w - lambda*h) to key m+j; then all tasks meet at a barrier (Appendix A
 * "Matrix factorization").  The tasks of a stratum must not share a worker or
 * a block (PS_ECONFLICT).  Each access inside a subepoch is local (Sec. 4.1)
 * and is counted as such: 2 local pulls and 2 local pushes per entry. */
int mf_sgd_epoch(ps_handle ps, const int32_t *tasks_host, const int32_t *stratum_ptr_host, int32_t num_strata,
                 float lr, float lambda, void *stream);

/* One pass over all blocks without barriers between subepochs: column blocks are handed from worker to worker
 * as they become free (the asynchronous form of the blocked schedule - NOMAD, which Sec. 2.2.2 names among the
 * algorithms that move parameters to the data; each move is a localize, Sec. 2.3).  Worker w keeps row block w for
 * the whole epoch (needs d_row <= num_workers; one workgroup per worker, one launch per epoch).  A column block is
 * free or held by one worker.  A worker that has finished a block gives its column block back and takes the first
 * one, in cyclic order after the one it had, that is free and that it has not had in this epoch (worker w starts
 * looking at column block floor(w d_col / d_row)); then it localizes its row block and that column block and
 * processes the block's entries in stored order.  Every block is processed once.  The order depends on timing
 * and is reported: order_host_out (host, 2 d_row d_col ints, may be NULL; passing it synchronizes the stream)
 * gets for worker w and its s-th block, at [2 (w d_col + s)], the column block and, next to it, how many workers
 * had that column block before in this epoch.  The factors, the owner map and the statistics are those of
 * mf_sgd_epoch over strata of one task each, (w, w, column block), in any sequence that agrees with both of
 * these orders - blocks that share neither a row block nor a column block commute.  If a deferred error stops the
 * epoch (see ps_status), the entries of the blocks that were not taken are -1.
 * Runs the grouped kernel only: rank <= 128, PS_OPT_MF_EXACT, PS_OPT_MF_CLASSIC off, PS_OPT_MF_GROUPED on
 * (PS_ELIMIT otherwise), d_col <= 4096.  Scratch is allocated by the library. */
int mf_sgd_epoch_handoff(ps_handle ps, float lr, float lambda, int32_t *order_host_out, void *stream);

/* Sum over the loaded entries of (v - <w_i, h_j>)^2, accumulated in fp64 from
 * the fp32 factors; synchronizes the stream.  Also reports a deferred error. */
int mf_train_sse(ps_handle ps, double *sse_host_out, void *stream);

/* With PS_OPT_MF_PROFILE on: synchronize the stream, return the summed duration (milliseconds) of the SGD
 * kernel launches recorded since the last call and their number, and forget them.  Both outputs are host
 * pointers.  For measurement only: the events cost a few microseconds per launch. */
int mf_profile_read(ps_handle ps, double *sgd_ms_host_out, int64_t *launches_host_out, void *stream);

/* ---- knowledge graph embeddings (Sec. 4.1 "Knowledge graph embeddings", Appendix A) ---- */
/* One mini-batch step of ComplEx training with AdaGrad and negative sampling, the AdaGrad accumulators stored in
 * the server next to the embeddings.  Entity e is key e, relation r is key num_entities + r; value_len = 4 * dim:
 * [0, dim) real parts, [dim, 2 dim) imaginary parts, [2 dim, 4 dim) the accumulators of those 2 dim numbers.
 * The batch has `batch` data points: positive triples (subj, rel, obj: device arrays of int32 indices), data point
 * b with n_neg_subj negatives that replace its subject by neg_subj[b * n_neg_subj + j] and n_neg_obj that replace
 * its object by neg_obj[b * n_neg_obj + j] (device; the paper perturbs both, 10 times).  A data point has
 * 3 + n_neg_subj + n_neg_obj key slots: subject, relation, object, subject negatives, object negatives.  The step
 * pulls the keys of all slots (values as they are before the step).  Per data point the loss is the sum over its
 * scored triples - label +1 for the positive, -1 for a negative - of log(1 + exp(-label score)), score = Re sum_k
 * e_s[k] w_r[k] conj(e_o[k]); the gradient g of that loss for the 2 dim numbers of a slot is the sum of the terms
 * of the triples the slot occurs in (subject: the positive and every object negative; relation: all; object: the
 * positive and every subject negative; a negative: its own), in the order positive, subject negatives, object
 * negatives; and the slot takes one AdaGrad step, dtheta = -lr g / sqrt(G + g^2 + eps), dG = g^2 (G: the pulled
 * accumulator) - AdaGrad per data point (Appendix A).  These are cumulative updates: the batch pushes one row per
 * slot, in the order (data point; subject, relation, object, subject negatives, object negatives), with ps_push's
 * rule for keys that fill several slots: the result depends on the arguments only.  Pull and push statistics
 * count every slot, as a ps_pull and a ps_push of those keys would.
 * worker: as for ps_pull / ps_push (locality statistics).  loss_host_out (may be NULL): sum of the losses of all
 * scored triples; asking for it synchronizes the stream.  dim <= 256, 1 + n_neg_subj + n_neg_obj <= 64
 * (PS_ELIMIT).  Scratch is allocated by the library and grows with the batch (a call that outgrows it waits
 * for the stream, frees and allocates). */
int kge_sgd_step(ps_handle ps, int32_t worker, int64_t num_entities, int32_t dim, int64_t batch, const int32_t *subj,
                 const int32_t *rel, const int32_t *obj, int32_t n_neg_subj, const int32_t *neg_subj, int32_t n_neg_obj,
                 const int32_t *neg_obj, float lr, float eps, double *loss_host_out, void *stream);

/* One epoch of that training over several workers with the parameters allocated where they are used (Appendix A:
 * "data clustering" for the relation parameters, "latency hiding" for the entity parameters).  The triples are
 * given grouped by worker - worker w has [part_ptr_host[w], part_ptr_host[w + 1]), all triples of a relation with
 * one worker - and every worker goes through its part in batches of `batch` triples, the workers taking turns
 * (worker 0's batch r, worker 1's batch r, ...), each batch one step as in kge_sgd_step.  With lookahead != 0 every
 * worker first localizes the relation keys of its part and the entity keys (subjects, objects, negatives) of its
 * first batch, and before it works on a batch it localizes the entity keys of its next one; an entity that another
 * worker localizes in between is then accessed remotely (a localization conflict; see the pull / push statistics).
 * With lookahead == 0 nothing is relocated.  The values are the same either way.  The localize calls and the
 * access statistics touch the owner map and the counters only and run on a second stream of the library's beside
 * the work on the values; the call returns with that stream joined into `stream`.  All indices are checked on the
 * device first (a bad one: PS_EKEY from the next status call, nothing is read through it).
 * subj, rel, obj, neg_subj, neg_obj: device arrays over all num_triples triples, as for kge_sgd_step;
 * part_ptr_host: num_parts + 1 offsets, num_parts <= the server's workers.  loss_host_out (may be NULL): sum of the
 * losses of all scored triples of the epoch; asking for it synchronizes the stream. */
int kge_sgd_epoch(ps_handle ps, int64_t num_entities, int32_t dim, int64_t num_triples, const int32_t *subj, const int32_t *rel,
                  const int32_t *obj, int32_t n_neg_subj, const int32_t *neg_subj, int32_t n_neg_obj, const int32_t *neg_obj,
                  const int64_t *part_ptr_host, int32_t num_parts, int64_t batch, int32_t lookahead, float lr, float eps,
                  double *loss_host_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DPAPS_H */
