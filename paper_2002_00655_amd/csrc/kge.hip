// One mini-batch step of knowledge-graph-embedding training through the parameter
// server (Sec. 4.1 "Knowledge graph embeddings" and Appendix A of the paper: SGD with
// AdaGrad and negative sampling, the AdaGrad metadata stored in the parameter server;
// model ComplEx, cited there, whose score Re sum_k e_s[k] w_r[k] conj(e_o[k]) is the
// standard one).  The step is what a worker does for a batch of data points: pull the
// parameters of the positive triples and of their negatives, compute the updates, push
// them.  Pull and push are accounted exactly like ps_pull and ps_push for every key
// occurrence (key check, locality statistics, message counts).  The pulled values are read
// from the store by the kernel that uses them instead of being copied out first, and the
// update terms that one data point has for the same key slot are added up before the push,
// which then runs as in ps_push (deterministic order of the cumulative updates).
//
// Key space: entity e is key e, relation r is key num_entities + r.  A value has 4 D
// numbers: [0, D) real parts, [D, 2 D) imaginary parts, [2 D, 4 D) the AdaGrad
// accumulators of those 2 D numbers.
#include "common.h"
#include "mf_device.h"

#include <algorithm>
#include <type_traits>

static inline unsigned grid_for(int64_t n, int block) { return (unsigned)((n + block - 1) / block); }

// the keys of the batch, in pull and push order: per data point its slots - subject, relation, object, subject
// negatives, object negatives
__global__ void k_kge_keys(int64_t num_entities, int64_t batch, const int32_t *subj, const int32_t *rel, const int32_t *obj,
                           int32_t ns, const int32_t *neg_subj, int32_t no, const int32_t *neg_obj, int64_t *keys) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int32_t rows = 3 + ns + no;
    if (i >= batch * rows) return;
    const int64_t b = i / rows;
    const int32_t j = (int32_t)(i - b * rows);
    int64_t k;
    if (j == 0) k = subj[b];
    else if (j == 1) k = num_entities + rel[b];
    else if (j == 2) k = obj[b];
    else if (j < 3 + ns) k = neg_subj[b * ns + (j - 3)];
    else k = neg_obj[b * no + (j - 3 - ns)];
    keys[i] = k;
}

// AdaGrad with the gradient g of a key slot and the accumulator G as pulled:
//   dtheta = -lr g / sqrt(G + g^2 + eps),  dG = g^2
// EXACT: root in double and a correctly rounded division, operation by operation what a sequential fp32 program
// does; otherwise the hardware's reciprocal square root, good to one unit in the last place (G + g^2 + eps >= eps > 0).
struct Upd { float dt, dg; };
template <bool EXACT>
__device__ __forceinline__ Upd adagrad(float g, float G, float lr, float eps) {
    if constexpr (EXACT) return {-lr * g / (float)sqrt((double)(G + g * g + eps)), g * g};
    else return {(-lr * g) * __builtin_amdgcn_rsqf(G + g * g + eps), g * g};
}

// One wavefront per data point - a positive triple and its negatives (Appendix A: the negatives are derived from
// the data point) -, lane l the components l, l + 64, ...  The values come from the store as it holds them (the
// pull).  The data point's loss is the sum over its scored triples; the gradient of a key slot - subject,
// relation, object, each negative - is the sum of the terms of the triples the slot occurs in, added in the order of
// the triples (positive, subject negatives, object negatives), and every slot takes one AdaGrad step on it: the
// data point pushes one row per slot.  The positive triple first, then every negative in one go: its row, its
// score, the derivative of its loss (the same in all lanes), its terms for the two slots it shares with the
// positive triple, its own AdaGrad step.  Score t is also kept in lane t, and the losses of all scored triples
// are evaluated together at the end.
//   loss = log(1 + exp(-label score)),  g = dloss/dscore * dscore/dtheta
// EXACT: every score is summed in index order (the lanes' terms one after the other), for bit-for-bit comparisons
// with a sequential program; otherwise per lane and then across the lanes.
// rows: (3 + ns + no) per data point in upd and in upd_keys (NULL: the caller has the keys already).  1 + ns + no <= 64.
template <int NC, bool EXACT>
__global__ __launch_bounds__(256) void k_kge_group(int64_t batch, int64_t num_entities, int32_t D, const int32_t *subj, const int32_t *rel,
                                                    const int32_t *obj, int32_t ns, const int32_t *neg_subj, int32_t no,
                                                    const int32_t *neg_obj, float lr, float eps, const float *__restrict__ store,
                                                    float *__restrict__ upd,
                                                    int64_t *upd_keys, double *loss, const int32_t *err) {
    if (__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    const int lane = threadIdx.x & 63;
    // the data point is the same for all lanes of a wavefront: said so, its keys and row addresses stay in scalar registers
    const int64_t b = (int64_t)blockIdx.x * (blockDim.x >> 6) + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (b >= batch) return;
    constexpr int CH = NC <= 2 ? 5 : 1;                              // negatives whose rows are in flight together
    const int L = 4 * D, rows = 3 + ns + no;
    const uint32_t Du = (uint32_t)D;                                 // row addresses and field offsets are scalars, k the only lane offset
    const int64_t ks = subj[b], kr = num_entities + rel[b], ko = obj[b];
    const float *vs = store + ks * L, *vr = store + kr * L, *vo = store + ko * L;
    float *u0 = upd + b * rows * L;
    if (lane == 0 && upd_keys) { upd_keys[b * rows + 0] = ks; upd_keys[b * rows + 1] = kr; upd_keys[b * rows + 2] = ko; }
    // the sum of the lanes' terms: term[c] belongs to component lane + 64 c
    auto total = [&](const float (&term)[NC]) {
        if constexpr (EXACT) {
            float acc = 0.0f;
            for (int k = 0; k < D; ++k) {
                float t = 0.0f;
#pragma unroll
                for (int c = 0; c < NC; ++c) t = (k >> 6) == c ? rl_f(term[c], k & 63) : t;
                acc = acc + t;
            }
            return acc;
        } else {
            float part = 0.0f;
#pragma unroll
            for (int c = 0; c < NC; ++c) part += term[c];
            return wave_sum(part);
        }
    };
    float sr[NC], si[NC], rr[NC], ri[NC], orl[NC], oi[NC];
    float score = 0.0f;                                              // lane t: score of scored triple t
    {
        float term[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const uint32_t k = (uint32_t)lane + 64u * c;
            const bool in = k < Du;
            sr[c] = in ? vs[k] : 0.0f; si[c] = in ? (vs + Du)[k] : 0.0f;
            rr[c] = in ? vr[k] : 0.0f; ri[c] = in ? (vr + Du)[k] : 0.0f;
            orl[c] = in ? vo[k] : 0.0f; oi[c] = in ? (vo + Du)[k] : 0.0f;
            // Re((sr + i si)(rr + i ri)(or - i oi))
            term[c] = sr[c] * rr[c] * orl[c] + si[c] * rr[c] * oi[c] + sr[c] * ri[c] * oi[c] - si[c] * ri[c] * orl[c];
        }
        const float sc = total(term);
        score = lane == 0 ? sc : score;
    }
    // dloss/dscore of one scored triple (the same value in every lane): -label sigmoid(-label score), written so that
    // nothing overflows; EXACT: the exponential in double and rounded to float, as a sequential fp32 program has it
    auto dloss = [](float label, float sc) {
        const float z = -label * sc;
        const float na = z >= 0.0f ? -z : z;                         // -|z|
        float ex;
        if constexpr (EXACT) ex = (float)exp((double)na);
        else ex = __builtin_amdgcn_exp2f(na * 1.44269504088896340736f);   // the hardware's 2^x, good to one unit in the last place
        const float sig = z >= 0.0f ? 1.0f / (1.0f + ex) : ex / (1.0f + ex);
        return -label * sig;
    };
    // the gradients of the subject's, the relation's and the object's slot, started by the positive triple
    float gs[NC][2], gr[NC][2], go[NC][2];
    {
        const float dl = dloss(1.0f, rl_f(score, 0));
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            gs[c][0] = 0.0f + dl * (rr[c] * orl[c] + ri[c] * oi[c]); gs[c][1] = 0.0f + dl * (rr[c] * oi[c] - ri[c] * orl[c]);
            gr[c][0] = 0.0f + dl * (sr[c] * orl[c] + si[c] * oi[c]); gr[c][1] = 0.0f + dl * (sr[c] * oi[c] - si[c] * orl[c]);
            go[c][0] = 0.0f + dl * (sr[c] * rr[c] - si[c] * ri[c]);  go[c][1] = 0.0f + dl * (si[c] * rr[c] + sr[c] * ri[c]);
        }
    }
    // The negatives, CH at a time: their rows (values and accumulators) are asked for together, so that a wavefront
    // waits for memory once per CH negatives, then per negative in order its score, the derivative of its loss,
    // its terms for the two slots it shares with the positive triple, and its own step.
    // OBJ false: subject replaced by n, the triple (n, r, o); true: object replaced by n, the triple (s, r, n); label -1
    auto negatives = [&](auto obj_tag, const int32_t *list, int n_list, int slot0) {
        constexpr bool OBJ = decltype(obj_tag)::value;
        for (int j0 = 0; j0 < n_list; j0 += CH) {
            float nr[CH][NC], ni[CH][NC], Gn[CH][NC][2], sc[CH];
#pragma unroll
            for (int q = 0; q < CH; ++q) {
                const bool valid = j0 + q < n_list;
                const int64_t kn = valid ? (int64_t)list[b * n_list + j0 + q] : ks;
                const float *vn = store + kn * L;
                if (lane == 0 && upd_keys && valid) upd_keys[b * rows + slot0 + j0 + q] = kn;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const uint32_t k = (uint32_t)lane + 64u * c;
                    const bool in = valid && k < Du;
                    nr[q][c] = in ? vn[k] : 0.0f; ni[q][c] = in ? (vn + Du)[k] : 0.0f;
                    Gn[q][c][0] = in ? (vn + 2 * Du)[k] : 0.0f; Gn[q][c][1] = in ? (vn + 3 * Du)[k] : 0.0f;
                }
            }
#pragma unroll
            for (int q = 0; q < CH; ++q) {
                float term[NC];
#pragma unroll
                for (int c = 0; c < NC; ++c)
                    term[c] = OBJ ? sr[c] * rr[c] * nr[q][c] + si[c] * rr[c] * ni[q][c] + sr[c] * ri[c] * ni[q][c] - si[c] * ri[c] * nr[q][c]
                                  : nr[q][c] * rr[c] * orl[c] + ni[q][c] * rr[c] * oi[c] + nr[q][c] * ri[c] * oi[c] - ni[q][c] * ri[c] * orl[c];
                sc[q] = total(term);
            }
#pragma unroll
            for (int q = 0; q < CH; ++q) {
                if (j0 + q >= n_list) break;
                float *un = u0 + (int64_t)(slot0 + j0 + q) * L;
                score = lane == slot0 - 2 + j0 + q ? sc[q] : score;
                const float dl = dloss(-1.0f, sc[q]);
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const uint32_t k = (uint32_t)lane + 64u * c;
                    if (k >= Du) continue;
                    float g0, g1;                                      // the negative's own slot
                    if constexpr (OBJ) {
                        gs[c][0] = gs[c][0] + dl * (rr[c] * nr[q][c] + ri[c] * ni[q][c]); gs[c][1] = gs[c][1] + dl * (rr[c] * ni[q][c] - ri[c] * nr[q][c]);
                        gr[c][0] = gr[c][0] + dl * (sr[c] * nr[q][c] + si[c] * ni[q][c]); gr[c][1] = gr[c][1] + dl * (sr[c] * ni[q][c] - si[c] * nr[q][c]);
                        g0 = 0.0f + dl * (sr[c] * rr[c] - si[c] * ri[c]); g1 = 0.0f + dl * (si[c] * rr[c] + sr[c] * ri[c]);
                    } else {
                        g0 = 0.0f + dl * (rr[c] * orl[c] + ri[c] * oi[c]); g1 = 0.0f + dl * (rr[c] * oi[c] - ri[c] * orl[c]);
                        gr[c][0] = gr[c][0] + dl * (nr[q][c] * orl[c] + ni[q][c] * oi[c]); gr[c][1] = gr[c][1] + dl * (nr[q][c] * oi[c] - ni[q][c] * orl[c]);
                        go[c][0] = go[c][0] + dl * (nr[q][c] * rr[c] - ni[q][c] * ri[c]);  go[c][1] = go[c][1] + dl * (ni[q][c] * rr[c] + nr[q][c] * ri[c]);
                    }
                    const Upd u_0 = adagrad<EXACT>(g0, Gn[q][c][0], lr, eps), u_1 = adagrad<EXACT>(g1, Gn[q][c][1], lr, eps);
                    un[k] = u_0.dt; (un + 2 * Du)[k] = u_0.dg;
                    (un + Du)[k] = u_1.dt; (un + 3 * Du)[k] = u_1.dg;
                }
            }
        }
    };
    negatives(std::false_type{}, neg_subj, ns, 3);
    negatives(std::true_type{}, neg_obj, no, 3 + ns);
    // the losses of all scored triples at once (lane t: triple t; the positive one is triple 0)
    {
        const float label = lane == 0 ? 1.0f : -1.0f;
        const float z = -label * score;
        const double en = exp((double)(z >= 0.0f ? -z : z));
        const double ls = z >= 0.0f ? (double)z + log1p(en) : log1p(en);
        double loss_sum = 0.0;
        for (int t = 0; t < 1 + ns + no; ++t) {
            const uint64_t bits = __builtin_bit_cast(uint64_t, ls);
            const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)bits, t);
            const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(bits >> 32), t);
            loss_sum += __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
        }
        if (lane == 0) loss[b] = loss_sum;
    }
    // subject, relation, object: one AdaGrad step each on the summed gradient, with the accumulators as pulled
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const uint32_t k = (uint32_t)lane + 64u * c;
        if (k >= Du) continue;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const uint32_t ft = p * Du, fg = (2 + p) * Du;              // the field of the values and that of their accumulators
            const Upd us = adagrad<EXACT>(gs[c][p], (vs + fg)[k], lr, eps);
            const Upd ur = adagrad<EXACT>(gr[c][p], (vr + fg)[k], lr, eps);
            const Upd uo = adagrad<EXACT>(go[c][p], (vo + fg)[k], lr, eps);
            (u0 + ft)[k] = us.dt; (u0 + fg)[k] = us.dg;
            (u0 + L + ft)[k] = ur.dt; (u0 + L + fg)[k] = ur.dg;
            (u0 + 2 * L + ft)[k] = uo.dt; (u0 + 2 * L + fg)[k] = uo.dg;
        }
    }
}

__global__ __launch_bounds__(256) void k_kge_loss_sum(const double *loss, int64_t n, double *out) {
    __shared__ double s[256];
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += 256) acc += loss[i];
    s[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) s[threadIdx.x] += s[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = s[0];
}

extern "C" int kge_sgd_step(ps_handle ps, int32_t worker, int64_t num_entities, int32_t dim, int64_t batch, const int32_t *subj,
                            const int32_t *rel, const int32_t *obj, int32_t n_neg_subj, const int32_t *neg_subj,
                            int32_t n_neg_obj, const int32_t *neg_obj, float lr, float eps, double *loss_host_out, void *stream) {
    if (!ps || batch < 0 || dim <= 0 || n_neg_subj < 0 || n_neg_obj < 0 || num_entities <= 0) return PS_EINVAL;
    if (4 * (int64_t)dim != ps->L || num_entities > ps->K) return PS_EINVAL;
    if (dim > 256 || 1 + (int64_t)n_neg_subj + n_neg_obj > 64) return PS_ELIMIT;
    if (worker < -1 || worker >= ps->W) return PS_EWORKER;
    if (batch > 0 && (!subj || !rel || !obj || (n_neg_subj > 0 && !neg_subj) || (n_neg_obj > 0 && !neg_obj))) return PS_EINVAL;
    if (loss_host_out) *loss_host_out = 0.0;
    if (batch == 0) return PS_OK;
    const int64_t rows = batch * (3 + n_neg_subj + n_neg_obj);        // keys pulled and pushed: the slots of the data points
    if (rows >= ((int64_t)1 << 31)) return PS_ELIMIT;
    hipStream_t st = (hipStream_t)stream;
    // scratch of the step: the keys of all slots, the update rows (one per slot), the losses
    const size_t off_upd = (size_t)((rows * 8 + 255) / 256 * 256);
    const size_t off_loss = off_upd + (size_t)((rows * ps->L * 4 + 255) / 256 * 256);
    const size_t bytes = off_loss + (size_t)(batch + 1) * 8;
    if (bytes > ps->kge_ws_bytes) {
        PS_HIP(ps, hipStreamSynchronize(st));
        if (ps->kge_ws) PS_HIP(ps, hipFree(ps->kge_ws));
        ps->kge_ws = nullptr; ps->kge_ws_bytes = 0;
        hipError_t e = hipMalloc(&ps->kge_ws, bytes);
        if (e != hipSuccess) { (void)hipGetLastError(); ps->last_error = "out of device memory for the step's scratch"; return PS_ENOMEM; }
        ps->kge_ws_bytes = bytes;
    }
    int64_t *ukeys = (int64_t *)ps->kge_ws;
    float *upd = (float *)((char *)ps->kge_ws + off_upd);
    double *loss = (double *)((char *)ps->kge_ws + off_loss);
    k_kge_keys<<<grid_for(rows, 256), 256, 0, st>>>(num_entities, batch, subj, rel, obj, n_neg_subj, neg_subj, n_neg_obj, neg_obj, ukeys);
    PS_HIP(ps, hipGetLastError());
    int rc = dpaps_check_keys(ps, ukeys, rows, st);                     // before anything indexes the store with them
    if (rc) return rc;
    // What needs the keys only - the sort of the push, and the statistics of the pull and of the push (every slot
    // is pulled, and pushed below) - runs on the library's second stream beside the kernel that computes the
    // update rows; the sums wait for the sort, the end of the step for the statistics.
    rc = dpaps_side_stream(ps);
    if (rc) return rc;
    hipStream_t bs = ps->side_stream;
    PS_HIP(ps, hipEventRecord(ps->ev_fork, st));
    PS_HIP(ps, hipStreamWaitEvent(bs, ps->ev_fork, 0));
    rc = dpaps_push_sort(ps, ukeys, rows, bs);
    if (rc) return rc;
    PS_HIP(ps, hipEventRecord(ps->ev_sorted, bs));
    rc = dpaps_route_pull_push(ps, worker, ukeys, rows, bs);
    if (rc) return rc;
    PS_HIP(ps, hipEventRecord(ps->ev_join, bs));
    const unsigned blocks = grid_for(batch * 64, 256);
#define KGE_GROUP(NC)                                                                                                                          \
    do {                                                                                                                                       \
        if (ps->opt_kge_exact) k_kge_group<NC, true><<<blocks, 256, 0, st>>>(batch, num_entities, dim, subj, rel, obj, n_neg_subj, neg_subj,     \
                                                                             n_neg_obj, neg_obj, lr, eps, ps->val, upd, nullptr, loss, ps->err); \
        else k_kge_group<NC, false><<<blocks, 256, 0, st>>>(batch, num_entities, dim, subj, rel, obj, n_neg_subj, neg_subj, n_neg_obj, neg_obj,  \
                                                            lr, eps, ps->val, upd, nullptr, loss, ps->err);                                      \
    } while (0)
    switch ((dim + 63) / 64) {
    case 1: KGE_GROUP(1); break;
    case 2: KGE_GROUP(2); break;
    case 3: KGE_GROUP(3); break;
    default: KGE_GROUP(4); break;
    }
#undef KGE_GROUP
    PS_HIP(ps, hipGetLastError());
    PS_HIP(ps, hipStreamWaitEvent(st, ps->ev_sorted, 0));
    rc = dpaps_push_add(ps, rows, upd, st);
    PS_HIP(ps, hipStreamWaitEvent(st, ps->ev_join, 0));
    if (rc) return rc;
    if (loss_host_out) {
        k_kge_loss_sum<<<1, 256, 0, st>>>(loss, batch, loss + batch);
        PS_HIP(ps, hipGetLastError());
        PS_HIP(ps, hipMemcpyAsync(loss_host_out, loss + batch, sizeof(double), hipMemcpyDeviceToHost, st));
        PS_HIP(ps, hipStreamSynchronize(st));
    }
    return PS_OK;
}

// ---------------------------------------------------------------------------
// One epoch over workers, with the parameters allocated where they are used (Appendix A of the paper)
// ---------------------------------------------------------------------------
// every index of the epoch's triples inside its range (the kernels that follow index the store with them)
__global__ void k_kge_validate(int64_t num_entities, int64_t num_relations, int64_t n, const int32_t *subj, const int32_t *rel,
                               const int32_t *obj, int32_t ns, const int32_t *neg_subj, int32_t no, const int32_t *neg_obj, int32_t *err) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= n) return;
    bool bad = subj[t] < 0 || subj[t] >= num_entities || obj[t] < 0 || obj[t] >= num_entities || rel[t] < 0 || rel[t] >= num_relations;
    for (int32_t j = 0; j < ns; ++j) bad |= neg_subj[t * ns + j] < 0 || neg_subj[t * ns + j] >= num_entities;
    for (int32_t j = 0; j < no; ++j) bad |= neg_obj[t * no + j] < 0 || neg_obj[t * no + j] >= num_entities;
    if (bad) atomicExch(err, PS_EKEY);
}

// the entity keys the triples [t0, t1) will access: per triple its subject, its object, its negatives
__global__ void k_kge_entity_keys(int64_t t0, int64_t t1, const int32_t *subj, const int32_t *obj, int32_t ns, const int32_t *neg_subj,
                                  int32_t no, const int32_t *neg_obj, int64_t *keys) {
    const int64_t t = t0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= t1) return;
    int64_t *k = keys + (t - t0) * (2 + ns + no);
    k[0] = subj[t]; k[1] = obj[t];
    for (int32_t j = 0; j < ns; ++j) k[2 + j] = neg_subj[t * ns + j];
    for (int32_t j = 0; j < no; ++j) k[2 + ns + j] = neg_obj[t * no + j];
}

__global__ void k_kge_relation_keys(int64_t num_entities, int64_t t0, int64_t t1, const int32_t *rel, int64_t *keys) {
    const int64_t t = t0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < t1) keys[t - t0] = num_entities + rel[t];
}

__global__ void k_kge_zero(double *x) { *x = 0.0; }

// *acc += the sum of loss[0 .. n)
__global__ __launch_bounds__(256) void k_kge_loss_add(const double *loss, int64_t n, double *acc) {
    __shared__ double s[256];
    double a = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += 256) a += loss[i];
    s[threadIdx.x] = a;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) s[threadIdx.x] += s[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *acc += s[0];
}

extern "C" int kge_sgd_epoch(ps_handle ps, int64_t num_entities, int32_t dim, int64_t num_triples, const int32_t *subj, const int32_t *rel,
                             const int32_t *obj, int32_t n_neg_subj, const int32_t *neg_subj, int32_t n_neg_obj, const int32_t *neg_obj,
                             const int64_t *part_ptr_host, int32_t num_parts, int64_t batch, int32_t lookahead, float lr, float eps,
                             double *loss_host_out, void *stream) {
    if (!ps || num_triples < 0 || dim <= 0 || n_neg_subj < 0 || n_neg_obj < 0 || num_entities <= 0 || batch <= 0 || !part_ptr_host) return PS_EINVAL;
    if (4 * (int64_t)dim != ps->L || num_entities > ps->K) return PS_EINVAL;
    if (dim > 256 || 1 + (int64_t)n_neg_subj + n_neg_obj > 64) return PS_ELIMIT;
    if (num_parts <= 0 || num_parts > ps->W) return PS_EWORKER;
    if (part_ptr_host[0] != 0 || part_ptr_host[num_parts] != num_triples) return PS_EINVAL;
    int64_t longest = 0;
    for (int32_t w = 0; w < num_parts; ++w) {
        if (part_ptr_host[w + 1] < part_ptr_host[w]) return PS_EINVAL;
        longest = std::max(longest, part_ptr_host[w + 1] - part_ptr_host[w]);
    }
    if (num_triples > 0 && (!subj || !rel || !obj || (n_neg_subj > 0 && !neg_subj) || (n_neg_obj > 0 && !neg_obj))) return PS_EINVAL;
    if (loss_host_out) *loss_host_out = 0.0;
    if (num_triples == 0) return PS_OK;
    const int32_t ns = n_neg_subj, no = n_neg_obj, per = 1 + ns + no, ent = 2 + ns + no;
    const int64_t bmax = std::min(batch, longest);
    if (bmax * (per + 2) >= ((int64_t)1 << 31) || longest * ent >= ((int64_t)1 << 31)) return PS_ELIMIT;
    hipStream_t vs = (hipStream_t)stream;                  // the work on the values
    {
        const int rc = dpaps_side_stream(ps);
        if (rc) return rc;
    }
    hipStream_t bs = ps->side_stream;                      // localize calls and statistics: owner map and counters only
    // scratch: localize keys (second stream), the slots' keys, update rows and the losses (first)
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    const int64_t rows_max = bmax * (3 + ns + no);
    const size_t off_loc = 0;
    const size_t off_ukeys = off_loc + up((size_t)std::max(longest, bmax * ent) * 8);
    const size_t off_upd = off_ukeys + up((size_t)rows_max * 8);
    const size_t off_loss = off_upd + up((size_t)rows_max * ps->L * 4);
    const size_t bytes = off_loss + (size_t)(bmax + 2) * 8;
    if (bytes > ps->kge_ws_bytes) {
        PS_HIP(ps, hipStreamSynchronize(vs));
        if (ps->kge_ws) PS_HIP(ps, hipFree(ps->kge_ws));
        ps->kge_ws = nullptr; ps->kge_ws_bytes = 0;
        hipError_t e = hipMalloc(&ps->kge_ws, bytes);
        if (e != hipSuccess) { (void)hipGetLastError(); ps->last_error = "out of device memory for the epoch's scratch"; return PS_ENOMEM; }
        ps->kge_ws_bytes = bytes;
    }
    int64_t *lkeys = (int64_t *)((char *)ps->kge_ws + off_loc);
    int64_t *ukeys = (int64_t *)((char *)ps->kge_ws + off_ukeys);
    float *upd = (float *)((char *)ps->kge_ws + off_upd);
    double *loss = (double *)((char *)ps->kge_ws + off_loss);
    double *loss_acc = loss + bmax;

    // every index is checked once; both streams start after that
    k_kge_validate<<<grid_for(num_triples, 256), 256, 0, vs>>>(num_entities, ps->K - num_entities, num_triples, subj, rel, obj, ns, neg_subj,
                                                             no, neg_obj, ps->err);
    PS_HIP(ps, hipGetLastError());
    k_kge_zero<<<1, 1, 0, vs>>>(loss_acc);
    PS_HIP(ps, hipGetLastError());
    PS_HIP(ps, hipEventRecord(ps->ev_fork, vs));
    PS_HIP(ps, hipStreamWaitEvent(bs, ps->ev_fork, 0));
    int rc = PS_OK;
    auto localize_entities = [&](int64_t t0, int64_t t1, int32_t w) {
        if (t1 <= t0) return (int)PS_OK;
        k_kge_entity_keys<<<grid_for(t1 - t0, 256), 256, 0, bs>>>(t0, t1, subj, obj, ns, neg_subj, no, neg_obj, lkeys);
        PS_HIP(ps, hipGetLastError());
        return dpaps_localize_checked(ps, lkeys, (t1 - t0) * ent, w, bs);
    };
    if (lookahead) {
        for (int32_t w = 0; w < num_parts && !rc; ++w) {              // relations go where their triples are
            const int64_t t0 = part_ptr_host[w], t1 = part_ptr_host[w + 1];
            if (t1 <= t0) continue;
            k_kge_relation_keys<<<grid_for(t1 - t0, 256), 256, 0, bs>>>(num_entities, t0, t1, rel, lkeys);
            PS_HIP(ps, hipGetLastError());
            rc = dpaps_localize_checked(ps, lkeys, t1 - t0, w, bs);
        }
        for (int32_t w = 0; w < num_parts && !rc; ++w)                // the first batch's entities
            rc = localize_entities(part_ptr_host[w], std::min(part_ptr_host[w] + batch, part_ptr_host[w + 1]), w);
    }
    int64_t steps_done = 0;
    for (int64_t r = 0; r * batch < longest && !rc; ++r) {
        for (int32_t w = 0; w < num_parts && !rc; ++w) {
            const int64_t t0 = part_ptr_host[w] + r * batch, end = part_ptr_host[w + 1];
            if (t0 >= end) continue;
            const int64_t t1 = std::min(t0 + batch, end), nb = t1 - t0;
            // second stream: the next batch's entities come to this worker, then this batch's accesses are counted
            if (lookahead && t1 < end) rc = localize_entities(t1, std::min(t1 + batch, end), w);
            if (rc) break;
            k_kge_keys<<<grid_for(nb * (3 + ns + no), 256), 256, 0, bs>>>(num_entities, nb, subj + t0, rel + t0, obj + t0, ns, neg_subj + t0 * ns,
                                                                          no, neg_obj + t0 * no, ukeys);
            PS_HIP(ps, hipGetLastError());
            rc = dpaps_route_pull_push(ps, w, ukeys, nb * (3 + ns + no), bs);
            if (rc) break;
            // ... and the push's sort, which needs the keys only, once the previous step's sums have read theirs
            if (steps_done > 0) PS_HIP(ps, hipStreamWaitEvent(bs, ps->ev_added, 0));
            rc = dpaps_push_sort(ps, ukeys, nb * (3 + ns + no), bs);
            if (rc) break;
            PS_HIP(ps, hipEventRecord(ps->ev_sorted, bs));
            // first stream: the values
            const unsigned blocks = grid_for(nb * 64, 256);
#define KGE_GROUP(NC)                                                                                                                              \
    do {                                                                                                                                           \
        if (ps->opt_kge_exact) k_kge_group<NC, true><<<blocks, 256, 0, vs>>>(nb, num_entities, dim, subj + t0, rel + t0, obj + t0, ns,               \
                                                                             neg_subj + t0 * ns, no, neg_obj + t0 * no, lr, eps, ps->val, upd, nullptr, \
                                                                             loss, ps->err);                                                        \
        else k_kge_group<NC, false><<<blocks, 256, 0, vs>>>(nb, num_entities, dim, subj + t0, rel + t0, obj + t0, ns, neg_subj + t0 * ns, no,         \
                                                            neg_obj + t0 * no, lr, eps, ps->val, upd, nullptr, loss, ps->err);                      \
    } while (0)
            switch ((dim + 63) / 64) {
            case 1: KGE_GROUP(1); break;
            case 2: KGE_GROUP(2); break;
            case 3: KGE_GROUP(3); break;
            default: KGE_GROUP(4); break;
            }
#undef KGE_GROUP
            PS_HIP(ps, hipGetLastError());
            PS_HIP(ps, hipStreamWaitEvent(vs, ps->ev_sorted, 0));
            rc = dpaps_push_add(ps, nb * (3 + ns + no), upd, vs);
            if (rc) break;
            PS_HIP(ps, hipEventRecord(ps->ev_added, vs));
            ++steps_done;
            if (loss_host_out) {
                k_kge_loss_add<<<1, 256, 0, vs>>>(loss, nb, loss_acc);
                PS_HIP(ps, hipGetLastError());
            }
        }
    }
    // the second stream joins the first
    PS_HIP(ps, hipEventRecord(ps->ev_join, bs));
    PS_HIP(ps, hipStreamWaitEvent(vs, ps->ev_join, 0));
    if (rc) return rc;
    if (loss_host_out) {
        PS_HIP(ps, hipMemcpyAsync(loss_host_out, loss_acc, sizeof(double), hipMemcpyDeviceToHost, vs));
        PS_HIP(ps, hipStreamSynchronize(vs));
    }
    return PS_OK;
}
