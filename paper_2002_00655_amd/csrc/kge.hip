// One mini-batch step of knowledge-graph-embedding training through the parameter
// server (Sec. 4.1 "Knowledge graph embeddings" and Appendix A of the paper: SGD with
// AdaGrad and negative sampling, the AdaGrad metadata stored in the parameter server;
// model ComplEx, cited there, whose score Re sum_k e_s[k] w_r[k] conj(e_o[k]) is the
// standard one).  The step is what a worker does for a batch of data points: pull the
// parameters of the positive triples and of their negatives, compute the updates, push
// them.  The pull is accounted exactly like ps_pull (key check, locality statistics,
// message counts) but its values are read from the store by the kernel that uses them
// instead of being copied out first; the push is ps_push, which gives the deterministic
// order of cumulative updates.
//
// Key space: entity e is key e, relation r is key num_entities + r.  A value has 4 D
// numbers: [0, D) real parts, [D, 2 D) imaginary parts, [2 D, 4 D) the AdaGrad
// accumulators of those 2 D numbers.
#include "common.h"
#include "mf_device.h"

int dpaps_account_pull(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, hipStream_t st);   // ps_store.hip

static inline unsigned grid_for(int64_t n, int block) { return (unsigned)((n + block - 1) / block); }

// the key occurrences of the batch, in push order: triple of the batch, then positive /
// subject-negatives / object-negatives, then role (subject, relation, object)
__global__ void k_kge_keys(int64_t num_entities, int64_t batch, const int32_t *subj, const int32_t *rel, const int32_t *obj,
                           int32_t ns, const int32_t *neg_subj, int32_t no, const int32_t *neg_obj, int64_t *keys) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;     // scored triple
    const int32_t per = 1 + ns + no;
    if (t >= batch * per) return;
    const int64_t b = t / per;
    const int32_t j = (int32_t)(t - b * per);
    int64_t s = subj[b], o = obj[b];
    if (j >= 1 && j <= ns) s = neg_subj[b * ns + (j - 1)];
    if (j > ns) o = neg_obj[b * no + (j - 1 - ns)];
    keys[3 * t + 0] = s;
    keys[3 * t + 1] = num_entities + rel[b];
    keys[3 * t + 2] = o;
}

// One wavefront per scored triple: its three values as the store holds them, score, loss,
// gradient, and the AdaGrad update of every occurrence, written to the occurrence's row of
// the update buffer (lane l handles components l, l + 64, ...).
//   loss = log(1 + exp(-label score)),  g = dloss/dscore * dscore/dtheta,
//   dtheta = -lr g / sqrt(G + g^2 + eps),  dG = g^2      (G: the pulled accumulator)
template <int NC>
__global__ __launch_bounds__(256) void k_kge_grad(int64_t ntriples, int32_t per, int32_t D, float lr, float eps, const int64_t *keys,
                                                   const float *store, float *upd, double *loss, const int32_t *err) {
    if (__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    const int lane = threadIdx.x & 63;
    const int64_t t = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    if (t >= ntriples) return;
    const int L = 4 * D;
    const float *vs = store + keys[3 * t + 0] * L, *vr = store + keys[3 * t + 1] * L, *vo = store + keys[3 * t + 2] * L;
    float *us = upd + (3 * t + 0) * L, *ur = upd + (3 * t + 1) * L, *uo = upd + (3 * t + 2) * L;
    float sr[NC], si[NC], rr[NC], ri[NC], orl[NC], oi[NC];
    float part = 0.0f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int k = lane + 64 * c;
        const bool in = k < D;
        sr[c] = in ? vs[k] : 0.0f; si[c] = in ? vs[D + k] : 0.0f;
        rr[c] = in ? vr[k] : 0.0f; ri[c] = in ? vr[D + k] : 0.0f;
        orl[c] = in ? vo[k] : 0.0f; oi[c] = in ? vo[D + k] : 0.0f;
        // Re((sr + i si)(rr + i ri)(or - i oi))
        part += sr[c] * rr[c] * orl[c] + si[c] * rr[c] * oi[c] + sr[c] * ri[c] * oi[c] - si[c] * ri[c] * orl[c];
    }
    const float score = wave_sum(part);
    const float label = (t % per) == 0 ? 1.0f : -1.0f;
    const float z = -label * score;
    // sigmoid(z) and log(1 + exp(z)), written so that neither overflows
    const float ex = (float)exp((double)(z >= 0.0f ? -z : z));
    const float sig = z >= 0.0f ? 1.0f / (1.0f + ex) : ex / (1.0f + ex);
    if (lane == 0) loss[t] = z >= 0.0f ? (double)z + log1p(exp((double)-z)) : log1p(exp((double)z));
    const float dl = -label * sig;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int k = lane + 64 * c;
        if (k >= D) continue;
        const float g[3][2] = {{dl * (rr[c] * orl[c] + ri[c] * oi[c]), dl * (rr[c] * oi[c] - ri[c] * orl[c])},
                               {dl * (sr[c] * orl[c] + si[c] * oi[c]), dl * (sr[c] * oi[c] - si[c] * orl[c])},
                               {dl * (sr[c] * rr[c] - si[c] * ri[c]), dl * (si[c] * rr[c] + sr[c] * ri[c])}};
        const float *v3[3] = {vs, vr, vo};
        float *u3[3] = {us, ur, uo};
#pragma unroll
        for (int role = 0; role < 3; ++role) {
#pragma unroll
            for (int p = 0; p < 2; ++p) {
                const float gg = g[role][p], G = v3[role][2 * D + p * D + k];
                u3[role][p * D + k] = -lr * gg / sqrtf(G + gg * gg + eps);
                u3[role][2 * D + p * D + k] = gg * gg;
            }
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
    if (dim > 256) return PS_ELIMIT;
    if (worker < -1 || worker >= ps->W) return PS_EWORKER;
    if (batch > 0 && (!subj || !rel || !obj || (n_neg_subj > 0 && !neg_subj) || (n_neg_obj > 0 && !neg_obj))) return PS_EINVAL;
    if (loss_host_out) *loss_host_out = 0.0;
    if (batch == 0) return PS_OK;
    const int32_t per = 1 + n_neg_subj + n_neg_obj;
    const int64_t ntr = batch * per, nocc = 3 * ntr;
    if (nocc >= ((int64_t)1 << 31)) return PS_ELIMIT;
    hipStream_t st = (hipStream_t)stream;
    // scratch of the step: keys, update terms, losses
    const size_t off_vals = (size_t)((nocc * 8 + 255) / 256 * 256);
    const size_t off_loss = off_vals + (size_t)((nocc * ps->L * 4 + 255) / 256 * 256);
    const size_t bytes = off_loss + (size_t)(ntr + 1) * 8;
    if (bytes > ps->kge_ws_bytes) {
        PS_HIP(ps, hipStreamSynchronize(st));
        if (ps->kge_ws) PS_HIP(ps, hipFree(ps->kge_ws));
        ps->kge_ws = nullptr; ps->kge_ws_bytes = 0;
        hipError_t e = hipMalloc(&ps->kge_ws, bytes);
        if (e != hipSuccess) { (void)hipGetLastError(); ps->last_error = "out of device memory for the step's scratch"; return PS_ENOMEM; }
        ps->kge_ws_bytes = bytes;
    }
    int64_t *keys = (int64_t *)ps->kge_ws;
    float *vals = (float *)((char *)ps->kge_ws + off_vals);
    double *loss = (double *)((char *)ps->kge_ws + off_loss);
    k_kge_keys<<<grid_for(ntr, 256), 256, 0, st>>>(num_entities, batch, subj, rel, obj, n_neg_subj, neg_subj, n_neg_obj, neg_obj, keys);
    PS_HIP(ps, hipGetLastError());
    int rc = dpaps_account_pull(ps, worker, keys, nocc, st);
    if (rc) return rc;
    const unsigned blocks = grid_for(ntr * 64, 256);
    switch ((dim + 63) / 64) {
    case 1: k_kge_grad<1><<<blocks, 256, 0, st>>>(ntr, per, dim, lr, eps, keys, ps->val, vals, loss, ps->err); break;
    case 2: k_kge_grad<2><<<blocks, 256, 0, st>>>(ntr, per, dim, lr, eps, keys, ps->val, vals, loss, ps->err); break;
    case 3: k_kge_grad<3><<<blocks, 256, 0, st>>>(ntr, per, dim, lr, eps, keys, ps->val, vals, loss, ps->err); break;
    default: k_kge_grad<4><<<blocks, 256, 0, st>>>(ntr, per, dim, lr, eps, keys, ps->val, vals, loss, ps->err); break;
    }
    PS_HIP(ps, hipGetLastError());
    rc = ps_push(ps, worker, keys, nocc, vals, stream);
    if (rc) return rc;
    if (loss_host_out) {
        k_kge_loss_sum<<<1, 256, 0, st>>>(loss, ntr, loss + ntr);
        PS_HIP(ps, hipGetLastError());
        PS_HIP(ps, hipMemcpyAsync(loss_host_out, loss + ntr, sizeof(double), hipMemcpyDeviceToHost, st));
        PS_HIP(ps, hipStreamSynchronize(st));
    }
    return PS_OK;
}
