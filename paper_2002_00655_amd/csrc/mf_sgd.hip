// Blocked latent-factor SGD through the parameter server (Sec. 2.2.2, Sec. 4.1,
// Appendix A "Matrix factorization" of the paper), for gfx950.
//
// One workgroup is one worker for one subepoch.  It owns a row block and a
// column block of the factor matrices (relocated to it by the localize step)
// and visits the entries of its data block in stored order, as far as that
// order can be observed: two entries that share neither row nor column touch
// disjoint parameters, so they may run concurrently; two entries of one column
// are taken by the same wavefront one after the other; two entries of one row
// are ordered by a per-row ticket counter in LDS.  The result is the one a
// sequential worker would produce, up to the rounding of each inner product.
//
// Where the parameters live during a subepoch ("localize" on one GPU):
//   - a column's factor row is held in the registers of the wavefront that
//     processes that column's entries, loaded once and written back once;
//   - the factor rows of rows with two or more entries in the block are copied
//     into the workgroup's LDS at the start and written back at the end (as
//     many as fit, busiest first); the others of that kind are handed from
//     wavefront to wavefront through global memory;
//   - a row with a single entry in the block is read and written in place.
#include "common.h"
#include "mf_device.h"

#include <algorithm>
#include <cstring>

static inline unsigned grid_for(int64_t n, int block) { return (unsigned)((n + block - 1) / block); }

__global__ __launch_bounds__(256) void k_mf_localize(LocalizeArgs a) {
    extern __shared__ uint32_t lds_loc[];
    if (*(volatile const int32_t *)a.err) return;
    mf_localize_task(a, lds_loc, (DPAPS_LOC_SLOTS + 1) * ((a.W + 31) / 32), a.tasks[3 * blockIdx.x], a.tasks[3 * blockIdx.x + 1],
                     a.tasks[3 * blockIdx.x + 2]);
}

// ---------------------------------------------------------------------------
// the SGD kernel
// ---------------------------------------------------------------------------
template <int NV>
__device__ __forceinline__ void load_row(const float *p, int lane, int L, float (&x)[NV]) {
#pragma unroll
    for (int c = 0; c < NV; ++c) { int k = lane + 64 * c; x[c] = k < L ? p[k] : 0.0f; }
}
template <int NV>
__device__ __forceinline__ void store_row(float *p, int lane, int L, const float (&x)[NV]) {
#pragma unroll
    for (int c = 0; c < NV; ++c) { int k = lane + 64 * c; if (k < L) p[k] = x[c]; }
}

// One SGD step on registers, in two parts so that other work can be issued
// between them.  w, h: the two factor rows (lane l holds components l, l+64,
// ...; components past L are zero).  Both rows are updated from their old values:
//   e = v - <w,h>;  w += lr (e h - lambda w);  h += lr (e w - lambda h).
// Part 1: the products of the inner product, per lane.
template <int NV, bool EXACT>
__device__ __forceinline__ void sgd_products(const float (&w)[NV], const float (&h)[NV], float (&prod)[NV]) {
    if constexpr (EXACT) {
#pragma unroll
        for (int c = 0; c < NV; ++c) prod[c] = w[c] * h[c];          // every product rounded on its own
    } else {
        float p = 0.0f;
#pragma unroll
        for (int c = 0; c < NV; ++c) p = __builtin_fmaf(w[c], h[c], p);
        prod[0] = p;
    }
}
// Part 2: the sum, the error and the two updates.
template <int NV, bool EXACT>
__device__ __forceinline__ void sgd_finish(float (&w)[NV], float (&h)[NV], const float (&prod)[NV], float v, float lr,
                                           float lambda, int L) {
    float dot;
    if constexpr (EXACT) {
        dot = 0.0f;                                                   // components summed in index order
#pragma unroll
        for (int c = 0; c < NV; ++c) {
            const int lim = min(64, L - 64 * c);
            for (int l = 0; l < lim; ++l) dot = dot + rl_f(prod[c], l);
        }
    } else {
        dot = wave_sum(prod[0]);
    }
    const float e = v - dot;
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        const float wo = w[c], ho = h[c];
        if constexpr (EXACT) {
            w[c] = wo + lr * (e * ho - lambda * wo);
            h[c] = ho + lr * (e * wo - lambda * ho);
        } else {
            w[c] = __builtin_fmaf(lr, __builtin_fmaf(e, ho, -(lambda * wo)), wo);
            h[c] = __builtin_fmaf(lr, __builtin_fmaf(e, wo, -(lambda * ho)), ho);
        }
    }
}

// D = entries per read-ahead group for rows that are updated in place.  A wavefront keeps the
// per-entry data of 64 consecutive entries of its run in registers, one entry per lane, and
// consumes 64 - D of them before it moves on, so that the entry after the current one and the
// rows of the next group are always found in the same registers.
template <int NV, bool EXACT, int D>
__global__ __launch_bounds__(1024) void k_mf_sgd(SgdArgs a) {
    extern __shared__ float lds_f[];
    if (__hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    constexpr int CONS = 64 - D;
    static_assert(CONS % D == 0, "a chunk is a whole number of groups");
    const int lane = threadIdx.x & 63;
    const int L = a.L;
    const bool tail = lane + 64 * (NV - 1) < L;
    float *cache = lds_f;                                              // cache_cap x L
    uint32_t *ticket = reinterpret_cast<uint32_t *>(lds_f + (size_t)a.cache_cap * L);   // ticket_cap
    __shared__ int next_run;
    __shared__ unsigned int done_entries;
    __shared__ uint32_t give_up;          // set when a bounded wait ran out, so that the other waits end at once

    const int32_t worker = a.tasks[3 * blockIdx.x], rb = a.tasks[3 * blockIdx.x + 1], cb = a.tasks[3 * blockIdx.x + 2];
    const int64_t b = (int64_t)rb * a.d_col + cb;
    const int64_t run0 = a.blk_run_ptr[b], run1 = a.blk_run_ptr[b + 1];
    const int64_t mp0 = a.blk_multi_ptr[b];
    const int nmulti = (int)(a.blk_multi_ptr[b + 1] - mp0);
    const int ncached = min(nmulti, a.cache_cap);

    // every parameter this worker will touch must be allocated to it (Sec. 4.1: all access is local)
    {
        const int64_t r0 = a.row_bounds[rb], r1 = a.row_bounds[rb + 1];
        const int64_t c0 = a.m + a.col_bounds[cb], c1 = a.m + a.col_bounds[cb + 1];
        bool bad = false;
        for (int64_t k = r0 + threadIdx.x; k < r1; k += blockDim.x) bad |= a.owner[k] != worker;
        for (int64_t k = c0 + threadIdx.x; k < c1; k += blockDim.x) bad |= a.owner[k] != worker;
        if (bad) atomicExch(a.err, PS_EREMOTE);
    }
    // pull the busiest rows into LDS (all threads, several loads in flight each); reset the tickets
    for (int t = threadIdx.x; t < nmulti; t += blockDim.x) ticket[t] = 0;
    {
        const int total = ncached * L;
#pragma unroll 4
        for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
            const int s = idx / L;
            cache[idx] = a.val[(int64_t)a.multi_row[mp0 + s] * L + (idx - s * L)];
        }
    }
    if (threadIdx.x == 0) { next_run = 0; done_entries = 0; give_up = 0; }
    __syncthreads();

    const float lr = a.lr, lambda = a.lambda;
    unsigned int done = 0;
    for (;;) {
        int run = 0;
        if (lane == 0) run = atomicAdd(&next_run, 1);
        run = __builtin_amdgcn_readfirstlane(run);
        const int64_t g = run0 + run;
        if (g >= run1) break;
        const int64_t s0 = a.run_start[g], s1 = a.run_start[g + 1];
        float *hrow = a.val + (a.m + a.run_col[g]) * (int64_t)L;
        // the long runs come first and everything else in the block ends up waiting for them
        if (run < 4) __builtin_amdgcn_s_setprio(3); else __builtin_amdgcn_s_setprio(1);
        float h[NV];
        load_row_t<NV>(hrow, lane, tail, h);

        int64_t pos = s0;
        int m_row = 0, m_info = (int)INFO_NONE;
        float m_val = 0.0f;
        if (pos + lane < s1) { m_row = a.e_row[pos + lane]; m_val = a.e_val[pos + lane]; m_info = (int)a.e_info[pos + lane]; }

        // Read-ahead for rows that are updated in place: while a group of D entries is processed
        // from `cur`, the rows of the next group are in flight into `nxt`.  Every slot is loaded
        // for every entry - from the column's own row when there is nothing to fetch - so that
        // the number of loads in flight does not depend on the data.
        float cur[D][NV], nxt[D][NV];
#pragma unroll
        for (int q = 0; q < D; ++q) {
            const uint32_t inf = (uint32_t)rl_i(m_info, q);
            const int r = rl_i(m_row, q);
            const float *src = (inf & 0xFFFFu) == INFO_SINGLE ? a.val + (int64_t)r * L : hrow;
            load_row_t<NV>(src, lane, tail, nxt[q]);
        }
        // Look-ahead for rows kept in LDS: ticket and row of the coming entry are read while the
        // current entry is being computed.
        uint32_t info_cur = (uint32_t)rl_i(m_info, 0);
        uint32_t pk_tk = 0;
        float pk_w[NV];
#pragma unroll
        for (int c = 0; c < NV; ++c) pk_w[c] = 0.0f;
        if ((info_cur & 0xFFFFu) < (uint32_t)ncached) {
            pk_tk = ticket_read(&ticket[info_cur & 0xFFFFu]);
            compiler_fence();
            load_row_t<NV>(cache + (size_t)(info_cur & 0xFFFFu) * L, lane, tail, pk_w);
        }

        while (pos < s1) {
            const int64_t left = s1 - pos;
            const int avail = left < 64 ? (int)left : 64;            // entries held in the chunk registers
            const int n_here = left < CONS ? (int)left : CONS;       // entries of this chunk to process
            // per-entry data of the chunk that follows
            int n_row = 0, n_info = (int)INFO_NONE;
            float n_val = 0.0f;
            {
                const int64_t p = pos + CONS + lane;
                if (p < s1) { n_row = a.e_row[p]; n_val = a.e_val[p]; n_info = (int)a.e_info[p]; }
            }
            for (int gb = 0; gb < n_here; gb += D) {
#pragma unroll
                for (int q = 0; q < D; ++q) {
#pragma unroll
                    for (int c = 0; c < NV; ++c) cur[q][c] = nxt[q][c];
                }
#pragma unroll
                for (int q = 0; q < D; ++q) {                         // rows of the next group
                    const uint32_t inf = (uint32_t)rl_i(m_info, gb + D + q);
                    const int r = rl_i(m_row, gb + D + q);
                    const float *src = (inf & 0xFFFFu) == INFO_SINGLE ? a.val + (int64_t)r * L : hrow;
                    load_row_t<NV>(src, lane, tail, nxt[q]);
                }
#pragma unroll
                for (int q = 0; q < D; ++q) {
                    const int u = gb + q;
                    if (u >= n_here) continue;
                    const uint32_t slot = info_cur & 0xFFFFu, seq = (info_cur >> 16) & 0x7FFFu;
                    const float v = rl_f(m_val, u);
                    const uint32_t info_nx = u + 1 < avail ? (uint32_t)rl_i(m_info, u + 1) : INFO_NONE;
                    const uint32_t slot_nx = info_nx & 0xFFFFu;
                    float w[NV], prod[NV];
                    // The three kinds of entry differ in where the row comes from and goes to; the
                    // step in between is the same: products, then (while they are summed) the reads
                    // for the coming entry, then the updates.
#define DPAPS_STEP()                                                                         \
    sgd_products<NV, EXACT>(w, h, prod);                                                     \
    __asm__ volatile("" : "+v"(prod[0]) : : "memory");                                       \
    if (slot_nx < (uint32_t)ncached) {                                                       \
        pk_tk = ticket_read(&ticket[slot_nx]);                                               \
        compiler_fence();                                                                    \
        load_row_t<NV>(cache + (size_t)slot_nx * L, lane, tail, pk_w);                       \
    }                                                                                        \
    sgd_finish<NV, EXACT>(w, h, prod, v, lr, lambda, L)
                    if (slot == INFO_SINGLE) {
                        // the row's only entry in the block: fetched ahead, updated in place
#pragma unroll
                        for (int c = 0; c < NV; ++c) w[c] = cur[q][c];
                        DPAPS_STEP();
                        store_row_t<NV>(a.val + (int64_t)rl_i(m_row, u) * L, lane, tail, w);
                    } else {
                        uint32_t *tk = &ticket[slot];
                        const bool cached = slot < (uint32_t)ncached;
                        bool have = false;
                        if (cached && (uint32_t)__builtin_amdgcn_readfirstlane((int)pk_tk) == seq) {
#pragma unroll
                            for (int c = 0; c < NV; ++c) w[c] = pk_w[c];
                            have = true;
                        } else {
                            // wait until the row's earlier entries (in stored order) are done
                            __builtin_amdgcn_s_setprio(0);
                            for (uint32_t spins = 0; ticket_read(tk) != seq;) {
                                __builtin_amdgcn_s_sleep(2);
                                // every wait ends: the predecessor always makes progress.  Should that ever
                                // fail (corrupt input tables), give up rather than hang the device.
                                if ((++spins & 1023u) == 0 && (spins > (1u << 21) || ticket_read(&give_up) != 0u)) {
                                    ticket_write(&give_up, 1u);
                                    atomicExch(a.err, PS_ESTALL);
                                    break;
                                }
                            }
                            compiler_fence();
                            if (run < 4) __builtin_amdgcn_s_setprio(3); else __builtin_amdgcn_s_setprio(1);
                        }
                        if (cached) {
                            float *lrow = cache + (size_t)slot * L;      // the row lives in LDS for this subepoch
                            if (!have) load_row_t<NV>(lrow, lane, tail, w);
                            DPAPS_STEP();
                            store_row_t<NV>(lrow, lane, tail, w);
                            compiler_fence();
                            ticket_write(tk, seq + 1u);
                        } else {
                            float *wrow = a.val + (int64_t)rl_i(m_row, u) * L;   // did not fit: handed over through memory
                            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                            load_row_t<NV>(wrow, lane, tail, w);
                            // wait for this load here, on the rare path, so that the common paths are
                            // not made to wait for the read-ahead in flight
                            __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0)
                            DPAPS_STEP();
                            store_row_t<NV>(wrow, lane, tail, w);
                            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                            ticket_write(tk, seq + 1u);
                        }
                    }
#undef DPAPS_STEP
                    info_cur = info_nx;
                }
            }
            done += (unsigned int)n_here;
            pos += CONS;
            m_row = n_row; m_val = n_val; m_info = n_info;
        }
        store_row_t<NV>(hrow, lane, tail, h);
    }
    __builtin_amdgcn_s_setprio(0);
    if (lane == 0 && done) atomicAdd(&done_entries, done);
    __syncthreads();
    // push the cached rows back
    {
        const int total = ncached * L;
#pragma unroll 4
        for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
            const int s = idx / L;
            a.val[(int64_t)a.multi_row[mp0 + s] * L + (idx - s * L)] = cache[idx];
        }
    }
    // each entry was one pull and one push of two local keys
    if (threadIdx.x == 0 && done_entries) {
        u64 *st = stat_slot(a.stats);
        atomicAdd(&st[PS_STAT_PULL_LOCAL], 2 * (u64)done_entries);
        atomicAdd(&st[PS_STAT_PUSH_LOCAL], 2 * (u64)done_entries);
    }
}


// ---------------------------------------------------------------------------
// training error
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_mf_sse(const int32_t *rows, const int32_t *cols, const float *vals, int64_t nnz,
                                                const float *val, int64_t m, int32_t L, double *partial) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t nw = ((int64_t)gridDim.x * blockDim.x) >> 6;
    double acc = 0.0;
    for (int64_t p = wave; p < nnz; p += nw) {
        const float *w = val + (int64_t)rows[p] * L, *h = val + (m + cols[p]) * (int64_t)L;
        double d = 0.0;
        for (int k = lane; k < L; k += 64) d += (double)w[k] * (double)h[k];
        for (int off = 32; off > 0; off >>= 1) d += __shfl_xor(d, off);
        const double e = (double)vals[p] - d;
        acc += e * e;             // identical in all lanes
    }
    __shared__ double s[4];
    if (lane == 0) s[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = (s[0] + s[1]) + (s[2] + s[3]);
}

// ---------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------
int dpaps_take_error(dpaps_ps *ps, hipStream_t st);   // ps_store.hip

template <int NV, bool EXACT>
static int launch_sgd(dpaps_ps *ps, const SgdArgs &a, int ntasks, int threads, size_t lds, hipStream_t st) {
    constexpr int D = NV <= 2 ? 16 : 8;       // read-ahead depth (D*NV registers per lane)
    static size_t configured = 0;
    if (lds > configured) {
        PS_HIP(ps, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mf_sgd<NV, EXACT, D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        configured = lds;
    }
    k_mf_sgd<NV, EXACT, D><<<ntasks, threads, lds, st>>>(a);
    PS_HIP(ps, hipGetLastError());
    return PS_OK;
}

// ---------------------------------------------------------------------------
// The epoch on a classic parameter server (Sec. 2.1: static allocation; the variants compared in Sec. 4.2 and
// Sec. 4.6): nothing is relocated and nothing stays with the worker.  One wavefront per task walks its block in
// stored order; every entry is a pull of its two keys from the store, the step, and a push that reads the
// stored values again and adds the update terms (in_place = 1: the worker updates the two rows where they are,
// without the second read - the variant of Sec. 4.4 in which workers operate on the server's own copy).  Every access is counted as
// local or remote by the owner map as it stands, with the messages a remote one costs (request to the home
// node, forward if the key lives elsewhere, reply; the two keys of a call share messages to one destination,
// Sec. 3.7).
// ---------------------------------------------------------------------------
struct ClassicArgs {
    const int32_t *tasks;
    float *val; const int32_t *owner;
    const int32_t *e_row, *e_col; const float *e_val;
    const int64_t *run_start, *blk_run_ptr;
    int64_t m, per_home;
    int32_t L, d_col, in_place;
    float lr, lambda;
    u64 *stats; int32_t *err;
};

template <int NV, bool EXACT>
__global__ __launch_bounds__(64) void k_mf_sgd_classic(ClassicArgs a) {
    if (__hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    const int lane = threadIdx.x;
    const int32_t worker = a.tasks[3 * blockIdx.x], rb = a.tasks[3 * blockIdx.x + 1], cb = a.tasks[3 * blockIdx.x + 2];
    const int64_t b = (int64_t)rb * a.d_col + cb;
    const int64_t p0 = a.run_start[a.blk_run_ptr[b]], p1 = a.run_start[a.blk_run_ptr[b + 1]];
    const int L = a.L;
    const float lr = a.lr, lambda = a.lambda;
    u64 n_local = 0, n_remote = 0, n_req = 0, n_fwd = 0, n_reply = 0;      // per call (a pull; the push costs the same)
    for (int64_t p = p0; p < p1; ++p) {
        const int64_t kr = a.e_row[p], kc = a.m + a.e_col[p];
        const float v = a.e_val[p];
        // where the two keys live, and what reaching them costs
        const int32_t o_r = a.owner[kr], o_c = a.owner[kc];
        const int32_t h_r = (int32_t)(kr / a.per_home), h_c = (int32_t)(kc / a.per_home);
        const bool rem_r = o_r != worker, rem_c = o_c != worker;
        n_local += (rem_r ? 0 : 1) + (rem_c ? 0 : 1);
        n_remote += (rem_r ? 1 : 0) + (rem_c ? 1 : 0);
        const bool req_r = rem_r && h_r != worker, req_c = rem_c && h_c != worker;
        n_req += (req_r ? 1 : 0) + (req_c && !(req_r && h_c == h_r) ? 1 : 0);
        const bool fwd_r = rem_r && h_r != o_r, fwd_c = rem_c && h_c != o_c;
        n_fwd += (fwd_r ? 1 : 0) + (fwd_c && !(fwd_r && h_c == h_r && o_c == o_r) ? 1 : 0);
        n_reply += (rem_r ? 1 : 0) + (rem_c && !(rem_r && o_c == o_r) ? 1 : 0);
        // pull
        float *pw = a.val + kr * L, *ph = a.val + kc * L;
        float w[NV], h[NV], prod[NV];
#pragma unroll
        for (int c = 0; c < NV; ++c) {
            const bool in = lane + 64 * c < L;
            w[c] = in ? pw[lane + 64 * c] : 0.0f;
            h[c] = in ? ph[lane + 64 * c] : 0.0f;
        }
        // the step
        sgd_products<NV, EXACT>(w, h, prod);
        float dot;
        if constexpr (EXACT) {
            dot = 0.0f;                                                   // components summed in index order
#pragma unroll
            for (int c = 0; c < NV; ++c) {
                const int lim = min(64, L - 64 * c);
                for (int l = 0; l < lim; ++l) dot = dot + rl_f(prod[c], l);
            }
        } else {
            dot = wave_sum(prod[0]);
        }
        const float e = v - dot;
        // push: the update terms are added to what the store holds
#pragma unroll
        for (int c = 0; c < NV; ++c) {
            if (lane + 64 * c >= L) continue;
            float dw, dh;
            if constexpr (EXACT) {
                dw = lr * (e * h[c] - lambda * w[c]);
                dh = lr * (e * w[c] - lambda * h[c]);
            } else {
                dw = lr * __builtin_fmaf(e, h[c], -(lambda * w[c]));
                dh = lr * __builtin_fmaf(e, w[c], -(lambda * h[c]));
            }
            float cw = w[c], ch = h[c];
            if (!a.in_place) {
                cw = __hip_atomic_load(&pw[lane + 64 * c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                ch = __hip_atomic_load(&ph[lane + 64 * c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            pw[lane + 64 * c] = cw + dw;
            ph[lane + 64 * c] = ch + dh;
        }
    }
    if (lane == 0) {
        u64 *st = stat_slot(a.stats);
        if (n_local) { atomicAdd(&st[PS_STAT_PULL_LOCAL], n_local); atomicAdd(&st[PS_STAT_PUSH_LOCAL], n_local); }
        if (n_remote) { atomicAdd(&st[PS_STAT_PULL_REMOTE], n_remote); atomicAdd(&st[PS_STAT_PUSH_REMOTE], n_remote); }
        if (n_req) atomicAdd(&st[PS_STAT_MSG_ACC_REQ], 2 * n_req);
        if (n_fwd) atomicAdd(&st[PS_STAT_MSG_ACC_FWD], 2 * n_fwd);
        if (n_reply) atomicAdd(&st[PS_STAT_MSG_ACC_REPLY], 2 * n_reply);
    }
}

template <int NV>
static int launch_classic(dpaps_ps *ps, const ClassicArgs &a, int ntasks, hipStream_t st) {
    if (ps->opt_exact) k_mf_sgd_classic<NV, true><<<ntasks, 64, 0, st>>>(a);
    else k_mf_sgd_classic<NV, false><<<ntasks, 64, 0, st>>>(a);
    PS_HIP(ps, hipGetLastError());
    return PS_OK;
}

// the arguments of the SGD kernels that do not depend on the launch
static SgdArgs sgd_args(dpaps_ps *ps, const int32_t *tasks, float lr, float lambda) {
    const MfData &f = ps->mf;
    SgdArgs a{};
    a.tasks = tasks; a.val = ps->val; a.owner = ps->owner;
    a.e_row = f.row; a.e_val = f.val; a.e_info = f.info;
    a.run_start = f.run_start; a.run_col = f.run_col; a.blk_run_ptr = f.blk_run_ptr;
    a.multi_row = f.multi_row; a.blk_multi_ptr = f.blk_multi_ptr;
    a.row_bounds = f.row_bounds; a.col_bounds = f.col_bounds;
    a.m = f.m; a.L = ps->L; a.d_col = f.d_col;
    a.blk_nheavy = f.blk_nheavy; a.blk_trun_ptr = f.blk_trun_ptr;
    a.trun_start = f.trun_start; a.trun_row = f.trun_row; a.trun_wait = f.trun_wait;
    a.trun_ci = f.trun_ci; a.trun_val = f.trun_val; a.trun_col = f.trun_col;
    a.t_cinfo = f.t_cinfo; a.t_val = f.t_val;
    a.run_gptr = f.run_gptr; a.gstart = f.gstart;
    a.lr = lr; a.lambda = lambda; a.stats = ps->stats; a.err = ps->err;
    a.W = ps->W; a.per_home = ps->per_home; a.owner_w = ps->owner;
    return a;
}

extern "C" int mf_sgd_epoch(ps_handle ps, const int32_t *tasks_host, const int32_t *stratum_ptr_host, int32_t num_strata,
                            float lr, float lambda, void *stream) {
    if (!ps || num_strata < 0 || (num_strata > 0 && (!tasks_host || !stratum_ptr_host))) return PS_EINVAL;
    MfData &f = ps->mf;
    if (!f.row) { ps->last_error = "mf_sgd_epoch before mf_load_ratings"; return PS_EINVAL; }
    if (ps->loc) { ps->last_error = "mf_sgd_epoch does not keep location caches: switch PS_OPT_LOCATION_CACHES off"; return PS_EINVAL; }
    if (num_strata == 0) return PS_OK;
    hipStream_t st = (hipStream_t)stream;
    if (stratum_ptr_host[0] != 0) return PS_EINVAL;
    const int64_t total = stratum_ptr_host[num_strata];
    // a stratum is a set of tasks that share no worker and no block (Sec. 2.2.2)
    {
        std::vector<int32_t> stamp((size_t)ps->W + f.d_row + f.d_col, -1);
        for (int32_t s = 0; s < num_strata; ++s) {
            if (stratum_ptr_host[s + 1] < stratum_ptr_host[s]) return PS_EINVAL;
            for (int32_t t = stratum_ptr_host[s]; t < stratum_ptr_host[s + 1]; ++t) {
                const int32_t w = tasks_host[3 * t], rb = tasks_host[3 * t + 1], cb = tasks_host[3 * t + 2];
                if (w < 0 || w >= ps->W) return PS_EWORKER;
                if (rb < 0 || rb >= f.d_row || cb < 0 || cb >= f.d_col) return PS_EINVAL;
                int32_t *x[3] = {&stamp[w], &stamp[(size_t)ps->W + rb], &stamp[(size_t)ps->W + f.d_row + cb]};
                for (int i = 0; i < 3; ++i) { if (*x[i] == s) return PS_ECONFLICT; }
                for (int i = 0; i < 3; ++i) *x[i] = s;
            }
        }
    }
    // stage the schedule on the device (skipped when it is the one already there)
    if (total > 0) {
        const size_t bytes = (size_t)total * 3 * sizeof(int32_t);
        bool same = ps->h_tasks_cached.size() == (size_t)total * 3 && std::memcmp(ps->h_tasks_cached.data(), tasks_host, bytes) == 0;
        if (!same) {
            if (total > ps->d_tasks_cap) {
                PS_HIP(ps, hipStreamSynchronize(st));
                if (ps->d_tasks) PS_HIP(ps, hipFree(ps->d_tasks));
                ps->d_tasks = nullptr; ps->d_tasks_cap = 0;
                PS_HIP(ps, hipMalloc(&ps->d_tasks, bytes));
                ps->d_tasks_cap = total;
            }
            PS_HIP(ps, hipStreamSynchronize(st));      // earlier epochs may still read the old schedule
            ps->h_tasks_cached.assign(tasks_host, tasks_host + total * 3);
            PS_HIP(ps, hipMemcpyAsync(ps->d_tasks, ps->h_tasks_cached.data(), bytes, hipMemcpyHostToDevice, st));
        }
    }
    // LDS plan: ticket counters for the busiest block, the rest for cached rows
    const int L = ps->L;
    const int NV = (L + 63) / 64;
    const int64_t ticket_cap = std::max<int64_t>(f.max_multi_in_block, 1);
    const int64_t budget = (int64_t)ps->lds_bytes - 1024;     // static LDS and slack
    if (ticket_cap * 4 > budget / 2) { ps->last_error = "too many rows with several entries in one block"; return PS_ELIMIT; }
    int64_t cache_cap = (budget - ticket_cap * 4) / ((int64_t)L * 4);
    cache_cap = std::min<int64_t>(cache_cap, f.max_multi_in_block);
    if (ps->opt_cache_rows >= 0) cache_cap = std::min<int64_t>(cache_cap, ps->opt_cache_rows);
    const size_t lds = (size_t)cache_cap * L * 4 + (size_t)ticket_cap * 4;
    const int waves = dpaps_mf_waves(ps);
    const int threads = 64 * waves;
    const size_t loc_lds = (DPAPS_LOC_SLOTS + 1) * (size_t)((ps->W + 31) / 32) * sizeof(uint32_t);

    for (int32_t s = 0; s < num_strata; ++s) {
        const int ntasks = stratum_ptr_host[s + 1] - stratum_ptr_host[s];
        if (ntasks == 0) continue;
        const int32_t *tasks = ps->d_tasks + 3 * (int64_t)stratum_ptr_host[s];
        const bool classic = ps->opt_classic != 0;
        const bool grouped = !classic && ps->opt_grouped && !ps->opt_exact && L <= 128 && f.sweep_ok;
        if (!grouped && !classic) {      // the grouped kernel does the localize step itself; a classic server has none
            LocalizeArgs la{tasks, ps->owner, f.row_bounds, f.col_bounds, f.m, ps->per_home, ps->W, ps->stats, ps->err};
            k_mf_localize<<<ntasks, 256, loc_lds, st>>>(la);
            PS_HIP(ps, hipGetLastError());
        }
        SgdArgs a = sgd_args(ps, tasks, lr, lambda);
        a.cache_cap = (int32_t)cache_cap; a.ticket_cap = (int32_t)ticket_cap;
        a.fuse_localize = grouped ? 1 : 0;
        int rc;
        hipEvent_t ev0 = nullptr, ev1 = nullptr;
        if (ps->opt_profile) {
            while (ps->ev_pool.size() < ps->ev_used + 2) {
                hipEvent_t e;
                PS_HIP(ps, hipEventCreate(&e));
                ps->ev_pool.push_back(e);
            }
            ev0 = ps->ev_pool[ps->ev_used]; ev1 = ps->ev_pool[ps->ev_used + 1];
            ps->ev_used += 2;
            PS_HIP(ps, hipEventRecord(ev0, st));
        }
        if (classic) {
            ClassicArgs ca{tasks, ps->val, ps->owner, f.row, f.col, f.val, f.run_start, f.blk_run_ptr, f.m, ps->per_home,
                           L, f.d_col, ps->opt_classic == 2 ? 1 : 0, lr, lambda, ps->stats, ps->err};
            switch (NV) {
            case 1: rc = launch_classic<1>(ps, ca, ntasks, st); break;
            case 2: rc = launch_classic<2>(ps, ca, ntasks, st); break;
            case 3: rc = launch_classic<3>(ps, ca, ntasks, st); break;
            default: rc = launch_classic<4>(ps, ca, ntasks, st); break;
            }
        } else if (grouped) {
            rc = dpaps_launch_sgd_chunk(ps, a, ntasks, waves, st);
        } else if (ps->opt_exact) {
            switch (NV) {
            case 1: rc = launch_sgd<1, true>(ps, a, ntasks, threads, lds, st); break;
            case 2: rc = launch_sgd<2, true>(ps, a, ntasks, threads, lds, st); break;
            case 3: rc = launch_sgd<3, true>(ps, a, ntasks, threads, lds, st); break;
            default: rc = launch_sgd<4, true>(ps, a, ntasks, threads, lds, st); break;
            }
        } else {
            switch (NV) {
            case 1: rc = launch_sgd<1, false>(ps, a, ntasks, threads, lds, st); break;
            case 2: rc = launch_sgd<2, false>(ps, a, ntasks, threads, lds, st); break;
            case 3: rc = launch_sgd<3, false>(ps, a, ntasks, threads, lds, st); break;
            default: rc = launch_sgd<4, false>(ps, a, ntasks, threads, lds, st); break;
            }
        }
        if (rc) return rc;
        if (ev1) PS_HIP(ps, hipEventRecord(ev1, st));
    }
    return PS_OK;
}

extern "C" int mf_sgd_epoch_handoff(ps_handle ps, float lr, float lambda, int32_t *order_host_out, void *stream) {
    if (!ps) return PS_EINVAL;
    MfData &f = ps->mf;
    if (!f.row) { ps->last_error = "mf_sgd_epoch_handoff before mf_load_ratings"; return PS_EINVAL; }
    if (ps->loc) { ps->last_error = "mf_sgd_epoch_handoff does not keep location caches: switch PS_OPT_LOCATION_CACHES off"; return PS_EINVAL; }
    hipStream_t st = (hipStream_t)stream;
    const int L = ps->L;
    if (f.d_row > ps->W) { ps->last_error = "mf_sgd_epoch_handoff: more row blocks than workers"; return PS_EWORKER; }
    if (f.d_col > DPAPS_HANDOFF_MAX_COLS) { ps->last_error = "mf_sgd_epoch_handoff: more than 4096 column blocks"; return PS_ELIMIT; }
    if (L > 128 || !f.sweep_ok || ps->opt_exact || ps->opt_classic || !ps->opt_grouped) {
        ps->last_error = "mf_sgd_epoch_handoff runs the grouped kernel only (rank <= 128, default options)";
        return PS_ELIMIT;
    }
    if (f.d_row == 0 || f.d_col == 0) return PS_OK;
    const size_t n_order = (size_t)f.d_row * f.d_col * 2;
    const size_t need = (size_t)DPAPS_HANDOFF_MAX_COLS * sizeof(uint32_t) + n_order * sizeof(int32_t);
    if (need > ps->handoff_ws_bytes) {
        PS_HIP(ps, hipStreamSynchronize(st));
        if (ps->handoff_ws) PS_HIP(ps, hipFree(ps->handoff_ws));
        ps->handoff_ws = nullptr; ps->handoff_ws_bytes = 0;
        PS_HIP(ps, hipMalloc(&ps->handoff_ws, need));
        ps->handoff_ws_bytes = need;
    }
    SgdArgs a = sgd_args(ps, nullptr, lr, lambda);
    a.ticket_cap = (int32_t)std::max<int64_t>(f.max_multi_in_block, 1);
    a.fuse_localize = 1;
    a.col_state = (uint32_t *)ps->handoff_ws;
    a.sched = (int32_t *)(a.col_state + DPAPS_HANDOFF_MAX_COLS);
    // every column block free and unvisited, no order recorded yet (-1: a worker that stopped on an error)
    PS_HIP(ps, hipMemsetAsync(a.col_state, 0, (size_t)DPAPS_HANDOFF_MAX_COLS * sizeof(uint32_t), st));
    PS_HIP(ps, hipMemsetAsync(a.sched, 0xFF, n_order * sizeof(int32_t), st));
    const int rc = dpaps_launch_sgd_handoff(ps, a, f.d_row, st);
    if (rc) return rc;
    if (order_host_out) {
        PS_HIP(ps, hipMemcpyAsync(order_host_out, a.sched, n_order * sizeof(int32_t), hipMemcpyDeviceToHost, st));
        PS_HIP(ps, hipStreamSynchronize(st));
    }
    return PS_OK;
}

extern "C" int mf_profile_read(ps_handle ps, double *sgd_ms_host_out, int64_t *launches_host_out, void *stream) {
    if (!ps || !sgd_ms_host_out || !launches_host_out) return PS_EINVAL;
    PS_HIP(ps, hipStreamSynchronize((hipStream_t)stream));
    double total = 0.0;
    for (size_t i = 0; i + 1 < ps->ev_used; i += 2) {
        float ms = 0.0f;
        PS_HIP(ps, hipEventElapsedTime(&ms, ps->ev_pool[i], ps->ev_pool[i + 1]));
        total += (double)ms;
    }
    *sgd_ms_host_out = total;
    *launches_host_out = (int64_t)(ps->ev_used / 2);
    ps->ev_used = 0;
    return PS_OK;
}

extern "C" int mf_train_sse(ps_handle ps, double *sse_host_out, void *stream) {
    if (!ps || !sse_host_out) return PS_EINVAL;
    MfData &f = ps->mf;
    if (!f.row) { ps->last_error = "mf_train_sse before mf_load_ratings"; return PS_EINVAL; }
    hipStream_t st = (hipStream_t)stream;
    const int blocks = 2048;
    int rc = dpaps_ws_reserve(ps, blocks * sizeof(double));
    if (rc) return rc;
    double *partial = (double *)ps->ws;
    k_mf_sse<<<blocks, 256, 0, st>>>(f.row, f.col, f.val, f.nnz, ps->val, f.m, ps->L, partial);
    PS_HIP(ps, hipGetLastError());
    std::vector<double> h(blocks);
    PS_HIP(ps, hipMemcpyAsync(h.data(), partial, blocks * sizeof(double), hipMemcpyDeviceToHost, st));
    rc = dpaps_take_error(ps, st);
    double sse = 0.0;
    for (int i = 0; i < blocks; ++i) sse += h[i];
    *sse_host_out = sse;
    return rc;
}
