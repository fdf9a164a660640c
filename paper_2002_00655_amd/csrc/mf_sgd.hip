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

#include <algorithm>
#include <cstring>

static inline unsigned grid_for(int64_t n, int block) { return (unsigned)((n + block - 1) / block); }

// ---------------------------------------------------------------------------
// wavefront sum over 64 lanes with DPP; the total is returned in every lane as a
// wave-uniform value.  Fixed reduction tree, so the result is reproducible.
// ---------------------------------------------------------------------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float x) {
    int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROW_MASK, 0xF, false);
    return x + __builtin_bit_cast(float, y);
}

__device__ __forceinline__ float wave_sum(float x) {
    x = dpp_add<0xB1, 0xF>(x);    // quad_perm [1,0,3,2]: pairs
    x = dpp_add<0x4E, 0xF>(x);    // quad_perm [2,3,0,1]: quads
    x = dpp_add<0x141, 0xF>(x);   // row_half_mirror: 8 lanes
    x = dpp_add<0x140, 0xF>(x);   // row_mirror: 16 lanes (every lane of a row holds the row's sum)
    x = dpp_add<0x142, 0xA>(x);   // row_bcast15 into rows 1 and 3
    x = dpp_add<0x143, 0xC>(x);   // row_bcast31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

__device__ __forceinline__ int rl_i(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ float rl_f(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// ---------------------------------------------------------------------------
// localize step of a subepoch: every task takes the keys of its row block and
// of its column block (Sec. 2.3).  One workgroup per task.  Message counts as
// for ps_localize; because the keys are two ascending ranges, their home nodes
// come in ascending runs, and the distinct old owners are collected per home
// node in an LDS bit set.
// ---------------------------------------------------------------------------
struct LocalizeArgs {
    const int32_t *tasks;      // (worker, row block, column block) triples of this stratum
    int32_t *owner;
    const int64_t *row_bounds, *col_bounds;
    int64_t m, per_home;
    int32_t W;
    u64 *stats;
    const int32_t *err;
};

__global__ __launch_bounds__(256) void k_mf_localize(LocalizeArgs a) {
    extern __shared__ uint32_t lds_u32[];
    if (*(volatile const int32_t *)a.err) return;
    const int words = (a.W + 31) / 32;
    uint32_t *bits_all = lds_u32, *bits_h = lds_u32 + words;
    __shared__ int s_reloc, s_req, s_instr;
    const int32_t worker = a.tasks[3 * blockIdx.x], rb = a.tasks[3 * blockIdx.x + 1], cb = a.tasks[3 * blockIdx.x + 2];
    const int64_t r0 = a.row_bounds[rb], r1 = a.row_bounds[rb + 1];
    const int64_t c0 = a.m + a.col_bounds[cb], c1 = a.m + a.col_bounds[cb + 1];
    for (int i = threadIdx.x; i < 2 * words; i += blockDim.x) lds_u32[i] = 0;
    if (threadIdx.x == 0) { s_reloc = 0; s_req = 0; s_instr = 0; }
    __syncthreads();
    // home nodes touched by the two key ranges (empty range: lo > hi)
    const int64_t hr_lo = r1 > r0 ? r0 / a.per_home : 1, hr_hi = r1 > r0 ? (r1 - 1) / a.per_home : 0;
    const int64_t hc_lo = c1 > c0 ? c0 / a.per_home : 1, hc_hi = c1 > c0 ? (c1 - 1) / a.per_home : 0;
    int reloc = 0;
    for (int part = 0; part < 2; ++part) {
        const int64_t lo = part == 0 ? hr_lo : hc_lo, hi = part == 0 ? hr_hi : hc_hi;
        for (int64_t h = lo; h <= hi; ++h) {
            if (part == 1 && h >= hr_lo && h <= hr_hi) continue;   // done together with the row range
            const int64_t k_lo = h * a.per_home, k_hi = k_lo + a.per_home;
            for (int sub = 0; sub < 2; ++sub) {
                const int64_t x0 = sub == 0 ? r0 : c0, x1 = sub == 0 ? r1 : c1;
                const int64_t s0 = x0 > k_lo ? x0 : k_lo, s1 = x1 < k_hi ? x1 : k_hi;
                for (int64_t k = s0 + threadIdx.x; k < s1; k += blockDim.x) {
                    int32_t old = a.owner[k];
                    if (old != worker) {
                        a.owner[k] = worker;             // the home node updates the location at once
                        ++reloc;
                        atomicOr(&bits_h[old >> 5], 1u << (old & 31));
                        atomicOr(&bits_all[old >> 5], 1u << (old & 31));
                    }
                }
            }
            __syncthreads();
            if (threadIdx.x < 64) {
                int cnt = 0;
                for (int i = threadIdx.x; i < words; i += 64) cnt += __popc(bits_h[i]);
                for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off);
                if (threadIdx.x == 0 && cnt > 0) {
                    if (h != worker) s_req += 1;
                    s_instr += cnt - (int)((bits_h[h >> 5] >> (h & 31)) & 1u);
                }
            }
            __syncthreads();
            for (int i = threadIdx.x; i < words; i += blockDim.x) bits_h[i] = 0;
            __syncthreads();
        }
    }
    if (reloc) atomicAdd(&s_reloc, reloc);
    __syncthreads();
    if (threadIdx.x < 64) {
        int cnt = 0;
        for (int i = threadIdx.x; i < words; i += 64) cnt += __popc(bits_all[i]);
        for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off);
        if (threadIdx.x == 0) {
            atomicAdd(&a.stats[PS_STAT_LOCALIZE_KEYS], (u64)((r1 - r0) + (c1 - c0)));
            if (s_reloc) atomicAdd(&a.stats[PS_STAT_RELOCATED], (u64)s_reloc);
            if (s_req) atomicAdd(&a.stats[PS_STAT_MSG_LOC_REQ], (u64)s_req);
            if (s_instr) atomicAdd(&a.stats[PS_STAT_MSG_LOC_INSTRUCT], (u64)s_instr);
            if (cnt) atomicAdd(&a.stats[PS_STAT_MSG_LOC_TRANSFER], (u64)cnt);
        }
    }
}

// ---------------------------------------------------------------------------
// the SGD kernel
// ---------------------------------------------------------------------------
struct SgdArgs {
    const int32_t *tasks;
    float *val;                 // the parameter store, K x L
    const int32_t *owner;
    const int32_t *e_row; const float *e_val; const uint32_t *e_info;
    const int64_t *run_start; const int32_t *run_col; const int64_t *blk_run_ptr;
    const int32_t *multi_row; const int64_t *blk_multi_ptr;
    const int64_t *row_bounds, *col_bounds;
    int64_t m;
    int32_t L, d_col;
    int32_t cache_cap;          // row factors that fit in LDS
    int32_t ticket_cap;         // ticket counters in LDS
    float lr, lambda;
    u64 *stats;
    int32_t *err;
};

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

// One SGD step on registers.  w, h: the two factor rows (lane l holds
// components l, l+64, ...; components past L are zero).  Both rows are
// updated from their old values:
//   e = v - <w,h>;  w += lr (e h - lambda w);  h += lr (e w - lambda h).
template <int NV, bool EXACT>
__device__ __forceinline__ void sgd_step(float (&w)[NV], float (&h)[NV], float v, float lr, float lambda, int L) {
    float dot;
    if constexpr (EXACT) {
        // components summed in index order, every product and sum rounded on its own
        float prod[NV];
#pragma unroll
        for (int c = 0; c < NV; ++c) prod[c] = w[c] * h[c];
        dot = 0.0f;
#pragma unroll
        for (int c = 0; c < NV; ++c) {
            const int lim = min(64, L - 64 * c);
            for (int l = 0; l < lim; ++l) dot = dot + rl_f(prod[c], l);
        }
    } else {
        float p = 0.0f;
#pragma unroll
        for (int c = 0; c < NV; ++c) p = __builtin_fmaf(w[c], h[c], p);
        dot = wave_sum(p);
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

template <int NV, bool EXACT>
__global__ __launch_bounds__(1024) void k_mf_sgd(SgdArgs a) {
    extern __shared__ float lds_f[];
    if (*(volatile const int32_t *)a.err) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int L = a.L;
    float *cache = lds_f;                                              // cache_cap x L
    uint32_t *ticket = reinterpret_cast<uint32_t *>(lds_f + (size_t)a.cache_cap * L);   // ticket_cap
    __shared__ int next_run;

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
    // pull the busiest rows into LDS; reset the tickets
    for (int t = threadIdx.x; t < nmulti; t += blockDim.x) ticket[t] = 0;
    for (int s = wave; s < ncached; s += nwaves) {
        const float *src = a.val + (int64_t)a.multi_row[mp0 + s] * L;
        for (int k = lane; k < L; k += 64) cache[(size_t)s * L + k] = src[k];
    }
    if (threadIdx.x == 0) next_run = 0;
    __syncthreads();

    const float lr = a.lr, lambda = a.lambda;
    u64 done = 0;
    for (;;) {
        int run = 0;
        if (lane == 0) run = atomicAdd(&next_run, 1);
        run = __builtin_amdgcn_readfirstlane(run);
        const int64_t g = run0 + run;
        if (g >= run1) break;
        const int64_t s0 = a.run_start[g], s1 = a.run_start[g + 1];
        float *hrow = a.val + (a.m + a.run_col[g]) * (int64_t)L;
        float h[NV];
        load_row<NV>(hrow, lane, L, h);
        for (int64_t base = s0; base < s1; base += 64) {
            const int cnt = (s1 - base) < 64 ? (int)(s1 - base) : 64;
            int my_row = 0; float my_val = 0.0f; int my_info = 0;
            if (lane < cnt) { my_row = a.e_row[base + lane]; my_val = a.e_val[base + lane]; my_info = (int)a.e_info[base + lane]; }
            for (int u = 0; u < cnt; ++u) {
                const int row = rl_i(my_row, u);
                const float v = rl_f(my_val, u);
                const uint32_t info = (uint32_t)rl_i(my_info, u);
                const uint32_t slot = info & 0xFFFFu, seq = info >> 16;
                float *wrow = a.val + (int64_t)row * L;
                float w[NV];
                if (slot == 0xFFFFu) {
                    // the only entry of this row in the block: read and write in place
                    load_row<NV>(wrow, lane, L, w);
                    sgd_step<NV, EXACT>(w, h, v, lr, lambda, L);
                    store_row<NV>(wrow, lane, L, w);
                } else {
                    // wait until the row's earlier entries (in stored order) are done
                    uint32_t *tk = &ticket[slot];
                    for (uint32_t spins = 0; __hip_atomic_load(tk, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) != seq;) {
                        __builtin_amdgcn_s_sleep(1);
                        // every wait ends: the predecessor always makes progress.  Should that ever fail
                        // (corrupt input tables), give up rather than hang the device.
                        if ((++spins & 1023u) == 0 && (spins > (1u << 22) || *(volatile const int32_t *)a.err)) {
                            atomicExch(a.err, PS_ESTALL);
                            break;
                        }
                    }
                    if (slot < (uint32_t)ncached) {
                        float *src = cache + (size_t)slot * L;          // the row lives in LDS for this subepoch
                        load_row<NV>(src, lane, L, w);
                        sgd_step<NV, EXACT>(w, h, v, lr, lambda, L);
                        store_row<NV>(src, lane, L, w);
                    } else {                                             // did not fit: handed over through memory
                        load_row<NV>(wrow, lane, L, w);
                        sgd_step<NV, EXACT>(w, h, v, lr, lambda, L);
                        store_row<NV>(wrow, lane, L, w);
                    }
                    __hip_atomic_store(tk, seq + 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
            done += (u64)cnt;
        }
        store_row<NV>(hrow, lane, L, h);
    }
    __syncthreads();
    // push the cached rows back
    for (int s = wave; s < ncached; s += nwaves) {
        float *dst = a.val + (int64_t)a.multi_row[mp0 + s] * L;
        for (int k = lane; k < L; k += 64) dst[k] = cache[(size_t)s * L + k];
    }
    // each entry was one pull and one push of two local keys
    if (lane == 0 && done) {
        atomicAdd(&a.stats[PS_STAT_PULL_LOCAL], 2 * done);
        atomicAdd(&a.stats[PS_STAT_PUSH_LOCAL], 2 * done);
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
    static size_t configured = 0;
    if (lds > configured) {
        PS_HIP(ps, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mf_sgd<NV, EXACT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        configured = lds;
    }
    k_mf_sgd<NV, EXACT><<<ntasks, threads, lds, st>>>(a);
    PS_HIP(ps, hipGetLastError());
    return PS_OK;
}

extern "C" int mf_sgd_epoch(ps_handle ps, const int32_t *tasks_host, const int32_t *stratum_ptr_host, int32_t num_strata,
                            float lr, float lambda, void *stream) {
    if (!ps || num_strata < 0 || (num_strata > 0 && (!tasks_host || !stratum_ptr_host))) return PS_EINVAL;
    MfData &f = ps->mf;
    if (!f.row) { ps->last_error = "mf_sgd_epoch before mf_load_ratings"; return PS_EINVAL; }
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
    const int threads = 64 * ps->opt_waves;
    const size_t loc_lds = 2 * (size_t)((ps->W + 31) / 32) * sizeof(uint32_t);

    for (int32_t s = 0; s < num_strata; ++s) {
        const int ntasks = stratum_ptr_host[s + 1] - stratum_ptr_host[s];
        if (ntasks == 0) continue;
        const int32_t *tasks = ps->d_tasks + 3 * (int64_t)stratum_ptr_host[s];
        LocalizeArgs la{tasks, ps->owner, f.row_bounds, f.col_bounds, f.m, ps->per_home, ps->W, ps->stats, ps->err};
        k_mf_localize<<<ntasks, 256, loc_lds, st>>>(la);
        PS_HIP(ps, hipGetLastError());
        SgdArgs a{tasks, ps->val, ps->owner, f.row, f.val, f.info, f.run_start, f.run_col, f.blk_run_ptr, f.multi_row,
                  f.blk_multi_ptr, f.row_bounds, f.col_bounds, f.m, L, f.d_col, (int32_t)cache_cap, (int32_t)ticket_cap,
                  lr, lambda, ps->stats, ps->err};
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
        if (ps->opt_exact) {
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
