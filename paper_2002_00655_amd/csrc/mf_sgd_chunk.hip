// Blocked latent-factor SGD, grouped form of the per-entry step (Sec. 2.2.2, Sec. 4.1,
// Appendix A "Matrix factorization" of the paper; same schedule, same stored order and
// same result, up to rounding, as the entry-by-entry kernel in mf_sgd.hip).
//
// Why.  All entries of one column update the same factor row h, so a column's entries
// form a serial chain, and measured on the device the entry-by-entry kernel is bound by
// the instruction issue of the wavefront that holds the longest chain, not by memory.
// The per-entry recursion
//     e_t = v_t - <w_t, h_{t-1}>,   h_t = c h_{t-1} + lr e_t w_t,   w_t' = c w_t + lr e_t h_{t-1}
// (c = 1 - lr lambda) is affine in h, so for a group of T consecutive entries of a column
// (distinct rows w_0 .. w_{T-1}, all final when the group starts) it can be regrouped:
//   1. X = [w_0; ...; w_{T-1}; h]  (16 x r with T = 15),  G = X X^T  - one dense 16x16xr
//      product (matrix cores); G[s][15] = <w_s, h> are the T inner products with the
//      incoming h, G[s][t] = <w_s, w_t>;
//   2. with p_s = <w_s, h> for the incoming h, the errors solve a lower-triangular system,
//      e_t = v_t - c^t p_t - sum_(u<t) lr c^(t-1-u) G[t][u] e_u, which in the scaled unknowns
//      e_t c^(-t) loses its powers of c: one dependent vector instruction per entry instead
//      of a length-r reduction;
//   3. all new rows are one more dense product X' = C X with the lower-triangular 16x16
//      coefficient matrix  C[t][t] = c,  C[t][s<t] = lr^2 e_t e_s c^(t-1-s),
//      C[t][15] = lr e_t c^t,  C[15][s] = lr e_s c^(T-1-s),  C[15][15] = c^T.
// c is never rounded to fp32 on its own (that would bias every update of a row the same
// way): products with c are formed as x - (lr lambda) x, and the dense product is taken
// as X' = X + (C - I) X with c - 1 and c^T - 1 computed in double.
// Dependencies between columns are unchanged: a row with several entries in the block is
// ordered by its ticket, and a group starts when the rows of all its entries are final.
// Groups are cut by the data alone (15 entries, the end of the column, or just before an
// entry whose row already occurs earlier in the same column), never by timing, so the
// arithmetic - and with it every bit of the result - is the same from run to run.  A
// group only waits for entries of earlier columns or earlier groups, so waiting ends.
//
// Two parts.  Grouping pays for long column runs; a short run would still cost a whole
// group, and because every column is walked by ascending row, each run's last group ends
// up waiting for the previous run's, one after the other.  So only the leading runs of a
// block that are long enough ("heavy" columns) are processed in groups, by the first few
// wavefronts.  The entries of all other runs are walked row by row: a wavefront takes a few
// consecutive rows, keeps a row's factor in registers for all of that row's entries, and
// the factors of the non-heavy columns live in LDS for the subepoch, each with a ticket
// counter that orders the column's entries as stored.  This is the same dependency graph
// as walking those runs one after the other - every row's entries in stored order, every
// column's entries in stored order - so the result is the same; it only takes the waiting
// out.  A row's entries in heavy runs precede its other entries in stored order (heavy
// runs lead the block), and the row's ticket tells when they are done.
#include "common.h"
#include "mf_device.h"

#include <algorithm>

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

#define CH 15                    // entries per group (the 16th row of X is the column's row)
#define AUX_SC1 16               // cache policy of a buffer access: agent scope
#define DPAPS_LONG_RUN_GROUPS 64 // data with a column run of at least this many groups in a block: see the recurrence

// x, which is the same in all lanes, as a scalar
__device__ __forceinline__ int64_t uniform_i64(int64_t x) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)x);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)x >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// value of `v` in lane `src` (any permutation; goes through the LDS crossbar, no memory)
__device__ __forceinline__ int bperm_i(int v, int src) { return __builtin_amdgcn_ds_bpermute(src << 2, v); }
__device__ __forceinline__ float bperm_f(float v, int src) {
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src << 2, __builtin_bit_cast(int, v)));
}

// One step of the triangular solve in sgd_block, with the terms of the new column factor that have become final
// (see there): with eps_U = acc of lane U of every row of 16 lanes, broadcast by the instruction itself,
//     hs[cc] += eps_U * w[cc]   (the entry's row, for the new h),     acc += eps_U * nl   (nl = -(lr / c) G[t][U] below
// the diagonal, zero elsewhere, so lanes t <= U keep their value).  The data hazard "a vector instruction writes a
// register, a DPP operand reads it" needs two wait states, which no instruction of the step can fill (all three read
// acc through DPP): hence the s_nop at the head, which also covers whatever the compiler puts in front.
template <int U, int NV>
__device__ __forceinline__ void solve_step(float &acc, float (&hs)[NV], const float (&w)[NV], float nl) {
    static_assert(NV == 1 || NV == 2, "a factor row has at most 128 components here");
    if constexpr (NV == 2)
        __asm__ volatile("s_nop 1\n\t"
                         "v_fmac_f32_dpp %1, %0, %3 row_newbcast:%6 row_mask:0xf bank_mask:0xf\n\t"
                         "v_fmac_f32_dpp %2, %0, %4 row_newbcast:%6 row_mask:0xf bank_mask:0xf\n\t"
                         "v_fmac_f32_dpp %0, %0, %5 row_newbcast:%6 row_mask:0xf bank_mask:0xf"
                         : "+v"(acc), "+v"(hs[0]), "+v"(hs[1])
                         : "v"(w[0]), "v"(w[1]), "v"(nl), "n"(U));
    else
        __asm__ volatile("s_nop 1\n\t"
                         "v_fmac_f32_dpp %1, %0, %2 row_newbcast:%4 row_mask:0xf bank_mask:0xf\n\t"
                         "v_fmac_f32_dpp %0, %0, %3 row_newbcast:%4 row_mask:0xf bank_mask:0xf"
                         : "+v"(acc), "+v"(hs[0])
                         : "v"(w[0]), "v"(nl), "n"(U));
}
// the last entry has nothing below it: only its term of the new h
template <int U, int NV>
__device__ __forceinline__ void solve_last(const float &acc, float (&hs)[NV], const float (&w)[NV]) {
    if constexpr (NV == 2)
        __asm__ volatile("s_nop 1\n\t"
                         "v_fmac_f32_dpp %0, %2, %3 row_newbcast:%5 row_mask:0xf bank_mask:0xf\n\t"
                         "v_fmac_f32_dpp %1, %2, %4 row_newbcast:%5 row_mask:0xf bank_mask:0xf"
                         : "+v"(hs[0]), "+v"(hs[1])
                         : "v"(acc), "v"(w[0]), "v"(w[1]), "n"(U));
    else
        __asm__ volatile("s_nop 1\n\t"
                         "v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
                         : "+v"(hs[0])
                         : "v"(acc), "v"(w[0]), "n"(U));
}
// in front of the first step: a DPP operand must also keep five wait states from a write of the execution mask
__device__ __forceinline__ void solve_first() { __asm__ volatile("s_nop 4"); }

// NT = number of 16-component tiles of a factor row (rank <= 16 NT); A4: the rank is a multiple of 4,
// so every row starts on a 16-byte boundary and is read in 16-byte pieces
// (otherwise in 8-byte pieces where the rank is even, in 4-byte pieces where it is odd)
// AGENT_H: the column factors and the owner map are read and written with agent-scope accesses, which the caches
// of a compute die pass through to memory, so that the workgroup that takes the column block next - on any die -
// reads what this one wrote, without a write-back or an invalidation of whole caches (the row factors need none
// of that: they stay with this workgroup).  Off: plain accesses; the kernel's end publishes everything.
// One call processes the block (rb, cb) for `worker`; all threads of the workgroup take part.
// LONG_RUNS: the variant of the recurrence for data with column runs of very many groups (see there).
// RICH: compiled for at most 12 wavefronts, so with a third more registers: what does not depend on the column's
// factor is then read ahead of the wait for it.
template <int NT, bool A4, bool AGENT_H, bool LONG_RUNS, bool RICH = false>
__device__ __forceinline__ void sgd_block(const SgdArgs &a, float *lds_f, const int32_t worker, const int32_t rb, const int32_t cb) {
    if constexpr (!AGENT_H) {     // (in the loop, the caller looks: there all threads must take the same way)
        if (__hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) return;
    }
    constexpr int RS = 16 * NT + 4;          // row stride of the staging area in floats (conflict-free for both read patterns)
    constexpr int NV = (NT + 3) / 4;         // 64-component slices of a row
    // Called in a loop (AGENT_H): the thread's number, the rank and the step sizes pass through empty asm
    // statements, so that what depends on them - the table of powers of c, lane offsets - is not computed ahead
    // of the loop and held in registers all the way through it.
    int tid = threadIdx.x, L_ = a.L;
    unsigned lr_ = __float_as_uint(a.lr), lambda_ = __float_as_uint(a.lambda);
    if constexpr (AGENT_H) {
        __asm__ volatile("" : "+v"(tid));
        __asm__ volatile("" : "+s"(L_), "+s"(lr_), "+s"(lambda_));
    }
    const int lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    const int n16_ = lane & 15, hi_ = lane >> 4;
    const int L = L_;
    const bool even_rank = (L & 1) == 0;     // (only looked at where the rank is no multiple of 4: rows then start on 8-byte boundaries)
    const bool tail = lane + 64 * (NV - 1) < L;
    const int hwaves = a.heavy_waves;                                  // wavefronts 0 .. hwaves-1 take the heavy runs
    float *stg = lds_f + (size_t)wave * 16 * RS;                       // this wavefront's X: 16 rows (heavy wavefronts only)
    float *cpow = lds_f + (size_t)hwaves * 16 * RS;                    // c^0 .. c^16
    float *cpm1 = cpow + 20;                                           // c^0 - 1 .. c^16 - 1
    float *cim1 = cpow + 40;                                           // c^-0 - 1 .. c^-16 - 1
    float *hshare = cpow + 60;                                         // DPAPS_HEAVY_MAX x 16 NT: the heavy columns' factors
    uint32_t *hseq = reinterpret_cast<uint32_t *>(hshare + DPAPS_HEAVY_MAX * 16 * NT);   // and how many groups each has absorbed
    uint32_t *ticket = hseq + DPAPS_HEAVY_MAX;                          // ticket_cap: one per row with several entries
    uint32_t *ctick = ticket + a.ticket_cap;                           // ctick_cap: one per non-heavy column
    float *hcache = reinterpret_cast<float *>(ctick + a.ctick_cap);    // hcache_cap x L: factors of non-heavy columns
    __shared__ int next_run;
    __shared__ int next_trow;
    __shared__ unsigned int done_entries;
    __shared__ uint32_t give_up;

    // (what is the same in all lanes is said to be: a value read from memory otherwise stays in vector registers
    // for the whole kernel)
    const int64_t b = (int64_t)rb * a.d_col + cb;
    const int64_t run0 = uniform_i64(a.blk_run_ptr[b]), run1 = uniform_i64(a.blk_run_ptr[b + 1]);
    const int nmulti = __builtin_amdgcn_readfirstlane((int)(a.blk_multi_ptr[b + 1] - a.blk_multi_ptr[b]));
    const int nruns = (int)(run1 - run0);
    const int nheavy = __builtin_amdgcn_readfirstlane(a.blk_nheavy[b]);
    const int ntcols = nruns - nheavy;                                 // non-heavy columns
    const int ncached = min(ntcols, a.hcache_cap);
    const int64_t tr0 = uniform_i64(a.blk_trun_ptr[b]), tr1 = uniform_i64(a.blk_trun_ptr[b + 1]);
    const float lr = __uint_as_float(lr_), lambda = __uint_as_float(lambda_);
    const float delta = (float)((double)lr * (double)lambda);         // c = 1 - delta
    const float nlrc = (float)(-(double)lr / (1.0 - (double)lr * (double)lambda));   // -lr / c
    // The factors of the block's rows and of its columns, each as a buffer: an access at an offset past
    // the end reads as zero and writes nothing, which is how lanes without a row are switched off
    // without branching.  (The host has checked that both spans are below 2 GiB.)
    const int64_t blk_r0 = uniform_i64(a.row_bounds[rb]), blk_c0 = uniform_i64(a.col_bounds[cb]);
    const uint32_t wspan = (uint32_t)__builtin_amdgcn_readfirstlane((int)((a.row_bounds[rb + 1] - blk_r0) * L * 4));
    const uint32_t hspan = (uint32_t)__builtin_amdgcn_readfirstlane((int)((a.col_bounds[cb + 1] - blk_c0) * L * 4));
    const __amdgpu_buffer_rsrc_t wbuf = __builtin_amdgcn_make_buffer_rsrc(a.val + blk_r0 * L, 0, (int)wspan, 0x00020000);
    const __amdgpu_buffer_rsrc_t hbuf = __builtin_amdgcn_make_buffer_rsrc(a.val + (a.m + blk_c0) * L, 0, (int)hspan, 0x00020000);

    // The column factors that will live in LDS are requested now and put there after the localize step, which
    // hides their way from memory: of the heavy columns' this thread's first element, of the others' its first HPRE.
    constexpr int HPRE = 8;
    auto heavy_elem = [&](int i) {
        const int r = i / (16 * NT), k = i - r * 16 * NT;
        return (r < nheavy && k < L) ? load_f<AGENT_H>(&a.val[(a.m + a.run_col[run0 + r]) * (int64_t)L + k]) : 0.0f;
    };
    auto cached_elem = [&](int idx) {
        const int s = idx / L;
        return load_f<AGENT_H>(&a.val[(a.m + a.run_col[run0 + nheavy + s]) * (int64_t)L + (idx - s * L)]);
    };
    const int ncached_elems = ncached * L;
    float pre_heavy = 0.0f, pre_cached[HPRE];
    if (tid < DPAPS_HEAVY_MAX * 16 * NT) pre_heavy = heavy_elem(tid);
#pragma unroll
    for (int q = 0; q < HPRE; ++q) {
        const int idx = tid + q * (int)blockDim.x;
        pre_cached[q] = idx < ncached_elems ? cached_elem(idx) : 0.0f;
    }

    if (a.fuse_localize) {
        // the localize step of this task (Sec. 2.3), which makes every parameter the worker will touch its own
        LocalizeArgs la{a.tasks, a.owner_w, a.row_bounds, a.col_bounds, a.m, a.per_home, a.W, a.stats, a.err};
        mf_localize_task<AGENT_H>(la, reinterpret_cast<uint32_t *>(lds_f), hwaves * 16 * RS, worker, rb, cb);
    } else {
        // every parameter this worker will touch must be allocated to it (Sec. 4.1: all access is local)
        const int64_t r0 = a.row_bounds[rb], r1 = a.row_bounds[rb + 1];
        const int64_t c0 = a.m + a.col_bounds[cb], c1 = a.m + a.col_bounds[cb + 1];
        bool bad = false;
        for (int64_t k = r0 + threadIdx.x; k < r1; k += blockDim.x) bad |= a.owner[k] != worker;
        for (int64_t k = c0 + threadIdx.x; k < c1; k += blockDim.x) bad |= a.owner[k] != worker;
        if (bad) atomicExch(a.err, PS_EREMOTE);
    }
    for (int t = threadIdx.x; t < nmulti; t += blockDim.x) ticket[t] = 0;
    for (int t = threadIdx.x; t < ntcols; t += blockDim.x) ctick[t] = 0;
    for (int i = threadIdx.x; i < hwaves * 16 * RS; i += blockDim.x) lds_f[i] = 0.0f;
    // the heavy columns' factors (components past the rank are zero) and their group counters
    if (tid < DPAPS_HEAVY_MAX * 16 * NT) hshare[tid] = pre_heavy;
    for (int i = tid + blockDim.x; i < DPAPS_HEAVY_MAX * 16 * NT; i += blockDim.x) hshare[i] = heavy_elem(i);
    if (threadIdx.x < DPAPS_HEAVY_MAX) hseq[threadIdx.x] = 0;
#pragma unroll
    for (int q = 0; q < HPRE; ++q) {
        const int idx = tid + q * (int)blockDim.x;
        if (idx < ncached_elems) hcache[idx] = pre_cached[q];
    }
#pragma unroll 4
    for (int idx = tid + HPRE * (int)blockDim.x; idx < ncached_elems; idx += blockDim.x) hcache[idx] = cached_elem(idx);
    if (threadIdx.x == 0) {
        const double cd = 1.0 - (double)lr * (double)lambda;
        double x = 1.0;
        for (int i = 0; i <= 16; ++i) { cpow[i] = (float)x; cpm1[i] = (float)(x - 1.0); cim1[i] = (float)(1.0 / x - 1.0); x = x * cd; }
        next_run = 0; next_trow = 0; done_entries = 0; give_up = 0;
    }
    __syncthreads();

    unsigned int done = 0;
    // ---- part 1: the heavy runs, in groups ----------------------------------------------
    // A heavy run is processed by a team of T wavefronts that take its groups in turn.  Only a small part
    // of a group's work depends on the column's factor h as the previous group left it: the inner products
    // <w_s, h>, the error recurrence and the new h.  That part is done with h in LDS (shared by the team)
    // and handed from group to group through a counter; the loads, the products <w_s, w_t> before it and
    // the new rows w_s after it overlap with the other wavefront's turn.
    if (wave < hwaves) {
        // The longest runs are what everything else ends up waiting for.  With 12 or more heavy wavefronts each
        // follows the block's plan: a team of T wavefronts on one long run (this one takes its groups mb, mb + T,
        // ...), or one wavefront that takes several short runs one after the other.  With fewer: one wavefront
        // per run, taking runs in turn.
        int T = 1, mb = 0, run_first = wave, run_last = nheavy, run_step = hwaves;
        if (a.team == 2) {
            const uint32_t pl = a.team_plan[b * 16 + wave];
            run_first = (int)(pl & 0xFFu); run_last = (int)((pl >> 8) & 0xFFu); T = (int)((pl >> 16) & 0xFFu); mb = (int)(pl >> 24);
            run_step = 1;
        }
        for (int run = run_first; run < run_last; run += run_step) {
            const int64_t g = run0 + run;
            const int64_t s0 = a.run_start[g], s1 = a.run_start[g + 1];
            const uint32_t hoff = (uint32_t)((a.run_col[g] - blk_c0) * L * 4);   // the column's row inside the column buffer
            const int64_t gb = a.run_gptr[g];
            const int ng = (int)(a.run_gptr[g + 1] - gb) - 1;                   // groups of this run
            float *hsh = hshare + run * 16 * NT;
            uint32_t *hsq = &hseq[run];
            __builtin_amdgcn_s_setprio(2);
            // where the groups start: 64 table entries, one per lane, from group gw on
            int gw = 0;
            int gs_win = a.gstart[gb + (lane <= ng ? lane : ng)];
            auto gs = [&](int gi) { return rl_i(gs_win, (gi < ng ? gi : ng) - gw); };   // start of group gi (the run's length past the last)

            // Read-ahead in two stages.  meta_load: the per-entry data of a group, entry pp + l into lane l.
            // plan: whether all rows of the group are final, and their gather, straight into the layout of
            // the dense products - lane (n16, hi) holds components 16 j + 4 hi .. + 3 of row n16 in xp[j].
            // (Always executed, with positions clamped into the run: a load that is only issued on some
            // paths makes the compiler copy its result into the loop's registers right away, which waits.)
            int mq_row = 0, mq_info = (int)INFO_NONE;
            float mq_val = 0.0f;
            auto meta_load = [&](int64_t pp) {
                int64_t q = pp + lane;
                q = q < s1 ? q : s1 - 1;
                mq_row = a.e_row[q]; mq_val = a.e_val[q]; mq_info = (int)a.e_info[q];
            };
            int pf_row = 0, pf_info = (int)INFO_NONE, pf_n = 0;
            float pf_val = 0.0f;
            bool pf_ready = false;
            f32x4 xp[NT];
            auto gather = [&](int n16, int hi) {
                const int rid = bperm_i(pf_row, n16);
                // byte offset of this lane's first piece; no entry: past the end, reads as zero
                const uint32_t goff = n16 < pf_n ? (uint32_t)((rid - (int)blk_r0) * L + 4 * hi) * 4u : wspan;
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    if constexpr (A4) {
                        // may run past the row's end (into the next row, or past the buffer's end)
                        xp[j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(wbuf, (int)goff + 64 * j, 0, 0));
                    } else if (even_rank) {
                        // rows start on 8-byte boundaries: two pieces of two components (both exist or neither)
#pragma unroll
                        for (int q = 0; q < 4; q += 2) {
                            const u32x2 pr = __builtin_amdgcn_raw_buffer_load_b64(
                                wbuf, (16 * j + 4 * hi + q < L ? (int)goff : (int)wspan) + 64 * j + 4 * q, 0, 0);
                            const uint32_t p0 = pr[0], p1 = pr[1];
                            xp[j][q] = __uint_as_float(p0); xp[j][q + 1] = __uint_as_float(p1);
                        }
                    } else {
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            xp[j][q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                wbuf, (16 * j + 4 * hi + q < L ? (int)goff : (int)wspan) + 64 * j + 4 * q, 0, 0));
                    }
                }
            };
            auto plan = [&](int n, int n16, int hi) {     // the group of n entries whose data meta_load has fetched
                pf_row = mq_row; pf_val = mq_val;
                pf_info = lane < n ? mq_info : (int)INFO_NONE;
                pf_n = n;
                const uint32_t slot = (uint32_t)pf_info & 0xFFFFu, seq = ((uint32_t)pf_info >> 16) & 0x7FFFu;
                bool ready = true;
                if (lane < n && slot != INFO_SINGLE) ready = ticket_read(&ticket[slot]) == seq;
                pf_ready = __ballot(ready) == ~0ull;      // all rows final now, before their loads are issued
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                gather(n16, hi);
            };

            int gi = mb;                                  // this wavefront's groups: mb, mb + T, ...
            meta_load(s0 + gs(gi));
            plan(gs(gi + 1) - gs(gi), n16_, hi_);
            meta_load(s0 + gs(gi + T));
            // everything asked for so far has arrived before the loop is entered, so that inside the loop
            // the read-ahead only ever has to wait for loads that were issued a whole group earlier
            __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
            for (; gi < ng; gi += T) {
                if (gi + 2 * T + 1 - gw >= 64) {         // move the table window (runs of more than 60 groups)
                    gw = gi;
                    const int q = gw + lane;
                    gs_win = a.gstart[gb + (q <= ng ? q : ng)];
                }
                int c_row = pf_row, c_info = pf_info;
                float c_val = pf_val;
                const int k = pf_n;                        // entries of this group
                // The lane's coordinates once more, opaque to the compiler: everything derived from them
                // (LDS addresses, offsets) is then recomputed per group with a few instructions instead of
                // being kept in registers across the loop, of which there are not enough.
                int n16 = n16_, hi = hi_, ln = lane;
                __asm__ volatile("" : "+v"(n16), "+v"(hi), "+v"(ln));
                if (!pf_ready) {
                    // some row was not final when it was read ahead: wait for its earlier entries (in stored
                    // order), then read the rows again
                    const uint32_t slot = (uint32_t)c_info & 0xFFFFu, seq = ((uint32_t)c_info >> 16) & 0x7FFFu;
                    const bool waits = ln < k && slot != INFO_SINGLE;
                    __builtin_amdgcn_s_setprio(0);
                    for (uint32_t spins = 0;;) {
                        bool ready = true;
                        if (waits) ready = ticket_read(&ticket[slot]) == seq;
                        if (__ballot(ready) == ~0ull) break;
                        __builtin_amdgcn_s_sleep(2);
                        // every wait ends: the predecessor always makes progress.  Should that ever fail
                        // (corrupt input tables), give up rather than hang the device.
                        if ((++spins & 1023u) == 0 && (spins > (1u << 21) || ticket_read(&give_up) != 0u)) {
                            ticket_write(&give_up, 1u);
                            atomicExch(a.err, PS_ESTALL);
                            break;
                        }
                    }
                    __builtin_amdgcn_s_setprio(2);
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                    gather(n16, hi);                      // same group, rows as they are now
                    // waited for here, on the rare path, so that where the paths join the common one is not
                    // made to wait for everything it has in flight
                    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
                }
                // X: rows 0 .. 14 from the read-ahead (components past the rank are zero) go to the staging
                // area; both dense products read X from there, so the registers of the read-ahead are free
                // again at once
                // (the first product and the inner products with h take them from the registers they are in)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (16 * (NT - 1) + 4 * hi + q >= L) xp[NT - 1][q] = 0.0f;
                if (n16 < 15) {
#pragma unroll
                    for (int j = 0; j < NT; ++j) *reinterpret_cast<f32x4 *>(&stg[n16 * RS + 16 * j + 4 * hi]) = xp[j];
                }
                // ---- <w_s, w_t>: G = X X^T (row 15 of X is an old copy of h here; its products are not used)
                f32x4 gm = {0.0f, 0.0f, 0.0f, 0.0f}, gm2 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const f32x4 xm = xp[j];
                    gm = __builtin_amdgcn_mfma_f32_16x16x4f32(xm[0], xm[0], gm, 0, 0, 0);
                    gm2 = __builtin_amdgcn_mfma_f32_16x16x4f32(xm[1], xm[1], gm2, 0, 0, 0);
                    gm = __builtin_amdgcn_mfma_f32_16x16x4f32(xm[2], xm[2], gm, 0, 0, 0);
                    gm2 = __builtin_amdgcn_mfma_f32_16x16x4f32(xm[3], xm[3], gm2, 0, 0, 0);
                    if (j & 1) __builtin_amdgcn_sched_barrier(0);   // two tiles in flight at most: registers are scarce
                }
                gm = gm + gm2;
                // lane (n16, hi) holds G[4 hi + v][n16] in gm[v].  The solve below needs, in every lane of row t = n16,
                // -(lr / c) G[t][u] for u < t and zero for u >= t: the lane that holds G[u][t] clears what is not below
                // the diagonal before the exchange
                float nl[CH - 1];
                {
                    float gmm[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) gmm[v] = 4 * hi + v < n16 ? gm[v] : 0.0f;
#pragma unroll
                    for (int u = 0; u < CH - 1; ++u) nl[u] = nlrc * bperm_f(gmm[u & 3], 16 * (u >> 2) + n16);
                }

                // v_t of the lane's row t = n16 in all four rows of 16 lanes (the per-entry data sits in lanes 0 .. 14),
                // scaled: v_t c^(-t) = v_t + (c^(-t) - 1) v_t
                const float v_row = bperm_f(c_val, n16);
                float vs = __builtin_fmaf(v_row, cim1[n16], v_row);
                float e_vec = 0.0f;                        // e_t in every lane with n16 == t
                {
                    // table entries for the new h, read before the wait as well
                    float cpm1_k = cpm1[k];
                    float lrck = lr * cpow[k > 0 ? k - 1 : 0];                            // lr c^(k-1): what eps_s w_s weighs in the new h
                    float cpm1_t = cpm1[n16];
                    // (all of this is computed here, ahead of the wait, not where it is first used)
#pragma unroll
                    for (int u = 0; u < CH - 1; ++u) __asm__ volatile("" : "+v"(nl[u]));
                    __asm__ volatile("" : "+v"(vs), "+v"(cpm1_k), "+v"(lrck), "+v"(cpm1_t));
                    // (this lane's quarter of row n16, for the inner products with h below, is xp: still in registers)
                    __builtin_amdgcn_sched_barrier(0);

                    // ---- the part that needs h as the previous group left it --------------------------------
                    f32x4 hq[NT];                          // h in quarters, for p_s = <w_s, h>
                    float ho[NV];                          // h as it is now, lane l its components l, l + 64 (lanes past the row's 16 NT floats: any)
                    int ck[NV];
#pragma unroll
                    for (int cc = 0; cc < NV; ++cc) ck[cc] = ln + 64 * cc < 16 * NT ? ln + 64 * cc : 0;
                    // the rows' components for the new h further down (lane l: components l, l + 64 of every row)
                    float wv[CH][NV];
                    if constexpr (RICH) {
#pragma unroll
                        for (int s = 0; s < CH; ++s)
#pragma unroll
                            for (int cc = 0; cc < NV; ++cc) wv[s][cc] = stg[s * RS + ck[cc]];
#pragma unroll
                        for (int s = 0; s < CH; ++s)
#pragma unroll
                            for (int cc = 0; cc < NV; ++cc) __asm__ volatile("" : "+v"(wv[s][cc]));
                    }
                    for (uint32_t spins = 0; ticket_read(hsq) != (uint32_t)gi;) {
                        if constexpr (!LONG_RUNS) __builtin_amdgcn_s_sleep(1);     // (where runs are very long, the wait is all there is)
                        if ((++spins & 1023u) == 0 && (spins > (1u << 21) || ticket_read(&give_up) != 0u)) {
                            ticket_write(&give_up, 1u);
                            atomicExch(a.err, PS_ESTALL);
                            break;
                        }
                    }
                    compiler_fence();
                    // from here to the hand-over every other wavefront of the team waits for this one
                    __builtin_amdgcn_s_setprio(3);
#pragma unroll
                    for (int j = 0; j < NT; ++j) hq[j] = *reinterpret_cast<const f32x4 *>(&hsh[16 * j + 4 * hi]);
#pragma unroll
                    for (int cc = 0; cc < NV; ++cc) ho[cc] = hsh[ck[cc]];
                    __builtin_amdgcn_sched_barrier(0);      // all of h asked for before the first product waits for its piece
                    float pq[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                    for (int j = 0; j < NT; ++j) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) pq[q] = __builtin_fmaf(xp[j][q], hq[j][q], pq[q]);
                    }
                    // (with fewer registers they are asked for now, so that they arrive while the errors are being computed)
                    if constexpr (!RICH) {
#pragma unroll
                        for (int s = 0; s < CH; ++s)
#pragma unroll
                            for (int cc = 0; cc < NV; ++cc) wv[s][cc] = stg[s * RS + ck[cc]];
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    float p = (pq[0] + pq[1]) + (pq[2] + pq[3]);
                    // the four quarters of a row sit in the same lane of the four rows of 16 lanes: two lane swaps in
                    // the vector unit add them up and leave the sum in all four
                    p = add_across_halves(p);
                    p = add_across_row_pairs(p);
                    // The errors.  With p_s = <w_s, h> for the incoming h, the per-entry recursion e_t = v_t - <w_t, h_(t-1)>
                    // is the lower-triangular system
                    //     e_t = v_t - c^t p_t - sum_(u<t) lr c^(t-1-u) G[t][u] e_u,
                    // and in the scaled unknowns eps_t = e_t c^(-t) its coefficients lose their powers of c:
                    //     eps_t = v_t c^(-t) - p_t - sum_(u<t) (lr / c) G[t][u] eps_u.
                    // Lane (t, any hi) starts with acc = v_t c^(-t) - p_t; step u adds -(lr / c) G[t][u] eps_u, eps_u = acc of lane u
                    // (final after step u - 1) broadcast inside each row of 16 lanes by the multiply-add itself: one
                    // dependent instruction per entry.  The new h = c^k h + lr c^(k-1) sum_s eps_s w_s collects its terms
                    // along the way with the same broadcast.  Steps past the group's end work on rows of X that are
                    // zero and on finite values, so what they compute changes nothing that is used; the chain has no
                    // branches.  Lane 15 (the row of X that holds h) computes something finite that is never used.
                    float acc = vs - p;
                    float hs[NV];
#pragma unroll
                    for (int cc = 0; cc < NV; ++cc) hs[cc] = 0.0f;
                    float hbase[NV];                           // c^k h
#pragma unroll
                    for (int cc = 0; cc < NV; ++cc) hbase[cc] = __builtin_fmaf(cpm1_k, ho[cc], ho[cc]);
                    solve_first();
                    solve_step<0, NV>(acc, hs, wv[0], nl[0]);   solve_step<1, NV>(acc, hs, wv[1], nl[1]);
                    solve_step<2, NV>(acc, hs, wv[2], nl[2]);   solve_step<3, NV>(acc, hs, wv[3], nl[3]);
                    solve_step<4, NV>(acc, hs, wv[4], nl[4]);   solve_step<5, NV>(acc, hs, wv[5], nl[5]);
                    solve_step<6, NV>(acc, hs, wv[6], nl[6]);   solve_step<7, NV>(acc, hs, wv[7], nl[7]);
                    solve_step<8, NV>(acc, hs, wv[8], nl[8]);   solve_step<9, NV>(acc, hs, wv[9], nl[9]);
                    solve_step<10, NV>(acc, hs, wv[10], nl[10]); solve_step<11, NV>(acc, hs, wv[11], nl[11]);
                    solve_step<12, NV>(acc, hs, wv[12], nl[12]); solve_step<13, NV>(acc, hs, wv[13], nl[13]);
                    solve_last<14, NV>(acc, hs, wv[14]);
                    static_assert(CH == 15, "the solve above is written out for 15 entries");
                    float hn[NV];                              // the new h = c^k h + lr c^(k-1) sum_s eps_s w_s
#pragma unroll
                    for (int cc = 0; cc < NV; ++cc) hn[cc] = __builtin_fmaf(lrck, hs[cc], hbase[cc]);
                    // the new h is complete: into LDS for the next group, which may start at once
                    {
#pragma unroll
                        for (int cc = 0; cc < NV; ++cc)
                            if (ln + 64 * cc < L) hsh[ln + 64 * cc] = hn[cc];
                        compiler_fence();
                        ticket_write(hsq, (uint32_t)gi + 1u);
                        compiler_fence();
                        // to memory as the run's last group leaves it (an offset past the end writes nothing)
#pragma unroll
                        for (int cc = 0; cc < NV; ++cc) {
                            const int off = (int)(ln + 64 * cc < L && gi + 1 == ng ? hoff + (uint32_t)(ln + 64 * cc) * 4u : hspan);
                            if constexpr (AGENT_H) __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(hn[cc]), hbuf, off, 0, AUX_SC1);
                            else __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(hn[cc]), hbuf, off, 0, 0);
                        }
                        __builtin_amdgcn_s_setprio(2);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    // e_t = eps_t c^t in every lane with n16 == t, for the new rows below
                    e_vec = __builtin_fmaf(acc, cpm1_t, acc);
                    // this wavefront's copy of h as it was (row 15 of X), for the new rows below
#pragma unroll
                    for (int cc = 0; cc < NV; ++cc)
                        if (ln + 64 * cc < 16 * NT) stg[15 * RS + ln + 64 * cc] = ho[cc];
                }
                // read ahead: the rows of this wavefront's next group, the per-entry data of the one after (not
                // earlier: the registers they arrive in are needed by the part above)
                {
                    const int p1 = gs(gi + T), p2 = gs(gi + T + 1);
                    plan(p2 - p1, n16, hi);
                    meta_load(s0 + gs(gi + 2 * T));
                }

                // ---- the new rows: X' = X + (C - I) X, tile by tile; rows 0 .. k-1 go to the store ----------
                // The product is formed transposed (X'^T = X^T (C - I)^T + X^T), which leaves lane (n16, hi) with
                // components 16 tile + 4 hi .. + 3 of row n16 - the layout the rows were gathered in - so a row
                // goes to the store in 16-byte pieces.  Byte offset of the lane's piece of tile 0 in the block's
                // row factors (past the end for rows without an entry, row 15 among them):
                const uint32_t dst = n16 < k ? (uint32_t)((bperm_i(c_row, n16) - (int)blk_r0) * L + 4 * hi) * 4u : wspan;
                float ca[4];                               // (C - I)[t = n16][s = 4 hi + v]; row 15 is not needed any more
                {
                    // (the exchanges and the table reads all first, then the arithmetic: one wait for LDS, not eight)
                    float es_all[4], cp[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) es_all[v] = bperm_f(e_vec, 4 * hi + v);   // lane s (< 16) holds e_s (all lanes take part in the exchange)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int s = 4 * hi + v, pw = s == 15 ? n16 : n16 - 1 - s;
                        cp[v] = cpow[pw > 0 ? pw : 0];
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int s = 4 * hi + v, t = n16;
                        const float es = s < k ? es_all[v] : 0.0f;
                        // C[t][s<t] = lr^2 e_t e_s c^(t-1-s),  C[t][t] - 1 = -lr lambda,  C[t][15] = lr e_t c^t
                        float x = 0.0f;
                        if (s < t) x = (lr * e_vec) * (lr * es) * cp[v];
                        if (s == t) x = -delta;
                        if (s == 15) x = lr * e_vec * cp[v];
                        ca[v] = t < 15 ? x : 0.0f;
                    }
                }
                // all of X is asked for (both layouts) before the first product waits for its operands: a tile's
                // four matrix instructions depend on each other, and seven trips to LDS in between would double
                // the time of this part
                float xn[NT][4];
                f32x4 xa[NT];
#pragma unroll
                for (int tile = 0; tile < NT; ++tile) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) xn[tile][v] = stg[(4 * hi + v) * RS + 16 * tile + n16];
                    xa[tile] = *reinterpret_cast<const f32x4 *>(&stg[n16 * RS + 16 * tile + 4 * hi]);   // the X of X + (C - I) X
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int tile = 0; tile < NT; ++tile) {
                    f32x4 acc = xa[tile];
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(xn[tile][v], ca[v], acc, 0, 0, 0);
                    if constexpr (A4) {
                        const bool comp = tile < NT - 1 || 16 * tile + 4 * hi < L;    // the piece exists (the rank is a multiple of 4)
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc), wbuf, (int)(comp ? dst : wspan) + 64 * tile, 0, 0);
                    } else {
                        // (element by element into scalars first: a bit cast applied to a vector element directly
                        // has been seen to pick element 0 every time)
                        const float r0 = acc[0], r1 = acc[1], r2 = acc[2], r3 = acc[3];
                        const float rr[4] = {r0, r1, r2, r3};
                        if (even_rank) {
#pragma unroll
                            for (int q = 0; q < 4; q += 2) {
                                const u32x2 pr = {__float_as_uint(rr[q]), __float_as_uint(rr[q + 1])};
                                __builtin_amdgcn_raw_buffer_store_b64(pr, wbuf, (int)(16 * tile + 4 * hi + q < L ? dst : wspan) + 64 * tile + 4 * q, 0, 0);
                            }
                        } else {
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(rr[q]), wbuf,
                                                                      (int)(16 * tile + 4 * hi + q < L ? dst : wspan) + 64 * tile + 4 * q, 0, 0);
                        }
                    }
                }
                // ---- hand the rows on: the stores must have completed before the tickets move ---------
                {
                    const uint32_t slot = (uint32_t)c_info & 0xFFFFu, seq = ((uint32_t)c_info >> 16) & 0x7FFFu;
                    const bool bump = ln < k && slot != INFO_SINGLE && slot != INFO_NONE;
                    if (__ballot(bump) != 0) {
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                        if (bump) ticket_write(&ticket[slot], seq + 1u);
                    }
                }
                done += (unsigned int)k;
            }
        }
    }

    // ---- part 2: the other runs, row by row ---------------------------------------------
    // A wavefront takes the next D consecutive row runs, waits until the heavy runs have passed these
    // rows, reads their entries and factors in one go, and then keeps going round its rows: whichever
    // row's next entry is the next of its column (by the column's ticket) is processed, the others are
    // looked at again in the next round.  Batches are taken in ascending order and no wavefront ever
    // waits for one particular entry, so the lowest unfinished entry of the block is always processed
    // in its wavefront's next round: every wait ends.
    __builtin_amdgcn_s_setprio(1);
    if constexpr (!LONG_RUNS) {
        if (tr1 > tr0) {
            constexpr int D = 4;
            const int ntrow = (int)(tr1 - tr0);
            for (;;) {
                int jb = 0;
                if (lane == 0) jb = atomicAdd(&next_trow, D);
                jb = __builtin_amdgcn_readfirstlane(jb);
                if (jb >= ntrow) break;
                // lane i < D: row run jb + i
                int r_row = -1;
                uint32_t r_e0 = 0, r_e1 = 0, r_wait = 0xFFFFFFFFu;
                if (lane < D && jb + lane < ntrow) {
                    r_row = a.trun_row[tr0 + jb + lane]; r_e0 = a.trun_start[tr0 + jb + lane]; r_e1 = a.trun_start[tr0 + jb + lane + 1];
                    r_wait = a.trun_wait[tr0 + jb + lane];
                }
                // entries of every row (one per lane) and its factor, once the row's entries in heavy runs are done
                float w[D][NV], ev[D];
                uint32_t ci[D], pos[D], wb[D];
                uint32_t pend = 0;
                bool stalled = false;
#pragma unroll
                for (int i = 0; i < D; ++i) {
                    const int row = rl_i(r_row, i);
                    const uint32_t e0 = (uint32_t)rl_i((int)r_e0, i), e1 = (uint32_t)rl_i((int)r_e1, i);
                    const uint32_t wt = (uint32_t)rl_i((int)r_wait, i);
                    ci[i] = 0; ev[i] = 0.0f; pos[i] = e0; wb[i] = e0;
#pragma unroll
                    for (int cc = 0; cc < NV; ++cc) w[i][cc] = 0.0f;
                    if (e0 + lane < e1) { ci[i] = a.t_cinfo[e0 + lane]; ev[i] = a.t_val[e0 + lane]; }
                    if (row >= 0 && !stalled) {
                        if (wt != 0xFFFFFFFFu) {
                            uint32_t *tk = &ticket[wt & 0xFFFFu];
                            __builtin_amdgcn_s_setprio(0);
                            for (uint32_t spins = 0; ticket_read(tk) != (wt >> 16);) {
                                __builtin_amdgcn_s_sleep(4);
                                if ((++spins & 1023u) == 0 && (spins > (1u << 21) || ticket_read(&give_up) != 0u)) {
                                    ticket_write(&give_up, 1u);
                                    atomicExch(a.err, PS_ESTALL);
                                    stalled = true;
                                    break;
                                }
                            }
                            __builtin_amdgcn_s_setprio(1);
                        }
                        if (!stalled) {
                            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                            load_row_t<NV>(a.val + (int64_t)row * L, lane, tail, w[i]);
                            pend |= 1u << i;
                        }
                    }
                }
                // rounds over the rows that still have entries; lane i holds the next entry of row i
                uint32_t cur_ci = 0;
#pragma unroll
                for (int i = 0; i < D; ++i) {
                    const uint32_t first = (uint32_t)rl_i((int)ci[i], 0);
                    cur_ci = lane == i ? first : cur_ci;
                }
                uint32_t idle_rounds = 0;
                while (pend != 0) {
                    // lane i looks at the ticket of the column of row i's next entry
                    uint32_t tkv = 0;
                    if (lane < D) tkv = ticket_read(&ctick[cur_ci & 0xFFFFu]);
                    const uint32_t ready = (uint32_t)__ballot(lane < D && ((pend >> lane) & 1u) != 0u && tkv == ((cur_ci >> 16) & 0x7FFFu));
                    const bool any = ready != 0u;
#pragma unroll
                    for (int i = 0; i < D; ++i) {
                        if (!((ready >> i) & 1u)) continue;         // done, or the column's earlier entries first
                        const uint32_t cinfo = (uint32_t)rl_i((int)cur_ci, i);
                        const uint32_t slot = cinfo & 0xFFFFu, seq = (cinfo >> 16) & 0x7FFFu;
                        const float v = rl_f(ev[i], (int)(pos[i] - wb[i]));
                        const uint32_t e1 = (uint32_t)rl_i((int)r_e1, i);
                        uint32_t *tk = &ctick[slot];
                        compiler_fence();
                        // one step on the row's factor (registers) and the column's factor h
                        auto step = [&](float (&h)[NV]) {
                            float pr = 0.0f;
#pragma unroll
                            for (int cc = 0; cc < NV; ++cc) pr = __builtin_fmaf(w[i][cc], h[cc], pr);
                            const float e = v - wave_sum(pr);
#pragma unroll
                            for (int cc = 0; cc < NV; ++cc) {
                                const float wo = w[i][cc], ho = h[cc];
                                w[i][cc] = __builtin_fmaf(lr, __builtin_fmaf(e, ho, -(lambda * wo)), wo);
                                h[cc] = __builtin_fmaf(lr, __builtin_fmaf(e, wo, -(lambda * ho)), ho);
                            }
                        };
                        float h[NV];
                        if (slot < (uint32_t)ncached) {            // the column's factor lives in LDS
                            float *hl = hcache + (size_t)slot * L;
                            load_row_t<NV>(hl, lane, tail, h);
                            step(h);
                            store_row_t<NV>(hl, lane, tail, h);
                            compiler_fence();
                        } else {                                   // did not fit: handed over through memory
                            float *hg = a.val + (a.m + a.run_col[run0 + nheavy + slot]) * (int64_t)L;
                            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                            load_row_t<NV, AGENT_H>(hg, lane, tail, h);
                            step(h);
                            store_row_t<NV, AGENT_H>(hg, lane, tail, h);
                            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                        }
                        ticket_write(tk, seq + 1u);
                        ++pos[i];
                        ++done;
                        if (pos[i] == e1) {
                            store_row_t<NV>(a.val + (int64_t)rl_i(r_row, i) * L, lane, tail, w[i]);
                            pend &= ~(1u << i);
                        } else {
                            if (pos[i] - wb[i] >= 64u) {       // a row with more than 64 entries here: next 64
                                wb[i] = pos[i];
                                ci[i] = 0; ev[i] = 0.0f;
                                if (wb[i] + lane < e1) { ci[i] = a.t_cinfo[wb[i] + lane]; ev[i] = a.t_val[wb[i] + lane]; }
                            }
                            const uint32_t nx = (uint32_t)rl_i((int)ci[i], (int)(pos[i] - wb[i]));
                            cur_ci = lane == i ? nx : cur_ci;
                        }
                    }
                    if (any) {
                        idle_rounds = 0;
                    } else {
                        __builtin_amdgcn_s_sleep(1);
                        if ((++idle_rounds & 1023u) == 0 && (idle_rounds > (1u << 21) || ticket_read(&give_up) != 0u)) {
                            ticket_write(&give_up, 1u);
                            atomicExch(a.err, PS_ESTALL);
                            break;
                        }
                    }
                }
                if (stalled) break;
            }
        }
    } else {
        // The same for data whose rows mostly have a single entry in a block.  What counts there is the number of
        // trips to memory a wavefront makes one after the other, so: batches of 8 rows; a row run's record holds its
        // first entry, and the records of the next batch are read while the current one is worked on; the column
        // factor of a first entry that is also its column's first entry in the block (nobody writes it before) is asked
        // for together with the row's factor; the rows of a round whose column factors are in memory are taken together
        // (loads, steps, stores); and a column's last entry in the block leaves no ticket and waits for no store.
        if (tr1 > tr0) {
            constexpr int D = 8;
            const int ntrow = (int)(tr1 - tr0);
            int n_jb = 0, n_row = -1, n_col = 0;
            uint32_t n_e0 = 0, n_e1 = 0, n_wait = 0xFFFFFFFFu, n_ci = 0;
            float n_val = 0.0f;
            auto claim = [&]() {                                 // takes the next batch; lane i < D: the record of row run n_jb + i
                int j = 0;
                if (lane == 0) j = atomicAdd(&next_trow, D);
                n_jb = __builtin_amdgcn_readfirstlane(j);
                n_row = -1; n_col = 0; n_e0 = 0; n_e1 = 0; n_wait = 0xFFFFFFFFu; n_ci = 0; n_val = 0.0f;
                if (lane < D && n_jb + lane < ntrow) {
                    const int64_t q = tr0 + n_jb + lane;
                    n_row = a.trun_row[q]; n_e0 = a.trun_start[q]; n_e1 = a.trun_start[q + 1]; n_wait = a.trun_wait[q];
                    n_ci = a.trun_ci[q]; n_val = a.trun_val[q]; n_col = a.trun_col[q];
                }
            };
            claim();
            __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0)
            bool stalled = false;
            while (n_jb < ntrow && !stalled) {
                const int r_row = n_row, f_col = n_col;
                const uint32_t r_e0 = n_e0, r_e1 = n_e1, r_wait = n_wait, f_ci = n_ci;
                const float f_val = n_val;
                claim();
                // the rows' factors once the heavy runs have passed them, the column factors that can be asked for
                // already, and the entries of rows that have more than one
                float w[D][NV], hc[D][NV], ev[D];
                uint32_t ci[D], pos[D], wb[D];
                uint32_t pend = 0, spec = 0, first = 0;
#pragma unroll
                for (int i = 0; i < D; ++i) {
                    const int row = rl_i(r_row, i);
                    const uint32_t e0 = (uint32_t)rl_i((int)r_e0, i), e1 = (uint32_t)rl_i((int)r_e1, i);
                    const uint32_t wt = (uint32_t)rl_i((int)r_wait, i);
                    ci[i] = 0; ev[i] = 0.0f; pos[i] = e0; wb[i] = e0;
#pragma unroll
                    for (int cc = 0; cc < NV; ++cc) { w[i][cc] = 0.0f; hc[i][cc] = 0.0f; }
                    if (row < 0 || stalled) continue;
                    if (wt != 0xFFFFFFFFu) {
                        uint32_t *tk = &ticket[wt & 0xFFFFu];
                        __builtin_amdgcn_s_setprio(0);
                        for (uint32_t spins = 0; ticket_read(tk) != (wt >> 16);) {
                            __builtin_amdgcn_s_sleep(4);
                            if ((++spins & 1023u) == 0 && (spins > (1u << 21) || ticket_read(&give_up) != 0u)) {
                                ticket_write(&give_up, 1u);
                                atomicExch(a.err, PS_ESTALL);
                                stalled = true;
                                break;
                            }
                        }
                        __builtin_amdgcn_s_setprio(1);
                        if (stalled) continue;
                    }
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                    load_row_t<NV>(a.val + (int64_t)row * L, lane, tail, w[i]);
                    pend |= 1u << i;
                    first |= 1u << i;
                    const uint32_t fci = (uint32_t)rl_i((int)f_ci, i);
                    if ((fci & 0xFFFFu) >= (uint32_t)ncached && ((fci >> 16) & 0x7FFFu) == 0u) {
                        load_row_t<NV, AGENT_H>(a.val + (a.m + rl_i(f_col, i)) * (int64_t)L, lane, tail, hc[i]);
                        spec |= 1u << i;
                    }
                    if (e1 - e0 > 1u && e0 + lane < e1) { ci[i] = a.t_cinfo[e0 + lane]; ev[i] = a.t_val[e0 + lane]; }
                }
                // Everything asked for so far is waited for here, once: the counter of outstanding memory operations
                // also counts stores, and a wait placed inside the rounds would wait for those in every round.
                __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
                uint32_t cur_ci = f_ci;                       // lane i: the next entry of row i
                uint32_t idle_rounds = 0;
                while (pend != 0) {
                    uint32_t tkv = 0;
                    if (lane < D) tkv = ticket_read(&ctick[cur_ci & 0xFFFFu]);
                    const uint32_t ready = (uint32_t)__ballot(lane < D && ((pend >> lane) & 1u) != 0u && tkv == ((cur_ci >> 16) & 0x7FFFu));
                    if (ready == 0u) {
                        __builtin_amdgcn_s_sleep(1);
                        if ((++idle_rounds & 1023u) == 0 && (idle_rounds > (1u << 21) || ticket_read(&give_up) != 0u)) {
                            ticket_write(&give_up, 1u);
                            atomicExch(a.err, PS_ESTALL);
                            stalled = true;
                            break;
                        }
                        continue;
                    }
                    idle_rounds = 0;
                    compiler_fence();
                    // what a row's entry leaves behind: its place in the row, the row's factor after its last entry
                    auto advance = [&](int i) {
                        const uint32_t e1 = (uint32_t)rl_i((int)r_e1, i);
                        ++pos[i];
                        ++done;
                        first &= ~(1u << i);
                        spec &= ~(1u << i);
                        if (pos[i] == e1) {
                            store_row_t<NV>(a.val + (int64_t)rl_i(r_row, i) * L, lane, tail, w[i]);
                            pend &= ~(1u << i);
                        } else {
                            if (pos[i] - wb[i] >= 64u) {       // a row with more than 64 entries here: next 64
                                wb[i] = pos[i];
                                ci[i] = 0; ev[i] = 0.0f;
                                if (wb[i] + lane < e1) { ci[i] = a.t_cinfo[wb[i] + lane]; ev[i] = a.t_val[wb[i] + lane]; }
                                __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0): see above
                            }
                            const uint32_t nx = (uint32_t)rl_i((int)ci[i], (int)(pos[i] - wb[i]));
                            cur_ci = lane == i ? nx : cur_ci;
                        }
                    };
                    // one step on row i's factor (registers) and the column's factor h
                    auto step = [&](int i, float (&h)[NV]) {
                        const float v = (first >> i) & 1u ? rl_f(f_val, i) : rl_f(ev[i], (int)(pos[i] - wb[i]));
                        float pr = 0.0f;
#pragma unroll
                        for (int cc = 0; cc < NV; ++cc) pr = __builtin_fmaf(w[i][cc], h[cc], pr);
                        const float e = v - wave_sum(pr);
#pragma unroll
                        for (int cc = 0; cc < NV; ++cc) {
                            const float wo = w[i][cc], ho = h[cc];
                            w[i][cc] = __builtin_fmaf(lr, __builtin_fmaf(e, ho, -(lambda * wo)), wo);
                            h[cc] = __builtin_fmaf(lr, __builtin_fmaf(e, wo, -(lambda * ho)), ho);
                        }
                    };
                    const uint32_t slot_v = cur_ci & 0xFFFFu;
                    // rows whose column factor did not fit in LDS: it is handed over through memory
                    const uint32_t in_mem = ready & (uint32_t)__ballot(lane < D && slot_v >= (uint32_t)ncached);
                    // the columns that live in LDS, one after the other; each is handed on at once
#pragma unroll
                    for (int i = 0; i < D; ++i) {
                        if (!(((ready & ~in_mem) >> i) & 1u)) continue;
                        const uint32_t cinfo = (uint32_t)rl_i((int)cur_ci, i);
                        float *hl = hcache + (size_t)(cinfo & 0xFFFFu) * L;
                        float h[NV];
                        load_row_t<NV>(hl, lane, tail, h);
                        step(i, h);
                        store_row_t<NV>(hl, lane, tail, h);
                        compiler_fence();
                        ticket_write(&ctick[cinfo & 0xFFFFu], ((cinfo >> 16) & 0x7FFFu) + 1u);
                        advance(i);
                    }
                    if (in_mem != 0u) {
                        const uint32_t old_ci = cur_ci;
                        // A column's first entry in the block finds its factor as the last launch left it, and after
                        // its last entry nobody in this block looks at the factor or its ticket again: the fences and
                        // the ticket are for the entries in between (a column with one entry needs neither).
                        const uint32_t to_load = in_mem & ~spec;
                        const uint32_t not_first = to_load & (uint32_t)__ballot(lane < D && ((cur_ci >> 16) & 0x7FFFu) != 0u);
                        const uint32_t not_last = in_mem & (uint32_t)__ballot(lane < D && (cur_ci >> 31) == 0u);
                        // the columns: of a row's first entry from its record, of later entries looked up
                        int32_t colv = f_col;
                        if (lane < D && ((in_mem & ~first) >> lane) & 1u) colv = a.run_col[run0 + nheavy + slot_v];
                        if (not_first != 0u) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                        int32_t col[D];
#pragma unroll
                        for (int i = 0; i < D; ++i) {
                            col[i] = 0;
                            if (!((in_mem >> i) & 1u)) continue;
                            col[i] = rl_i(colv, i);
                            if ((to_load >> i) & 1u) load_row_t<NV, AGENT_H>(a.val + (a.m + col[i]) * (int64_t)L, lane, tail, hc[i]);
                        }
#pragma unroll
                        for (int i = 0; i < D; ++i)
                            if ((in_mem >> i) & 1u) step(i, hc[i]);
#pragma unroll
                        for (int i = 0; i < D; ++i)
                            if ((in_mem >> i) & 1u) store_row_t<NV, AGENT_H>(a.val + (a.m + col[i]) * (int64_t)L, lane, tail, hc[i]);
                        compiler_fence();
                        if (not_last != 0u) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
#pragma unroll
                        for (int i = 0; i < D; ++i) {
                            if (!((in_mem >> i) & 1u)) continue;
                            const uint32_t cinfo = (uint32_t)rl_i((int)old_ci, i);
                            if ((not_last >> i) & 1u) ticket_write(&ctick[cinfo & 0xFFFFu], ((cinfo >> 16) & 0x7FFFu) + 1u);
                            advance(i);
                        }
                    }
                }
            }
        }
    }
    __builtin_amdgcn_s_setprio(0);
    if (lane == 0 && done) atomicAdd(&done_entries, done);
    __syncthreads();
    // write the cached column factors back
    {
        const int total = ncached * L;
#pragma unroll 4
        for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
            const int s = idx / L;
            store_f<AGENT_H>(&a.val[(a.m + a.run_col[run0 + nheavy + s]) * (int64_t)L + (idx - s * L)], hcache[idx]);
        }
    }
    // each entry was one pull and one push of two local keys
    if (threadIdx.x == 0 && done_entries) {
        u64 *st = stat_slot(a.stats);
        atomicAdd(&st[PS_STAT_PULL_LOCAL], 2 * (u64)done_entries);
        atomicAdd(&st[PS_STAT_PUSH_LOCAL], 2 * (u64)done_entries);
    }
}

// One workgroup per task of a stratum.
// MAXT: the largest workgroup the kernel is compiled for (12 wavefronts leave each of them a third more registers
// than 16 do, which the first part needs)
template <int NT, bool A4, int MAXT, bool LONG_RUNS>
__global__ __launch_bounds__(MAXT) void k_mf_sgd_chunk(SgdArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    sgd_block<NT, A4, false, LONG_RUNS, MAXT <= 768>(a, lds_f, a.tasks[3 * blockIdx.x], a.tasks[3 * blockIdx.x + 1], a.tasks[3 * blockIdx.x + 2]);
}

// ---- an epoch without barriers: column blocks handed from worker to worker ----------------------------------
// (the asynchronous form of the blocked schedule - NOMAD, which Sec. 2.2.2 lists among the algorithms that move
// parameters to where the data is; the move is a localize, Sec. 2.3.)  Workgroup w is worker w and keeps row block
// w for the whole epoch.  A column block is either free or held by one worker; state word c = visits << 1 | held.
// A worker that has finished a block gives its column block back and takes another: the first one, in cyclic
// order after the one it just had, that is free and that it has not had in this epoch.  It never waits while it
// holds a block, so every wait ends.  Which order results depends on timing; it is written down (sched) so that
// the epoch can be replayed.

// Wavefront 0 of the workgroup: take a column block; returns it (and how many workers had it before), or -1 when
// an error is pending or the wait ran out.
__device__ __forceinline__ int handoff_take(const SgdArgs &a, const uint32_t *todo, int start, int &visit) {
    const int lane = threadIdx.x, d_col = a.d_col;
    if (rl_i(__hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), 0) != 0) return -1;
    for (uint32_t spins = 1;; ++spins) {
        for (int base = 0; base < d_col; base += 64) {
            int c = start + base + lane;
            c = c >= d_col ? c - d_col : c;
            uint32_t sv = 1u;
            if (base + lane < d_col && ((todo[c >> 5] >> (c & 31)) & 1u)) sv = __hip_atomic_load(&a.col_state[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            unsigned long long free_mask = __ballot((sv & 1u) == 0u);
            while (free_mask) {
                const int l = __ffsll((long long)free_mask) - 1;
                free_mask &= free_mask - 1;
                const int cc = rl_i(c, l);
                const uint32_t expect = (uint32_t)rl_i((int)sv, l);
                int won = 0;
                if (lane == 0) won = atomicCAS(&a.col_state[cc], expect, expect | 1u) == expect ? 1 : 0;
                if (rl_i(won, 0)) { visit = (int)(expect >> 1); return cc; }
            }
        }
        __builtin_amdgcn_s_sleep(8);
        if ((spins & 63u) == 0u) {
            if (rl_i(__hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), 0) != 0) return -1;
            if (spins > a.take_spins) { atomicExch(a.err, PS_ESTALL); return -1; }
        }
    }
}

template <int NT, bool A4, bool LONG_RUNS>
__global__ __launch_bounds__(1024) void k_mf_sgd_handoff(SgdArgs a) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    __shared__ uint32_t todo[DPAPS_HANDOFF_MAX_COLS / 32];
    __shared__ int s_cb, s_visit;
    const int32_t worker = blockIdx.x;
    const int d_col = a.d_col;
    for (int i = threadIdx.x; i < DPAPS_HANDOFF_MAX_COLS / 32; i += blockDim.x) {
        const int left = d_col - 32 * i;
        todo[i] = left >= 32 ? 0xFFFFFFFFu : (left > 0 ? (1u << left) - 1u : 0u);
    }
    __syncthreads();
    int start = (int)((int64_t)worker * d_col / gridDim.x);       // the workers start spread over the column blocks
    for (int step = 0; step < d_col; ++step) {
        if (threadIdx.x < 64) {
            int visit = 0;
            const int got = handoff_take(a, todo, start, visit);
            if (threadIdx.x == 0) {
                s_cb = got; s_visit = visit;
                if (got >= 0) {
                    todo[got >> 5] &= ~(1u << (got & 31));
                    a.sched[2 * ((int64_t)worker * d_col + step)] = got;
                    a.sched[2 * ((int64_t)worker * d_col + step) + 1] = visit;
                }
            }
        }
        __syncthreads();
        const int cb = __builtin_amdgcn_readfirstlane(s_cb);          // the same in all lanes: block addresses stay scalar
        const int visit = __builtin_amdgcn_readfirstlane(s_visit);
        if (cb < 0) break;
        sgd_block<NT, A4, true, LONG_RUNS>(a, lds_f, worker, worker, cb);
        // every store of this wavefront has reached memory before the barrier, every wavefront's before the release
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (threadIdx.x == 0) __hip_atomic_store(&a.col_state[cb], ((uint32_t)visit + 1u) << 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        start = cb + 1 < d_col ? cb + 1 : 0;
    }
}

// Which variant of the kernels the loaded data gets (LONG_RUNS): a column run of very many groups in some block, or
// rows that mostly have a single entry per block - there the second part is bound by trips to memory, not by
// the order of a row's entries.
static bool dpaps_wide_like(const MfData &f) {
    return f.max_run_groups >= DPAPS_LONG_RUN_GROUPS || (f.num_truns > 0 && 2 * f.num_tail < 3 * f.num_truns);
}

// Wavefronts per workgroup of the SGD kernels: what PS_OPT_MF_WAVES says, else 16 - or 12 where the grouped kernel
// runs on data of that kind: its second part has little to wait for there, and with 12 wavefronts each has a third
// more registers, which the first part uses to read ahead of its wait for the column's factor (measured on the
// 10M x 1M configuration: 2 % less time per launch than with 16).
int dpaps_mf_waves(const dpaps_ps *ps) {
    if (ps->opt_waves > 0) return ps->opt_waves;
    const bool grouped = !ps->opt_classic && ps->opt_grouped && !ps->opt_exact && ps->L <= 128 && ps->mf.sweep_ok;
    return grouped && dpaps_wide_like(ps->mf) ? 12 : 16;
}

// LDS plan of sgd_block: staging areas, tables and the heavy columns' factors, the two kinds of ticket counters,
// then as many other column factors as fit.  Fills in a.ctick_cap, a.hcache_cap.
template <int NT>
static int plan_block_lds(dpaps_ps *ps, SgdArgs &a, size_t *lds_out) {
    const MfData &f = ps->mf;
    const int L = a.L;
    // the kernel addresses the factors of a block's rows, and of its columns, with 32-bit byte offsets
    if ((int64_t)f.max_block_rows * L * 4 >= ((int64_t)1 << 31) - 4096 || (int64_t)f.max_block_cols * L * 4 >= ((int64_t)1 << 31) - 4096) {
        ps->last_error = "a block's factors span 2 GiB or more: use the entry-by-entry kernel (PS_OPT_MF_GROUPED 0)";
        return PS_ELIMIT;
    }
    if (!f.sweep_ok) { ps->last_error = "the grouped SGD kernel needs rows in ascending order inside the short column runs"; return PS_ELAYOUT; }
    a.ctick_cap = f.max_tail_cols > 1 ? f.max_tail_cols : 1;
    const int64_t fixed = ((int64_t)a.heavy_waves * 16 * (16 * NT + 4) + 60 + DPAPS_HEAVY_MAX * 16 * NT + DPAPS_HEAVY_MAX) * 4 +
                          ((int64_t)a.ticket_cap + a.ctick_cap) * 4;
    const int64_t budget = (int64_t)ps->lds_bytes - 1024;         // static LDS and slack
    if (fixed > budget) { ps->last_error = "not enough LDS for the grouped SGD kernel"; return PS_ELIMIT; }
    int64_t hcap = (budget - fixed) / ((int64_t)L * 4);
    if (hcap > f.max_tail_cols) hcap = f.max_tail_cols;
    if (ps->opt_cache_rows >= 0 && hcap > ps->opt_cache_rows) hcap = ps->opt_cache_rows;
    a.hcache_cap = (int32_t)hcap;
    *lds_out = (size_t)(fixed + hcap * L * 4);
    return PS_OK;
}

template <int NT, bool A4, int MAXT, bool LONG_RUNS>
static int launch_chunk_t(dpaps_ps *ps, SgdArgs a, int ntasks, int waves, hipStream_t st) {
    size_t lds = 0;
    const int rc = plan_block_lds<NT>(ps, a, &lds);
    if (rc) return rc;
    static size_t configured = 0;
    if (lds > configured) {
        PS_HIP(ps, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mf_sgd_chunk<NT, A4, MAXT, LONG_RUNS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        configured = lds;
    }
    k_mf_sgd_chunk<NT, A4, MAXT, LONG_RUNS><<<ntasks, 64 * waves, lds, st>>>(a);
    PS_HIP(ps, hipGetLastError());
    return PS_OK;
}

template <int NT, bool A4>
static int launch_chunk(dpaps_ps *ps, SgdArgs a, int ntasks, int waves, hipStream_t st) {
    if (dpaps_wide_like(ps->mf))
        return waves <= 12 ? launch_chunk_t<NT, A4, 768, true>(ps, a, ntasks, waves, st) : launch_chunk_t<NT, A4, 1024, true>(ps, a, ntasks, waves, st);
    return waves <= 12 ? launch_chunk_t<NT, A4, 768, false>(ps, a, ntasks, waves, st) : launch_chunk_t<NT, A4, 1024, false>(ps, a, ntasks, waves, st);
}

// The plan of a block: word w of its 16 = run_first | run_last << 8 | T << 16 | mb << 24 for heavy wavefront w
// (T = 0, no runs: the wavefront goes straight to the second part).  Every heavy run gets a wavefront of its
// own, so that all runs advance side by side (the last groups of consecutive runs tend to wait for each
// other, and a run that started late would make everything after it late).  The wavefronts that are left
// join the runs one by one, each time the run with the most groups per wavefront, up to tmax per run.
__global__ void k_team_plan(const int64_t *blk_run_ptr, const int32_t *blk_nheavy, const int64_t *run_gptr, int64_t nb, int H, int tmax,
                            uint32_t *plan) {
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= nb) return;
    const int64_t run0 = blk_run_ptr[b];
    int nh = blk_nheavy[b] < DPAPS_HEAVY_MAX ? blk_nheavy[b] : DPAPS_HEAVY_MAX;
    if (nh > H) nh = H;
    int g[DPAPS_HEAVY_MAX], T[DPAPS_HEAVY_MAX];
    for (int i = 0; i < nh; ++i) {
        g[i] = (int)(run_gptr[run0 + i + 1] - run_gptr[run0 + i]) - 1;
        T[i] = 1;
    }
    for (int left = H - nh; left > 0 && nh > 0; --left) {
        int best = -1;
        for (int i = 0; i < nh; ++i)
            if (T[i] < tmax && g[i] > T[i] && (best < 0 || (int64_t)g[i] * T[best] > (int64_t)g[best] * T[i])) best = i;
        if (best < 0) break;
        ++T[best];
    }
    int w = 0;
    for (int i = 0; i < nh; ++i)
        for (int q = 0; q < T[i]; ++q, ++w) plan[b * 16 + w] = (uint32_t)i | (uint32_t)(i + 1) << 8 | (uint32_t)T[i] << 16 | (uint32_t)q << 24;
    for (; w < 16; ++w) plan[b * 16 + w] = 0;
}

template <int NT, bool A4, bool LONG_RUNS>
static int launch_handoff_t(dpaps_ps *ps, SgdArgs a, int workers, hipStream_t st) {
    size_t lds = 0;
    const int rc = plan_block_lds<NT>(ps, a, &lds);
    if (rc) return rc;
    static size_t configured = 0;
    if (lds > configured) {
        PS_HIP(ps, hipFuncSetAttribute(reinterpret_cast<const void *>(&k_mf_sgd_handoff<NT, A4, LONG_RUNS>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds));
        configured = lds;
    }
    k_mf_sgd_handoff<NT, A4, LONG_RUNS><<<workers, 1024, lds, st>>>(a);
    PS_HIP(ps, hipGetLastError());
    return PS_OK;
}

template <int NT, bool A4>
static int launch_handoff(dpaps_ps *ps, SgdArgs a, int workers, hipStream_t st) {
    return dpaps_wide_like(ps->mf) ? launch_handoff_t<NT, A4, true>(ps, a, workers, st)
                                                          : launch_handoff_t<NT, A4, false>(ps, a, workers, st);
}

// how the wavefronts of a workgroup share the heavy runs: with 12 or more wavefronts, 12 (14 of 16) of them take
// heavy runs as the block's plan says; else at most one per heavy run
static int plan_teams(dpaps_ps *ps, SgdArgs &a, int waves, hipStream_t st) {
    a.team = waves >= 12 ? 2 : 1;
    a.heavy_waves = waves >= 16 ? 14 : (waves >= 12 ? 12 : (waves < DPAPS_HEAVY_MAX ? waves : DPAPS_HEAVY_MAX));
    a.team_plan = nullptr;
    if (a.team == 2) {
        MfData &f = ps->mf;
        // Most wavefronts per run: what PS_OPT_MF_TEAM_MAX says, else one per vector unit - or two where runs are
        // very long and the workgroup has 12 wavefronts: a wavefront then has the registers to overlap its own
        // work with its neighbour's, and a run of a thousand groups is all its block has (measured on the
        // 10M x 1M configuration: 4 % less time per launch than with 4, while 6 is no better than 4).
        const int tmax = ps->opt_team_max > 0 ? ps->opt_team_max : (dpaps_wide_like(f) && waves <= 12 ? 8 : 4);
        if (!f.team_plan) PS_HIP(ps, hipMalloc(&f.team_plan, (size_t)f.num_blocks * 16 * sizeof(uint32_t)));
        if (f.team_plan_waves != a.heavy_waves * 100 + tmax) {
            k_team_plan<<<(unsigned)((f.num_blocks + 255) / 256), 256, 0, st>>>(f.blk_run_ptr, f.blk_nheavy, f.run_gptr, f.num_blocks, a.heavy_waves,
                                                                               tmax, f.team_plan);
            PS_HIP(ps, hipGetLastError());
            f.team_plan_waves = a.heavy_waves * 100 + tmax;
        }
        a.team_plan = f.team_plan;
    }
    return PS_OK;
}

// One launch for a whole epoch: `workers` workgroups of 16 wavefronts, worker w on row block w (see k_mf_sgd_handoff).
int dpaps_launch_sgd_handoff(dpaps_ps *ps, const SgdArgs &a_in, int workers, hipStream_t st) {
    SgdArgs a = a_in;
    // A worker without a block looks again about every microsecond.  While it waits, the blocks it still needs are
    // being worked on by others, and in the worst case it is the last to get each of them: the bound on its looks
    // covers the whole epoch at a generous microsecond per entry (2 million looks at least) - it is there for
    // inconsistent tables, not to time out a slow epoch.
    const int64_t looks = std::max<int64_t>((int64_t)1 << 21, 8 * ps->mf.nnz);
    a.take_spins = (uint32_t)std::min<int64_t>(looks, 0x7FFFFFFF);
    const int rc = plan_teams(ps, a, 16, st);
    if (rc) return rc;
    switch ((a.L + 15) / 16) {
    case 1: return a.L % 4 == 0 ? launch_handoff<1, true>(ps, a, workers, st) : launch_handoff<1, false>(ps, a, workers, st);
    case 2: return a.L % 4 == 0 ? launch_handoff<2, true>(ps, a, workers, st) : launch_handoff<2, false>(ps, a, workers, st);
    case 3: return a.L % 4 == 0 ? launch_handoff<3, true>(ps, a, workers, st) : launch_handoff<3, false>(ps, a, workers, st);
    case 4: return a.L % 4 == 0 ? launch_handoff<4, true>(ps, a, workers, st) : launch_handoff<4, false>(ps, a, workers, st);
    case 5: return a.L % 4 == 0 ? launch_handoff<5, true>(ps, a, workers, st) : launch_handoff<5, false>(ps, a, workers, st);
    case 6: return a.L % 4 == 0 ? launch_handoff<6, true>(ps, a, workers, st) : launch_handoff<6, false>(ps, a, workers, st);
    case 7: return a.L % 4 == 0 ? launch_handoff<7, true>(ps, a, workers, st) : launch_handoff<7, false>(ps, a, workers, st);
    case 8: return a.L % 4 == 0 ? launch_handoff<8, true>(ps, a, workers, st) : launch_handoff<8, false>(ps, a, workers, st);
    default: return PS_ELIMIT;
    }
}

int dpaps_launch_sgd_chunk(dpaps_ps *ps, const SgdArgs &a_in, int ntasks, int waves, hipStream_t st) {
    SgdArgs a = a_in;
    const int rc = plan_teams(ps, a, waves, st);
    if (rc) return rc;
    switch ((a.L + 15) / 16) {
    case 1: return a.L % 4 == 0 ? launch_chunk<1, true>(ps, a, ntasks, waves, st) : launch_chunk<1, false>(ps, a, ntasks, waves, st);
    case 2: return a.L % 4 == 0 ? launch_chunk<2, true>(ps, a, ntasks, waves, st) : launch_chunk<2, false>(ps, a, ntasks, waves, st);
    case 3: return a.L % 4 == 0 ? launch_chunk<3, true>(ps, a, ntasks, waves, st) : launch_chunk<3, false>(ps, a, ntasks, waves, st);
    case 4: return a.L % 4 == 0 ? launch_chunk<4, true>(ps, a, ntasks, waves, st) : launch_chunk<4, false>(ps, a, ntasks, waves, st);
    case 5: return a.L % 4 == 0 ? launch_chunk<5, true>(ps, a, ntasks, waves, st) : launch_chunk<5, false>(ps, a, ntasks, waves, st);
    case 6: return a.L % 4 == 0 ? launch_chunk<6, true>(ps, a, ntasks, waves, st) : launch_chunk<6, false>(ps, a, ntasks, waves, st);
    case 7: return a.L % 4 == 0 ? launch_chunk<7, true>(ps, a, ntasks, waves, st) : launch_chunk<7, false>(ps, a, ntasks, waves, st);
    case 8: return a.L % 4 == 0 ? launch_chunk<8, true>(ps, a, ntasks, waves, st) : launch_chunk<8, false>(ps, a, ntasks, waves, st);
    default: return PS_ELIMIT;
    }
}
