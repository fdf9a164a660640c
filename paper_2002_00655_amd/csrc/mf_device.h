// Device helpers shared by the SGD kernels: wavefront reduction, lane reads, LDS
// tickets, factor-row access in the "lane l holds components l, l+64, ..." layout.
#pragma once

#include "common.h"

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

// x of lane T of the same row of 16 lanes, in every lane (row_newbcast)
template <int T>
__device__ __forceinline__ float row_bcast_lane(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x150 + T, 0xF, 0xF, true));
}

// x[l] + x[l ^ 32] in every lane: the swap leaves the lower half of x in both halves of one result and the upper
// half in both halves of the other.  (Element by element into scalars: a bit cast applied to a vector element
// directly has been seen to pick element 0.)
__device__ __forceinline__ float add_across_halves(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const unsigned lo = r[0], hi = r[1];
    return __uint_as_float(lo) + __uint_as_float(hi);
}
// x[l] + x[l ^ 16] in every lane, likewise with the swap of the odd and even rows of 16 lanes
__device__ __forceinline__ float add_across_row_pairs(float x) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const unsigned even = r[0], odd = r[1];
    return __uint_as_float(even) + __uint_as_float(odd);
}

__device__ __forceinline__ int rl_i(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }
__device__ __forceinline__ float rl_f(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// LDS accesses of one wavefront are executed in program order, so for data that
// lives in LDS a ticket needs no waiting on counters: the writer issues the
// row's ds_writes and then the ticket's ds_write; a reader that issues the
// ticket's ds_read and then the row's ds_read and finds the expected ticket
// value has read the finished row.  The empty asm statements only keep the
// compiler from reordering the accesses around the (relaxed) ticket access.
__device__ __forceinline__ void compiler_fence() { __asm__ volatile("" ::: "memory"); }
__device__ __forceinline__ uint32_t ticket_read(uint32_t *tk) {
    return __hip_atomic_load(tk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void ticket_write(uint32_t *tk, uint32_t v) {
    __hip_atomic_store(tk, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Row access with lane l holding components l, l+64, ...: only the last of the
// NV slices can reach past the end of the row, and `tail` says whether this
// lane's component of that slice exists.
// AGENT: an agent-scope access, which the caches of a compute die pass through, for data that workgroups on
// different dies hand to each other inside one launch.
template <bool AGENT>
__device__ __forceinline__ float load_f(const float *p) {
    if constexpr (AGENT) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else return *p;
}
template <bool AGENT>
__device__ __forceinline__ void store_f(float *p, float x) {
    if constexpr (AGENT) __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = x;
}
template <int NV, bool AGENT = false>
__device__ __forceinline__ void load_row_t(const float *p, int lane, bool tail, float (&x)[NV]) {
#pragma unroll
    for (int c = 0; c < NV - 1; ++c) x[c] = load_f<AGENT>(p + lane + 64 * c);
    x[NV - 1] = tail ? load_f<AGENT>(p + lane + 64 * (NV - 1)) : 0.0f;
}
template <int NV, bool AGENT = false>
__device__ __forceinline__ void store_row_t(float *p, int lane, bool tail, const float (&x)[NV]) {
#pragma unroll
    for (int c = 0; c < NV - 1; ++c) store_f<AGENT>(p + lane + 64 * c, x[c]);
    if (tail) store_f<AGENT>(p + lane + 64 * (NV - 1), x[NV - 1]);
}

#define INFO_SINGLE 0xFFFFu      // low 16 bits of an info word: the row's only entry in the block
#define INFO_NONE 0xFFFEu        // filler for lanes past the end of a run: neither single nor in LDS

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

// Home nodes (at most) whose keys one task may touch for all of them to be handled in one pass.
#define DPAPS_LOC_SLOTS 16

// All threads of the workgroup call this.  lds_u32: scratch_words words of LDS scratch, at least 2 * ceil(W / 32);
// with (home nodes touched + 1) * ceil(W / 32) words (at most DPAPS_LOC_SLOTS home nodes) the keys of all home
// nodes are handled in one pass, otherwise home node by home node.
// AGENT: the owner map is read and written with agent-scope accesses (see load_f).
template <bool AGENT = false>
__device__ __forceinline__ void mf_localize_task(const LocalizeArgs &a, uint32_t *lds_u32, int scratch_words, int32_t worker, int32_t rb,
                                                 int32_t cb) {
    const int words = (a.W + 31) / 32;
    __shared__ int s_reloc, s_req, s_instr;
    const int64_t r0 = a.row_bounds[rb], r1 = a.row_bounds[rb + 1];
    const int64_t c0 = a.m + a.col_bounds[cb], c1 = a.m + a.col_bounds[cb + 1];
    // home nodes touched by the two key ranges (empty range: lo > hi)
    const int64_t hr_lo = r1 > r0 ? r0 / a.per_home : 1, hr_hi = r1 > r0 ? (r1 - 1) / a.per_home : 0;
    const int64_t hc_lo = c1 > c0 ? c0 / a.per_home : 1, hc_hi = c1 > c0 ? (c1 - 1) / a.per_home : 0;
    // the owner of a key before; takes the key if it is another's
    auto take = [&](int64_t k) -> int32_t {
        int32_t old;
        if constexpr (AGENT) old = __hip_atomic_load(&a.owner[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else old = a.owner[k];
        if (old != worker) {
            // the home node updates the location at once
            if constexpr (AGENT) __hip_atomic_store(&a.owner[k], worker, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else a.owner[k] = worker;
        }
        return old;
    };
    int reloc = 0;
    // slot of a home node: those of the row range first, those only in the column range behind them
    const int nslot_r = (int)(hr_hi - hr_lo + 1 > 0 ? hr_hi - hr_lo + 1 : 0);
    const int nslot_c = (int)(hc_hi - hc_lo + 1 > 0 ? hc_hi - hc_lo + 1 : 0);
    const int nslots = nslot_r + nslot_c;
    const bool one_pass = nslots <= DPAPS_LOC_SLOTS && (nslots + 1) * words <= scratch_words;
    uint32_t *bits_all = one_pass ? lds_u32 + nslots * words : lds_u32;       // the old owners over all home nodes
    if (one_pass) {
        // per home node a bit set of the old owners, all filled in one sweep over the keys
        for (int i = threadIdx.x; i < (nslots + 1) * words; i += blockDim.x) lds_u32[i] = 0;
        if (threadIdx.x == 0) { s_reloc = 0; s_req = 0; s_instr = 0; }
        __syncthreads();
        for (int sub = 0; sub < 2; ++sub) {
            const int64_t x0 = sub == 0 ? r0 : c0, x1 = sub == 0 ? r1 : c1;
            const int64_t lo = sub == 0 ? hr_lo : hc_lo, hi = sub == 0 ? hr_hi : hc_hi;
            for (int64_t h = lo; h <= hi; ++h) {
                const int slot = sub == 0 || (h >= hr_lo && h <= hr_hi) ? (int)(h - hr_lo) : nslot_r + (int)(h - hc_lo);
                uint32_t *bits_h = lds_u32 + slot * words;
                const int64_t k_lo = h * a.per_home, k_hi = k_lo + a.per_home;
                const int64_t s0 = x0 > k_lo ? x0 : k_lo, s1 = x1 < k_hi ? x1 : k_hi;
                for (int64_t k = s0 + threadIdx.x; k < s1; k += blockDim.x) {
                    const int32_t old = take(k);
                    if (old != worker) {
                        ++reloc;
                        atomicOr(&bits_h[old >> 5], 1u << (old & 31));
                    }
                }
            }
        }
        __syncthreads();
        if (threadIdx.x < 64) {
            int req = 0, instr = 0;
            for (int slot = 0; slot < nslots; ++slot) {
                const int64_t h = slot < nslot_r ? hr_lo + slot : hc_lo + (slot - nslot_r);
                if (slot >= nslot_r && h >= hr_lo && h <= hr_hi) continue;     // counted with the row range's slot
                const uint32_t *bits_h = lds_u32 + slot * words;
                int cnt = 0;
                for (int i = threadIdx.x; i < words; i += 64) {
                    cnt += __popc(bits_h[i]);
                    if (bits_h[i]) atomicOr(&bits_all[i], bits_h[i]);
                }
                for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off);
                if (cnt > 0) {
                    if (h != worker) req += 1;
                    instr += cnt - (int)((bits_h[h >> 5] >> (h & 31)) & 1u);
                }
            }
            if (threadIdx.x == 0) { s_req = req; s_instr = instr; }
        }
    } else {
        // home node by home node, one bit set reused
        uint32_t *bits_h = lds_u32 + words;
        for (int i = threadIdx.x; i < 2 * words; i += blockDim.x) lds_u32[i] = 0;
        if (threadIdx.x == 0) { s_reloc = 0; s_req = 0; s_instr = 0; }
        __syncthreads();
        for (int part = 0; part < 2; ++part) {
            const int64_t lo = part == 0 ? hr_lo : hc_lo, hi = part == 0 ? hr_hi : hc_hi;
            for (int64_t h = lo; h <= hi; ++h) {
                if (part == 1 && h >= hr_lo && h <= hr_hi) continue;   // done together with the row range
                const int64_t k_lo = h * a.per_home, k_hi = k_lo + a.per_home;
                for (int sub = 0; sub < 2; ++sub) {
                    const int64_t x0 = sub == 0 ? r0 : c0, x1 = sub == 0 ? r1 : c1;
                    const int64_t s0 = x0 > k_lo ? x0 : k_lo, s1 = x1 < k_hi ? x1 : k_hi;
                    for (int64_t k = s0 + threadIdx.x; k < s1; k += blockDim.x) {
                        const int32_t old = take(k);
                        if (old != worker) {
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
    }
    if (reloc) atomicAdd(&s_reloc, reloc);
    __syncthreads();
    int n_transfer = 0, n_reloc = 0, n_req = 0, n_instr = 0;
    if (threadIdx.x < 64) {
        for (int i = threadIdx.x; i < words; i += 64) n_transfer += __popc(bits_all[i]);
        for (int off = 32; off > 0; off >>= 1) n_transfer += __shfl_xor(n_transfer, off);
        n_reloc = s_reloc; n_req = s_req; n_instr = s_instr;
    }
    __syncthreads();            // the scratch and the three counters may be used again
    // (after the barrier, so that nobody waits for these additions to arrive: the next barrier of the caller does)
    if (threadIdx.x == 0) {
        u64 *st = stat_slot(a.stats);
        atomicAdd(&st[PS_STAT_LOCALIZE_KEYS], (u64)((r1 - r0) + (c1 - c0)));
        if (n_reloc) atomicAdd(&st[PS_STAT_RELOCATED], (u64)n_reloc);
        if (n_req) atomicAdd(&st[PS_STAT_MSG_LOC_REQ], (u64)n_req);
        if (n_instr) atomicAdd(&st[PS_STAT_MSG_LOC_INSTRUCT], (u64)n_instr);
        if (n_transfer) atomicAdd(&st[PS_STAT_MSG_LOC_TRANSFER], (u64)n_transfer);
    }
}
