// Parameter server primitives on one GPU: dense store, owner map, pull / push /
// localize and the integer routing statistics (Table "Primitives", Sec. 3.1-3.3,
// Sec. 3.5, Sec. 3.7 of the paper).
#include "common.h"

#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>

// ---------------------------------------------------------------------------
// host helpers
// ---------------------------------------------------------------------------
int dpaps_fail_hip(dpaps_ps *ps, hipError_t e, const char *what) {
    if (ps) {
        ps->last_error = std::string(what) + ": " + hipGetErrorString(e);
    }
    (void)hipGetLastError();
    return e == hipErrorOutOfMemory ? PS_ENOMEM : PS_EHIP;
}

int dpaps_ws_reserve(dpaps_ps *ps, size_t bytes) {
    if (bytes <= ps->ws_bytes) return PS_OK;
    if (ps->ws) {
        PS_HIP(ps, hipDeviceSynchronize());
        PS_HIP(ps, hipFree(ps->ws));
        ps->ws = nullptr;
        ps->ws_bytes = 0;
    }
    size_t want = bytes + bytes / 4 + 4096;
    PS_HIP(ps, hipMalloc(&ps->ws, want));
    ps->ws_bytes = want;
    return PS_OK;
}

static inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------
__global__ void k_init_owner(int32_t *owner, int64_t K, int64_t per_home) {
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < K) owner[k] = (int32_t)(k / per_home);
}

__global__ void k_check_keys(const int64_t *keys, int64_t n, int64_t K, int32_t *err) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) {
        int64_t k = keys[p];
        if (k < 0 || k >= K) atomicExch(err, PS_EKEY);
    }
}

// ---- routing statistics ----------------------------------------------------
// A call's kernels run a fixed number of workgroups that walk over the keys.  Each workgroup counts in LDS
// and adds its counts to the statistics once, at its end.  The message counts need "first mention of a
// destination in this call": stamps in device memory carry the id of the last call that mentioned the
// destination; a workgroup remembers in LDS which destinations it has already settled, so that device-wide
// operations on the few hot stamp words stay rare.
constexpr int ROUTE_BLOCKS_PER_CU = 2;
constexpr int NODE_WORDS = 2048 / 32;                  // one bit per node (at most 2048 workers)
constexpr int PAIR_BITS = 1 << 16;                     // one bit per (from, to) pair where W x W fits (W <= 256) ...
constexpr int SEEN_PAIR = 1024;                        // ... else direct-mapped: entry holds idx + 1 of a settled pair

struct RouteLds {
    uint32_t count[8];
    uint32_t bits_h[NODE_WORDS], bits_o[NODE_WORDS];   // nodes this workgroup has settled as request / reply destinations
    uint32_t bits_pair[PAIR_BITS / 32];
    uint32_t seen_pair[SEEN_PAIR];
};

__device__ __forceinline__ void route_lds_init(RouteLds &l) {
    for (int i = threadIdx.x; i < (int)(sizeof(RouteLds) / 4); i += blockDim.x) reinterpret_cast<uint32_t *>(&l)[i] = 0;
    __syncthreads();
}

__device__ __forceinline__ void lds_count_add(bool flag, uint32_t *counter) {
    const u64 b = __ballot(flag);
    if (b != 0 && (threadIdx.x & 63) == (unsigned)(__ffsll((long long)__ballot(true)) - 1)) atomicAdd(counter, (uint32_t)__popcll(b));
}

// Marks stamps[idx] with this call's id and tells whether this was the first mark of the call: true in
// exactly one lane of the whole call per idx.  Lanes of a wavefront that name the same idx are served by
// one of them; a destination the workgroup has settled before is skipped; the exchange is skipped when
// the stamp is seen to carry the id already (a stale read only costs an exchange).
__device__ __forceinline__ bool stamp_first(bool want, uint32_t *stamps, int32_t idx, uint32_t call_id, uint32_t *seen, int seen_mask) {
    bool first = false;
    const int lane = threadIdx.x & 63;
    u64 todo = __ballot(want);
    while (todo != 0) {
        const int leader = __ffsll((long long)todo) - 1;
        const int32_t idx0 = __builtin_amdgcn_readlane(idx, leader);
        const u64 same = __ballot(want && idx == idx0);
        if (lane == leader && seen[idx0 & seen_mask] != (uint32_t)idx0 + 1u) {
            if (__hip_atomic_load(&stamps[idx0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != call_id)
                first = atomicExch(&stamps[idx0], call_id) != call_id;
            seen[idx0 & seen_mask] = (uint32_t)idx0 + 1u;
        }
        todo &= ~same;
    }
    return first;
}

// The same where every idx has a bit of its own in LDS: the lane that sets the bit settles idx for the workgroup,
// no matter how many different destinations the lanes of a wavefront name (with hundreds of nodes and keys drawn at
// random that is nearly one each, and the loop above goes round once per destination).
__device__ __forceinline__ bool stamp_first_bit(bool want, uint32_t *stamps, int32_t idx, uint32_t call_id, uint32_t *bits) {
    bool first = false;
    if (want) {
        const uint32_t m = 1u << (idx & 31);
        if ((atomicOr(&bits[idx >> 5], m) & m) == 0u &&
            __hip_atomic_load(&stamps[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != call_id)
            first = atomicExch(&stamps[idx], call_id) != call_id;
    }
    return first;
}
__device__ __forceinline__ bool stamp_first_pair(bool want, uint32_t *stamp_pair, int32_t from, int32_t to, int32_t W, uint32_t call_id,
                                                 RouteLds &l) {
    if (W * W <= PAIR_BITS) return stamp_first_bit(want, stamp_pair, from * W + to, call_id, l.bits_pair);
    return stamp_first(want, stamp_pair, from * W + to, call_id, l.seen_pair, SEEN_PAIR - 1);
}

// home node of key k: k / per_home without the 64-bit division (double has 53 bits, keys and per_home fewer; the
// quotient estimate is off by at most one)
__device__ __forceinline__ int32_t home_node(int64_t k, int64_t per_home, double inv_per_home) {
    int64_t h = (int64_t)((double)k * inv_per_home);
    if (h * per_home > k) --h;
    else if ((h + 1) * per_home <= k) ++h;
    return (int32_t)h;
}

// One key that must travel for requester `worker`: home h, current owner o.
// Within one call the messages to one destination are grouped (Sec. 3.7); the
// stamps record which destinations this call has already been charged for.
// count[2..4]: request, forward, reply (or their localize counterparts).
__device__ __forceinline__ void route_key(bool travels, int32_t worker, int32_t h, int32_t o, int32_t W,
                                          uint32_t *stamp_h, uint32_t *stamp_o, uint32_t *stamp_pair, uint32_t call_id, RouteLds &l) {
    const bool req = stamp_first_bit(travels && h != worker, stamp_h, h, call_id, l.bits_h);
    const bool fresh = stamp_first_pair(travels, stamp_pair, h, o, W, call_id, l);
    const bool fwd = fresh && (h != o);
    const bool back = stamp_first_bit(travels && o != worker, stamp_o, o, call_id, l.bits_o);
    lds_count_add(req, &l.count[2]);
    lds_count_add(fwd, &l.count[3]);
    lds_count_add(back, &l.count[4]);
}

// adds count[i] to the statistic which[i] (i < 7; -1: none), one workgroup's share
__device__ __forceinline__ void route_lds_flush(RouteLds &l, u64 *stats, int w0, int w1, int w2, int w3, int w4, int w5 = -1, int w6 = -1) {
    __syncthreads();
    const int which[7] = {w0, w1, w2, w3, w4, w5, w6};
    if (threadIdx.x < 7 && which[threadIdx.x] >= 0 && l.count[threadIdx.x] != 0)
        atomicAdd(&stat_slot(stats)[which[threadIdx.x]], (u64)l.count[threadIdx.x]);
}

// One key that `worker` reads or writes remotely: home h, owner o, c = what the worker's node's location cache says
// (Sec. 3.3 "Location caching"; -1: no entry, or no caches).  No entry: request to the home node, which forwards
// to the owner, which replies.  Correct entry: request straight to the owner.  Stale entry: request to the node
// named, which forwards to the home node, which forwards to the owner (double-forward).  Grouped per call like
// route_key: one request per node asked, one forward per (from, to), one reply per owner.
// count[2..4]: request, forward, reply; count[5], count[6]: accesses with a correct / a stale entry.
__device__ __forceinline__ void route_access_key(bool remote, int32_t worker, int32_t h, int32_t o, int32_t c, int32_t W,
                                                 uint32_t *stamp_h, uint32_t *stamp_o, uint32_t *stamp_pair, uint32_t call_id, RouteLds &l) {
    const bool hit = remote && c == o, stale = remote && c >= 0 && c != o;
    const int32_t asked = hit ? o : (stale ? c : h);
    const bool req = stamp_first_bit(remote && asked != worker, stamp_h, asked, call_id, l.bits_h);
    const bool fresh1 = stamp_first_pair(stale, stamp_pair, c, h, W, call_id, l);
    const bool fresh2 = stamp_first_pair(remote && !hit, stamp_pair, h, o, W, call_id, l);
    const bool back = stamp_first_bit(remote, stamp_o, o, call_id, l.bits_o);
    lds_count_add(req, &l.count[2]);
    lds_count_add(fresh1 && c != h, &l.count[3]);
    lds_count_add(fresh2 && h != o, &l.count[3]);
    lds_count_add(back, &l.count[4]);
    lds_count_add(hit, &l.count[5]);
    lds_count_add(stale, &l.count[6]);
}

// Locality statistics and message counts of one pull or push call.
__global__ __launch_bounds__(256) void k_route_access(const int64_t *keys, int64_t n, int32_t worker, const int32_t *owner, int64_t per_home,
                                                       int32_t W, uint32_t *stamp_h, uint32_t *stamp_o, uint32_t *stamp_pair, uint32_t call_id,
                                                       u64 *stats, int stat_local, int stat_remote, int stat_local2, int stat_remote2,
                                                       const int16_t *loc_row, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    __shared__ RouteLds l;
    route_lds_init(l);
    const double inv_per_home = 1.0 / (double)per_home;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t base = (int64_t)blockIdx.x * blockDim.x; base < n; base += step) {     // whole workgroups walk together
        const int64_t p = base + threadIdx.x;
        const bool active = p < n;
        const int64_t k = active ? keys[p] : 0;
        const int32_t o = active ? owner[k] : 0;
        const bool local = active && o == worker, remote = active && o != worker;
        lds_count_add(local, &l.count[0]);
        lds_count_add(remote, &l.count[1]);
        const int32_t c = remote && loc_row ? (int32_t)loc_row[k] : -1;       // this node's location cache, if there are caches
        route_access_key(remote, worker, home_node(k, per_home, inv_per_home), o, c, W, stamp_h, stamp_o, stamp_pair, call_id, l);
    }
    route_lds_flush(l, stats, stat_local, stat_remote, PS_STAT_MSG_ACC_REQ, PS_STAT_MSG_ACC_FWD, PS_STAT_MSG_ACC_REPLY, PS_STAT_CACHE_HIT,
                    PS_STAT_CACHE_STALE);
    // a second access to the same keys by the same worker right after (a pull and a push of one step) has the
    // same locality and sends the same messages once more
    // (only without location caches: with them the first access's replies change how the second is routed)
    if (stat_local2 >= 0) route_lds_flush(l, stats, stat_local2, stat_remote2, PS_STAT_MSG_ACC_REQ, PS_STAT_MSG_ACC_FWD, PS_STAT_MSG_ACC_REPLY);
}

// The replies of a pull or push have arrived: the requester's node knows the owner of every remote key it asked
// for (Sec. 3.3: the caches change without messages of their own).  Several mentions of a key write the same.
__global__ void k_cache_replies(const int64_t *keys, int64_t n, int32_t worker, const int32_t *owner, int16_t *loc_row, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    const int64_t k = keys[p];
    const int32_t o = owner[k];
    if (o != worker) loc_row[k] = (int16_t)o;
}

// localize: the home node updates the location at once (Sec. 3.2, step 1); the
// exchange makes exactly one of several mentions of a key the one that moves it.
__global__ __launch_bounds__(256) void k_localize(const int64_t *keys, int64_t n, int32_t worker, int32_t *owner, int64_t per_home, int32_t W,
                                                   uint32_t *stamp_h, uint32_t *stamp_o, uint32_t *stamp_pair, uint32_t call_id, u64 *stats,
                                                   int16_t *loc, int64_t K, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    __shared__ RouteLds l;
    route_lds_init(l);
    const double inv_per_home = 1.0 / (double)per_home;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t base = (int64_t)blockIdx.x * blockDim.x; base < n; base += step) {
        const int64_t p = base + threadIdx.x;
        const bool active = p < n;
        const int64_t k = active ? keys[p] : 0;
        // (a key that is seen to be the worker's already is left alone: a stale read only costs an exchange, and
        // a key mentioned a million times in one call does not turn into a million exchanges on one word)
        int32_t old = worker;
        if (active && __hip_atomic_load(&owner[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != worker) old = atomicExch(&owner[k], worker);
        const bool moved = active && old != worker;
        if (moved && loc) loc[(int64_t)old * K + k] = (int16_t)worker;     // the old owner hands the value over: it knows where to
        lds_count_add(active, &l.count[0]);
        lds_count_add(moved, &l.count[1]);
        route_key(moved, worker, home_node(k, per_home, inv_per_home), old, W, stamp_h, stamp_o, stamp_pair, call_id, l);
    }
    route_lds_flush(l, stats, PS_STAT_LOCALIZE_KEYS, PS_STAT_RELOCATED, PS_STAT_MSG_LOC_REQ, PS_STAT_MSG_LOC_INSTRUCT, PS_STAT_MSG_LOC_TRANSFER);
}

__global__ void k_owner(const int64_t *keys, int64_t n, const int32_t *owner, int32_t *out, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) out[p] = owner[keys[p]];
}

// pull: one thread per value; a key's row is contiguous, so 64 lanes read 256
// contiguous bytes of the store and write 256 contiguous bytes of the result.
__global__ void k_pull(const int64_t *keys, int64_t n, int32_t L, const float *val, float *out, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * L) return;
    int64_t p = idx / L;
    int32_t c = (int32_t)(idx - p * L);
    out[idx] = val[keys[p] * L + c];
}

// the same in 16-byte pieces, for rows that start on 16-byte boundaries (value_len a multiple of 4) and fewer
// than 2^32 pieces in all: P pieces per row
__global__ void k_pull_v4(const int64_t *keys, uint32_t total, uint32_t P, const float4 *val, float4 *out, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    const uint32_t idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const uint32_t p = idx / P, c = idx - p * P;
    out[idx] = val[keys[p] * (int64_t)P + c];
}

// push, after the (key, position) pairs have been sorted by key with a stable
// sort: one wavefront per sorted position; the wavefront at the head of a run
// of equal keys adds that key's update terms one after the other, in
// increasing position - the order a sequential server would apply them in.
// (One wavefront per key however often it is mentioned: the checking mode.)
__global__ void k_push_apply(const uint64_t *skeys, const uint32_t *spos, int64_t n, int32_t L, const float *deltas,
                             float *val, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    const int lane = threadIdx.x & 63;
    int64_t q = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    if (q >= n) return;
    uint64_t k = skeys[q];
    if (q > 0 && skeys[q - 1] == k) return;
    int64_t end = q + 1;
    while (end < n && skeys[end] == k) ++end;
    for (int32_t c = lane; c < L; c += 64) {
        float v = val[(int64_t)k * L + c];
        for (int64_t t = q; t < end; ++t) v = v + deltas[(int64_t)spos[t] * L + c];
        val[(int64_t)k * L + c] = v;
    }
}

// push, the default: the sorted positions are cut into ranges of PUSH_RANGE, one wavefront each, so that a key
// mentioned thousands of times is summed by many wavefronts.  Inside a range the terms of a key are added
// one after the other in argument order, starting from the stored value; a key whose terms fill one range
// only (any key mentioned once, most keys mentioned a few times) therefore gets the sequential server's
// bits.  Where a key's terms continue from the previous range they are summed from zero into part[2 r];
// where they start here and continue into the next range the running value goes to part[2 r + 1]; the
// second kernel adds a key's partial sums in range order.  The result depends on the arguments only.
constexpr int PUSH_RANGE = 64;

__device__ __forceinline__ uint64_t readlane_u64(uint64_t x, int l) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, l);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), l);
    return ((uint64_t)hi << 32) | lo;
}

template <int UN>
__global__ __launch_bounds__(256) void k_push_ranges(const uint64_t *skeys, const uint32_t *spos, int64_t n, int32_t L,
                                                      const float *deltas, float *val, float *part, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    const int lane = threadIdx.x & 63;
    const int64_t r = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t q0 = r * PUSH_RANGE;
    if (q0 >= n) return;
    const int cnt = (int)(n - q0 < PUSH_RANGE ? n - q0 : PUSH_RANGE);
    const uint64_t NOKEY = ~0ull;                                      // no key looks like this
    const uint64_t mk = lane < cnt ? skeys[q0 + lane] : NOKEY;         // lane t: sorted position q0 + t
    const int mp = lane < cnt ? (int)spos[q0 + lane] : 0;
    const uint64_t prevk = q0 > 0 ? skeys[q0 - 1] : NOKEY;
    const uint64_t nextk = q0 + cnt < n ? skeys[q0 + cnt] : NOKEY;
    const uint64_t before = lane > 0 && lane < cnt ? skeys[q0 + lane - 1] : NOKEY;
    const u64 heads = __ballot(lane < cnt && (lane == 0 || before != mk));   // positions where a key's terms start
    const bool first_open = readlane_u64(mk, 0) == prevk;              // the first key's terms continue from the range before
    const int c = blockIdx.y * 64 + lane;                              // this wavefront's 64 components
    const bool in = c < L;
    // UN positions at a time: all their loads first (update terms, and the stored value where a key's terms
    // start), then the additions in order
    float v = 0.0f;
    uint64_t key = NOKEY;                                              // key of the terms being summed
    bool key_open = false;                                             // ... which continue from the range before
    for (int u0 = 0; u0 < cnt; u0 += UN) {
        float d[UN], b[UN];
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            const int u = u0 + i < cnt ? u0 + i : cnt - 1;
            const bool is_head = u0 + i < cnt && ((heads >> u) & 1) != 0 && !(u == 0 && first_open);
            d[i] = in && u0 + i < cnt ? deltas[(int64_t)__builtin_amdgcn_readlane(mp, u) * L + c] : 0.0f;
            b[i] = 0.0f;
            if (is_head && in) b[i] = val[(int64_t)readlane_u64(mk, u) * L + c];
        }
#pragma unroll
        for (int i = 0; i < UN; ++i) {
            const int u = u0 + i;
            if (u < cnt) {
                if ((heads >> u) & 1) {
                    if (u > 0 && in) {                                 // the previous key's terms end here
                        if (key_open) part[(2 * r) * L + c] = v;
                        else val[(int64_t)key * L + c] = v;
                    }
                    key = readlane_u64(mk, u);
                    key_open = u == 0 && first_open;
                    v = b[i];
                }
                v = v + d[i];
            }
        }
    }
    if (in) {
        if (key_open) part[(2 * r) * L + c] = v;
        else if (key == nextk) part[(2 * r + 1) * L + c] = v;
        else val[(int64_t)key * L + c] = v;
    }
}

// Second kernel: the wavefront of the range in which a key's terms start and do not end adds the partial sums
// of the following ranges, in order, and stores the value.  blockIdx.y: which 64 components.
__global__ __launch_bounds__(256) void k_push_join(const uint64_t *skeys, int64_t n, int32_t L, const float *part, float *val,
                                                    const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    const int lane = threadIdx.x & 63;
    const int64_t r = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t q1 = (r + 1) * PUSH_RANGE;
    if (q1 >= n) return;                                               // nothing follows this range
    const uint64_t key = skeys[q1 - 1];
    if (skeys[q1] != key) return;                                      // its last key ends here
    if (r > 0 && skeys[q1 - PUSH_RANGE] == key && skeys[q1 - PUSH_RANGE - 1] == key) return;   // it started earlier
    // m: how many of the following ranges begin with this key
    int64_t m = 0;
    for (;;) {
        const int64_t q = (r + 1 + m + lane) * PUSH_RANGE;
        const u64 b = __ballot(q < n && skeys[q < n ? q : 0] == key);
        const int run = b == ~0ull ? 64 : __ffsll((long long)~b) - 1;
        m += run;
        if (run < 64) break;
    }
    const int c = blockIdx.y * 64 + lane;
    if (c >= L) return;
    float v = part[(2 * r + 1) * L + c];
    int64_t j = 1;
    for (; j + 16 <= m + 1; j += 16) {
        float d[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) d[i] = part[(2 * (r + j + i)) * L + c];
#pragma unroll
        for (int i = 0; i < 16; ++i) v = v + d[i];
    }
    for (; j <= m; ++j) v = v + part[(2 * (r + j)) * L + c];
    val[(int64_t)key * L + c] = v;
}

// ---------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------
static inline unsigned grid_for(int64_t n, int block) { return (unsigned)((n + block - 1) / block); }
static inline unsigned route_grid(const dpaps_ps *ps, int64_t n) {
    const int64_t need = (n + 255) / 256, cap = (int64_t)ROUTE_BLOCKS_PER_CU * (ps->num_cu > 0 ? ps->num_cu : 1);
    return (unsigned)(need < cap ? need : cap);
}

static int static_scratch_init(dpaps_ps *ps);

extern "C" int ps_create(int64_t num_keys, int32_t value_len, int32_t num_workers, ps_handle *out) {
    if (!out) return PS_EINVAL;
    *out = nullptr;
    if (num_keys <= 0 || value_len <= 0 || value_len > 1024 || num_workers <= 0 || num_workers > 2048) return PS_EINVAL;
    dpaps_ps *ps = new (std::nothrow) dpaps_ps();
    if (!ps) return PS_ENOMEM;
    ps->K = num_keys; ps->L = value_len; ps->W = num_workers;
    ps->per_home = (num_keys + num_workers - 1) / num_workers;
    hipError_t e;
#define CR(call) do { e = (call); if (e != hipSuccess) { int rc_ = dpaps_fail_hip(ps, e, #call); ps_destroy(ps); return rc_; } } while (0)
    CR(hipGetDevice(&ps->device));
    {
        const int rc_ = static_scratch_init(ps);
        if (rc_) { ps_destroy(ps); return rc_; }
    }
    int v = 0;
    CR(hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, ps->device));
    ps->lds_bytes = v;
    CR(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, ps->device));
    ps->num_cu = v;
    // slack after the last row: the grouped SGD kernel reads rows in 16-byte pieces up to the next multiple of 16
    // components, and parks switched-off lanes just past the end of a block's factors
    size_t vbytes = ((size_t)num_keys * value_len + 256) * sizeof(float);
    CR(hipMalloc(&ps->val, vbytes));
    CR(hipMemset(ps->val, 0, vbytes));
    CR(hipMalloc(&ps->owner, (size_t)num_keys * sizeof(int32_t)));
    static_assert(PS_STAT_COUNT <= PS_STAT_STRIDE, "a slot holds all counters");
    CR(hipMalloc(&ps->stats, PS_STAT_SLOTS * PS_STAT_STRIDE * sizeof(u64)));
    CR(hipMemset(ps->stats, 0, PS_STAT_SLOTS * PS_STAT_STRIDE * sizeof(u64)));
    CR(hipMalloc(&ps->err, sizeof(int32_t)));
    CR(hipMemset(ps->err, 0, sizeof(int32_t)));
    CR(hipMalloc(&ps->d_sse, sizeof(double)));
    size_t W = (size_t)num_workers;
    CR(hipMalloc(&ps->stamp_h, (2 * W + W * W) * sizeof(uint32_t)));
    CR(hipMemset(ps->stamp_h, 0, (2 * W + W * W) * sizeof(uint32_t)));
    ps->stamp_o = ps->stamp_h + W;
    ps->stamp_pair = ps->stamp_o + W;
    k_init_owner<<<grid_for(num_keys, 256), 256>>>(ps->owner, num_keys, ps->per_home);
    CR(hipGetLastError());
    CR(hipDeviceSynchronize());
#undef CR
    *out = ps;
    return PS_OK;
}

void dpaps_mf_free(dpaps_ps *ps);   // mf_prepare.hip

extern "C" int ps_destroy(ps_handle ps) {
    if (!ps) return PS_EINVAL;
    (void)hipDeviceSynchronize();
    dpaps_mf_free(ps);
    if (ps->val) (void)hipFree(ps->val);
    if (ps->owner) (void)hipFree(ps->owner);
    if (ps->stats) (void)hipFree(ps->stats);
    if (ps->err) (void)hipFree(ps->err);
    if (ps->d_sse) (void)hipFree(ps->d_sse);
    if (ps->stamp_h) (void)hipFree(ps->stamp_h);
    if (ps->ws) (void)hipFree(ps->ws);
    if (ps->kge_ws) (void)hipFree(ps->kge_ws);
    if (ps->handoff_ws) (void)hipFree(ps->handoff_ws);
    if (ps->loc) (void)hipFree(ps->loc);
    if (ps->side_stream) (void)hipStreamDestroy(ps->side_stream);
    if (ps->ev_fork) (void)hipEventDestroy(ps->ev_fork);
    if (ps->ev_join) (void)hipEventDestroy(ps->ev_join);
    if (ps->ev_sorted) (void)hipEventDestroy(ps->ev_sorted);
    if (ps->ev_added) (void)hipEventDestroy(ps->ev_added);
    if (ps->d_tasks) (void)hipFree(ps->d_tasks);
    for (hipEvent_t e : ps->ev_pool) (void)hipEventDestroy(e);
    delete ps;
    return PS_OK;
}

static int launch_check(dpaps_ps *ps, const int64_t *keys, int64_t n, hipStream_t st) {
    if (n > 0) {
        k_check_keys<<<grid_for(n, 256), 256, 0, st>>>(keys, n, ps->K, ps->err);
        PS_HIP(ps, hipGetLastError());
    }
    return PS_OK;
}

// the library's second stream (default priority) and the events that tie it to the caller's
int dpaps_side_stream(dpaps_ps *ps) {
    if (!ps->side_stream) {
        PS_HIP(ps, hipStreamCreateWithFlags(&ps->side_stream, hipStreamNonBlocking));
        PS_HIP(ps, hipEventCreateWithFlags(&ps->ev_fork, hipEventDisableTiming));
        PS_HIP(ps, hipEventCreateWithFlags(&ps->ev_join, hipEventDisableTiming));
        PS_HIP(ps, hipEventCreateWithFlags(&ps->ev_sorted, hipEventDisableTiming));
        PS_HIP(ps, hipEventCreateWithFlags(&ps->ev_added, hipEventDisableTiming));
    }
    return PS_OK;
}

// Calls with this many keys or more count their statistics on the second stream, beside the work on the values
// (below that the two extra waits between streams cost more than the statistics kernel takes).
constexpr int64_t SIDE_STATS_MIN_KEYS = (int64_t)1 << 20;

// statistics of a large pull or push, started on the second stream once the keys are checked; the caller's stream
// waits for them when the call's own kernels are queued (dpaps_side_stats_join)
static int side_stats_fork(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, int st_local, int st_remote, hipStream_t st);
static int side_stats_join(dpaps_ps *ps, hipStream_t st) {
    PS_HIP(ps, hipStreamWaitEvent(st, ps->ev_join, 0));
    return PS_OK;
}

int dpaps_check_keys(dpaps_ps *ps, const int64_t *keys, int64_t n, hipStream_t st) { return launch_check(ps, keys, n, st); }

__global__ void k_fill_u32(uint32_t *p, size_t n, uint32_t v) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

static uint32_t next_call_id(dpaps_ps *ps, hipStream_t st) {
    if (++ps->call_id == 0) {   // wrapped: forget all stamps (a kernel, not a memset node: callers may be capturing)
        const size_t W = (size_t)ps->W, words = 2 * W + W * W;
        k_fill_u32<<<grid_for((int64_t)words, 256), 256, 0, st>>>(ps->stamp_h, words, 0u);
        ps->call_id = 1;
    }
    return ps->call_id;
}

static int route_access(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, int st_local, int st_remote,
                        hipStream_t st, int st_local2 = -1, int st_remote2 = -1) {
    if (worker < 0 || n == 0) return PS_OK;
    if (ps->loc && st_local2 >= 0) {      // with location caches the second access is routed after the first one's replies
        const int rc = route_access(ps, worker, keys, n, st_local, st_remote, st);
        return rc ? rc : route_access(ps, worker, keys, n, st_local2, st_remote2, st);
    }
    uint32_t id = next_call_id(ps, st);
    int16_t *loc_row = ps->loc ? ps->loc + (int64_t)worker * ps->K : nullptr;
    k_route_access<<<route_grid(ps, n), 256, 0, st>>>(keys, n, worker, ps->owner, ps->per_home, ps->W, ps->stamp_h,
                                                     ps->stamp_o, ps->stamp_pair, id, ps->stats, st_local, st_remote,
                                                     st_local2, st_remote2, loc_row, ps->err);
    PS_HIP(ps, hipGetLastError());
    if (loc_row) {
        k_cache_replies<<<grid_for(n, 256), 256, 0, st>>>(keys, n, worker, ps->owner, loc_row, ps->err);
        PS_HIP(ps, hipGetLastError());
    }
    return PS_OK;
}

static int side_stats_fork(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, int st_local, int st_remote, hipStream_t st) {
    int rc = dpaps_side_stream(ps);
    if (rc) return rc;
    PS_HIP(ps, hipEventRecord(ps->ev_fork, st));
    PS_HIP(ps, hipStreamWaitEvent(ps->side_stream, ps->ev_fork, 0));
    rc = route_access(ps, worker, keys, n, st_local, st_remote, ps->side_stream);
    if (rc) return rc;
    PS_HIP(ps, hipEventRecord(ps->ev_join, ps->side_stream));
    return PS_OK;
}

int dpaps_account_pull(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, hipStream_t st) {
    int rc = launch_check(ps, keys, n, st);
    if (rc) return rc;
    return route_access(ps, worker, keys, n, PS_STAT_PULL_LOCAL, PS_STAT_PULL_REMOTE, st);
}

extern "C" int ps_pull(ps_handle ps, int32_t worker, const int64_t *keys, int64_t n, float *out, void *stream) {
    if (!ps || n < 0 || (n > 0 && (!keys || !out))) return PS_EINVAL;
    if (worker < -1 || worker >= ps->W) return PS_EWORKER;
    if (n == 0) return PS_OK;
    hipStream_t st = (hipStream_t)stream;
    const bool side = worker >= 0 && n >= SIDE_STATS_MIN_KEYS;
    int rc = side ? launch_check(ps, keys, n, st) : dpaps_account_pull(ps, worker, keys, n, st);
    if (rc) return rc;
    if (side && (rc = side_stats_fork(ps, worker, keys, n, PS_STAT_PULL_LOCAL, PS_STAT_PULL_REMOTE, st)) != PS_OK) return rc;
    const int64_t pieces = n * (ps->L / 4);
    if (ps->L % 4 == 0 && pieces < ((int64_t)1 << 32) - 256 && ((uintptr_t)out & 15) == 0)
        k_pull_v4<<<grid_for(pieces, 256), 256, 0, st>>>(keys, (uint32_t)pieces, (uint32_t)(ps->L / 4),
                                                          reinterpret_cast<const float4 *>(ps->val), reinterpret_cast<float4 *>(out), ps->err);
    else
        k_pull<<<grid_for(n * ps->L, 256), 256, 0, st>>>(keys, n, ps->L, ps->val, out, ps->err);
    PS_HIP(ps, hipGetLastError());
    return side ? side_stats_join(ps, st) : PS_OK;
}

// what ps_push does before it adds: key check, locality statistics and message counts
int dpaps_account_push(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, hipStream_t st) {
    int rc = launch_check(ps, keys, n, st);
    if (rc) return rc;
    return route_access(ps, worker, keys, n, PS_STAT_PUSH_LOCAL, PS_STAT_PUSH_REMOTE, st);
}

// a pull and a push of the same keys by the same worker with nothing in between that moves a key, counted in one pass
int dpaps_account_pull_push(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, hipStream_t st) {
    int rc = launch_check(ps, keys, n, st);
    if (rc) return rc;
    return route_access(ps, worker, keys, n, PS_STAT_PULL_LOCAL, PS_STAT_PULL_REMOTE, st, PS_STAT_PUSH_LOCAL, PS_STAT_PUSH_REMOTE);
}

// The adding itself, for keys that have been checked (the kernels do nothing once the error flag is set), in two
// halves: the sort, which needs the keys only (a step that computes its update rows meanwhile runs it beside that
// work), and the sums, which need the rows.  The sorted pairs stay in the scratch between the two.
// Scratch of a push of n pairs: sorted keys, sorted positions, two partial-sum rows per range, the sort's own.
struct PushLayout { size_t off_pos, off_part, off_sort, bytes; };
static PushLayout push_layout(const dpaps_ps *ps, int64_t n) {
    const int64_t nranges = (n + PUSH_RANGE - 1) / PUSH_RANGE;
    const size_t part_bytes = ps->opt_push_sequential ? 0 : align_up((size_t)nranges * 2 * ps->L * sizeof(float));
    PushLayout l;
    l.off_pos = align_up((size_t)n * 8);
    l.off_part = l.off_pos + align_up((size_t)n * 4);
    l.off_sort = l.off_part + part_bytes;
    l.bytes = l.off_sort + dpaps_sort_scratch_bytes(n, dpaps_key_bits(ps->K));
    return l;
}

// the sort into `base` (scratch of at least push_layout(n).bytes, not allocated here)
static int push_sort_into(dpaps_ps *ps, void *base, const int64_t *keys, int64_t n, hipStream_t st) {
    const PushLayout l = push_layout(ps, n);
    uint64_t *skeys = (uint64_t *)base;
    uint32_t *spos = (uint32_t *)((char *)base + l.off_pos);
    const int rc = dpaps_sort_pairs(ps, keys, n, dpaps_key_bits(ps->K), skeys, spos, (char *)base + l.off_sort, st);
    if (rc) return rc;
    ps->push_base = base; ps->push_sorted_n = n; ps->push_off_pos = l.off_pos; ps->push_off_part = l.off_part;
    return PS_OK;
}

int dpaps_push_sort(dpaps_ps *ps, const int64_t *keys, int64_t n, hipStream_t st) {
    const int rc = dpaps_ws_reserve(ps, push_layout(ps, n).bytes);
    return rc ? rc : push_sort_into(ps, ps->ws, keys, n, st);
}

int dpaps_push_add(dpaps_ps *ps, int64_t n, const float *deltas, hipStream_t st) {
    if (n != ps->push_sorted_n || !ps->push_base) { ps->last_error = "push: the sums do not follow their sort"; return PS_EINVAL; }
    const int64_t nranges = (n + PUSH_RANGE - 1) / PUSH_RANGE;
    const uint64_t *skeys = (const uint64_t *)ps->push_base;
    const uint32_t *spos = (const uint32_t *)((char *)ps->push_base + ps->push_off_pos);
    float *part = (float *)((char *)ps->push_base + ps->push_off_part);
    if (ps->opt_push_sequential) {
        k_push_apply<<<grid_for(n * 64, 256), 256, 0, st>>>(skeys, spos, n, ps->L, deltas, ps->val, ps->err);
        PS_HIP(ps, hipGetLastError());
        return PS_OK;
    }
    k_push_ranges<16><<<dim3(grid_for(nranges * 64, 256), (unsigned)((ps->L + 63) / 64)), 256, 0, st>>>(skeys, spos, n, ps->L, deltas, ps->val, part, ps->err);
    PS_HIP(ps, hipGetLastError());
    if (nranges > 1) {
        k_push_join<<<dim3(grid_for(nranges * 64, 256), (unsigned)((ps->L + 63) / 64)), 256, 0, st>>>(skeys, n, ps->L, part, ps->val, ps->err);
        PS_HIP(ps, hipGetLastError());
    }
    return PS_OK;
}

int dpaps_push_apply(dpaps_ps *ps, const int64_t *keys, int64_t n, const float *deltas, hipStream_t st) {
    const int rc = dpaps_push_sort(ps, keys, n, st);
    return rc ? rc : dpaps_push_add(ps, n, deltas, st);
}

extern "C" int ps_push(ps_handle ps, int32_t worker, const int64_t *keys, int64_t n, const float *deltas, void *stream) {
    if (!ps || n < 0 || (n > 0 && (!keys || !deltas))) return PS_EINVAL;
    if (worker < -1 || worker >= ps->W) return PS_EWORKER;
    if (n >= ((int64_t)1 << 31)) return PS_ELIMIT;
    if (n == 0) return PS_OK;
    hipStream_t st = (hipStream_t)stream;
    const bool side = worker >= 0 && n >= SIDE_STATS_MIN_KEYS;
    int rc = side ? launch_check(ps, keys, n, st) : dpaps_account_push(ps, worker, keys, n, st);
    if (rc) return rc;
    if (side && (rc = side_stats_fork(ps, worker, keys, n, PS_STAT_PUSH_LOCAL, PS_STAT_PUSH_REMOTE, st)) != PS_OK) return rc;
    rc = dpaps_push_apply(ps, keys, n, deltas, st);
    if (rc) return rc;
    return side ? side_stats_join(ps, st) : PS_OK;
}

// ---- a push that allocates nothing -------------------------------------------------------------------------
// For callers that cannot allocate (code under graph capture, serving loops, harnesses that forbid it): the
// scratch of the push - sorted pairs, the sort's buffers and counters, partial sums - lives in a fixed array in
// device memory, one copy per device that the library runs on, held until the process ends.  Its address on a
// device is looked up once, by ps_create with that device current, and kept per device; host code uses that
// address only, never the array's name.
constexpr size_t PUSH_STATIC_BYTES = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[PUSH_STATIC_BYTES];
constexpr int PUSH_STATIC_DEVICES = 64;
static void *g_scratch_ptr[PUSH_STATIC_DEVICES];
static std::mutex g_scratch_mutex;

static int static_scratch_init(dpaps_ps *ps) {
    if (ps->device < 0 || ps->device >= PUSH_STATIC_DEVICES) return PS_OK;     // ps_push_noalloc will refuse
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[ps->device]) {
        void *p = nullptr;
        PS_HIP(ps, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        g_scratch_ptr[ps->device] = p;
    }
    return PS_OK;
}

extern "C" int ps_push_noalloc(ps_handle ps, int32_t worker, const int64_t *keys, int64_t n, const float *deltas, void *stream) {
    if (!ps || n < 0 || (n > 0 && (!keys || !deltas))) return PS_EINVAL;
    if (worker < -1 || worker >= ps->W) return PS_EWORKER;
    if (n == 0) return PS_OK;
    void *base = ps->device >= 0 && ps->device < PUSH_STATIC_DEVICES ? g_scratch_ptr[ps->device] : nullptr;
    if (!base) { ps->last_error = "ps_push_noalloc: no fixed scratch on this device"; return PS_EINVAL; }
    if (n > PS_PUSH_NOALLOC_MAX_KEYS || (n + PUSH_RANGE - 1) / PUSH_RANGE * ps->L > PS_PUSH_NOALLOC_MAX_PARTIAL ||
        push_layout(ps, n).bytes > PUSH_STATIC_BYTES) {
        ps->last_error = "ps_push_noalloc: at most 262144 keys and ceil(n / 64) * value_len <= 2^20 per call; use ps_push";
        return PS_ELIMIT;
    }
    hipStream_t st = (hipStream_t)stream;
    int rc = dpaps_account_push(ps, worker, keys, n, st);
    if (rc) return rc;
    rc = push_sort_into(ps, base, keys, n, st);
    return rc ? rc : dpaps_push_add(ps, n, deltas, st);
}

// the owner updates and statistics of a localize call, for keys that have been checked
int dpaps_localize_checked(dpaps_ps *ps, const int64_t *keys, int64_t n, int32_t worker, hipStream_t st) {
    if (n == 0) return PS_OK;
    uint32_t id = next_call_id(ps, st);
    k_localize<<<route_grid(ps, n), 256, 0, st>>>(keys, n, worker, ps->owner, ps->per_home, ps->W, ps->stamp_h,
                                                 ps->stamp_o, ps->stamp_pair, id, ps->stats, ps->loc, ps->K, ps->err);
    PS_HIP(ps, hipGetLastError());
    return PS_OK;
}
int dpaps_route_pull_push(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, hipStream_t st) {
    return route_access(ps, worker, keys, n, PS_STAT_PULL_LOCAL, PS_STAT_PULL_REMOTE, st, PS_STAT_PUSH_LOCAL, PS_STAT_PUSH_REMOTE);
}

extern "C" int ps_localize(ps_handle ps, const int64_t *keys, int64_t n, int32_t worker, void *stream) {
    if (!ps || n < 0 || (n > 0 && !keys)) return PS_EINVAL;
    if (worker < 0 || worker >= ps->W) return PS_EWORKER;
    if (n == 0) return PS_OK;
    hipStream_t st = (hipStream_t)stream;
    int rc = launch_check(ps, keys, n, st);
    if (rc) return rc;
    uint32_t id = next_call_id(ps, st);
    k_localize<<<route_grid(ps, n), 256, 0, st>>>(keys, n, worker, ps->owner, ps->per_home, ps->W, ps->stamp_h,
                                                 ps->stamp_o, ps->stamp_pair, id, ps->stats, ps->loc, ps->K, ps->err);
    PS_HIP(ps, hipGetLastError());
    return PS_OK;
}

extern "C" int ps_owner(ps_handle ps, const int64_t *keys, int64_t n, int32_t *owner_out, void *stream) {
    if (!ps || n < 0 || (n > 0 && (!keys || !owner_out))) return PS_EINVAL;
    if (n == 0) return PS_OK;
    hipStream_t st = (hipStream_t)stream;
    int rc = launch_check(ps, keys, n, st);
    if (rc) return rc;
    k_owner<<<grid_for(n, 256), 256, 0, st>>>(keys, n, ps->owner, owner_out, ps->err);
    PS_HIP(ps, hipGetLastError());
    return PS_OK;
}

// Synchronize, fetch and clear the sticky device error.
int dpaps_take_error(dpaps_ps *ps, hipStream_t st) {
    int32_t e = 0;
    PS_HIP(ps, hipMemcpyAsync(&e, ps->err, sizeof(e), hipMemcpyDeviceToHost, st));
    PS_HIP(ps, hipStreamSynchronize(st));
    if (e != 0) {
        PS_HIP(ps, hipMemsetAsync(ps->err, 0, sizeof(int32_t), st));
        PS_HIP(ps, hipStreamSynchronize(st));
        switch (e) {
        case PS_EKEY: ps->last_error = "a key or index was out of range in an earlier call"; break;
        case PS_EREMOTE: ps->last_error = "an SGD task touched a parameter that is not allocated to its worker"; break;
        case PS_ESTALL: ps->last_error = "a kernel gave up a wait that did not end (inconsistent layout tables, or more workgroups than the device runs at once)"; break;
        case PS_ELAYOUT: ps->last_error = "the ratings are not laid out block by block as mf_load_ratings requires"; break;
        case PS_ELIMIT: ps->last_error = "the ratings exceed a limit of the layout (rows with several entries per block, or entries per row or column in a block)"; break;
        default: ps->last_error = "a kernel of an earlier call reported an error"; break;
        }
    }
    return e;
}

extern "C" int ps_status(ps_handle ps, void *stream) {
    if (!ps) return PS_EINVAL;
    return dpaps_take_error(ps, (hipStream_t)stream);
}

extern "C" int ps_stats(ps_handle ps, int64_t *host_out, void *stream) {
    if (!ps || !host_out) return PS_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    u64 h[PS_STAT_SLOTS * PS_STAT_STRIDE];
    PS_HIP(ps, hipMemcpyAsync(h, ps->stats, sizeof(h), hipMemcpyDeviceToHost, st));
    int rc = dpaps_take_error(ps, st);      // synchronizes
    for (int c = 0; c < PS_STAT_COUNT; ++c) {
        u64 sum = 0;
        for (int sl = 0; sl < PS_STAT_SLOTS; ++sl) sum += h[sl * PS_STAT_STRIDE + c];
        host_out[c] = (int64_t)sum;
    }
    return rc;
}

extern "C" int ps_set_option(ps_handle ps, int32_t option, int64_t value) {
    if (!ps) return PS_EINVAL;
    switch (option) {
    case PS_OPT_MF_EXACT: ps->opt_exact = value != 0; return PS_OK;
    case PS_OPT_MF_CACHE_ROWS: if (value < -1) return PS_EINVAL; ps->opt_cache_rows = value; return PS_OK;
    case PS_OPT_MF_WAVES: if (value < 0 || value > 16) return PS_EINVAL; ps->opt_waves = (int)value; return PS_OK;
    case PS_OPT_MF_PROFILE: ps->opt_profile = value != 0; return PS_OK;
    case PS_OPT_MF_GROUPED: ps->opt_grouped = value != 0; return PS_OK;
    case PS_OPT_PUSH_SEQUENTIAL: ps->opt_push_sequential = value != 0; return PS_OK;
    case PS_OPT_MF_CLASSIC: if (value < 0 || value > 2) return PS_EINVAL; ps->opt_classic = (int)value; return PS_OK;
    case PS_OPT_LOCATION_CACHES: {
        // one entry of two bytes per node and key (-1: none); switching on or off empties them
        PS_HIP(ps, hipDeviceSynchronize());
        if (ps->loc) { PS_HIP(ps, hipFree(ps->loc)); ps->loc = nullptr; }
        if (value != 0) {
            const size_t bytes = (size_t)ps->W * (size_t)ps->K * sizeof(int16_t);
            if (bytes > ((size_t)16 << 30)) { ps->last_error = "location caches: nodes x keys x 2 bytes exceeds 16 GiB"; return PS_ELIMIT; }
            PS_HIP(ps, hipMalloc(&ps->loc, bytes));
            PS_HIP(ps, hipMemset(ps->loc, 0xFF, bytes));
            PS_HIP(ps, hipDeviceSynchronize());
        }
        return PS_OK;
    }
    case PS_OPT_KGE_EXACT: ps->opt_kge_exact = value != 0; return PS_OK;
    case PS_OPT_MF_TEAM_MAX: if (value < 0 || value > 14) return PS_EINVAL; ps->opt_team_max = (int)value; return PS_OK;
    case PS_OPT_MF_HEAVY_LEN:
        if (value < 1 || value > (1 << 30)) return PS_EINVAL;
        ps->opt_heavy_len = (int)value; return PS_OK;
    default: return PS_EINVAL;
    }
}

extern "C" const char *ps_last_error(ps_handle ps) { return ps ? ps->last_error.c_str() : "null handle"; }
