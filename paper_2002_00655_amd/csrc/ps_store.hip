// Parameter server primitives on one GPU: dense store, owner map, pull / push /
// localize and the integer routing statistics (Table "Primitives", Sec. 3.1-3.3,
// Sec. 3.5, Sec. 3.7 of the paper).
#include "common.h"

#include <cstring>
#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>
#include <rocprim/iterator/counting_iterator.hpp>

#include <cstdio>
#include <cstring>
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

__device__ __forceinline__ void wave_count_add(bool flag, u64 *counter) {
    u64 b = __ballot(flag);
    if (b != 0 && (threadIdx.x & 63) == (unsigned)(__ffsll((long long)__ballot(true)) - 1)) atomicAdd(counter, (u64)__popcll(b));
}

// One key that must travel for requester `worker`: home h, current owner o.
// Within one call the messages to one destination are grouped (Sec. 3.7); the
// stamps record which destinations this call has already been charged for.
__device__ __forceinline__ void route_key(bool travels, int32_t worker, int32_t h, int32_t o, int32_t W,
                                          uint32_t *stamp_h, uint32_t *stamp_o, uint32_t *stamp_pair, uint32_t call_id,
                                          u64 *c_req, u64 *c_fwd, u64 *c_back) {
    bool req = false, fwd = false, back = false;
    if (travels) {
        if (h != worker) req = atomicExch(&stamp_h[h], call_id) != call_id;
        bool fresh = atomicExch(&stamp_pair[(int64_t)h * W + o], call_id) != call_id;
        fwd = fresh && (h != o);
        if (o != worker) back = atomicExch(&stamp_o[o], call_id) != call_id;
    }
    wave_count_add(req, c_req);
    wave_count_add(fwd, c_fwd);
    wave_count_add(back, c_back);
}

// Locality statistics and message counts of one pull or push call.
__global__ void k_route_access(const int64_t *keys, int64_t n, int32_t worker, const int32_t *owner, int64_t per_home,
                               int32_t W, uint32_t *stamp_h, uint32_t *stamp_o, uint32_t *stamp_pair, uint32_t call_id,
                               u64 *stats, int stat_local, int stat_remote, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    stats = stat_slot(stats);
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool active = p < n;
    int64_t k = active ? keys[p] : 0;
    int32_t o = active ? owner[k] : 0;
    bool local = active && o == worker, remote = active && o != worker;
    wave_count_add(local, &stats[stat_local]);
    wave_count_add(remote, &stats[stat_remote]);
    route_key(remote, worker, (int32_t)(k / per_home), o, W, stamp_h, stamp_o, stamp_pair, call_id,
              &stats[PS_STAT_MSG_ACC_REQ], &stats[PS_STAT_MSG_ACC_FWD], &stats[PS_STAT_MSG_ACC_REPLY]);
}

// localize: the home node updates the location at once (Sec. 3.2, step 1); the
// exchange makes exactly one of several mentions of a key the one that moves it.
__global__ void k_localize(const int64_t *keys, int64_t n, int32_t worker, int32_t *owner, int64_t per_home, int32_t W,
                           uint32_t *stamp_h, uint32_t *stamp_o, uint32_t *stamp_pair, uint32_t call_id, u64 *stats,
                           const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    stats = stat_slot(stats);
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool active = p < n;
    int64_t k = active ? keys[p] : 0;
    int32_t old = worker;
    if (active) old = atomicExch(&owner[k], worker);
    bool moved = active && old != worker;
    wave_count_add(active, &stats[PS_STAT_LOCALIZE_KEYS]);
    wave_count_add(moved, &stats[PS_STAT_RELOCATED]);
    route_key(moved, worker, (int32_t)(k / per_home), old, W, stamp_h, stamp_o, stamp_pair, call_id,
              &stats[PS_STAT_MSG_LOC_REQ], &stats[PS_STAT_MSG_LOC_INSTRUCT], &stats[PS_STAT_MSG_LOC_TRANSFER]);
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

// push, after the (key, position) pairs have been sorted by key with a stable
// sort: one wavefront per sorted position; the wavefront at the head of a run
// of equal keys adds that key's update terms one after the other, in
// increasing position - the order a sequential server would apply them in.
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

// ---------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------
static inline unsigned grid_for(int64_t n, int block) { return (unsigned)((n + block - 1) / block); }

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

static uint32_t next_call_id(dpaps_ps *ps, hipStream_t st) {
    if (++ps->call_id == 0) {   // wrapped: forget all stamps
        size_t W = (size_t)ps->W;
        (void)hipMemsetAsync(ps->stamp_h, 0, (2 * W + W * W) * sizeof(uint32_t), st);
        ps->call_id = 1;
    }
    return ps->call_id;
}

static int route_access(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, int st_local, int st_remote,
                        hipStream_t st) {
    if (worker < 0 || n == 0) return PS_OK;
    uint32_t id = next_call_id(ps, st);
    k_route_access<<<grid_for(n, 256), 256, 0, st>>>(keys, n, worker, ps->owner, ps->per_home, ps->W, ps->stamp_h,
                                                     ps->stamp_o, ps->stamp_pair, id, ps->stats, st_local, st_remote,
                                                     ps->err);
    PS_HIP(ps, hipGetLastError());
    return PS_OK;
}

extern "C" int ps_pull(ps_handle ps, int32_t worker, const int64_t *keys, int64_t n, float *out, void *stream) {
    if (!ps || n < 0 || (n > 0 && (!keys || !out))) return PS_EINVAL;
    if (worker < -1 || worker >= ps->W) return PS_EWORKER;
    if (n == 0) return PS_OK;
    hipStream_t st = (hipStream_t)stream;
    int rc = launch_check(ps, keys, n, st);
    if (rc) return rc;
    rc = route_access(ps, worker, keys, n, PS_STAT_PULL_LOCAL, PS_STAT_PULL_REMOTE, st);
    if (rc) return rc;
    k_pull<<<grid_for(n * ps->L, 256), 256, 0, st>>>(keys, n, ps->L, ps->val, out, ps->err);
    PS_HIP(ps, hipGetLastError());
    return PS_OK;
}

extern "C" int ps_push(ps_handle ps, int32_t worker, const int64_t *keys, int64_t n, const float *deltas, void *stream) {
    if (!ps || n < 0 || (n > 0 && (!keys || !deltas))) return PS_EINVAL;
    if (worker < -1 || worker >= ps->W) return PS_EWORKER;
    if (n >= ((int64_t)1 << 31)) return PS_ELIMIT;
    if (n == 0) return PS_OK;
    hipStream_t st = (hipStream_t)stream;
    int rc = launch_check(ps, keys, n, st);
    if (rc) return rc;
    rc = route_access(ps, worker, keys, n, PS_STAT_PUSH_LOCAL, PS_STAT_PUSH_REMOTE, st);
    if (rc) return rc;

    // stable sort of (key, position) by key; the positions come from a counting iterator
    int key_bits = 1;
    while (key_bits < 63 && ((int64_t)1 << key_bits) < ps->K) ++key_bits;
    size_t temp_bytes = 0;
    const uint64_t *kin = reinterpret_cast<const uint64_t *>(keys);
    rocprim::counting_iterator<uint32_t> iota(0);
    PS_HIP(ps, rocprim::radix_sort_pairs(nullptr, temp_bytes, kin, (uint64_t *)nullptr, iota, (uint32_t *)nullptr,
                                         (size_t)n, 0, key_bits, st));
    size_t off_keys = 0, off_pos = align_up((size_t)n * 8), off_tmp = off_pos + align_up((size_t)n * 4);
    rc = dpaps_ws_reserve(ps, off_tmp + temp_bytes);
    if (rc) return rc;
    uint64_t *skeys = (uint64_t *)((char *)ps->ws + off_keys);
    uint32_t *spos = (uint32_t *)((char *)ps->ws + off_pos);
    void *tmp = (char *)ps->ws + off_tmp;
    PS_HIP(ps, rocprim::radix_sort_pairs(tmp, temp_bytes, kin, skeys, iota, spos, (size_t)n, 0, key_bits, st));
    k_push_apply<<<grid_for(n * 64, 256), 256, 0, st>>>(skeys, spos, n, ps->L, deltas, ps->val, ps->err);
    PS_HIP(ps, hipGetLastError());
    return PS_OK;
}

extern "C" int ps_localize(ps_handle ps, const int64_t *keys, int64_t n, int32_t worker, void *stream) {
    if (!ps || n < 0 || (n > 0 && !keys)) return PS_EINVAL;
    if (worker < 0 || worker >= ps->W) return PS_EWORKER;
    if (n == 0) return PS_OK;
    hipStream_t st = (hipStream_t)stream;
    int rc = launch_check(ps, keys, n, st);
    if (rc) return rc;
    uint32_t id = next_call_id(ps, st);
    k_localize<<<grid_for(n, 256), 256, 0, st>>>(keys, n, worker, ps->owner, ps->per_home, ps->W, ps->stamp_h,
                                                 ps->stamp_o, ps->stamp_pair, id, ps->stats, ps->err);
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
        ps->last_error = "a key or index was out of range in an earlier call";
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
    case PS_OPT_MF_WAVES: if (value < 1 || value > 16) return PS_EINVAL; ps->opt_waves = (int)value; return PS_OK;
    case PS_OPT_MF_PROFILE: ps->opt_profile = value != 0; return PS_OK;
    case PS_OPT_MF_GROUPED: ps->opt_grouped = value != 0; return PS_OK;
    case PS_OPT_MF_HEAVY_LEN:
        if (value < 1 || value > (1 << 30)) return PS_EINVAL;
        ps->opt_heavy_len = (int)value; return PS_OK;
    default: return PS_EINVAL;
    }
}

extern "C" const char *ps_last_error(ps_handle ps) { return ps ? ps->last_error.c_str() : "null handle"; }
