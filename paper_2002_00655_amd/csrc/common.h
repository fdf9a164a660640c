// Internal declarations shared by the translation units of libdpaps.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "dpaps.h"

typedef unsigned long long u64;

#define PS_STAT_SLOTS 64
#define PS_STAT_STRIDE 16             // u64 per slot: one 128-byte line
__device__ __forceinline__ u64 *stat_slot(u64 *stats) { return stats + (size_t)(blockIdx.x % PS_STAT_SLOTS) * PS_STAT_STRIDE; }

// Device-resident description of the loaded ratings (built by mf_load_ratings).
struct MfData {
    int64_t m = 0, n = 0, nnz = 0;
    int32_t d_row = 0, d_col = 0;
    int64_t num_blocks = 0, num_runs = 0, num_multi = 0;
    int32_t max_multi_in_block = 0;   // largest number of rows with >= 2 entries in any block
    // per entry, in stored order
    int32_t *row = nullptr;           // global row index
    float *val = nullptr;
    uint32_t *info = nullptr;         // bits 0-15: ticket slot of the row in its block (0xFFFF: only entry of that
                                      // row in the block); bits 16-30: rank among the row's entries in the block;
                                      // bit 31: the row's previous entry is in the same column
    int32_t *col = nullptr;           // column of the entry (kept for mf_train_sse)
    // per column run (maximal group of consecutive entries of one column inside a block)
    int64_t *run_start = nullptr;     // num_runs + 1
    int32_t *run_col = nullptr;       // num_runs
    int64_t *blk_run_ptr = nullptr;   // num_blocks + 1, index into runs
    // rows with >= 2 entries in a block, per block, most frequent first
    int32_t *multi_row = nullptr;     // num_multi
    int64_t *blk_multi_ptr = nullptr; // num_blocks + 1
    // Split of every block for the grouped SGD kernel: its leading column runs of at least heavy_len entries
    // ("heavy" columns) are processed column by column, the entries of the other runs row by row.  That part
    // is kept a second time, ordered by (block, row, stored position):
    int64_t max_block_rows = 0, max_block_cols = 0;   // largest row block and column block
    int32_t heavy_len = 0;            // the threshold this split was made with
    bool sweep_ok = false;            // rows ascend inside every run of the second part (needed to walk it by rows)
    int32_t *blk_nheavy = nullptr;    // num_blocks: heavy runs of the block
    int64_t num_tail = 0, num_truns = 0;
    int32_t max_tail_cols = 0;        // largest number of non-heavy runs in any block
    uint32_t *t_cinfo = nullptr;      // num_tail: bits 0-15 index of the entry's run among the block's non-heavy runs,
                                      // bits 16-30 its rank inside that run, bit 31: it is the run's last entry
    float *t_val = nullptr;           // num_tail
    uint32_t *trun_start = nullptr;   // num_truns + 1: first entry of a row run
    int32_t *trun_row = nullptr;      // num_truns: global row index
    uint32_t *trun_wait = nullptr;    // num_truns: bits 0-15 ticket slot of the row, bits 16-31 the row's entries in heavy
                                      // runs (the ticket value to wait for); 0xFFFFFFFF: none
    uint32_t *trun_ci = nullptr;      // num_truns: t_cinfo, value and column of the row run's first entry, so that one
    float *trun_val = nullptr;        // read brings everything a row with a single entry needs
    int32_t *trun_col = nullptr;
    int64_t *blk_trun_ptr = nullptr;  // num_blocks + 1, index into row runs
    // where the groups of the heavy runs start: run r has run_gptr[r+1] - run_gptr[r] - 1 groups (none if it is not
    // heavy); gstart[run_gptr[r] + g] is the start of group g relative to the run's first entry, one more entry = length
    int64_t *run_gptr = nullptr;      // num_runs + 1
    int32_t *gstart = nullptr;        // num_gstart
    uint32_t *team_plan = nullptr;    // 16 words per block: which heavy runs each wavefront takes (built on first use)
    int team_plan_waves = 0;          // the number of heavy wavefronts it was built for
    int64_t num_gstart = 0;
    int32_t max_run_groups = 0;       // most groups of any heavy run
    // block geometry
    int64_t *row_bounds = nullptr;    // device copy, d_row + 1
    int64_t *col_bounds = nullptr;    // device copy, d_col + 1
    std::vector<int64_t> h_row_bounds, h_col_bounds, h_block_ptr;
};

struct dpaps_ps {
    int device = 0;
    int64_t K = 0;
    int32_t L = 0, W = 0;
    int64_t per_home = 0;
    float *val = nullptr;             // K x L, row-major, packed
    int32_t *owner = nullptr;         // K
    u64 *stats = nullptr;             // PS_STAT_SLOTS x PS_STAT_COUNT partial counters on the device (a workgroup
                                      // adds to slot blockIdx.x % PS_STAT_SLOTS, so that the atomics of one launch
                                      // spread over many cache lines); ps_stats adds the slots up
    int32_t *err = nullptr;           // sticky device error flag (0 = fine)
    // stamps for counting the distinct destinations of one call's messages
    uint32_t *stamp_h = nullptr, *stamp_o = nullptr, *stamp_pair = nullptr;
    uint32_t call_id = 0;
    // growable scratch for ps_push
    void *ws = nullptr;
    size_t ws_bytes = 0;
    void *push_base = nullptr;        // what the sort of a push left for its sums: the scratch it used,
    int64_t push_sorted_n = -1;       // the number of pairs,
    size_t push_off_pos = 0, push_off_part = 0;   // the offsets of the sorted positions and of the partial sums
    // schedule staging for mf_sgd_epoch
    int32_t *d_tasks = nullptr;
    int64_t d_tasks_cap = 0;
    std::vector<int32_t> h_tasks_cached;
    // options
    int opt_exact = 0;
    int64_t opt_cache_rows = -1;
    int opt_waves = 0;              // wavefronts per workgroup of the SGD kernels; 0: chosen by the library (dpaps_mf_waves)
    int opt_profile = 0;
    int opt_push_sequential = 0;      // 1: ps_push adds each key's terms strictly one after the other
    int opt_classic = 0;              // 1, 2: mf_sgd_epoch as on a classic parameter server (2: updates in place)
    int opt_team_max = 0;             // most wavefronts that share one heavy run; 0: chosen by the library (plan_teams)
    int opt_grouped = 1;              // 1: use the grouped SGD kernel where it applies
    int opt_kge_exact = 0;            // 1: the knowledge-graph step sums and divides in the order of a sequential fp32 program
    int opt_heavy_len = 48;           // column runs of a block at least this long are processed in groups
    // event pairs around the SGD kernel launches (only while profiling is on)
    std::vector<hipEvent_t> ev_pool;
    size_t ev_used = 0;
    // device limits
    int lds_bytes = 65536;
    int num_cu = 0;
    MfData mf;
    double *d_sse = nullptr;
    void *kge_ws = nullptr;           // scratch of kge_sgd_step (grows)
    size_t kge_ws_bytes = 0;
    int16_t *loc = nullptr;           // location caches (PS_OPT_LOCATION_CACHES): W x K, node n's belief where key k is, -1 none
    void *handoff_ws = nullptr;       // column block states and the recorded order of mf_sgd_epoch_handoff (grows)
    size_t handoff_ws_bytes = 0;
    hipStream_t side_stream = nullptr;   // default priority: the localize calls and statistics of kge_sgd_epoch run here
    hipEvent_t ev_fork = nullptr, ev_join = nullptr, ev_sorted = nullptr, ev_added = nullptr;
    std::string last_error;
};

// Heavy runs of a block at most.
#define DPAPS_HEAVY_MAX 8
// Column blocks at most in an epoch with hand-over (one bit each in LDS).
#define DPAPS_HANDOFF_MAX_COLS 4096

// Arguments of the SGD kernels (one launch = the tasks of one stratum).
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
    // second part of a block (grouped kernel only)
    const int32_t *blk_nheavy; const int64_t *blk_trun_ptr;
    const uint32_t *trun_start; const int32_t *trun_row; const uint32_t *trun_wait;
    const uint32_t *trun_ci; const float *trun_val; const int32_t *trun_col;
    const uint32_t *t_cinfo; const float *t_val;
    const int64_t *run_gptr; const int32_t *gstart;
    int32_t heavy_waves;        // wavefronts that take heavy runs (each has a staging area in LDS)
    int32_t team;               // 2: the heavy wavefronts follow team_plan; 1: one wavefront per heavy run, in turn
    const uint32_t *team_plan;  // 16 words per block (see k_team_plan)
    // the localize step of the subepoch, done by the same workgroup first (grouped kernel only)
    int32_t fuse_localize; int32_t W; int64_t per_home; int32_t *owner_w;
    int32_t ctick_cap;          // column ticket counters in LDS
    int32_t hcache_cap;         // column factors that fit in LDS
    float lr, lambda;
    u64 *stats;
    int32_t *err;
    // an epoch with hand-over of column blocks instead of barriers (k_mf_sgd_handoff only)
    uint32_t *col_state;        // d_col words: visits << 1 | held
    int32_t *sched;             // per worker and step: column block, visits before
    uint32_t take_spins;        // looks for a free column block after which a worker gives up (PS_ESTALL)
};

// mf_sgd_chunk.hip: the kernel that processes a column's entries in groups (see there)
int dpaps_launch_sgd_chunk(dpaps_ps *ps, const SgdArgs &a, int ntasks, int waves, hipStream_t st);
int dpaps_launch_sgd_handoff(dpaps_ps *ps, const SgdArgs &a, int workers, hipStream_t st);
int dpaps_mf_waves(const dpaps_ps *ps);

// ps_store.hip: the two halves of ps_pull and ps_push, for steps that read the store where they use the values
// and add up the update terms of one data point before they push them
int dpaps_account_pull(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, hipStream_t st);
int dpaps_account_push(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, hipStream_t st);
int dpaps_account_pull_push(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, hipStream_t st);
int dpaps_route_pull_push(dpaps_ps *ps, int32_t worker, const int64_t *keys, int64_t n, hipStream_t st);   // without the key check
int dpaps_localize_checked(dpaps_ps *ps, const int64_t *keys, int64_t n, int32_t worker, hipStream_t st);
int dpaps_push_apply(dpaps_ps *ps, const int64_t *keys, int64_t n, const float *deltas, hipStream_t st);
int dpaps_push_sort(dpaps_ps *ps, const int64_t *keys, int64_t n, hipStream_t st);     // the two halves of dpaps_push_apply
int dpaps_push_add(dpaps_ps *ps, int64_t n, const float *deltas, hipStream_t st);
int dpaps_check_keys(dpaps_ps *ps, const int64_t *keys, int64_t n, hipStream_t st);     // the key check of the dpaps_account_* calls

// key_sort.hip: stable sort of (key, position) pairs by key (see there)
int dpaps_key_bits(int64_t num_keys);
size_t dpaps_sort_scratch_bytes(int64_t n, int key_bits);
int dpaps_sort_pairs(dpaps_ps *ps, const int64_t *keys, int64_t n, int key_bits, uint64_t *skeys, uint32_t *spos, void *scratch, hipStream_t st);

int dpaps_side_stream(dpaps_ps *ps);   // creates the library's second stream and its events on first use
int dpaps_fail_hip(dpaps_ps *ps, hipError_t e, const char *what);
int dpaps_ws_reserve(dpaps_ps *ps, size_t bytes);

#define PS_HIP(ps, call)                                                   \
    do {                                                                   \
        hipError_t e_ = (call);                                            \
        if (e_ != hipSuccess) return dpaps_fail_hip((ps), e_, #call);      \
    } while (0)

__host__ __device__ inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }
