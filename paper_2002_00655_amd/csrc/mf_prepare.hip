// Data layout for parameter blocking (Sec. 2.2.2): storing the revealed entries
// block by block (mf_block_ratings) and deriving, from the stored order, what the
// SGD kernel needs to keep that order where it matters (mf_load_ratings).
// Integer work only; sorting and scanning use rocPRIM's device primitives.
#include "common.h"

#include <cstring>
#include <rocprim/device/device_radix_sort.hpp>
#include <rocprim/device/device_scan.hpp>
#include <rocprim/iterator/counting_iterator.hpp>

#include <algorithm>
#include <cstring>

static inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
static inline unsigned grid_for(int64_t n, int block) { return (unsigned)((n + block - 1) / block); }

#define HIPRC(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { rc = dpaps_fail_hip(ps, e_, #call); goto done; } } while (0)

// Simple bump allocator over one device allocation.
struct Arena {
    char *base = nullptr;
    size_t cap = 0, used = 0;
    template <class T> T *take(size_t count) {
        size_t off = align_up(used);
        used = off + count * sizeof(T);
        return base ? reinterpret_cast<T *>(base + off) : nullptr;
    }
};

// ---------------------------------------------------------------------------
// small kernels
// ---------------------------------------------------------------------------
// largest b with bounds[b] <= id (bounds[0] = 0, bounds non-decreasing; among equal bounds the last)
__device__ __forceinline__ int32_t block_of(const int64_t *bounds, int32_t d, int64_t id) {
    int32_t lo = 0, hi = d;   // invariant: bounds[lo] <= id < bounds[hi] (bounds[d] = size)
    while (hi - lo > 1) {
        int32_t mid = (lo + hi) >> 1;
        if (bounds[mid] <= id) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ void k_block_ids(const int32_t *rows, const int32_t *cols, int64_t nnz, int64_t m, int64_t n,
                            const int64_t *row_bounds, const int64_t *col_bounds, int32_t d_row, int32_t d_col,
                            uint32_t *blk, uint32_t *colcount /* d_row x n */, u64 *blk_hist, int32_t *err) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= nnz) return;
    int64_t i = rows[p], j = cols[p];
    if (i < 0 || i >= m || j < 0 || j >= n) { atomicExch(err, PS_EKEY); blk[p] = 0; return; }
    int32_t rb = block_of(row_bounds, d_row, i), cb = block_of(col_bounds, d_col, j);
    uint32_t b = (uint32_t)rb * (uint32_t)d_col + (uint32_t)cb;
    blk[p] = b;
    atomicAdd(&colcount[(int64_t)rb * n + j], 1u);
    atomicAdd(&blk_hist[b], (u64)1);
}

__global__ void k_iota(uint32_t *a, int64_t n) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) a[p] = (uint32_t)p;
}

__global__ void k_gather_u32(const int32_t *src, const uint32_t *perm, int64_t n, uint32_t *dst) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < n) dst[p] = (uint32_t)src[perm[p]];
}

// key = block (high 32 bits) | 2^32-1 - (entries of this column in this row block) (low 32 bits)
__global__ void k_block_key(const uint32_t *blk, const int32_t *cols, const uint32_t *colcount, const uint32_t *perm,
                            int64_t nnz, int64_t n, int32_t d_col, uint64_t *key) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= nnz) return;
    uint32_t src = perm[p];
    uint32_t b = blk[src];
    uint32_t cnt = colcount[(int64_t)(b / (uint32_t)d_col) * n + cols[src]];
    key[p] = ((uint64_t)b << 32) | (uint64_t)(0xFFFFFFFFu - cnt);
}

__global__ void k_permute_entries(const int32_t *rows, const int32_t *cols, const float *vals, const uint32_t *perm,
                                  int64_t nnz, int32_t *rows_out, int32_t *cols_out, float *vals_out) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= nnz) return;
    uint32_t s = perm[p];
    rows_out[p] = rows[s]; cols_out[p] = cols[s]; vals_out[p] = vals[s];
}

// ---------------------------------------------------------------------------
// mf_block_ratings
// ---------------------------------------------------------------------------
static int check_bounds(const int64_t *b, int32_t d, int64_t size) {
    if (!b || b[0] != 0 || b[d] != size) return PS_EINVAL;
    for (int32_t i = 0; i < d; ++i) if (b[i + 1] < b[i]) return PS_EINVAL;
    return PS_OK;
}

extern "C" int mf_block_ratings(int64_t m, int64_t n, int64_t nnz, const int32_t *rows, const int32_t *cols,
                                const float *vals, int32_t d_row, int32_t d_col, const int64_t *row_bounds_host,
                                const int64_t *col_bounds_host, int32_t *rows_out, int32_t *cols_out, float *vals_out,
                                int64_t *block_ptr_host_out, void *stream) {
    dpaps_ps *ps = nullptr;
    if (m <= 0 || n <= 0 || nnz < 0 || d_row <= 0 || d_col <= 0 || !block_ptr_host_out) return PS_EINVAL;
    if (nnz > 0 && (!rows || !cols || !vals || !rows_out || !cols_out || !vals_out)) return PS_EINVAL;
    if (m >= ((int64_t)1 << 31) || n >= ((int64_t)1 << 31) || nnz >= ((int64_t)1 << 32)) return PS_ELIMIT;
    if ((int64_t)d_row * d_col >= ((int64_t)1 << 31)) return PS_ELIMIT;
    if (check_bounds(row_bounds_host, d_row, m) || check_bounds(col_bounds_host, d_col, n)) return PS_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    const int64_t nb = (int64_t)d_row * d_col;
    int rc = PS_OK;
    char *dev = nullptr;
    std::vector<u64> hist((size_t)nb);
    int32_t h_err = 0;

    // sizes of the sort scratch (the same for all three passes: take the 64-bit one)
    size_t tmp32 = 0, tmp64 = 0;
    Arena a;
    for (int pass = 0; pass < 2; ++pass) {   // pass 0 measures, pass 1 hands out
        a.used = 0;
        int64_t *d_rb = a.take<int64_t>(d_row + 1), *d_cb = a.take<int64_t>(d_col + 1);
        uint32_t *blk = a.take<uint32_t>(nnz), *colcount = a.take<uint32_t>((size_t)d_row * n);
        u64 *blk_hist = a.take<u64>(nb);
        int32_t *d_err = a.take<int32_t>(1);
        uint32_t *perm_a = a.take<uint32_t>(nnz), *perm_b = a.take<uint32_t>(nnz);
        uint32_t *k32_a = a.take<uint32_t>(nnz), *k32_b = a.take<uint32_t>(nnz);
        uint64_t *k64_a = a.take<uint64_t>(nnz), *k64_b = a.take<uint64_t>(nnz);
        if (pass == 0) {
            HIPRC(rocprim::radix_sort_pairs(nullptr, tmp32, k32_a, k32_b, perm_a, perm_b, (size_t)nnz, 0, 32, st));
            HIPRC(rocprim::radix_sort_pairs(nullptr, tmp64, k64_a, k64_b, perm_a, perm_b, (size_t)nnz, 0, 64, st));
        }
        char *tmp = a.take<char>(std::max(tmp32, tmp64) + 256);
        if (pass == 0) {
            HIPRC(hipMalloc(&dev, a.used + 256));
            a.base = dev;
            continue;
        }
        HIPRC(hipMemcpyAsync(d_rb, row_bounds_host, (d_row + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
        HIPRC(hipMemcpyAsync(d_cb, col_bounds_host, (d_col + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
        HIPRC(hipMemsetAsync(colcount, 0, (size_t)d_row * n * sizeof(uint32_t), st));
        HIPRC(hipMemsetAsync(blk_hist, 0, nb * sizeof(u64), st));
        HIPRC(hipMemsetAsync(d_err, 0, sizeof(int32_t), st));
        if (nnz > 0) {
            k_block_ids<<<grid_for(nnz, 256), 256, 0, st>>>(rows, cols, nnz, m, n, d_rb, d_cb, d_row, d_col, blk, colcount,
                                                            blk_hist, d_err);
            // three stable passes, least significant key first: row, column, (block, busiest column first)
            k_iota<<<grid_for(nnz, 256), 256, 0, st>>>(perm_a, nnz);
            k_gather_u32<<<grid_for(nnz, 256), 256, 0, st>>>(rows, perm_a, nnz, k32_a);
            int row_bits = 1; while (((int64_t)1 << row_bits) < m) ++row_bits;
            int col_bits = 1; while (((int64_t)1 << col_bits) < n) ++col_bits;
            HIPRC(rocprim::radix_sort_pairs(tmp, tmp32, k32_a, k32_b, perm_a, perm_b, (size_t)nnz, 0, row_bits, st));
            k_gather_u32<<<grid_for(nnz, 256), 256, 0, st>>>(cols, perm_b, nnz, k32_a);
            HIPRC(rocprim::radix_sort_pairs(tmp, tmp32, k32_a, k32_b, perm_b, perm_a, (size_t)nnz, 0, col_bits, st));
            k_block_key<<<grid_for(nnz, 256), 256, 0, st>>>(blk, cols, colcount, perm_a, nnz, n, d_col, k64_a);
            int blk_bits = 1; while (((int64_t)1 << blk_bits) < nb) ++blk_bits;
            HIPRC(rocprim::radix_sort_pairs(tmp, tmp64, k64_a, k64_b, perm_a, perm_b, (size_t)nnz, 0, 32 + blk_bits, st));
            k_permute_entries<<<grid_for(nnz, 256), 256, 0, st>>>(rows, cols, vals, perm_b, nnz, rows_out, cols_out, vals_out);
            HIPRC(hipGetLastError());
        }
        HIPRC(hipMemcpyAsync(hist.data(), blk_hist, nb * sizeof(u64), hipMemcpyDeviceToHost, st));
        HIPRC(hipMemcpyAsync(&h_err, d_err, sizeof(int32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipStreamSynchronize(st));
    }
    if (h_err) { rc = h_err; goto done; }
    block_ptr_host_out[0] = 0;
    for (int64_t b = 0; b < nb; ++b) block_ptr_host_out[b + 1] = block_ptr_host_out[b] + (int64_t)hist[(size_t)b];
done:
    if (dev) (void)hipFree(dev);
    return rc;
}

// ---------------------------------------------------------------------------
// mf_load_ratings
// ---------------------------------------------------------------------------
void dpaps_mf_free(dpaps_ps *ps) {
    MfData &f = ps->mf;
    void *ptrs[] = {f.row, f.val, f.info, f.col, f.run_start, f.run_col, f.blk_run_ptr, f.multi_row, f.blk_multi_ptr,
                    f.row_bounds, f.col_bounds, f.blk_nheavy, f.t_cinfo, f.t_val, f.trun_start, f.trun_row, f.trun_wait, f.trun_ci, f.trun_val, f.trun_col,
                    f.blk_trun_ptr, f.run_gptr, f.gstart, f.team_plan};
    for (void *p : ptrs) if (p) (void)hipFree(p);
    ps->mf = MfData();
}

// block of each stored position, from the block pointer array
__global__ void k_pos_block(const int64_t *block_ptr, int64_t nb, int64_t nnz, uint32_t *blk) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= nnz) return;
    int64_t lo = 0, hi = nb;          // block_ptr[lo] <= p < block_ptr[hi]
    while (hi - lo > 1) {
        int64_t mid = (lo + hi) >> 1;
        if (block_ptr[mid] <= p) lo = mid; else hi = mid;
    }
    blk[p] = (uint32_t)lo;
}

// checks every entry against its block's ranges, flags the heads of column
// runs, and marks each (row block, column) pair once per run: a pair marked
// twice means a column's entries are not contiguous inside the block.
__global__ void k_run_heads(const int32_t *rows, const int32_t *cols, const uint32_t *blk, const int64_t *block_ptr,
                            const int64_t *row_bounds, const int64_t *col_bounds, int32_t d_col, int64_t m, int64_t n,
                            int64_t nnz, uint32_t *head, uint32_t *seen_bits, int32_t *err) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= nnz) return;
    uint32_t b = blk[p];
    int32_t rb = (int32_t)(b / (uint32_t)d_col), cb = (int32_t)(b % (uint32_t)d_col);
    int64_t i = rows[p], j = cols[p];
    if (i < 0 || i >= m || j < 0 || j >= n) { atomicExch(err, PS_EKEY); head[p] = 0; return; }
    if (i < row_bounds[rb] || i >= row_bounds[rb + 1] || j < col_bounds[cb] || j >= col_bounds[cb + 1]) {
        atomicExch(err, PS_ELAYOUT); head[p] = 0; return;
    }
    bool is_head = (p == block_ptr[b]) || cols[p - 1] != (int32_t)j;
    head[p] = is_head ? 1u : 0u;
    if (is_head) {
        int64_t bit = (int64_t)rb * n + j;
        uint32_t mask = 1u << (bit & 31);
        if (atomicOr(&seen_bits[bit >> 5], mask) & mask) atomicExch(err, PS_ELAYOUT);
    }
}

__global__ void k_run_fill(const uint32_t *head, const uint32_t *run_idx /* exclusive scan of head */,
                           const int32_t *cols, int64_t nnz, int64_t *run_start, int32_t *run_col) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= nnz) return;
    if (head[p]) { run_start[run_idx[p]] = p; run_col[run_idx[p]] = cols[p]; }
}

__global__ void k_blk_ptr_from_scan(const int64_t *block_ptr, int64_t nb, int64_t nnz, const uint32_t *excl,
                                    int64_t total, int64_t *out /* nb+1 */) {
    int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b > nb) return;
    int64_t p = b == nb ? nnz : block_ptr[b];
    out[b] = p >= nnz ? total : (int64_t)excl[p];
}

__global__ void k_row_key(const uint32_t *blk, const int32_t *rows, int64_t nnz, uint64_t *key) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p < nnz) key[p] = ((uint64_t)blk[p] << 32) | (uint32_t)rows[p];
}

// in the order sorted by (block, row): head of a group of equal keys
__global__ void k_seg_heads(const uint64_t *skey, int64_t nnz, uint32_t *head) {
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q < nnz) head[q] = (q == 0 || skey[q] != skey[q - 1]) ? 1u : 0u;
}

__global__ void k_seg_starts(const uint32_t *head, const uint32_t *seg_idx, int64_t nnz, uint32_t *seg_start) {
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q < nnz && head[q]) seg_start[seg_idx[q]] = (uint32_t)q;
}

// a group with two or more entries is a "multi" row of its block
__global__ void k_multi_flags(const uint32_t *seg_start, int64_t nseg, int64_t nnz, uint32_t *is_multi) {
    int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= nseg) return;
    int64_t end = s + 1 < nseg ? seg_start[s + 1] : nnz;
    is_multi[s] = (end - seg_start[s]) >= 2 ? 1u : 0u;
}

// multi rows in (block, row) order: sort key = block | 65535 - min(count, 65535), so that a stable sort
// puts, inside a block, the busiest rows first and rows of equal count by increasing row
__global__ void k_multi_fill(const uint32_t *seg_start, const uint32_t *is_multi, const uint32_t *multi_idx,
                             const uint64_t *skey, int64_t nseg, int64_t nnz, uint64_t *mkey, uint32_t *mseg,
                             u64 *blk_multi_hist) {
    int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= nseg || !is_multi[s]) return;
    int64_t end = s + 1 < nseg ? seg_start[s + 1] : nnz;
    int64_t cnt = end - seg_start[s];
    uint64_t b = skey[seg_start[s]] >> 32;
    uint32_t mi = multi_idx[s];
    mkey[mi] = (b << 16) | (uint64_t)(65535 - (cnt > 65535 ? 65535 : cnt));
    mseg[mi] = (uint32_t)s;
    atomicAdd(&blk_multi_hist[b], (u64)1);
}

// after sorting the multi rows by that key: slot = rank inside the block
__global__ void k_multi_slots(const uint64_t *mkey_sorted, const uint32_t *mseg_sorted, int64_t nmulti,
                              const int64_t *blk_multi_ptr, const uint32_t *seg_start, const uint64_t *skey,
                              int32_t *multi_row, uint32_t *seg_slot, int32_t *err) {
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nmulti) return;
    uint64_t b = mkey_sorted[t] >> 16;
    int64_t slot = t - blk_multi_ptr[b];
    uint32_t s = mseg_sorted[t];
    multi_row[t] = (int32_t)(uint32_t)(skey[seg_start[s]] & 0xFFFFFFFFu);
    if (slot >= 65535) { atomicExch(err, PS_ELIMIT); slot = 65534; }
    seg_slot[s] = (uint32_t)slot;
}

// info word of every entry: bits 0-15 ticket slot of its row in the block (0xFFFF: the row's only entry
// there), bits 16-30 rank among that row's entries in the block, bit 31 set when the row's previous entry
// belongs to the same column (a cell revealed twice)
__global__ void k_entry_info(const uint32_t *spos, const uint32_t *seg_idx, const uint32_t *seg_start,
                             const uint32_t *is_multi, const uint32_t *seg_slot, const int32_t *cols, int64_t nnz,
                             uint32_t *info, int32_t *err) {
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= nnz) return;
    uint32_t s = seg_idx[q];
    uint32_t w = 0xFFFFu;
    if (is_multi[s]) {
        uint32_t seq = (uint32_t)q - seg_start[s];
        if (seq > 32767u) { atomicExch(err, PS_ELIMIT); seq = 32767u; }
        uint32_t repeat = (seq > 0 && cols[spos[q]] == cols[spos[q - 1]]) ? 1u : 0u;
        w = seg_slot[s] | (seq << 16) | (repeat << 31);
    }
    info[spos[q]] = w;
}

__global__ void k_incl_to_seg_idx(const uint32_t *incl, int64_t n, uint32_t *idx) {
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q < n) idx[q] = incl[q] - 1u;
}

// ---- split of a block into heavy column runs and the rest -----------------------------------------------
// heavy runs of a block: its leading runs of at least heavy_len entries, at most heavy_max of them (one per
// wavefront that processes heavy runs, so that all of them advance through the rows together)
__global__ void k_block_nheavy(const int64_t *blk_run_ptr, const int64_t *run_start, int64_t nb, int32_t heavy_len,
                               int32_t heavy_max, int32_t *nheavy, int32_t *max_tail_cols) {
    int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= nb) return;
    int64_t g0 = blk_run_ptr[b], g1 = blk_run_ptr[b + 1], g = g0;
    while (g < g1 && g - g0 < heavy_max && run_start[g + 1] - run_start[g] >= heavy_len) ++g;
    nheavy[b] = (int32_t)(g - g0);
    atomicMax(max_tail_cols, (int32_t)(g1 - g));
}

// per stored position: index of its run; whether it belongs to a non-heavy run; and the check that rows do
// not descend inside a non-heavy run
__global__ void k_tail_flags(const uint32_t *head, const uint32_t *run_excl, const uint32_t *blk, const int64_t *blk_run_ptr,
                             const int32_t *nheavy, const int32_t *rows, int64_t nnz, uint32_t *runidx, uint32_t *tflag,
                             int32_t *descends) {
    int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= nnz) return;
    uint32_t g = run_excl[p] + head[p] - 1u;
    uint32_t b = blk[p];
    bool tail = (int64_t)g >= blk_run_ptr[b] + nheavy[b];
    runidx[p] = g;
    tflag[p] = tail ? 1u : 0u;
    if (tail && !head[p] && rows[p] < rows[p - 1]) atomicExch(descends, 1);
}

// in the order sorted by (block, row): is the entry in the second part, and does it start a row run there
// (inside a row's group the entries of heavy runs come first, because heavy runs lead the block)
__global__ void k_tail_sorted(const uint32_t *spos, const uint32_t *tflag, const uint32_t *seg_idx, const uint32_t *seg_start,
                              int64_t nnz, uint32_t *tq, uint32_t *thead) {
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= nnz) return;
    uint32_t t = tflag[spos[q]];
    tq[q] = t;
    thead[q] = (t && (q == seg_start[seg_idx[q]] || !tflag[spos[q - 1]])) ? 1u : 0u;
}

__global__ void k_tail_fill(const uint32_t *spos, const uint32_t *tq, const uint32_t *tpos, const uint32_t *thead,
                            const uint32_t *tri, const uint32_t *seg_idx, const uint32_t *seg_start, const uint32_t *is_multi,
                            const uint32_t *seg_slot, const uint32_t *runidx, const uint32_t *blk, const int64_t *blk_run_ptr,
                            const int32_t *nheavy, const int64_t *run_start, const int32_t *rows, const float *vals,
                            int64_t nnz, uint32_t *t_cinfo, float *t_val, uint32_t *trun_start, int32_t *trun_row,
                            uint32_t *trun_wait, const int32_t *run_col, uint32_t *trun_ci, float *trun_val, int32_t *trun_col,
                            int32_t *err) {
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= nnz || !tq[q]) return;
    uint32_t p = spos[q], t = tpos[q], g = runidx[p], b = blk[p];
    int64_t cslot = (int64_t)g - (blk_run_ptr[b] + nheavy[b]);
    int64_t cseq = (int64_t)p - run_start[g];
    if (cslot >= 65535 || cseq > 32767) { atomicExch(err, PS_ELIMIT); cslot = 0; cseq = 0; }
    const uint32_t last = (int64_t)p + 1 == run_start[g + 1] ? 0x80000000u : 0u;      // the column's last entry in this block
    t_cinfo[t] = (uint32_t)cslot | ((uint32_t)cseq << 16) | last;
    t_val[t] = vals[p];
    if (thead[q]) {
        uint32_t j = tri[q], s = seg_idx[q];
        trun_ci[j] = (uint32_t)cslot | ((uint32_t)cseq << 16) | last;
        trun_val[j] = vals[p];
        trun_col[j] = run_col[g];
        uint32_t before = (uint32_t)q - seg_start[s];       // the row's entries in heavy runs
        trun_start[j] = t;
        trun_row[j] = rows[p];
        trun_wait[j] = (before > 0 && is_multi[s]) ? (seg_slot[s] | (before << 16)) : 0xFFFFFFFFu;
    }
}

// ---- groups of a heavy run ------------------------------------------------------------------------------
// A heavy run is processed in groups of at most 15 consecutive entries; a group also ends before an entry
// whose row's previous entry lies in the same column (so that the rows of a group are distinct).  Where the
// groups start depends on the data only, so it is worked out once: one thread per run walks its entries.
// fill == 0: cnt[r] = number of table entries of run r (groups + 1 for a heavy run, else 0);
// fill == 1: gstart[gptr[r] + g] = start of group g relative to the run's first entry, the last one = its length.
__global__ void k_run_groups(const int64_t *run_start, const uint32_t *blk, const int64_t *blk_run_ptr, const int32_t *nheavy,
                             const uint32_t *info, int64_t num_runs, int fill, uint32_t *cnt, const uint32_t *gptr,
                             int32_t *gstart) {
    int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= num_runs) return;
    const int64_t s0 = run_start[r], s1 = run_start[r + 1];
    const uint32_t b = blk[s0];
    if (r - blk_run_ptr[b] >= nheavy[b]) { if (!fill) cnt[r] = 0; return; }
    uint32_t ng = 0;
    int64_t p = s0;
    while (p < s1) {
        if (fill) gstart[gptr[r] + ng] = (int32_t)(p - s0);
        ++ng;
        int64_t q = p + 1;
        while (q < s1 && q - p < 15 && !((info[q] & 0xFFFFu) != 0xFFFFu && (info[q] >> 31) != 0u)) ++q;
        p = q;
    }
    if (fill) gstart[gptr[r] + ng] = (int32_t)(s1 - s0); else cnt[r] = ng + 1;
}

// out = max(out, the largest of src[0 .. n)) (out starts at zero)
__global__ void k_max_u32(const uint32_t *src, int64_t n, uint32_t *out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t v = i < n ? src[i] : 0u;
    for (int off = 32; off > 0; off >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, off));
    if ((threadIdx.x & 63) == 0 && v > 0) atomicMax(out, v);
}

__global__ void k_widen_u32(const uint32_t *src, int64_t n, int64_t last, int64_t *dst) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i]; else if (i == n) dst[i] = last;
}

extern "C" int mf_load_ratings(ps_handle ps, int64_t m, int64_t n, int64_t nnz, const int32_t *rows, const int32_t *cols,
                               const float *vals, int32_t d_row, int32_t d_col, const int64_t *row_bounds_host,
                               const int64_t *col_bounds_host, const int64_t *block_ptr_host, void *stream) {
    if (!ps || m <= 0 || n <= 0 || nnz < 0 || d_row <= 0 || d_col <= 0 || !block_ptr_host) return PS_EINVAL;
    if (m + n != ps->K) return PS_EINVAL;
    if (ps->L > 256) { ps->last_error = "the SGD kernels take ranks up to 256"; return PS_ELIMIT; }
    if (nnz > 0 && (!rows || !cols || !vals)) return PS_EINVAL;
    if (m >= ((int64_t)1 << 31) || n >= ((int64_t)1 << 31) || nnz >= ((int64_t)1 << 32)) return PS_ELIMIT;
    if ((int64_t)d_row * d_col >= ((int64_t)1 << 31)) return PS_ELIMIT;
    if (check_bounds(row_bounds_host, d_row, m) || check_bounds(col_bounds_host, d_col, n)) return PS_EINVAL;
    const int64_t nb = (int64_t)d_row * d_col;
    if (block_ptr_host[0] != 0 || block_ptr_host[nb] != nnz) return PS_EINVAL;
    for (int64_t b = 0; b < nb; ++b) if (block_ptr_host[b + 1] < block_ptr_host[b]) return PS_EINVAL;

    hipStream_t st = (hipStream_t)stream;
    int rc = PS_OK;
    char *dev = nullptr;
    int32_t h_err = 0;
    uint32_t h_last[2] = {0, 0};
    int64_t num_runs = 0, nseg = 0, nmulti = 0;
    std::vector<u64> mhist;
    std::vector<int64_t> h_bmp;
    dpaps_mf_free(ps);
    MfData &f = ps->mf;

    size_t tmp_sort64 = 0, tmp_scan = 0, tmp_sortm = 0;
    Arena a;
    int64_t *d_bp = nullptr; uint32_t *blk = nullptr, *head = nullptr, *scan = nullptr, *seen = nullptr;
    int32_t *d_err = nullptr; uint64_t *key_a = nullptr, *key_b = nullptr; uint32_t *pos_a = nullptr, *pos_b = nullptr;
    uint32_t *seg_idx = nullptr, *seg_start = nullptr, *is_multi = nullptr, *multi_idx = nullptr, *seg_slot = nullptr;
    u64 *bm_hist = nullptr; char *tmp = nullptr;
    uint32_t *runidx = nullptr, *tflag = nullptr, *tq = nullptr, *tpos = nullptr;
    int32_t *d_aux = nullptr;          // [0] largest number of non-heavy runs in a block, [1] rows descend in such a run
    int32_t h_aux[2] = {0, 0};
    uint32_t h_tail[4] = {0, 0, 0, 0};
    int64_t nt = 0, ntr = 0;
    const size_t seen_words = (size_t)(((int64_t)d_row * n + 31) / 32);
    for (int pass = 0; pass < 2; ++pass) {
        a.used = 0;
        d_bp = a.take<int64_t>(nb + 1);
        blk = a.take<uint32_t>(nnz); head = a.take<uint32_t>(nnz + 1); scan = a.take<uint32_t>(nnz + 1);
        seen = a.take<uint32_t>(seen_words);
        d_err = a.take<int32_t>(1);
        key_a = a.take<uint64_t>(nnz); key_b = a.take<uint64_t>(nnz);
        pos_a = a.take<uint32_t>(nnz); pos_b = a.take<uint32_t>(nnz);
        seg_idx = a.take<uint32_t>(nnz); seg_start = a.take<uint32_t>(nnz + 1);
        is_multi = a.take<uint32_t>(nnz + 1); multi_idx = a.take<uint32_t>(nnz + 1); seg_slot = a.take<uint32_t>(nnz + 1);
        bm_hist = a.take<u64>(nb);
        runidx = a.take<uint32_t>(nnz + 1); tflag = a.take<uint32_t>(nnz + 1);
        tq = a.take<uint32_t>(nnz + 1); tpos = a.take<uint32_t>(nnz + 1);
        d_aux = a.take<int32_t>(2);
        if (pass == 0) {
            HIPRC(rocprim::radix_sort_pairs(nullptr, tmp_sort64, key_a, key_b, pos_a, pos_b, (size_t)std::max<int64_t>(nnz, 1), 0, 64, st));
            HIPRC(rocprim::exclusive_scan(nullptr, tmp_scan, head, scan, 0u, (size_t)std::max<int64_t>(nnz, 1), rocprim::plus<uint32_t>(), st));
            size_t t2 = 0;
            HIPRC(rocprim::inclusive_scan(nullptr, t2, head, scan, (size_t)std::max<int64_t>(nnz, 1), rocprim::plus<uint32_t>(), st));
            tmp_scan = std::max(tmp_scan, t2);
        }
        tmp = a.take<char>(std::max(tmp_sort64, tmp_scan) + 256);
        if (pass == 0) {
            HIPRC(hipMalloc(&dev, a.used + 256));
            a.base = dev;
        }
    }
    (void)tmp_sortm;

    // persistent arrays
    f.m = m; f.n = n; f.nnz = nnz; f.d_row = d_row; f.d_col = d_col; f.num_blocks = nb;
    f.h_row_bounds.assign(row_bounds_host, row_bounds_host + d_row + 1);
    f.h_col_bounds.assign(col_bounds_host, col_bounds_host + d_col + 1);
    f.h_block_ptr.assign(block_ptr_host, block_ptr_host + nb + 1);
    for (int32_t i = 0; i < d_row; ++i) f.max_block_rows = std::max(f.max_block_rows, row_bounds_host[i + 1] - row_bounds_host[i]);
    for (int32_t i = 0; i < d_col; ++i) f.max_block_cols = std::max(f.max_block_cols, col_bounds_host[i + 1] - col_bounds_host[i]);
    HIPRC(hipMalloc(&f.row_bounds, (d_row + 1) * sizeof(int64_t)));
    HIPRC(hipMalloc(&f.col_bounds, (d_col + 1) * sizeof(int64_t)));
    HIPRC(hipMalloc(&f.blk_run_ptr, (nb + 1) * sizeof(int64_t)));
    HIPRC(hipMalloc(&f.blk_multi_ptr, (nb + 1) * sizeof(int64_t)));
    HIPRC(hipMalloc(&f.row, std::max<size_t>(nnz, 1) * sizeof(int32_t)));
    HIPRC(hipMalloc(&f.col, std::max<size_t>(nnz, 1) * sizeof(int32_t)));
    HIPRC(hipMalloc(&f.val, std::max<size_t>(nnz, 1) * sizeof(float)));
    HIPRC(hipMalloc(&f.info, std::max<size_t>(nnz, 1) * sizeof(uint32_t)));
    HIPRC(hipMemcpyAsync(f.row_bounds, row_bounds_host, (d_row + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
    HIPRC(hipMemcpyAsync(f.col_bounds, col_bounds_host, (d_col + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
    HIPRC(hipMemcpyAsync(d_bp, block_ptr_host, (nb + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
    HIPRC(hipMemsetAsync(d_err, 0, sizeof(int32_t), st));
    HIPRC(hipMemsetAsync(seen, 0, seen_words * sizeof(uint32_t), st));
    HIPRC(hipMemsetAsync(bm_hist, 0, nb * sizeof(u64), st));

    if (nnz > 0) {
        HIPRC(hipMemcpyAsync(f.row, rows, nnz * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        HIPRC(hipMemcpyAsync(f.col, cols, nnz * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        HIPRC(hipMemcpyAsync(f.val, vals, nnz * sizeof(float), hipMemcpyDeviceToDevice, st));
        // --- column runs -------------------------------------------------
        k_pos_block<<<grid_for(nnz, 256), 256, 0, st>>>(d_bp, nb, nnz, blk);
        k_run_heads<<<grid_for(nnz, 256), 256, 0, st>>>(f.row, f.col, blk, d_bp, f.row_bounds, f.col_bounds, d_col, m, n, nnz,
                                                        head, seen, d_err);
        HIPRC(rocprim::exclusive_scan(tmp, tmp_scan, head, scan, 0u, (size_t)nnz, rocprim::plus<uint32_t>(), st));
        HIPRC(hipMemcpyAsync(&h_last[0], scan + (nnz - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipMemcpyAsync(&h_last[1], head + (nnz - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipMemcpyAsync(&h_err, d_err, sizeof(int32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipStreamSynchronize(st));
        if (h_err) { rc = h_err; goto done; }
        num_runs = (int64_t)h_last[0] + h_last[1];
    }
    f.num_runs = num_runs;
    HIPRC(hipMalloc(&f.run_start, (num_runs + 1) * sizeof(int64_t)));
    HIPRC(hipMalloc(&f.run_col, std::max<int64_t>(num_runs, 1) * sizeof(int32_t)));
    HIPRC(hipMemcpyAsync(f.run_start + num_runs, &f.nnz, sizeof(int64_t), hipMemcpyHostToDevice, st));
    if (nnz > 0) {
        k_run_fill<<<grid_for(nnz, 256), 256, 0, st>>>(head, scan, f.col, nnz, f.run_start, f.run_col);
    }
    k_blk_ptr_from_scan<<<grid_for(nb + 1, 256), 256, 0, st>>>(d_bp, nb, nnz, scan, num_runs, f.blk_run_ptr);
    HIPRC(hipGetLastError());
    // --- heavy runs and the rest ---------------------------------------------
    f.heavy_len = ps->opt_heavy_len;
    HIPRC(hipMalloc(&f.blk_nheavy, nb * sizeof(int32_t)));
    HIPRC(hipMalloc(&f.blk_trun_ptr, (nb + 1) * sizeof(int64_t)));
    HIPRC(hipMemsetAsync(d_aux, 0, 2 * sizeof(int32_t), st));
    k_block_nheavy<<<grid_for(nb, 256), 256, 0, st>>>(f.blk_run_ptr, f.run_start, nb, f.heavy_len, DPAPS_HEAVY_MAX, f.blk_nheavy, d_aux);
    if (nnz > 0) {
        k_tail_flags<<<grid_for(nnz, 256), 256, 0, st>>>(head, scan, blk, f.blk_run_ptr, f.blk_nheavy, f.row, nnz, runidx, tflag,
                                                         d_aux + 1);
    }
    HIPRC(hipGetLastError());

    if (nnz > 0) {
        // --- rows with several entries in a block --------------------------
        int blk_bits = 1; while (((int64_t)1 << blk_bits) < nb) ++blk_bits;
        k_row_key<<<grid_for(nnz, 256), 256, 0, st>>>(blk, f.row, nnz, key_a);
        k_iota<<<grid_for(nnz, 256), 256, 0, st>>>(pos_a, nnz);
        HIPRC(rocprim::radix_sort_pairs(tmp, tmp_sort64, key_a, key_b, pos_a, pos_b, (size_t)nnz, 0, 32 + blk_bits, st));
        // key_b / pos_b: sorted by (block, row), equal keys in stored order
        k_seg_heads<<<grid_for(nnz, 256), 256, 0, st>>>(key_b, nnz, head);
        HIPRC(rocprim::inclusive_scan(tmp, tmp_scan, head, scan, (size_t)nnz, rocprim::plus<uint32_t>(), st));
        k_incl_to_seg_idx<<<grid_for(nnz, 256), 256, 0, st>>>(scan, nnz, seg_idx);
        HIPRC(hipMemcpyAsync(&h_last[0], scan + (nnz - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipStreamSynchronize(st));
        nseg = h_last[0];
        k_seg_starts<<<grid_for(nnz, 256), 256, 0, st>>>(head, seg_idx, nnz, seg_start);
        k_multi_flags<<<grid_for(nseg, 256), 256, 0, st>>>(seg_start, nseg, nnz, is_multi);
        HIPRC(rocprim::exclusive_scan(tmp, tmp_scan, is_multi, multi_idx, 0u, (size_t)nseg, rocprim::plus<uint32_t>(), st));
        HIPRC(hipMemcpyAsync(&h_last[0], multi_idx + (nseg - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipMemcpyAsync(&h_last[1], is_multi + (nseg - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipStreamSynchronize(st));
        nmulti = (int64_t)h_last[0] + h_last[1];
    }
    f.num_multi = nmulti;
    HIPRC(hipMalloc(&f.multi_row, std::max<int64_t>(nmulti, 1) * sizeof(int32_t)));
    mhist.assign((size_t)nb, 0);
    h_bmp.assign((size_t)nb + 1, 0);
    if (nmulti > 0) {
        // key_a (as mkey) and pos_a (as mseg) are free again
        uint64_t *mkey = key_a; uint32_t *mseg = pos_a;
        uint64_t *mkey_s = key_a + (nnz + 1) / 2;          // nmulti <= nnz / 2
        uint32_t *mseg_s = pos_a + (nnz + 1) / 2;
        k_multi_fill<<<grid_for(nseg, 256), 256, 0, st>>>(seg_start, is_multi, multi_idx, key_b, nseg, nnz, mkey, mseg, bm_hist);
        int blk_bits = 1; while (((int64_t)1 << blk_bits) < nb) ++blk_bits;
        size_t need = 0;
        HIPRC(rocprim::radix_sort_pairs(nullptr, need, mkey, mkey_s, mseg, mseg_s, (size_t)nmulti, 0, 16 + blk_bits, st));
        if (need > std::max(tmp_sort64, tmp_scan)) { rc = PS_ENOMEM; ps->last_error = "sort scratch too small"; goto done; }
        HIPRC(rocprim::radix_sort_pairs(tmp, need, mkey, mkey_s, mseg, mseg_s, (size_t)nmulti, 0, 16 + blk_bits, st));
        HIPRC(hipMemcpyAsync(mhist.data(), bm_hist, nb * sizeof(u64), hipMemcpyDeviceToHost, st));
        HIPRC(hipStreamSynchronize(st));
        int64_t mx = 0;
        for (int64_t b = 0; b < nb; ++b) { h_bmp[b + 1] = h_bmp[b] + (int64_t)mhist[(size_t)b]; mx = std::max<int64_t>(mx, (int64_t)mhist[(size_t)b]); }
        f.max_multi_in_block = (int32_t)std::min<int64_t>(mx, 65535);
        HIPRC(hipMemcpyAsync(f.blk_multi_ptr, h_bmp.data(), (nb + 1) * sizeof(int64_t), hipMemcpyHostToDevice, st));
        k_multi_slots<<<grid_for(nmulti, 256), 256, 0, st>>>(mkey_s, mseg_s, nmulti, f.blk_multi_ptr, seg_start, key_b,
                                                            f.multi_row, seg_slot, d_err);
    } else {
        HIPRC(hipMemsetAsync(f.blk_multi_ptr, 0, (nb + 1) * sizeof(int64_t), st));
    }
    if (nnz > 0) {
        k_entry_info<<<grid_for(nnz, 256), 256, 0, st>>>(pos_b, seg_idx, seg_start, is_multi, seg_slot, f.col, nnz, f.info, d_err);
        HIPRC(hipGetLastError());
        HIPRC(hipMemcpyAsync(&h_err, d_err, sizeof(int32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipStreamSynchronize(st));
        if (h_err) { rc = h_err; goto done; }
    }
    // --- the non-heavy part once more, by (block, row, stored position) --------
    if (nnz > 0) {
        k_tail_sorted<<<grid_for(nnz, 256), 256, 0, st>>>(pos_b, tflag, seg_idx, seg_start, nnz, tq, head);
        HIPRC(rocprim::exclusive_scan(tmp, tmp_scan, tq, tpos, 0u, (size_t)nnz, rocprim::plus<uint32_t>(), st));
        HIPRC(rocprim::exclusive_scan(tmp, tmp_scan, head, scan, 0u, (size_t)nnz, rocprim::plus<uint32_t>(), st));
        HIPRC(hipMemcpyAsync(&h_tail[0], tpos + (nnz - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipMemcpyAsync(&h_tail[1], tq + (nnz - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipMemcpyAsync(&h_tail[2], scan + (nnz - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipMemcpyAsync(&h_tail[3], head + (nnz - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    }
    HIPRC(hipMemcpyAsync(h_aux, d_aux, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIPRC(hipStreamSynchronize(st));
    nt = (int64_t)h_tail[0] + h_tail[1];
    ntr = (int64_t)h_tail[2] + h_tail[3];
    f.num_tail = nt; f.num_truns = ntr;
    f.max_tail_cols = h_aux[0];
    f.sweep_ok = h_aux[1] == 0;
    HIPRC(hipMalloc(&f.t_cinfo, std::max<int64_t>(nt, 1) * sizeof(uint32_t)));
    HIPRC(hipMalloc(&f.t_val, std::max<int64_t>(nt, 1) * sizeof(float)));
    HIPRC(hipMalloc(&f.trun_start, (ntr + 1) * sizeof(uint32_t)));
    HIPRC(hipMalloc(&f.trun_row, std::max<int64_t>(ntr, 1) * sizeof(int32_t)));
    HIPRC(hipMalloc(&f.trun_wait, std::max<int64_t>(ntr, 1) * sizeof(uint32_t)));
    HIPRC(hipMalloc(&f.trun_ci, std::max<int64_t>(ntr, 1) * sizeof(uint32_t)));
    HIPRC(hipMalloc(&f.trun_val, std::max<int64_t>(ntr, 1) * sizeof(float)));
    HIPRC(hipMalloc(&f.trun_col, std::max<int64_t>(ntr, 1) * sizeof(int32_t)));
    {
        const uint32_t end = (uint32_t)nt;
        HIPRC(hipMemcpyAsync(f.trun_start + ntr, &end, sizeof(uint32_t), hipMemcpyHostToDevice, st));
    }
    if (nnz > 0) {
        k_tail_fill<<<grid_for(nnz, 256), 256, 0, st>>>(pos_b, tq, tpos, head, scan, seg_idx, seg_start, is_multi, seg_slot, runidx,
                                                        blk, f.blk_run_ptr, f.blk_nheavy, f.run_start, f.row, f.val, nnz, f.t_cinfo,
                                                        f.t_val, f.trun_start, f.trun_row, f.trun_wait, f.run_col, f.trun_ci, f.trun_val,
                                                        f.trun_col, d_err);
    }
    k_blk_ptr_from_scan<<<grid_for(nb + 1, 256), 256, 0, st>>>(d_bp, nb, nnz, scan, ntr, f.blk_trun_ptr);
    HIPRC(hipGetLastError());
    HIPRC(hipMemcpyAsync(&h_err, d_err, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIPRC(hipStreamSynchronize(st));
    if (h_err) { rc = h_err; goto done; }
    // --- where the groups of the heavy runs start (head / scan are free again) ----------------------
    HIPRC(hipMalloc(&f.run_gptr, (num_runs + 1) * sizeof(int64_t)));
    if (num_runs > 0) {
        if (num_runs >= ((int64_t)1 << 31)) { rc = PS_ELIMIT; goto done; }
        k_run_groups<<<grid_for(num_runs, 128), 128, 0, st>>>(f.run_start, blk, f.blk_run_ptr, f.blk_nheavy, f.info, num_runs, 0,
                                                              head, nullptr, nullptr);
        HIPRC(rocprim::exclusive_scan(tmp, tmp_scan, head, scan, 0u, (size_t)num_runs, rocprim::plus<uint32_t>(), st));
        HIPRC(hipMemcpyAsync(&h_tail[0], scan + (num_runs - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipMemcpyAsync(&h_tail[1], head + (num_runs - 1), sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        // the most groups of any run (head[r] = groups + 1 of a heavy run), into the error word, which is zero here
        uint32_t h_max = 0;
        k_max_u32<<<grid_for(num_runs, 256), 256, 0, st>>>(head, num_runs, reinterpret_cast<uint32_t *>(d_err));
        HIPRC(hipMemcpyAsync(&h_max, d_err, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        HIPRC(hipStreamSynchronize(st));
        f.num_gstart = (int64_t)h_tail[0] + h_tail[1];
        f.max_run_groups = h_max > 0 ? (int32_t)(h_max - 1) : 0;
    }
    HIPRC(hipMalloc(&f.gstart, std::max<int64_t>(f.num_gstart, 1) * sizeof(int32_t)));
    k_widen_u32<<<grid_for(num_runs + 1, 256), 256, 0, st>>>(scan, num_runs, f.num_gstart, f.run_gptr);
    if (num_runs > 0) {
        k_run_groups<<<grid_for(num_runs, 128), 128, 0, st>>>(f.run_start, blk, f.blk_run_ptr, f.blk_nheavy, f.info, num_runs, 1,
                                                              nullptr, scan, f.gstart);
    }
    HIPRC(hipGetLastError());
    HIPRC(hipStreamSynchronize(st));
done:
    if (dev) (void)hipFree(dev);
    if (rc != PS_OK) dpaps_mf_free(ps);
    return rc;
}
