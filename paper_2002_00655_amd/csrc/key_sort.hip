// Stable sort of (key, position) pairs by key, for the cumulative push (Sec. 2.1: a push
// adds an update term to the stored value; Sec. 3.7: the operations on one key are applied
// one after the other).  A push with repeated keys must apply a key's terms in argument
// order, so the pairs are brought into the order (key, position) first.
//
// What is known here and a general sort cannot assume: keys are below num_keys (19 bits for
// half a million keys, 24 for eleven million), and positions are 0 .. n-1 in input order,
// so a stable sort by the key's digits alone yields (key, position) order and the positions
// need not be read in the first pass.  Least-significant-digit passes; each pass is
//   1. k_sort_count    one workgroup per tile of the input: how many pairs of the tile fall
//                      into each bucket (LDS counters), written bucket-major;
//   2. k_sort_rowsum   one workgroup per bucket: the bucket's total;
//   3. k_sort_scan     one workgroup per bucket: where the bucket starts (pairs in lower
//                      buckets) and, from there, where each tile's share of it starts;
//   4. k_sort_scatter  one workgroup per tile: a wavefront takes 64 consecutive pairs at a
//                      time; lanes with the same digit find each other with one ballot per
//                      bit of the digit, the first of them advances the wavefront's own
//                      counter of that bucket in LDS, the others take their place behind it
//                      in lane order; the wavefronts' counters are then turned into
//                      offsets in wavefront order, so that pairs of one bucket keep their
//                      input order - the pass is stable - and every pair is stored.
// Integer work only: the result is the same bit for bit whatever the scheduling.
#include "common.h"

namespace {

constexpr int SORT_THREADS = 256;          // 4 wavefronts per tile
constexpr int SORT_WAVES = SORT_THREADS / 64;
constexpr int SORT_MAX_BITS = 10;          // bits of a digit at most: 1024 buckets

__device__ __forceinline__ uint32_t digit_of(uint64_t key, int shift, uint32_t mask) { return (uint32_t)(key >> shift) & mask; }

// FIRST: the input is the caller's key array (int64, checked to be in range or the handle is frozen) and the
// positions are the indices; otherwise the pairs come from the previous pass.
template <int ITEMS, bool FIRST>
__global__ __launch_bounds__(SORT_THREADS) void k_sort_count(const int64_t *keys_in, const uint64_t *pk_in, int64_t n, int shift, int bits,
                                                             int64_t num_tiles, uint32_t *hist, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    __shared__ uint32_t cnt[1 << SORT_MAX_BITS];
    const int R = 1 << bits;
    const uint32_t mask = (uint32_t)R - 1u;
    for (int i = threadIdx.x; i < R; i += SORT_THREADS) cnt[i] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * (SORT_THREADS * ITEMS);
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        const int64_t q = base + (int64_t)r * SORT_THREADS + threadIdx.x;
        if (q < n) {
            const uint64_t k = FIRST ? (uint64_t)keys_in[q] : pk_in[q];
            atomicAdd(&cnt[digit_of(k, shift, mask)], 1u);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < R; i += SORT_THREADS) hist[(int64_t)i * num_tiles + blockIdx.x] = cnt[i];
}

__global__ __launch_bounds__(256) void k_sort_rowsum(const uint32_t *hist, int64_t num_tiles, uint32_t *row_total, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    __shared__ uint32_t s[256];
    const uint32_t *row = hist + (int64_t)blockIdx.x * num_tiles;
    uint32_t acc = 0;
    for (int64_t t = threadIdx.x; t < num_tiles; t += 256) acc += row[t];
    s[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) s[threadIdx.x] += s[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) row_total[blockIdx.x] = s[0];
}

// hist[b][t] <- pairs in buckets below b + pairs of bucket b in tiles before t
__global__ __launch_bounds__(256) void k_sort_scan(uint32_t *hist, int64_t num_tiles, const uint32_t *row_total, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    __shared__ uint32_t s[256];
    __shared__ uint32_t carry;
    const int b = blockIdx.x;
    uint32_t acc = 0;
    for (int i = threadIdx.x; i < b; i += 256) acc += row_total[i];
    s[threadIdx.x] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) s[threadIdx.x] += s[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) carry = s[0];
    __syncthreads();
    uint32_t *row = hist + (int64_t)b * num_tiles;
    for (int64_t t0 = 0; t0 < num_tiles; t0 += 256) {
        const int64_t t = t0 + threadIdx.x;
        const uint32_t v = t < num_tiles ? row[t] : 0u;
        // inclusive scan of the 256 values in LDS (Hillis-Steele, two buffers in one array by barriers)
        s[threadIdx.x] = v;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const uint32_t add = (int)threadIdx.x >= off ? s[threadIdx.x - off] : 0u;
            __syncthreads();
            s[threadIdx.x] += add;
            __syncthreads();
        }
        const uint32_t incl = s[threadIdx.x], c = carry;
        if (t < num_tiles) row[t] = c + incl - v;
        __syncthreads();
        if (threadIdx.x == 255) carry = c + incl;
        __syncthreads();
    }
}

template <int ITEMS, bool FIRST>
__global__ __launch_bounds__(SORT_THREADS) void k_sort_scatter(const int64_t *keys_in, const uint64_t *pk_in, const uint32_t *pp_in, int64_t n,
                                                               int shift, int bits, int64_t num_tiles, const uint32_t *hist, uint64_t *pk_out,
                                                               uint32_t *pp_out, const int32_t *err) {
    if (*(volatile const int32_t *)err) return;
    __shared__ uint32_t wh[SORT_WAVES][1 << SORT_MAX_BITS];
    const int R = 1 << bits;
    const uint32_t mask = (uint32_t)R - 1u;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < SORT_WAVES * (1 << SORT_MAX_BITS); i += SORT_THREADS) (&wh[0][0])[i] = 0;
    __syncthreads();
    // wavefront w takes the pairs [base + w * 64 * ITEMS, + 64 * ITEMS), 64 consecutive ones per round
    const int64_t base = (int64_t)blockIdx.x * (SORT_THREADS * ITEMS) + (int64_t)wave * 64 * ITEMS;
    uint64_t key[ITEMS];
    uint32_t pos[ITEMS], rank[ITEMS];
    const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        const int64_t q = base + r * 64 + lane;
        const bool valid = q < n;
        key[r] = 0; pos[r] = 0;
        if (valid) {
            key[r] = FIRST ? (uint64_t)keys_in[q] : pk_in[q];
            pos[r] = FIRST ? (uint32_t)q : pp_in[q];
        }
        const uint32_t d = digit_of(key[r], shift, mask);
        uint64_t same = __ballot(valid);
        for (int b = 0; b < bits; ++b) {
            const bool bit = ((d >> b) & 1u) != 0u;
            const uint64_t v = __ballot(valid && bit);
            same &= bit ? v : ~v;
        }
        // `same`: the valid lanes with this lane's digit (meaningful in valid lanes only)
        uint32_t before = 0;
        const int leader = valid ? __ffsll((long long)same) - 1 : lane;
        if (valid && lane == leader) {
            before = wh[wave][d];
            wh[wave][d] = before + (uint32_t)__popcll(same);
        }
        before = (uint32_t)__shfl((int)before, leader);
        rank[r] = before + (uint32_t)__popcll(same & below);
    }
    __syncthreads();
    // a wavefront's counters become the offsets of its first pair of each bucket
    for (int b = threadIdx.x; b < R; b += SORT_THREADS) {
        uint32_t run = hist[(int64_t)b * num_tiles + blockIdx.x];
#pragma unroll
        for (int w = 0; w < SORT_WAVES; ++w) {
            const uint32_t c = wh[w][b];
            wh[w][b] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        const int64_t q = base + r * 64 + lane;
        if (q < n) {
            const uint32_t dst = wh[wave][digit_of(key[r], shift, mask)] + rank[r];
            pk_out[dst] = key[r];
            pp_out[dst] = pos[r];
        }
    }
}

inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }

struct SortPlan {
    int items;            // pairs per thread: a tile holds 256 * items
    int passes;
    int bits[8];
    int64_t num_tiles;
    size_t off_pk, off_pp, off_hist, off_tot, bytes;   // the second pair of buffers, the counts, the bucket totals
};

SortPlan sort_plan(int64_t n, int key_bits) {
    SortPlan p{};
    p.items = n < ((int64_t)1 << 20) ? 4 : 16;
    // short inputs are bound by the number of launches: wide digits, few passes; long ones by memory
    // traffic, where narrower digits keep a tile's pairs of one bucket next to each other in the output
    const int max_bits = n < ((int64_t)1 << 20) ? SORT_MAX_BITS : 8;
    p.passes = (key_bits + max_bits - 1) / max_bits;
    if (p.passes < 1) p.passes = 1;
    for (int i = 0, left = key_bits; i < p.passes; ++i) {
        p.bits[i] = (left + (p.passes - i) - 1) / (p.passes - i);
        if (p.bits[i] < 1) p.bits[i] = 1;
        left -= p.bits[i];
    }
    p.num_tiles = (n + (int64_t)SORT_THREADS * p.items - 1) / ((int64_t)SORT_THREADS * p.items);
    if (p.num_tiles < 1) p.num_tiles = 1;
    p.off_pk = 0;
    p.off_pp = up256((size_t)n * 8);
    p.off_hist = p.off_pp + up256((size_t)n * 4);
    p.off_tot = p.off_hist + up256((size_t)(1 << SORT_MAX_BITS) * (size_t)p.num_tiles * 4);
    p.bytes = p.off_tot + up256((size_t)(1 << SORT_MAX_BITS) * 4);
    return p;
}

template <int ITEMS>
int sort_run(dpaps_ps *ps, const SortPlan &p, const int64_t *keys, int64_t n, uint64_t *skeys, uint32_t *spos, void *scratch, hipStream_t st) {
    uint64_t *alt_k = (uint64_t *)((char *)scratch + p.off_pk);
    uint32_t *alt_p = (uint32_t *)((char *)scratch + p.off_pp);
    uint32_t *hist = (uint32_t *)((char *)scratch + p.off_hist);
    uint32_t *tot = (uint32_t *)((char *)scratch + p.off_tot);
    // the last pass must write (skeys, spos): with an even number of passes the first one writes there too
    uint64_t *out_k = (p.passes & 1) ? skeys : alt_k, *in_k = nullptr;
    uint32_t *out_p = (p.passes & 1) ? spos : alt_p, *in_p = nullptr;
    const unsigned tiles = (unsigned)p.num_tiles;
    int shift = 0;
    for (int i = 0; i < p.passes; ++i) {
        const int bits = p.bits[i], R = 1 << bits;
        if (i == 0) k_sort_count<ITEMS, true><<<tiles, SORT_THREADS, 0, st>>>(keys, nullptr, n, shift, bits, p.num_tiles, hist, ps->err);
        else k_sort_count<ITEMS, false><<<tiles, SORT_THREADS, 0, st>>>(nullptr, in_k, n, shift, bits, p.num_tiles, hist, ps->err);
        PS_HIP(ps, hipGetLastError());
        k_sort_rowsum<<<R, 256, 0, st>>>(hist, p.num_tiles, tot, ps->err);
        PS_HIP(ps, hipGetLastError());
        k_sort_scan<<<R, 256, 0, st>>>(hist, p.num_tiles, tot, ps->err);
        PS_HIP(ps, hipGetLastError());
        if (i == 0) k_sort_scatter<ITEMS, true><<<tiles, SORT_THREADS, 0, st>>>(keys, nullptr, nullptr, n, shift, bits, p.num_tiles, hist, out_k, out_p, ps->err);
        else k_sort_scatter<ITEMS, false><<<tiles, SORT_THREADS, 0, st>>>(nullptr, in_k, in_p, n, shift, bits, p.num_tiles, hist, out_k, out_p, ps->err);
        PS_HIP(ps, hipGetLastError());
        in_k = out_k; in_p = out_p;
        out_k = in_k == skeys ? alt_k : skeys;
        out_p = in_p == spos ? alt_p : spos;
        shift += bits;
    }
    return PS_OK;
}

}  // namespace

// bits needed for keys below num_keys
int dpaps_key_bits(int64_t num_keys) {
    int b = 1;
    while (b < 63 && ((int64_t)1 << b) < num_keys) ++b;
    return b;
}

// scratch (bytes) that dpaps_sort_pairs needs for n pairs, besides its two output arrays
size_t dpaps_sort_scratch_bytes(int64_t n, int key_bits) { return sort_plan(n, key_bits).bytes; }

// skeys[q], spos[q] (n each) <- the pairs (keys[p], p) ordered by key, equal keys by p.  Keys must be in
// [0, 2^key_bits) (the kernels do nothing once the handle's error flag is set, which the key check before sets
// for a key out of range).  Allocates nothing; asynchronous on st.
int dpaps_sort_pairs(dpaps_ps *ps, const int64_t *keys, int64_t n, int key_bits, uint64_t *skeys, uint32_t *spos, void *scratch, hipStream_t st) {
    if (n <= 0) return PS_OK;
    const SortPlan p = sort_plan(n, key_bits);
    return p.items == 4 ? sort_run<4>(ps, p, keys, n, skeys, spos, scratch, st) : sort_run<16>(ps, p, keys, n, skeys, spos, scratch, st);
}
