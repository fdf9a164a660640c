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
template <int NV>
__device__ __forceinline__ void load_row_t(const float *p, int lane, bool tail, float (&x)[NV]) {
#pragma unroll
    for (int c = 0; c < NV - 1; ++c) x[c] = p[lane + 64 * c];
    x[NV - 1] = tail ? p[lane + 64 * (NV - 1)] : 0.0f;
}
template <int NV>
__device__ __forceinline__ void store_row_t(float *p, int lane, bool tail, const float (&x)[NV]) {
#pragma unroll
    for (int c = 0; c < NV - 1; ++c) p[lane + 64 * c] = x[c];
    if (tail) p[lane + 64 * (NV - 1)] = x[NV - 1];
}

#define INFO_SINGLE 0xFFFFu      // low 16 bits of an info word: the row's only entry in the block
#define INFO_NONE 0xFFFEu        // filler for lanes past the end of a run: neither single nor in LDS

