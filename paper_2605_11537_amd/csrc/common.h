// Internal helpers shared by the kernels of the library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/moe_mpmc.h"

namespace moe {

void set_error(const char *fmt, ...);

#define MOE_REQUIRE(cond, code, ...)     \
    do {                                 \
        if (!(cond)) {                   \
            moe::set_error(__VA_ARGS__); \
            return (code);               \
        }                                \
    } while (0)

// Check the launch that was just enqueued.
#define MOE_CHECK_LAUNCH(what)                                                      \
    do {                                                                            \
        hipError_t e__ = hipGetLastError();                                         \
        if (e__ != hipSuccess) {                                                    \
            moe::set_error("%s: launch failed: %s", (what), hipGetErrorString(e__)); \
            return MOE_ERR_HIP;                                                     \
        }                                                                           \
    } while (0)

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

constexpr int WAVE = 64;

// ---------------------------------------------------------------- bf16 <-> f32 on device
typedef unsigned short bf16_t;  // raw bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round to nearest, ties to even; NaN kept quiet
// binary32 -> bf16, round to nearest even, by the hardware conversion (v_cvt_pk_bf16_f32: one instruction
// per pair; the same rounding spelled out in integer operations is seven per value)
typedef float moe_f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 moe_bf16x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const moe_f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, moe_bf16x2_t));
}

__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

// XCD-aware remap of a linear workgroup id.  Hardware deals consecutive workgroup ids to the
// 8 XCDs in turn, so ids congruent mod 8 share an L2.  The n_valid units of work are cut into 8
// contiguous ranges, one per XCD: neighbours in the logical order (which share operands) meet
// in one L2, and every XCD gets the same share even when the grid was sized for a worst case
// larger than n_valid.  Returns -1 for a workgroup with nothing to do.
__device__ __forceinline__ int xcd_remap(int bid, int n_valid)
{
    int per = (n_valid + 7) >> 3;
    int slot = bid >> 3;
    int lid = (bid & 7) * per + slot;
    return (slot < per && lid < n_valid) ? lid : -1;
}

// Workgroup id -> (item, column tile) for a grouped GEMM over n_items row tiles x n_nt column
// tiles, XCD-aware (consecutive hardware workgroup ids go to the 8 XCDs in turn).
//   group == 0: the n_items*n_nt tiles are cut into 8 contiguous ranges, one per XCD.  Every
//     tile costs the same when the weight stream binds, so this balances exactly, and the
//     column tiles of an item (which share its token rows) meet in one L2.
//   group  > 0: items are dealt to the XCDs in chunks of `group` consecutive items, and inside
//     a chunk the order is column-tile-major.  The workgroups resident on an XCD then share
//     one 32-column-strip set of weights and `group` row tiles, both far below the L2 size,
//     so a hot expert's weights are not re-fetched for each of its hundreds of row tiles; and
//     its tiles spread over all XCDs.
// The grid must hold 8*ceil(ceil(n_items/group)/8)*group*n_nt workgroups in the second case.
__device__ __forceinline__ bool grouped_tile_of(int bid, int n_items, int n_nt, int group, int &item, int &nt)
{
    if (group <= 0) {
        int lid = xcd_remap(bid, n_items * n_nt);
        if (lid < 0) return false;
        item = lid / n_nt;
        nt = lid - item * n_nt;
        return true;
    }
    const int per_chunk = group * n_nt;
    const int j = bid >> 3;                        // index among this XCD's workgroups
    const int chunk = (j / per_chunk) * 8 + (bid & 7);
    const int within = j % per_chunk;
    const int first = chunk * group;
    if (first >= n_items) return false;
    const int g = n_items - first < group ? n_items - first : group;   // items in this chunk
    if (within >= g * n_nt) return false;
    nt = within / g;
    item = first + within % g;
    return true;
}

// Exclusive scan of one int per thread over a 1024-thread workgroup.  Returns the prefix and
// leaves the grand total in *total_out (LDS).  wave_sums is LDS scratch of 16 ints.
__device__ __forceinline__ int block_scan_excl_1024(int v, int *wave_sums, int *total_out)
{
    int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int n = __shfl_up(inc, o, 64);
        if (lane >= o) inc += n;
    }
    if (lane == 63) wave_sums[w] = inc;
    __syncthreads();
    if (w == 0) {
        int s = lane < 16 ? wave_sums[lane] : 0;
        int si = s;
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
            int n = __shfl_up(si, o, 64);
            if (lane >= o) si += n;
        }
        if (lane < 16) wave_sums[lane] = si - s;
        if (lane == 15) *total_out = si;
    }
    __syncthreads();
    int r = wave_sums[w] + inc - v;
    __syncthreads();
    return r;
}

}  // namespace moe
