// moe_combine: scale expert outputs by the gate probability and scatter them back to token
// order; tokens over capacity are copied through bit for bit.  HBM-bound: every 16-byte
// piece of x, y_perm and out is touched once.
#include "common.h"

namespace moe {

constexpr int CMB_THREADS = 256;

// one thread per 16-byte piece of an output row
template <bool BF16>
__global__ __launch_bounds__(CMB_THREADS) void combine_kernel(const uint4 *__restrict__ y_perm,
                                                              const uint4 *__restrict__ x,
                                                              const int32_t *__restrict__ inv,
                                                              const float *__restrict__ prob, int T,
                                                              int vec_per_row, int residual,
                                                              uint4 *__restrict__ out)
{
    long long total = (long long)T * vec_per_row;
    for (long long i = (long long)blockIdx.x * CMB_THREADS + threadIdx.x; i < total;
         i += (long long)gridDim.x * CMB_THREADS) {
        int s = (int)(i / vec_per_row);
        int c = (int)(i - (long long)s * vec_per_row);
        int pos = inv[s];
        uint4 xv;
        if (pos < 0 || residual) xv = x[i];
        if (pos < 0) {
            out[i] = xv;
            continue;
        }
        float p = prob[s];
        uint4 yv = y_perm[(size_t)pos * vec_per_row + c];
        uint4 o;
        if (BF16) {
            const uint32_t *yy = &yv.x, *xx = &xv.x;
            uint32_t *oo = &o.x;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float y0 = __uint_as_float(yy[k] << 16), y1 = __uint_as_float(yy[k] & 0xffff0000u);
                float r0 = 0.f, r1 = 0.f;
                if (residual) {
                    r0 = __uint_as_float(xx[k] << 16);
                    r1 = __uint_as_float(xx[k] & 0xffff0000u);
                }
                oo[k] = pack_bf16x2(fmaf(p, y0, r0), fmaf(p, y1, r1));
            }
        } else {
            const float *yy = reinterpret_cast<const float *>(&yv);
            const float *xx = reinterpret_cast<const float *>(&xv);
            float *oo = reinterpret_cast<float *>(&o);
#pragma unroll
            for (int k = 0; k < 4; ++k) oo[k] = fmaf(p, yy[k], residual ? xx[k] : 0.f);
        }
        out[i] = o;
    }
}

// top-k: k gathered rows per token, accumulated in choice order in binary32, one rounding
template <bool BF16>
__global__ __launch_bounds__(CMB_THREADS) void combine_topk_kernel(const uint4 *__restrict__ y_perm,
                                                                   const uint4 *__restrict__ x,
                                                                   const int32_t *__restrict__ inv,
                                                                   const float *__restrict__ weight, int T, int k,
                                                                   int vec_per_row, int residual,
                                                                   uint4 *__restrict__ out)
{
    long long total = (long long)T * vec_per_row;
    for (long long i = (long long)blockIdx.x * CMB_THREADS + threadIdx.x; i < total;
         i += (long long)gridDim.x * CMB_THREADS) {
        int s = (int)(i / vec_per_row);
        int c = (int)(i - (long long)s * vec_per_row);
        int pos[MOE_MAX_TOPK];
        bool any = false;
#pragma unroll
        for (int j = 0; j < MOE_MAX_TOPK; ++j) {
            pos[j] = j < k ? inv[(size_t)j * T + s] : -1;
            any = any || pos[j] >= 0;
        }
        uint4 xv;
        if (!any || residual) xv = x[i];
        if (!any) {
            out[i] = xv;
            continue;
        }
        float acc[8];
        if (BF16) {
            const uint32_t *xx = &xv.x;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                acc[2 * q] = residual ? __uint_as_float(xx[q] << 16) : 0.f;
                acc[2 * q + 1] = residual ? __uint_as_float(xx[q] & 0xffff0000u) : 0.f;
            }
        } else {
            const float *xx = reinterpret_cast<const float *>(&xv);
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = residual ? xx[q] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < MOE_MAX_TOPK; ++j) {
            if (pos[j] < 0) continue;
            const float p = weight[(size_t)j * T + s];
            const uint4 yv = y_perm[(size_t)pos[j] * vec_per_row + c];
            if (BF16) {
                const uint32_t *yy = &yv.x;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc[2 * q] = fmaf(p, __uint_as_float(yy[q] << 16), acc[2 * q]);
                    acc[2 * q + 1] = fmaf(p, __uint_as_float(yy[q] & 0xffff0000u), acc[2 * q + 1]);
                }
            } else {
                const float *yy = reinterpret_cast<const float *>(&yv);
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] = fmaf(p, yy[q], acc[q]);
            }
        }
        uint4 o;
        if (BF16) {
            uint32_t *oo = &o.x;
#pragma unroll
            for (int q = 0; q < 4; ++q) oo[q] = pack_bf16x2(acc[2 * q], acc[2 * q + 1]);
        } else {
            float *oo = reinterpret_cast<float *>(&o);
#pragma unroll
            for (int q = 0; q < 4; ++q) oo[q] = acc[q];
        }
        out[i] = o;
    }
}

}  // namespace moe

using namespace moe;

extern "C" int moe_combine(const void *y_perm, const void *x, const int32_t *inv, const float *expert_prob,
                           int T, int d, int dtype, int residual, void *out, void *stream)
{
    MOE_REQUIRE(T >= 0 && d > 0, MOE_ERR_INVALID_ARG, "moe_combine: T=%d d=%d out of range", T, d);
    MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_ERR_INVALID_ARG, "moe_combine: unknown dtype %d",
                dtype);
    MOE_REQUIRE(residual == 0 || residual == 1, MOE_ERR_INVALID_ARG, "moe_combine: residual must be 0 or 1");
    if (T == 0) return MOE_OK;
    MOE_REQUIRE(y_perm && x && inv && expert_prob && out, MOE_ERR_INVALID_ARG, "moe_combine: null pointer");
    MOE_REQUIRE(out != x && out != y_perm, MOE_ERR_INVALID_ARG, "moe_combine: out aliases an input");
    size_t esz = dtype == MOE_F32 ? 4 : 2;
    MOE_REQUIRE(((size_t)d * esz) % 16 == 0, MOE_ERR_INVALID_ARG,
                "moe_combine: row size %zu bytes is not a multiple of 16", (size_t)d * esz);
    MOE_REQUIRE(aligned16(y_perm) && aligned16(x) && aligned16(out), MOE_ERR_INVALID_ARG,
                "moe_combine: tensor misaligned");
    int vec_per_row = (int)((size_t)d * esz / 16);
    long long total = (long long)T * vec_per_row;
    long long want = (total + CMB_THREADS - 1) / CMB_THREADS;
    int grid = (int)(want < 256 * 16 ? want : 256 * 16);
    hipStream_t st = (hipStream_t)stream;
    if (dtype == MOE_BF16)
        hipLaunchKernelGGL(combine_kernel<true>, dim3(grid), dim3(CMB_THREADS), 0, st, (const uint4 *)y_perm,
                           (const uint4 *)x, inv, expert_prob, T, vec_per_row, residual, (uint4 *)out);
    else
        hipLaunchKernelGGL(combine_kernel<false>, dim3(grid), dim3(CMB_THREADS), 0, st, (const uint4 *)y_perm,
                           (const uint4 *)x, inv, expert_prob, T, vec_per_row, residual, (uint4 *)out);
    MOE_CHECK_LAUNCH("moe_combine");
    return MOE_OK;
}

extern "C" int moe_combine_topk(const void *y_perm, const void *x, const int32_t *inv, const float *expert_weight,
                                int T, int k, int d, int dtype, int residual, void *out, void *stream)
{
    MOE_REQUIRE(T >= 0 && d > 0 && k >= 1 && k <= MOE_MAX_TOPK, MOE_ERR_INVALID_ARG,
                "moe_combine_topk: T=%d d=%d k=%d out of range (k <= %d)", T, d, k, MOE_MAX_TOPK);
    MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_ERR_INVALID_ARG, "moe_combine_topk: unknown dtype %d",
                dtype);
    MOE_REQUIRE(residual == 0 || residual == 1, MOE_ERR_INVALID_ARG, "moe_combine_topk: residual must be 0 or 1");
    if (T == 0) return MOE_OK;
    MOE_REQUIRE(y_perm && x && inv && expert_weight && out, MOE_ERR_INVALID_ARG, "moe_combine_topk: null pointer");
    MOE_REQUIRE(out != x && out != y_perm, MOE_ERR_INVALID_ARG, "moe_combine_topk: out aliases an input");
    size_t esz = dtype == MOE_F32 ? 4 : 2;
    MOE_REQUIRE(((size_t)d * esz) % 16 == 0, MOE_ERR_INVALID_ARG,
                "moe_combine_topk: row size %zu bytes is not a multiple of 16", (size_t)d * esz);
    MOE_REQUIRE(aligned16(y_perm) && aligned16(x) && aligned16(out), MOE_ERR_INVALID_ARG,
                "moe_combine_topk: tensor misaligned");
    int vec_per_row = (int)((size_t)d * esz / 16);
    long long total = (long long)T * vec_per_row;
    long long want = (total + CMB_THREADS - 1) / CMB_THREADS;
    int grid = (int)(want < 256 * 16 ? want : 256 * 16);
    hipStream_t st = (hipStream_t)stream;
    if (dtype == MOE_BF16)
        hipLaunchKernelGGL(combine_topk_kernel<true>, dim3(grid), dim3(CMB_THREADS), 0, st, (const uint4 *)y_perm,
                           (const uint4 *)x, inv, expert_weight, T, k, vec_per_row, residual, (uint4 *)out);
    else
        hipLaunchKernelGGL(combine_topk_kernel<false>, dim3(grid), dim3(CMB_THREADS), 0, st, (const uint4 *)y_perm,
                           (const uint4 *)x, inv, expert_weight, T, k, vec_per_row, residual, (uint4 *)out);
    MOE_CHECK_LAUNCH("moe_combine_topk");
    return MOE_OK;
}
