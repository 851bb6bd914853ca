// moe_route: router logits, softmax probability of the winner and argmax, fused: the logits
// of a 64-token tile live in accumulators / LDS and reach HBM only when the caller asks.
//
//   bf16, E a multiple of 128 (<= 256): matrix-core kernel.  The [d,E] router matrix is first
//     re-laid into the packed k-major image the MFMA B operand wants (a few hundred KB, one
//     small kernel into the workspace), then each workgroup multiplies a 32-token tile with
//     all E columns and reduces each row (max, first arg-max, sum of exponentials) in LDS.
//   anything else (fp32 tensors, small or odd E): one wavefront per token, lanes over
//     experts, binary32 FMA in ascending k.
#include "gemm_bf16.h"
#include "route.h"
#include "route_resident.h"

namespace moe {

constexpr int RT_BK = 128;

__device__ __forceinline__ void argmax_merge(float &v, int &i, float ov, int oi)
{
    if (ov > v || (ov == v && oi < i)) {
        v = ov;
        i = oi;
    }
}

// in [K][N] bf16 row-major -> packed image, 16-byte piece ((n/32)*(K/8) + k/8)*32 + n%32
__global__ __launch_bounds__(256) void pack_matrix_kernel(const bf16_t *__restrict__ in, int K, int N,
                                                          uint4 *__restrict__ out)
{
    int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= (K / 8) * N) return;
    int kg = i / N, n = i - kg * N;
    const bf16_t *src = in + (size_t)kg * 8 * N + n;
    uint32_t v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        v[j] = (uint32_t)src[(size_t)(2 * j) * N] | ((uint32_t)src[(size_t)(2 * j + 1) * N] << 16);
    out[((size_t)(n >> 5) * (K / 8) + kg) * 32 + (n & 31)] = make_uint4(v[0], v[1], v[2], v[3]);
}

// MB row blocks of 32 tokens per workgroup: 1 for small batches (many small workgroups hide the
// k-loop latency), 2 above 8192 tokens (every workgroup reads the whole packed router matrix from L2, so
// taller tiles cut that traffic; the 256-expert shapes go to route_resident_kernel from 16384 tokens on).
template <int NB, int MB>
__global__ __launch_bounds__(GEMM_THREADS) void route_mfma_kernel(const bf16_t *__restrict__ x,
                                                                  const bf16_t *__restrict__ wr_packed,
                                                                  const float *__restrict__ bias, int T, int d,
                                                                  int top_k, int renormalize,
                                                                  int32_t *__restrict__ idx, float *__restrict__ prob,
                                                                  float *__restrict__ logits_opt)
{
    constexpr int E = NB * 128;
    constexpr int LDL = E + 8;                    // 8 threads per row, 4 rows per half wavefront: bank 8 r + sub
    constexpr int RT_BM = MB * 32;
    constexpr int BK = RT_BK;
    constexpr int STAGE_BYTES = gemm_lds_elems<MB, BK>() * 2, TILE_BYTES = 32 * LDL * 4;
    // the logits tile reuses the A staging buffers, which are free once the product is done
    __shared__ __attribute__((aligned(16))) char smem[STAGE_BYTES > TILE_BYTES ? STAGE_BYTES : TILE_BYTES];
    bf16_t *lds = reinterpret_cast<bf16_t *>(smem);
    float *tile = reinterpret_cast<float *>(smem);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int row0 = blockIdx.x * RT_BM;
    const int nrows = T - row0 < RT_BM ? T - row0 : RT_BM;
    f32x16_t acc[MB][NB];
    zero_acc<MB, NB>(acc);
    gemm_tile_bf16<MB, NB, BK>(x + (size_t)row0 * d, d, nrows, wr_packed, 0, d, lds, acc);

    float b[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) b[nb] = bias ? bias[(w * NB + nb) * 32 + (lane & 31)] : 0.f;

#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                tile[acc_row(v, lane) * LDL + (w * NB + nb) * 32 + (lane & 31)] = acc[mb][nb][v] + b[nb];
        __syncthreads();
        // 8 threads per row, each over E/8 strided columns held in registers (one batch of independent LDS
        // reads: read one by one inside the loops below, every read was a full LDS round trip in a
        // dependent chain, and this step took as long as the product), then a 3-step butterfly
        const int r = tid >> 3, sub = tid & 7;
        const float *row = tile + r * LDL;
        constexpr int PER = E / 8;
        float lv[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) lv[i] = row[sub + 8 * i];
        float best = lv[0];
        int bi = sub;
#pragma unroll
        for (int i = 1; i < PER; ++i) argmax_merge(best, bi, lv[i], sub + 8 * i);
#pragma unroll
        for (int o = 1; o < 8; o <<= 1) {
            float ov = __shfl_xor(best, o, 64);
            int oi = __shfl_xor(bi, o, 64);
            argmax_merge(best, bi, ov, oi);
        }
        float z = 0.f;
#pragma unroll
        for (int i = 0; i < PER; ++i) z += expf(lv[i] - best);
#pragma unroll
        for (int o = 1; o < 8; o <<= 1) z += __shfl_xor(z, o, 64);
        const int grow = row0 + mb * 32 + r;
        if (top_k == 1) {
            if (sub == 0 && mb * 32 + r < nrows) {
                idx[grow] = bi;
                prob[grow] = 1.f / z;
            }
        } else {
            // choice j: the largest logit after choice j-1 in the order (logit descending, id ascending)
            int ci[MOE_MAX_TOPK];
            float cw[MOE_MAX_TOPK];
            ci[0] = bi;
            cw[0] = 1.f / z;
            float pv = best, wsum = cw[0];
            int pi = bi;
#pragma unroll
            for (int j = 1; j < MOE_MAX_TOPK; ++j) {
                if (j < top_k) {
                    float v = -INFINITY;
                    int vi = 0x7fffffff;
#pragma unroll
                    for (int i = 0; i < PER; ++i) {
                        const float t = lv[i];
                        const int c = sub + 8 * i;
                        if (t < pv || (t == pv && c > pi)) argmax_merge(v, vi, t, c);
                    }
#pragma unroll
                    for (int o = 1; o < 8; o <<= 1) {
                        float ov = __shfl_xor(v, o, 64);
                        int oi = __shfl_xor(vi, o, 64);
                        argmax_merge(v, vi, ov, oi);
                    }
                    ci[j] = vi;
                    cw[j] = expf(v - best) / z;
                    wsum += cw[j];
                    pv = v;
                    pi = vi;
                }
            }
            if (sub == 0 && mb * 32 + r < nrows) {
#pragma unroll
                for (int j = 0; j < MOE_MAX_TOPK; ++j)
                    if (j < top_k) {
                        idx[(size_t)j * T + grow] = ci[j];
                        prob[(size_t)j * T + grow] = renormalize ? cw[j] / wsum : cw[j];
                    }
            }
        }
        if (logits_opt) {
            for (int i = tid; i < 32 * E; i += GEMM_THREADS) {
                int rr = i / E, cc = i - rr * E;
                if (mb * 32 + rr < nrows) logits_opt[(size_t)(row0 + mb * 32 + rr) * E + cc] = tile[rr * LDL + cc];
            }
        }
        __syncthreads();
    }
}

// one wavefront per token; lanes over experts
template <bool BF16>
__global__ __launch_bounds__(256) void route_generic_kernel(const void *__restrict__ xv, const void *__restrict__ wv,
                                                            const float *__restrict__ bias, int T, int d, int E,
                                                            int top_k, int renormalize,
                                                            int32_t *__restrict__ idx, float *__restrict__ prob,
                                                            float *__restrict__ logits_opt)
{
    const int lane = threadIdx.x & 63;
    const int s = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (s >= T) return;
    constexpr int PER = MOE_MAX_EXPERTS / WAVE;
    float l[PER];
    float best = -INFINITY;
    int bi = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        int e = lane + i * WAVE;
        l[i] = -INFINITY;
        if (e < E) {
            float acc = 0.f;
            if (BF16) {
                const bf16_t *x = (const bf16_t *)xv + (size_t)s * d;
                const bf16_t *w = (const bf16_t *)wv + e;
                for (int k = 0; k < d; ++k) acc = fmaf(bf16_to_f32(x[k]), bf16_to_f32(w[(size_t)k * E]), acc);
            } else {
                const float *x = (const float *)xv + (size_t)s * d;
                const float *w = (const float *)wv + e;
                for (int k = 0; k < d; ++k) acc = fmaf(x[k], w[(size_t)k * E], acc);
            }
            l[i] = acc + (bias ? bias[e] : 0.f);
            if (logits_opt) logits_opt[(size_t)s * E + e] = l[i];
            argmax_merge(best, bi, l[i], e);
        }
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        float ov = __shfl_xor(best, o, 64);
        int oi = __shfl_xor(bi, o, 64);
        argmax_merge(best, bi, ov, oi);
    }
    float z = 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i)
        if (lane + i * WAVE < E) z += expf(l[i] - best);
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) z += __shfl_xor(z, o, 64);
    if (top_k == 1) {
        if (lane == 0) {
            idx[s] = bi;
            prob[s] = 1.f / z;
        }
        return;
    }
    int ci[MOE_MAX_TOPK];
    float cw[MOE_MAX_TOPK];
    ci[0] = bi;
    cw[0] = 1.f / z;
    float pv = best, wsum = cw[0];
    int pi = bi;
#pragma unroll
    for (int j = 1; j < MOE_MAX_TOPK; ++j) {
        if (j < top_k) {
            float v = -INFINITY;
            int vi = 0x7fffffff;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int e = lane + i * WAVE;
                if (e < E && (l[i] < pv || (l[i] == pv && e > pi))) argmax_merge(v, vi, l[i], e);
            }
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                float ov = __shfl_xor(v, o, 64);
                int oi = __shfl_xor(vi, o, 64);
                argmax_merge(v, vi, ov, oi);
            }
            ci[j] = vi;
            cw[j] = expf(v - best) / z;
            wsum += cw[j];
            pv = v;
            pi = vi;
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int j = 0; j < MOE_MAX_TOPK; ++j)
            if (j < top_k) {
                idx[(size_t)j * T + s] = ci[j];
                prob[(size_t)j * T + s] = renormalize ? cw[j] / wsum : cw[j];
            }
    }
}

static inline bool route_uses_mfma(int d, int E, int dtype)
{
    return dtype == MOE_BF16 && (E == 128 || E == 256) && d % RT_BK == 0;
}

int pack_matrix_launch(const void *in, int K, int N, void *out, hipStream_t st, const char *who)
{
    int n = (K / 8) * N;
    hipLaunchKernelGGL(pack_matrix_kernel, dim3(ceil_div(n, 256)), dim3(256), 0, st, (const bf16_t *)in, K, N,
                       (uint4 *)out);
    MOE_CHECK_LAUNCH(who);
    return MOE_OK;
}

// shared with sru_predict (its head is the same product + argmax)
int route_launch(const void *x, const void *w_router, int w_layout, const float *b_router, int T, int d, int E,
                 int dtype, int top_k, int renormalize, int32_t *idx, float *prob, float *logits_opt, void *ws,
                 hipStream_t st, const char *who)
{
    if (route_uses_mfma(d, E, dtype)) {
        const void *wp = w_router;
        if (w_layout == MOE_LAYOUT_PLAIN) {
            int rc = pack_matrix_launch(w_router, d, E, ws, st, who);
            if (rc != MOE_OK) return rc;
            wp = ws;
        }
        // large batches of the 256-expert shapes: persistent workgroups with the router matrix in registers
        if (E == RR_E && T >= RR_MIN_T && (d == 768 || d == 512 || d == 256)) {
            int dev = 0, n_cu = 0;
            if (hipGetDevice(&dev) != hipSuccess ||
                hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1) {
                set_error("%s: cannot read the compute unit count", who);
                return MOE_ERR_HIP;
            }
            const int n_tiles = ceil_div(T, RR_BM);
            const int grid = n_tiles < n_cu ? n_tiles : n_cu;
#define MOE_ROUTE_RESIDENT(KS_)                                                                                  \
    if (top_k > 1)                                                                                               \
        hipLaunchKernelGGL((route_resident_kernel<KS_, true>), dim3(grid), dim3(GEMM_THREADS), 0, st,            \
                           (const bf16_t *)x, (const bf16_t *)wp, b_router, T, top_k, renormalize, idx, prob,    \
                           logits_opt);                                                                          \
    else                                                                                                         \
        hipLaunchKernelGGL((route_resident_kernel<KS_, false>), dim3(grid), dim3(GEMM_THREADS), 0, st,           \
                           (const bf16_t *)x, (const bf16_t *)wp, b_router, T, top_k, renormalize, idx, prob,    \
                           logits_opt)
            if (d == 768) {
                MOE_ROUTE_RESIDENT(48);
            } else if (d == 512) {
                MOE_ROUTE_RESIDENT(32);
            } else {
                MOE_ROUTE_RESIDENT(16);
            }
#undef MOE_ROUTE_RESIDENT
            MOE_CHECK_LAUNCH(who);
            return MOE_OK;
        }
        const int mbk = T <= 8192 ? 1 : 2;
        int grid = ceil_div(T, 32 * mbk);
#define MOE_ROUTE_LAUNCH(NB_, MB_)                                                                            \
    hipLaunchKernelGGL((route_mfma_kernel<NB_, MB_>), dim3(grid), dim3(GEMM_THREADS), 0, st, (const bf16_t *)x, \
                       (const bf16_t *)wp, b_router, T, d, top_k, renormalize, idx, prob, logits_opt)
        if (E == 128) {
            if (mbk == 1) MOE_ROUTE_LAUNCH(1, 1);
            else MOE_ROUTE_LAUNCH(1, 2);
        } else {
            if (mbk == 1) MOE_ROUTE_LAUNCH(2, 1);
            else MOE_ROUTE_LAUNCH(2, 2);
        }
#undef MOE_ROUTE_LAUNCH
    } else if (dtype == MOE_BF16) {
        hipLaunchKernelGGL(route_generic_kernel<true>, dim3(ceil_div(T, 4)), dim3(256), 0, st, x, w_router, b_router, T,
                           d, E, top_k, renormalize, idx, prob, logits_opt);
    } else {
        hipLaunchKernelGGL(route_generic_kernel<false>, dim3(ceil_div(T, 4)), dim3(256), 0, st, x, w_router, b_router,
                           T, d, E, top_k, renormalize, idx, prob, logits_opt);
    }
    MOE_CHECK_LAUNCH(who);
    return MOE_OK;
}

size_t route_ws_bytes(int d, int E, int dtype)
{
    return route_uses_mfma(d, E, dtype) ? align_up((size_t)d * E * 2, 256) : 256;
}

}  // namespace moe

using namespace moe;

extern "C" size_t moe_route_workspace_bytes(int T, int d, int E, int dtype)
{
    (void)T;
    if (d <= 0 || E <= 0) return 0;
    return route_ws_bytes(d, E, dtype);
}

static int route_checked(const char *who, const void *x, const void *w_router, int w_layout, const float *b_router,
                         int T, int d, int E, int dtype, int top_k, int renormalize, int32_t *expert_idx,
                         float *expert_prob, float *logits_opt, void *ws, size_t ws_bytes, void *stream)
{
    MOE_REQUIRE(w_layout == MOE_LAYOUT_PLAIN || w_layout == MOE_LAYOUT_PACKED, MOE_ERR_INVALID_ARG,
                "%s: unknown weight layout %d", who, w_layout);
    MOE_REQUIRE(T >= 0 && d > 0 && E > 0, MOE_ERR_INVALID_ARG, "%s: T=%d d=%d E=%d out of range", who, T, d, E);
    MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, dtype);
    MOE_REQUIRE(E <= MOE_MAX_EXPERTS, MOE_ERR_UNSUPPORTED, "%s: E=%d exceeds %d", who, E, MOE_MAX_EXPERTS);
    MOE_REQUIRE(top_k >= 1 && top_k <= MOE_MAX_TOPK && top_k <= E, MOE_ERR_INVALID_ARG,
                "%s: k=%d outside 1..min(%d, E=%d)", who, top_k, MOE_MAX_TOPK, E);
    MOE_REQUIRE((long long)T * top_k <= 0x7fffffffLL, MOE_ERR_INVALID_ARG, "%s: T*k=%lld does not fit 31 bits", who,
                (long long)T * top_k);
    MOE_REQUIRE(renormalize == 0 || renormalize == 1, MOE_ERR_INVALID_ARG, "%s: renormalize must be 0 or 1", who);
    MOE_REQUIRE(d % 8 == 0, MOE_ERR_INVALID_ARG, "%s: d=%d is not a multiple of 8", who, d);
    MOE_REQUIRE(w_layout == MOE_LAYOUT_PLAIN || route_uses_mfma(d, E, dtype), MOE_ERR_UNSUPPORTED,
                "%s: a packed router matrix needs bf16, E = 128 or 256 and d a multiple of %d", who, RT_BK);
    if (T == 0) return MOE_OK;
    MOE_REQUIRE(x && w_router && expert_idx && expert_prob, MOE_ERR_INVALID_ARG, "%s: null pointer", who);
    MOE_REQUIRE(aligned16(x) && aligned16(w_router), MOE_ERR_INVALID_ARG, "%s: tensor misaligned", who);
    size_t need = route_ws_bytes(d, E, dtype);
    MOE_REQUIRE(ws && aligned16(ws) && ws_bytes >= need, MOE_ERR_WORKSPACE,
                "%s: workspace of %zu bytes needed, %zu given", who, need, ws_bytes);
    return route_launch(x, w_router, w_layout, b_router, T, d, E, dtype, top_k, renormalize, expert_idx, expert_prob,
                        logits_opt, ws, (hipStream_t)stream, who);
}

extern "C" int moe_route(const void *x, const void *w_router, int w_layout, const float *b_router, int T, int d,
                         int E, int dtype, int32_t *expert_idx, float *expert_prob, float *logits_opt, void *ws,
                         size_t ws_bytes, void *stream)
{
    return route_checked("moe_route", x, w_router, w_layout, b_router, T, d, E, dtype, 1, 0, expert_idx, expert_prob,
                         logits_opt, ws, ws_bytes, stream);
}

extern "C" int moe_route_topk(const void *x, const void *w_router, int w_layout, const float *b_router, int T,
                              int d, int E, int dtype, int k, int renormalize, int32_t *expert_idx,
                              float *expert_weight, float *logits_opt, void *ws, size_t ws_bytes, void *stream)
{
    return route_checked("moe_route_topk", x, w_router, w_layout, b_router, T, d, E, dtype, k, renormalize, expert_idx,
                         expert_weight, logits_opt, ws, ws_bytes, stream);
}
