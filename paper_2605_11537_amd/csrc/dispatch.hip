// moe_dispatch: capacity-limited, stable dispatch of tokens to expert slots.
//
// Three kernels, no global atomics, so the permutation is the stable one whatever the
// hardware scheduling:
//   hist     one workgroup per 1024 tokens: LDS histogram of expert ids -> block_hist[b][e]
//   scan     one workgroup: per expert, exclusive prefix over the token blocks; kept counts,
//            expert offsets (scan over experts), slot offsets (balanced split per expert)
//   permute  one workgroup per 1024 tokens: rank of every token among the tokens of its expert
//            = prefix over earlier blocks + prefix over earlier 64-token chunks of the block
//            (LDS table) + rank inside the chunk (wavefront ballots, one per id bit);
//            writes inv / perm and copies the kept rows with 16-byte accesses.
#include "common.h"

namespace moe {

constexpr int DSP_THREADS = 256;
constexpr int DSP_TOKENS = 1024;  // tokens per workgroup
constexpr int DSP_CHUNKS = DSP_TOKENS / WAVE;

__global__ __launch_bounds__(DSP_THREADS) void dispatch_hist_kernel(const int32_t *__restrict__ idx, int T,
                                                                    int E, int32_t *__restrict__ block_hist)
{
    __shared__ int hist[MOE_MAX_EXPERTS];
    for (int e = threadIdx.x; e < E; e += DSP_THREADS) hist[e] = 0;
    __syncthreads();
    int base = blockIdx.x * DSP_TOKENS;
#pragma unroll
    for (int i = 0; i < DSP_TOKENS / DSP_THREADS; ++i) {
        int t = base + i * DSP_THREADS + threadIdx.x;
        if (t < T) {
            int e = idx[t];
            if (e >= 0 && e < E) atomicAdd(&hist[e], 1);
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += DSP_THREADS) block_hist[(size_t)blockIdx.x * E + e] = hist[e];
}

__global__ __launch_bounds__(1024) void dispatch_scan_kernel(int32_t *__restrict__ block_hist, int nb, int E,
                                                              const int32_t *__restrict__ replicas, int C,
                                                              int max_slots, int32_t *__restrict__ counts,
                                                              int32_t *__restrict__ kept,
                                                              int32_t *__restrict__ expert_offset,
                                                              int32_t *__restrict__ slot_offset)
{
    __shared__ int wave_sums[16];
    __shared__ int total_k, total_p;
    int e = threadIdx.x;
    int n = 0, r = 0, kp = 0;
    if (e < E) {
        for (int b = 0; b < nb; ++b) {
            int v = block_hist[(size_t)b * E + e];
            block_hist[(size_t)b * E + e] = n;
            n += v;
        }
        r = replicas ? replicas[e] : 1;
        if (r < 1) r = 1;
        long long cap = (long long)r * C;
        kp = (long long)n < cap ? n : (int)cap;
        counts[e] = n;
        kept[e] = kp;
    }
    int off = block_scan_excl_1024(kp, wave_sums, &total_k);
    int sb = block_scan_excl_1024(r, wave_sums, &total_p);
    int K = total_k, P = total_p;
    if (e < E) {
        expert_offset[e] = off;
        if (slot_offset) {
            int q = kp / r, rem = kp % r;
            for (int k = 0; k < r; ++k) {
                int p = sb + k;
                if (p <= max_slots) slot_offset[p] = off + k * q + (k < rem ? k : rem);
            }
        }
    }
    if (e == 0) expert_offset[E] = K;
    if (slot_offset)
        for (int p = P + e; p <= max_slots; p += 1024) slot_offset[p] = K;
}

template <typename VecT>
__global__ __launch_bounds__(DSP_THREADS) void dispatch_permute_kernel(
    const VecT *__restrict__ x, const int32_t *__restrict__ idx, const int32_t *__restrict__ replicas, int T,
    int vec_per_row, int E, int nbits, int C, const int32_t *__restrict__ block_base,
    const int32_t *__restrict__ expert_offset, int32_t *__restrict__ perm, int32_t *__restrict__ inv,
    VecT *__restrict__ x_perm)
{
    __shared__ unsigned short chunk_cnt[DSP_CHUNKS][MOE_MAX_EXPERTS];
    __shared__ int dest_of[DSP_TOKENS];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int base = blockIdx.x * DSP_TOKENS;
    for (int i = tid; i < DSP_CHUNKS * E; i += DSP_THREADS) chunk_cnt[i / E][i % E] = 0;
    __syncthreads();

    int my_e[4], my_rank[4];
#pragma unroll
    for (int rd = 0; rd < 4; ++rd) {
        int c = rd * 4 + w;
        int t = base + c * WAVE + lane;
        bool valid = t < T;
        int e = valid ? idx[t] : 0;
        valid = valid && e >= 0 && e < E;
        unsigned long long mask = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            bool bit = (e >> b) & 1;
            unsigned long long bal = __ballot(bit);
            mask &= bit ? bal : ~bal;
        }
        int rank = __popcll(mask & ((1ull << lane) - 1ull));
        if (valid && rank == 0) chunk_cnt[c][e] = (unsigned short)__popcll(mask);
        my_e[rd] = valid ? e : -1;
        my_rank[rd] = rank;
    }
    __syncthreads();
    for (int e = tid; e < E; e += DSP_THREADS) {
        int run = 0;
#pragma unroll
        for (int c = 0; c < DSP_CHUNKS; ++c) {
            int v = chunk_cnt[c][e];
            chunk_cnt[c][e] = (unsigned short)run;
            run += v;
        }
    }
    __syncthreads();
    const int K = expert_offset[E];
#pragma unroll
    for (int rd = 0; rd < 4; ++rd) {
        int c = rd * 4 + w;
        int t = base + c * WAVE + lane;
        int dest = -1;
        int e = my_e[rd];
        if (e >= 0) {
            int j = block_base[(size_t)blockIdx.x * E + e] + chunk_cnt[c][e] + my_rank[rd];
            int r = replicas ? replicas[e] : 1;
            if (r < 1) r = 1;
            long long cap = (long long)r * C;
            if ((long long)j < cap) dest = expert_offset[e] + j;
        }
        dest_of[c * WAVE + lane] = dest;
        if (t < T) {
            inv[t] = dest;
            if (dest >= 0) perm[dest] = t;
            if (t >= K) perm[t] = -1;
        }
    }
    __syncthreads();
    if (!x) return;
    int rows = T - base < DSP_TOKENS ? T - base : DSP_TOKENS;
    int total = rows * vec_per_row;
    const VecT *src = x + (size_t)base * vec_per_row;
    for (int i = tid; i < total; i += DSP_THREADS * 4) {
        VecT v[4];
        int dst[4], col[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int ii = i + u * DSP_THREADS;
            dst[u] = -1;
            if (ii < total) {
                int row = ii / vec_per_row;
                col[u] = ii - row * vec_per_row;
                dst[u] = dest_of[row];
                if (dst[u] >= 0) v[u] = src[ii];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (dst[u] >= 0) x_perm[(size_t)dst[u] * vec_per_row + col[u]] = v[u];
    }
}

}  // namespace moe

using namespace moe;

extern "C" size_t moe_dispatch_workspace_bytes(int T, int E)
{
    if (T < 0 || E <= 0) return 0;
    size_t nb = (size_t)ceil_div(T, DSP_TOKENS);
    return align_up((nb > 0 ? nb : 1) * (size_t)E * sizeof(int32_t), 256);
}

extern "C" int moe_dispatch(const void *x, const int32_t *expert_idx, const int32_t *replicas, int T, int d,
                            int E, int slot_capacity, int max_slots, int dtype, int32_t *counts,
                            int32_t *kept, int32_t *expert_offset, int32_t *slot_offset, int32_t *perm,
                            int32_t *inv, void *x_perm, void *ws, size_t ws_bytes, void *stream)
{
    MOE_REQUIRE(T >= 0 && d > 0 && E > 0 && slot_capacity >= 1 && max_slots >= 0, MOE_ERR_INVALID_ARG,
                "moe_dispatch: T=%d d=%d E=%d slot_capacity=%d max_slots=%d out of range", T, d, E,
                slot_capacity, max_slots);
    MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_ERR_INVALID_ARG, "moe_dispatch: unknown dtype %d",
                dtype);
    MOE_REQUIRE(E <= MOE_MAX_EXPERTS, MOE_ERR_UNSUPPORTED, "moe_dispatch: E=%d exceeds %d", E,
                MOE_MAX_EXPERTS);
    MOE_REQUIRE(counts && kept && expert_offset && (T == 0 || (expert_idx && perm && inv)),
                MOE_ERR_INVALID_ARG, "moe_dispatch: null output or id pointer");
    MOE_REQUIRE((x == nullptr) == (x_perm == nullptr), MOE_ERR_INVALID_ARG,
                "moe_dispatch: x and x_perm must both be given or both be NULL");
    MOE_REQUIRE(!slot_offset || max_slots >= E, MOE_ERR_INVALID_ARG,
                "moe_dispatch: max_slots=%d smaller than E=%d", max_slots, E);
    size_t esz = dtype == MOE_F32 ? 4 : 2;
    MOE_REQUIRE(((size_t)d * esz) % 16 == 0, MOE_ERR_INVALID_ARG,
                "moe_dispatch: row size %zu bytes is not a multiple of 16", (size_t)d * esz);
    MOE_REQUIRE(aligned16(x) && aligned16(x_perm), MOE_ERR_INVALID_ARG, "moe_dispatch: x / x_perm misaligned");
    MOE_REQUIRE(ws && ws_bytes >= moe_dispatch_workspace_bytes(T, E), MOE_ERR_WORKSPACE,
                "moe_dispatch: workspace of %zu bytes needed, %zu given", moe_dispatch_workspace_bytes(T, E),
                ws_bytes);
    hipStream_t st = (hipStream_t)stream;
    int nb = ceil_div(T, DSP_TOKENS);
    int32_t *block_hist = (int32_t *)ws;
    if (nb > 0) {
        hipLaunchKernelGGL(dispatch_hist_kernel, dim3(nb), dim3(DSP_THREADS), 0, st, expert_idx, T, E, block_hist);
        MOE_CHECK_LAUNCH("moe_dispatch/hist");
    }
    hipLaunchKernelGGL(dispatch_scan_kernel, dim3(1), dim3(1024), 0, st, block_hist, nb, E, replicas,
                       slot_capacity, max_slots, counts, kept, expert_offset, slot_offset);
    MOE_CHECK_LAUNCH("moe_dispatch/scan");
    if (nb > 0) {
        int nbits = 0;
        while ((1 << nbits) < E) ++nbits;
        int vec_per_row = (int)((size_t)d * esz / 16);
        hipLaunchKernelGGL(dispatch_permute_kernel<uint4>, dim3(nb), dim3(DSP_THREADS), 0, st, (const uint4 *)x,
                           expert_idx, replicas, T, vec_per_row, E, nbits, slot_capacity, block_hist,
                           expert_offset, perm, inv, (uint4 *)x_perm);
        MOE_CHECK_LAUNCH("moe_dispatch/permute");
    }
    return MOE_OK;
}
