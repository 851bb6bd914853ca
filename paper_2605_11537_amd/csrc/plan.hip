// replica_plan: per-expert replica counts from (predicted) expert ids, within a slot budget.
//
// One workgroup of 1024 threads (for batches above 8192 ids the histogram is first built by one
// workgroup per 8192 ids into the workspace and summed here).  All threads build the histogram of
// ids in LDS (ids that share a wavefront load are pre-counted with ballots, so a hot expert does
// not serialise the LDS atomics).  Wavefront 0 then runs the integer allocation entirely in
// registers: lane l owns experts l, l+64, ..., sums and arg-max searches are wavefront reductions,
// so the one-by-one hand-out of the slots left by the floors needs no barrier.  All threads
// finally scan the replica counts into slot_base and write the slot -> expert table.
#include "plan_alloc.h"
#include "route.h"

namespace moe {

// large batches: one workgroup per PLAN_BLOCK_TOKENS ids writes its histogram to partial[b][E]
__global__ __launch_bounds__(PLAN_THREADS) void replica_plan_partial_kernel(const int32_t *__restrict__ idx, int T,
                                                                            int E, int nbits,
                                                                            int32_t *__restrict__ partial)
{
    __shared__ int hist[MOE_MAX_EXPERTS];
    for (int e = threadIdx.x; e < E; e += PLAN_THREADS) hist[e] = 0;
    __syncthreads();
    int t0 = blockIdx.x * PLAN_BLOCK_TOKENS;
    int t1 = t0 + PLAN_BLOCK_TOKENS < T ? t0 + PLAN_BLOCK_TOKENS : T;
    plan_histogram(idx, t0, t1, E, nbits, hist);
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += PLAN_THREADS) partial[(size_t)blockIdx.x * E + e] = hist[e];
}

// PLAN_PER_LANE = experts per lane of wavefront 0 (E <= 64 * PLAN_PER_LANE).
// n_partial == 0: the histogram is built here from idx; otherwise it is the sum of n_partial
// partial histograms.
template <int PLAN_PER_LANE>
__global__ __launch_bounds__(PLAN_THREADS) void replica_plan_kernel(
    const int32_t *__restrict__ idx, int T, int E, int nbits, int R, int C, int policy,
    const int32_t *__restrict__ partial, int n_partial, int32_t *__restrict__ plan_counts,
    int32_t *__restrict__ replicas, int32_t *__restrict__ slot_base, int32_t *__restrict__ slot_expert,
    int32_t *__restrict__ n_slots)
{
    __shared__ int hist[MOE_MAX_EXPERTS];
    __shared__ int rep[MOE_MAX_EXPERTS];
    __shared__ int wave_sums[16];
    __shared__ int total_p;
    const int tid = threadIdx.x, lane = tid & 63;
    for (int e = tid; e < MOE_MAX_EXPERTS; e += PLAN_THREADS) {
        int h = 0;
        if (n_partial > 0 && e < E)
            for (int b = 0; b < n_partial; ++b) h += partial[(size_t)b * E + e];
        hist[e] = h;
        rep[e] = 0;
    }
    __syncthreads();
    if (n_partial == 0) plan_histogram(idx, 0, T, E, nbits, hist);
    __syncthreads();

    if (tid < WAVE) plan_allocate_wave<PLAN_PER_LANE>(hist, rep, T, E, R, C, policy, replicas, plan_counts);
    __syncthreads();

    // slot_base = exclusive scan of the replica counts (one expert per thread)
    int v = tid < E ? rep[tid] : 0;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int nn = __shfl_up(inc, o, 64);
        if (lane >= o) inc += nn;
    }
    if (lane == 63) wave_sums[tid >> 6] = inc;
    __syncthreads();
    if (tid < WAVE) {
        int s = lane < 16 ? wave_sums[lane] : 0, si = s;
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
            int nn = __shfl_up(si, o, 64);
            if (lane >= o) si += nn;
        }
        if (lane < 16) wave_sums[lane] = si - s;
        if (lane == 15) total_p = si;
    }
    __syncthreads();
    int base = wave_sums[tid >> 6] + inc - v;
    int P = total_p;
    if (tid < E) {
        if (slot_base) slot_base[tid] = base;
        if (slot_expert)
            for (int k = 0; k < v; ++k) slot_expert[base + k] = tid;
    }
    if (tid == 0) {
        if (slot_base) slot_base[E] = P;
        if (n_slots) n_slots[0] = P;
    }
    if (slot_expert)
        for (int p = P + tid; p < E + R; p += PLAN_THREADS) slot_expert[p] = -1;
}

int plan_partial_block() { return PLAN_BLOCK_TOKENS; }

int plan_partial_launch(const int32_t *idx, int T, int E, int32_t *partial, hipStream_t st, const char *who)
{
    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;
    hipLaunchKernelGGL(replica_plan_partial_kernel, dim3(ceil_div(T, PLAN_BLOCK_TOKENS)), dim3(PLAN_THREADS), 0, st, idx,
                       T, E, nbits, partial);
    MOE_CHECK_LAUNCH(who);
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" size_t replica_plan_workspace_bytes(int T, int E)
{
    if (T <= PLAN_BLOCK_TOKENS || E <= 0) return 0;   // one workgroup does it all
    return align_up((size_t)ceil_div(T, PLAN_BLOCK_TOKENS) * E * sizeof(int32_t), 256);
}

extern "C" int replica_plan(const int32_t *idx, int T, int E, int budget, int slot_capacity, int policy,
                            int32_t *plan_counts, int32_t *replicas, int32_t *slot_base,
                            int32_t *slot_expert, int32_t *n_slots, void *ws, size_t ws_bytes, void *stream)
{
    MOE_REQUIRE(T >= 0 && E > 0 && budget >= 0 && slot_capacity >= 1, MOE_ERR_INVALID_ARG,
                "replica_plan: T=%d E=%d budget=%d slot_capacity=%d out of range", T, E, budget,
                slot_capacity);
    MOE_REQUIRE(policy == 0 || policy == 1, MOE_ERR_INVALID_ARG, "replica_plan: unknown policy %d", policy);
    MOE_REQUIRE(E <= MOE_MAX_EXPERTS, MOE_ERR_UNSUPPORTED, "replica_plan: E=%d exceeds %d", E, MOE_MAX_EXPERTS);
    MOE_REQUIRE((long long)E + budget <= MOE_MAX_SLOTS, MOE_ERR_UNSUPPORTED,
                "replica_plan: E+budget=%lld exceeds %d", (long long)E + budget, MOE_MAX_SLOTS);
    MOE_REQUIRE((T == 0 || idx) && plan_counts && replicas, MOE_ERR_INVALID_ARG, "replica_plan: null pointer");
    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;
    size_t need = replica_plan_workspace_bytes(T, E);
    MOE_REQUIRE(need == 0 || (ws && ws_bytes >= need), MOE_ERR_WORKSPACE,
                "replica_plan: workspace of %zu bytes needed, %zu given", need, ws_bytes);
    int n_partial = 0;
    if (need > 0) {
        n_partial = ceil_div(T, PLAN_BLOCK_TOKENS);
        hipLaunchKernelGGL(replica_plan_partial_kernel, dim3(n_partial), dim3(PLAN_THREADS), 0, (hipStream_t)stream,
                           idx, T, E, nbits, (int32_t *)ws);
        MOE_CHECK_LAUNCH("replica_plan/partial");
    }
    auto kern = E <= 128 ? replica_plan_kernel<2> : E <= 256 ? replica_plan_kernel<4> : replica_plan_kernel<16>;
    hipLaunchKernelGGL(kern, dim3(1), dim3(PLAN_THREADS), 0, (hipStream_t)stream, idx, T, E, nbits, budget,
                       slot_capacity, policy, (const int32_t *)ws, n_partial, plan_counts, replicas, slot_base,
                       slot_expert, n_slots);
    MOE_CHECK_LAUNCH("replica_plan");
    return MOE_OK;
}
