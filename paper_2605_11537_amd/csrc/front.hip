// moe_plan_dispatch: replica_plan followed by the index tables of moe_dispatch, as one call.
//
// For small batches (at most FRONT_MAX_TOKENS ids on either side, E <= FRONT_MAX_EXPERTS) both run in
// ONE workgroup of 1024 threads: the separate calls are three dependent launches (plan, histogram,
// permute) of a few microseconds each in front of the expert FFN, each a chain of two or three memory
// round trips, and at a few thousand tokens that chain is a tenth of the layer.  Steps:
//   A  histogram of the plan ids and, from the routed ids, per 64-token chunk and expert the number of
//      tokens (lanes with equal ids are matched through LDS; a token keeps its rank inside the chunk)
//   B  wavefront 0: the integer allocation of the plan; the other wavefronts: per expert, prefix of the
//      chunk counts (two levels: inside segments of 8 chunks, then over the segments) and the total.
//      When the plan ids ARE the routed ids, they are read and matched once for both.
//   C  per expert: kept = min(total, replicas * C); scans over experts for the first row of every expert
//      and the first slot; slot tables
//   D  per token: row = first row of its expert + prefix of its chunk + rank in the chunk, if kept
// Larger inputs: block histograms of the ids, then the dispatch's permute kernel with the plan made inside it
// (every workgroup for itself), two or three launches instead of four.  Same tables, bit for bit, either way.
#include "plan_alloc.h"
#include "route.h"

namespace moe {

constexpr int FRONT_MAX_TOKENS = 8192;
constexpr int FRONT_MAX_EXPERTS = 256;
constexpr int FRONT_CHUNKS = FRONT_MAX_TOKENS / WAVE;              // 128
constexpr int FRONT_ROUNDS = FRONT_MAX_TOKENS / PLAN_THREADS;      // chunks per wavefront

constexpr int FRONT_SEG = 8;                                       // chunks per segment of the two-level prefix
constexpr int FRONT_SEGS = FRONT_CHUNKS / FRONT_SEG;               // 16
constexpr int FRONT_LD = FRONT_MAX_EXPERTS + 2;                    // row stride of the chunk table (bank spread)

// Exclusive scans of two ints per thread over the first 256 threads (experts) of the workgroup in one
// pass; every thread calls it.  sums: LDS scratch of 10 ints; totals come back in tot0 / tot1.
__device__ __forceinline__ void expert_scan2(int v0, int v1, int &ex0, int &ex1, int &tot0, int &tot1, int *sums)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int i0 = v0, i1 = v1;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int a = __shfl_up(i0, o, 64), b = __shfl_up(i1, o, 64);
        if (lane >= o) {
            i0 += a;
            i1 += b;
        }
    }
    if (w < 4 && lane == 63) {
        sums[w] = i0;
        sums[4 + w] = i1;
    }
    __syncthreads();
    int b0 = 0, b1 = 0, t0 = 0, t1 = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int a = sums[i], b = sums[4 + i];
        b0 += i < w ? a : 0;
        b1 += i < w ? b : 0;
        t0 += a;
        t1 += b;
    }
    ex0 = b0 + i0 - v0;
    ex1 = b1 + i1 - v1;
    tot0 = t0;
    tot1 = t1;
}

// SAME: the plan is made from the routed ids themselves (no predictor): their histogram is gathered
// along with the chunk counts, the plan ids are not read a second time.
template <int PLAN_PER_LANE, bool SAME>
__global__ __launch_bounds__(PLAN_THREADS) void plan_dispatch_small_kernel(
    const int32_t *__restrict__ plan_idx, int n_plan, const int32_t *__restrict__ idx, int T, int n_tokens, int E,
    int R, int C, int policy, int max_slots, int32_t *__restrict__ plan_counts,
    int32_t *__restrict__ replicas, int32_t *__restrict__ slot_base, int32_t *__restrict__ slot_expert,
    int32_t *__restrict__ n_slots, int32_t *__restrict__ counts, int32_t *__restrict__ kept,
    int32_t *__restrict__ expert_offset, int32_t *__restrict__ slot_offset, int32_t *__restrict__ perm,
    int32_t *__restrict__ inv, int32_t *__restrict__ row_token)
{
    __shared__ unsigned short chunk_cnt[FRONT_CHUNKS][FRONT_LD];   // count, then prefix inside its segment
    __shared__ int seg_tot[FRONT_MAX_EXPERTS][FRONT_SEGS + 1];     // per expert: segment totals, then their prefix
    __shared__ unsigned long long match[PLAN_THREADS / WAVE][FRONT_MAX_EXPERTS];   // per wavefront and expert: lanes
    __shared__ int hist[MOE_MAX_EXPERTS];
    __shared__ int rep[MOE_MAX_EXPERTS];
    __shared__ int tot_e[FRONT_MAX_EXPERTS], eoff_e[FRONT_MAX_EXPERTS], cap_e[FRONT_MAX_EXPERTS];
    __shared__ int wave_sums[16];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n_chunks = (T + WAVE - 1) / WAVE;
    const int n_segs = (n_chunks + FRONT_SEG - 1) / FRONT_SEG;

    // all ids of this thread are fetched up front, so both sets are one memory round trip
    int my_e[FRONT_ROUNDS], my_rank[FRONT_ROUNDS], plan_e[FRONT_ROUNDS];
#pragma unroll
    for (int rd = 0; rd < FRONT_ROUNDS; ++rd) {
        const int t = (rd * 16 + w) * WAVE + lane;
        my_e[rd] = t < T ? idx[t] : -1;
        plan_e[rd] = (!SAME && t < n_plan) ? plan_idx[t] : -1;
    }
    for (int e = tid; e < MOE_MAX_EXPERTS; e += PLAN_THREADS) {
        hist[e] = 0;
        rep[e] = 0;
    }
    for (int i = lane; i < E; i += WAVE) match[w][i] = 0ull;
    for (int i = tid; i < n_segs * FRONT_SEG * (FRONT_LD / 2); i += PLAN_THREADS)
        reinterpret_cast<unsigned int *>(&chunk_cnt[0][0])[i] = 0u;
    __syncthreads();

    // ---- A: lanes of a wavefront with equal ids find each other through a 64-bit lane mask per expert in
    // LDS (one atomic OR, one read, one clear per 64 ids; a ballot per id bit costs ~100 vector
    // instructions per 64 ids, and with 16 wavefronts on one CU this step is bound by instruction issue)
    auto match_lanes = [&](int e, bool valid) {
        unsigned long long *slot = &match[w][valid ? e : 0];
        if (valid) atomicOr(slot, 1ull << lane);
        const unsigned long long m = valid ? __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) : 0ull;
        if (valid && (m & ((1ull << lane) - 1ull)) == 0)
            __hip_atomic_store(slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);   // for the next 64 ids
        return m;
    };
#pragma unroll
    for (int rd = 0; rd < FRONT_ROUNDS; ++rd) {
        const int c = rd * 16 + w;
        if (!SAME && c * WAVE < n_plan) {           // uniform per wavefront
            const int e = plan_e[rd];
            const bool valid = e >= 0 && e < E;
            const unsigned long long mask = match_lanes(e, valid);
            if (valid && (mask & ((1ull << lane) - 1ull)) == 0) atomicAdd(&hist[e], __popcll(mask));
        }
        my_rank[rd] = 0;
        if (c < n_chunks) {
            const int e = my_e[rd];
            const bool valid = e >= 0 && e < E;
            const unsigned long long mask = match_lanes(e, valid);
            const int rank = __popcll(mask & ((1ull << lane) - 1ull));
            if (valid && rank == 0) {
                chunk_cnt[c][e] = (unsigned short)__popcll(mask);
                if (SAME) atomicAdd(&hist[e], __popcll(mask));      // the plan's histogram is the same count
            }
            my_e[rd] = valid ? e : -1;
            my_rank[rd] = rank;
        }
    }
    __syncthreads();

    // ---- B: wavefront 0 runs the allocation; the others the prefix of the chunk counts inside segments of
    // 8 chunks (one expert and segment per thread)
    if (tid < WAVE) {
        plan_allocate_wave<PLAN_PER_LANE>(hist, rep, SAME ? T : n_plan, E, R, C, policy, replicas, plan_counts);
    } else {
        for (int i = tid - WAVE; i < E * n_segs; i += PLAN_THREADS - WAVE) {
            const int e = i % E, g = i / E;
            int v[FRONT_SEG];
#pragma unroll
            for (int u = 0; u < FRONT_SEG; ++u) v[u] = chunk_cnt[g * FRONT_SEG + u][e];
            int run = 0;
#pragma unroll
            for (int u = 0; u < FRONT_SEG; ++u) {
                chunk_cnt[g * FRONT_SEG + u][e] = (unsigned short)run;
                run += v[u];
            }
            seg_tot[e][g] = run;
        }
    }
    __syncthreads();
    // per expert: prefix over its segments, total
    if (tid < E) {
        int v[FRONT_SEGS];
#pragma unroll
        for (int g = 0; g < FRONT_SEGS; ++g) v[g] = g < n_segs ? seg_tot[tid][g] : 0;
        int run = 0;
#pragma unroll
        for (int g = 0; g < FRONT_SEGS; ++g) {
            seg_tot[tid][g] = run;
            run += v[g];
        }
        tot_e[tid] = run;
    }
    __syncthreads();

    // ---- C: thread e owns expert e
    const int r_e = tid < E ? rep[tid] : 0;
    const int n_e = tid < E ? tot_e[tid] : 0;
    const long long cap = (long long)r_e * C;
    const int k_e = (long long)n_e < cap ? n_e : (int)cap;
    int off_e, sb_e, K, P;
    expert_scan2(k_e, r_e, off_e, sb_e, K, P, wave_sums);
    if (tid < E) {
        eoff_e[tid] = off_e;
        cap_e[tid] = k_e;
        counts[tid] = n_e;
        kept[tid] = k_e;
        expert_offset[tid] = off_e;
        if (slot_base) slot_base[tid] = sb_e;
        const int q = k_e / r_e, rem = k_e % r_e;      // r_e >= 1 for every expert
        for (int j = 0; j < r_e; ++j) {
            const int p = sb_e + j;
            if (slot_expert) slot_expert[p] = tid;
            if (slot_offset && p <= max_slots) slot_offset[p] = off_e + j * q + (j < rem ? j : rem);
        }
    }
    if (tid == 0) {
        expert_offset[E] = K;
        if (slot_base) slot_base[E] = P;
        if (n_slots) n_slots[0] = P;
    }
    if (slot_expert)
        for (int p = P + tid; p < E + R; p += PLAN_THREADS) slot_expert[p] = -1;
    if (slot_offset)
        for (int p = P + tid; p <= max_slots; p += PLAN_THREADS) slot_offset[p] = K;
    __syncthreads();

    // ---- D
#pragma unroll
    for (int rd = 0; rd < FRONT_ROUNDS; ++rd) {
        const int c = rd * 16 + w;
        const int t = c * WAVE + lane;
        if (t >= T) continue;
        int dest = -1;
        const int e = my_e[rd];
        if (e >= 0) {
            const int j = seg_tot[e][c / FRONT_SEG] + chunk_cnt[c][e] + my_rank[rd];
            if (j < cap_e[e]) dest = eoff_e[e] + j;
        }
        inv[t] = dest;
        if (dest >= 0) perm[dest] = t;
        if (t >= K) perm[t] = -1;
        if (row_token) {
            if (dest >= 0) row_token[dest] = t % n_tokens;
            if (t >= K) row_token[t] = -1;
        }
    }
}

}  // namespace moe

using namespace moe;

static inline bool front_fused(int n_plan, int A, int E)
{
    return n_plan <= FRONT_MAX_TOKENS && A <= FRONT_MAX_TOKENS && E <= FRONT_MAX_EXPERTS;
}

extern "C" size_t moe_plan_dispatch_workspace_bytes(int n_plan, int T, int k, int E)
{
    if (n_plan < 0 || T < 0 || k < 1 || E <= 0 || (long long)T * k > 0x7fffffffLL) return 0;
    if (front_fused(n_plan, T * k, E)) return 0;
    return dispatch_block_hist_bytes(T * k, E) +
           align_up((size_t)(ceil_div(n_plan, plan_partial_block()) + 1) * E * sizeof(int32_t), 256);
}

extern "C" int moe_plan_dispatch(const int32_t *plan_idx, int n_plan, const int32_t *expert_idx, int T, int k,
                                 int E, int budget, int slot_capacity, int policy, int32_t *plan_counts,
                                 int32_t *replicas, int32_t *slot_base, int32_t *slot_expert, int32_t *n_slots,
                                 int32_t *counts, int32_t *kept, int32_t *expert_offset, int32_t *slot_offset,
                                 int32_t *perm, int32_t *inv, int32_t *row_token, void *ws, size_t ws_bytes,
                                 void *stream)
{
    MOE_REQUIRE(n_plan >= 0 && T >= 0 && E > 0 && budget >= 0 && slot_capacity >= 1, MOE_ERR_INVALID_ARG,
                "moe_plan_dispatch: n_plan=%d T=%d E=%d budget=%d slot_capacity=%d out of range", n_plan, T, E,
                budget, slot_capacity);
    MOE_REQUIRE(k >= 1 && k <= MOE_MAX_TOPK && (long long)T * k <= 0x7fffffffLL, MOE_ERR_INVALID_ARG,
                "moe_plan_dispatch: k=%d out of range (k <= %d, T*k < 2^31)", k, MOE_MAX_TOPK);
    MOE_REQUIRE(policy == 0 || policy == 1, MOE_ERR_INVALID_ARG, "moe_plan_dispatch: unknown policy %d", policy);
    MOE_REQUIRE(E <= MOE_MAX_EXPERTS, MOE_ERR_UNSUPPORTED, "moe_plan_dispatch: E=%d exceeds %d", E, MOE_MAX_EXPERTS);
    MOE_REQUIRE((long long)E + budget <= MOE_MAX_SLOTS, MOE_ERR_UNSUPPORTED,
                "moe_plan_dispatch: E+budget=%lld exceeds %d", (long long)E + budget, MOE_MAX_SLOTS);
    const int A = T * k;
    MOE_REQUIRE((n_plan == 0 || plan_idx) && plan_counts && replicas && slot_base && slot_expert && n_slots &&
                    counts && kept && expert_offset && slot_offset && (A == 0 || (expert_idx && perm && inv)),
                MOE_ERR_INVALID_ARG, "moe_plan_dispatch: null pointer");
    MOE_REQUIRE(k == 1 || A == 0 || row_token, MOE_ERR_INVALID_ARG, "moe_plan_dispatch: null row_token with k > 1");
    const int max_slots = E + budget;
    const bool same = plan_idx == expert_idx && n_plan == A;
    if (!front_fused(n_plan, A, E)) {
        // block histograms of the routed ids (and of the plan ids, if they are others), then one kernel that
        // makes the plan and the permutation
        const size_t hist_bytes = dispatch_block_hist_bytes(A, E);
        const size_t need = moe_plan_dispatch_workspace_bytes(n_plan, T, k, E);
        MOE_REQUIRE(ws && aligned16(ws) && ws_bytes >= need, MOE_ERR_WORKSPACE,
                    "moe_plan_dispatch: workspace of %zu bytes needed, %zu given", need, ws_bytes);
        int32_t *block_hist = (int32_t *)ws;
        int32_t *partial = nullptr;
        int n_partial = 0;
        if (!same) {
            partial = (int32_t *)((char *)ws + hist_bytes);
            n_partial = ceil_div(n_plan, plan_partial_block());
            if (n_partial > 0) {
                int rc = plan_partial_launch(plan_idx, n_plan, E, partial, (hipStream_t)stream, "moe_plan_dispatch");
                if (rc != MOE_OK) return rc;
            }
        }
        return dispatch_planned_launch(expert_idx, A, T, E, slot_capacity, budget, policy, partial, n_partial,
                                       same ? A : n_plan, block_hist, plan_counts, replicas, slot_base, slot_expert,
                                       n_slots, counts, kept, expert_offset, slot_offset, perm, inv, row_token,
                                       (hipStream_t)stream, "moe_plan_dispatch");
    }
    auto kern = E <= 128 ? (same ? plan_dispatch_small_kernel<2, true> : plan_dispatch_small_kernel<2, false>)
                         : (same ? plan_dispatch_small_kernel<4, true> : plan_dispatch_small_kernel<4, false>);
    hipLaunchKernelGGL(kern, dim3(1), dim3(PLAN_THREADS), 0, (hipStream_t)stream, plan_idx, n_plan, expert_idx, A,
                       T > 0 ? T : 1, E, budget, slot_capacity, policy, max_slots, plan_counts, replicas,
                       slot_base, slot_expert, n_slots, counts, kept, expert_offset, slot_offset, perm, inv,
                       row_token);
    MOE_CHECK_LAUNCH("moe_plan_dispatch");
    return MOE_OK;
}
