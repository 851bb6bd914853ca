// moe_dispatch: capacity-limited, stable dispatch of tokens to expert slots.
//
// Three kernels, no global atomics, so the permutation is the stable one whatever the
// hardware scheduling:
//   hist     one workgroup per 1024 tokens: LDS histogram of expert ids -> block_hist[b][e]
//   permute  one workgroup per 1024 tokens: per expert, prefix over the earlier token blocks,
//            kept counts, expert offsets (scan over experts), slot offsets (balanced split
//            per expert); then the rank of every token among the tokens of its expert
//            = prefix over earlier blocks + prefix over earlier 64-token chunks of the block
//            (LDS table) + rank inside the chunk (wavefront ballots, one per id bit);
//            writes inv / perm
//   gather   whole-chip copy of the kept rows, x_perm[pos] = x[perm[pos]], 16-byte accesses
#include <mutex>

#include "plan_alloc.h"
#include "route.h"

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

// exclusive scan over E <= 1024 values held 4 per thread (thread t owns experts 4t .. 4t+3)
__device__ __forceinline__ void block_scan4_256(const int (&v)[4], int (&excl)[4], int *wave_sums, int *total_out)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int local = v[0] + v[1] + v[2] + v[3];
    int inc = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int n = __shfl_up(inc, o, 64);
        if (lane >= o) inc += n;
    }
    if (lane == 63) wave_sums[w] = inc;
    __syncthreads();
    int base = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) base += i < w ? wave_sums[i] : 0;
    if (threadIdx.x == DSP_THREADS - 1) *total_out = base + inc;
    int run = base + inc - local;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        excl[i] = run;
        run += v[i];
    }
    __syncthreads();
}

// One workgroup per 1024 tokens.  Every workgroup first rebuilds, from the per-block
// histograms, the per-expert totals, its own prefix over earlier blocks, the kept counts and
// the expert offsets (a few KB of reads; cheaper than a separate single-workgroup launch in
// the dependency chain); workgroup 0 also writes those tables and the slot offsets out.
//
// PPL > 0: the replica plan is made here as well (PPL = experts per lane of the allocating wavefront), by
// every workgroup for itself from the same counts -- the plan's own ids' histograms in plan_partial, or, when
// that is NULL, the routed ids' totals just rebuilt (a plan made from the routed ids themselves) -- so the
// plan kernels and their place in the dependency chain go away; workgroup 0 writes the plan's tables.
struct PlanArgs {
    const int32_t *plan_partial;
    int n_partial, n_plan_ids, R, policy;
    int32_t *plan_counts, *replicas, *slot_base, *slot_expert, *n_slots;
};

template <int PPL>
__global__ __launch_bounds__(DSP_THREADS) void dispatch_permute_kernel(
    const int32_t *__restrict__ idx, const int32_t *__restrict__ replicas, int T, int E, int nbits, int C, int nb,
    int max_slots, const int32_t *__restrict__ block_hist, int32_t *__restrict__ counts, int32_t *__restrict__ kept,
    int32_t *__restrict__ expert_offset, int32_t *__restrict__ slot_offset, int32_t *__restrict__ perm,
    int32_t *__restrict__ inv, int n_tokens, int32_t *__restrict__ row_token, PlanArgs pa)
{
    __shared__ unsigned short chunk_cnt[DSP_CHUNKS][MOE_MAX_EXPERTS];
    __shared__ int before_e[MOE_MAX_EXPERTS];   // tokens of e in earlier blocks
    __shared__ int eoff_e[MOE_MAX_EXPERTS];     // first permuted row of e
    __shared__ int cap_e[MOE_MAX_EXPERTS];      // kept count of e
    __shared__ int wave_sums[4];
    __shared__ int total_k, total_p;
    __shared__ int plan_hist[PPL > 0 ? MOE_MAX_EXPERTS : 1];
    __shared__ int rep[PPL > 0 ? MOE_MAX_EXPERTS : 1];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int base = blockIdx.x * DSP_TOKENS;
    for (int i = tid; i < DSP_CHUNKS * E; i += DSP_THREADS) chunk_cnt[i / E][i % E] = 0;

    // ---- tables.  Pass 1: thread per expert (strided), coalesced over the block histograms.
    for (int e = tid; e < E; e += DSP_THREADS) {
        int tot = 0, bef = 0;
        // 16 loads in flight per thread: at 64 blocks this loop is four memory round trips instead of eight
#pragma unroll 16
        for (int b = 0; b < nb; ++b) {
            int v = block_hist[(size_t)b * E + e];
            bef += b < (int)blockIdx.x ? v : 0;
            tot += v;
        }
        before_e[e] = bef;
        eoff_e[e] = tot;      // total count, replaced by the offset below
        if (PPL > 0) {
            int h = tot;
            if (pa.plan_partial) {
                h = 0;
                for (int b = 0; b < pa.n_partial; ++b) h += pa.plan_partial[(size_t)b * E + e];
            }
            plan_hist[e] = h;
        } else {
            int r = replicas ? replicas[e] : 1;
            if (r < 1) r = 1;
            long long cap = (long long)r * C;
            cap_e[e] = (long long)tot < cap ? tot : (int)cap;
        }
    }
    // ---- ranks inside the block.  With the plan made in here, wavefront 0 is busy with the allocation (a
    // dependent chain of microseconds) and the other three rank all 16 chunks meanwhile; otherwise all four
    // wavefronts take four chunks each.
    constexpr int RANK_WAVES = PPL > 0 ? DSP_THREADS / WAVE - 1 : DSP_THREADS / WAVE;
    constexpr int RANK_ROUNDS = (DSP_CHUNKS + RANK_WAVES - 1) / RANK_WAVES;
    const int rank_w = PPL > 0 ? w - 1 : w;          // -1: this wavefront ranks nothing
    int my_e[RANK_ROUNDS], my_rank[RANK_ROUNDS];
    auto rank_chunks = [&]() {
#pragma unroll
        for (int rd = 0; rd < RANK_ROUNDS; ++rd) {
            const int c = rd * RANK_WAVES + rank_w;
            my_e[rd] = -1;
            my_rank[rd] = 0;
            if (c >= DSP_CHUNKS) continue;            // uniform per wavefront
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
    };
    if (PPL > 0) {
        for (int e = E + tid; e < MOE_MAX_EXPERTS; e += DSP_THREADS) plan_hist[e] = 0;
        __syncthreads();                  // the chunk table is clear, the plan's histogram complete
        if (tid < WAVE)
            plan_allocate_wave<(PPL > 0 ? PPL : 1)>(plan_hist, rep, pa.n_plan_ids, E, pa.R, C, pa.policy, pa.replicas,
                                                    pa.plan_counts, blockIdx.x == 0);
        else
            rank_chunks();
        __syncthreads();
        for (int e = tid; e < E; e += DSP_THREADS) {
            const long long cap = (long long)rep[e] * C;
            cap_e[e] = (long long)eoff_e[e] < cap ? eoff_e[e] : (int)cap;
        }
    }
    __syncthreads();
    // Pass 2: thread t owns experts 4t..4t+3 for the scans over experts
    int n4[4], r4[4], k4[4], off4[4], sb4[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int e = tid * 4 + i;
        n4[i] = e < E ? eoff_e[e] : 0;
        k4[i] = e < E ? cap_e[e] : 0;
        int r = (e < E) ? (PPL > 0 ? rep[e] : (replicas ? replicas[e] : 1)) : 0;
        if (e < E && r < 1) r = 1;
        r4[i] = r;
    }
    __syncthreads();
    block_scan4_256(k4, off4, wave_sums, &total_k);
    block_scan4_256(r4, sb4, wave_sums, &total_p);
    const int K = total_k, P = total_p;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int e = tid * 4 + i;
        if (e < E) eoff_e[e] = off4[i];
    }
    if (blockIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int e = tid * 4 + i;
            if (e < E) {
                counts[e] = n4[i];
                kept[e] = k4[i];
                expert_offset[e] = off4[i];
                if (slot_offset) {
                    int q = k4[i] / r4[i], rem = k4[i] % r4[i];
                    for (int k = 0; k < r4[i]; ++k) {
                        int p = sb4[i] + k;
                        if (p <= max_slots) slot_offset[p] = off4[i] + k * q + (k < rem ? k : rem);
                    }
                }
                if (PPL > 0) {
                    if (pa.slot_base) pa.slot_base[e] = sb4[i];
                    if (pa.slot_expert)
                        for (int k = 0; k < r4[i]; ++k) pa.slot_expert[sb4[i] + k] = e;
                }
            }
        }
        if (tid == 0) expert_offset[E] = K;
        if (slot_offset)
            for (int p = P + tid; p <= max_slots; p += DSP_THREADS) slot_offset[p] = K;
        if (PPL > 0) {
            if (tid == 0) {
                if (pa.slot_base) pa.slot_base[E] = P;
                if (pa.n_slots) pa.n_slots[0] = P;
            }
            if (pa.slot_expert)
                for (int p = P + tid; p < E + pa.R; p += DSP_THREADS) pa.slot_expert[p] = -1;
        }
    }
    if (T == 0) return;

    if (PPL == 0) rank_chunks();
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
#pragma unroll
    for (int rd = 0; rd < RANK_ROUNDS; ++rd) {
        int c = rd * RANK_WAVES + rank_w;
        if (rank_w < 0 || c >= DSP_CHUNKS) continue;
        int t = base + c * WAVE + lane;
        int dest = -1;
        int e = my_e[rd];
        if (e >= 0) {
            int j = before_e[e] + chunk_cnt[c][e] + my_rank[rd];
            if (j < cap_e[e]) dest = eoff_e[e] + j;
        }
        if (t < T) {
            inv[t] = dest;
            if (dest >= 0) perm[dest] = t;
            if (t >= K) perm[t] = -1;
            if (row_token) {        // top-k: entry t is assignment (t / n_tokens, t % n_tokens)
                if (dest >= 0) row_token[dest] = t % n_tokens;
                if (t >= K) row_token[t] = -1;
            }
        }
    }
}

// x_perm[pos] = x[perm[pos]] for pos < K (K is not read: the permutation ends in -1 entries).  32 lanes per row, 8 rows per workgroup, 16-byte
// pieces: the scattered row reads and the contiguous writes are both whole lines, the row
// index is read once per row, and all of a lane's loads are independent.
constexpr int GATHER_ROWS = DSP_THREADS / 32;
__global__ __launch_bounds__(DSP_THREADS) void dispatch_gather_kernel(const uint4 *__restrict__ x,
                                                                      const int32_t *__restrict__ perm, int T,
                                                                      int n_tokens, int vec_per_row,
                                                                      uint4 *__restrict__ x_perm)
{
    const int pos = blockIdx.x * GATHER_ROWS + (threadIdx.x >> 5);
    const int l = threadIdx.x & 31;
    if (pos >= T) return;
    int row = perm[pos];
    if (row < 0) return;                      // past the kept rows (perm holds -1 there): nothing to copy
    if (row >= n_tokens) row %= n_tokens;     // top-k: assignment -> its token
    const uint4 *src = x + (size_t)row * vec_per_row;
    uint4 *dst = x_perm + (size_t)pos * vec_per_row;
    int c = l;
    for (; c + 96 < vec_per_row; c += 128) {
        uint4 v0 = src[c], v1 = src[c + 32], v2 = src[c + 64], v3 = src[c + 96];
        dst[c] = v0;
        dst[c + 32] = v1;
        dst[c + 64] = v2;
        dst[c + 96] = v3;
    }
    uint4 v[3];
#pragma unroll
    for (int u = 0; u < 3; ++u)
        if (c + u * 32 < vec_per_row) v[u] = src[c + u * 32];
#pragma unroll
    for (int u = 0; u < 3; ++u)
        if (c + u * 32 < vec_per_row) dst[c + u * 32] = v[u];
}

size_t dispatch_block_hist_bytes(int T, int E)
{
    size_t nb = (size_t)ceil_div(T, DSP_TOKENS);
    return align_up((nb > 0 ? nb : 1) * (size_t)E * sizeof(int32_t), 256);
}

int dispatch_planned_launch(const int32_t *expert_idx, int T, int n_tokens, int E, int slot_capacity, int budget,
                            int policy, const int32_t *plan_partial, int n_partial, int n_plan_ids,
                            int32_t *block_hist, int32_t *plan_counts, int32_t *replicas, int32_t *slot_base,
                            int32_t *slot_expert, int32_t *n_slots, int32_t *counts, int32_t *kept,
                            int32_t *expert_offset, int32_t *slot_offset, int32_t *perm, int32_t *inv,
                            int32_t *row_token, hipStream_t st, const char *who)
{
    const int nb = ceil_div(T, DSP_TOKENS);
    if (nb > 0) {
        hipLaunchKernelGGL(dispatch_hist_kernel, dim3(nb), dim3(DSP_THREADS), 0, st, expert_idx, T, E, block_hist);
        MOE_CHECK_LAUNCH(who);
    }
    int nbits = 0;
    while ((1 << nbits) < E) ++nbits;
    PlanArgs pa{plan_partial, n_partial, n_plan_ids, budget, policy, plan_counts, replicas, slot_base, slot_expert,
                n_slots};
    auto kern = E <= 128 ? dispatch_permute_kernel<2> : E <= 256 ? dispatch_permute_kernel<4> : dispatch_permute_kernel<16>;
    hipLaunchKernelGGL(kern, dim3(nb > 0 ? nb : 1), dim3(DSP_THREADS), 0, st, expert_idx, (const int32_t *)nullptr, T, E,
                       nbits, slot_capacity, nb, E + budget, block_hist, counts, kept, expert_offset, slot_offset, perm,
                       inv, n_tokens > 0 ? n_tokens : 1, row_token, pa);
    MOE_CHECK_LAUNCH(who);
    return MOE_OK;
}

// ------------------------------------------------------------------ allocation-free variant
// The per-block histograms of moe_dispatch_static live in this file-scope device array instead of a
// caller's workspace.  Every GPU the library runs on holds its own copy at its own address until the
// process ends.  In host code the array's name is only a stand-in for the symbol: its device address is
// asked of the runtime once per device and that pointer is what the kernels get.
constexpr size_t DSP_STATIC_BYTES = (size_t)1 << 20;   // 262144 table entries: e.g. 256 blocks x 1024 experts
static __device__ __align__(256) int32_t scratch[DSP_STATIC_BYTES / sizeof(int32_t)];

constexpr int DSP_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static int32_t *g_scratch_ptr[DSP_MAX_DEVICES];        // device address of `scratch` per device ordinal

static int32_t *static_scratch_of_current_device(const char *who)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= DSP_MAX_DEVICES) {
        set_error("%s: cannot tell the current device (ordinal %d, at most %d devices)", who, dev, DSP_MAX_DEVICES);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_error("%s: hipGetSymbolAddress(scratch) failed on device %d: %s", who, dev, hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = (int32_t *)p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace moe

using namespace moe;

extern "C" size_t moe_dispatch_workspace_bytes(int T, int E)
{
    if (T < 0 || E <= 0) return 0;
    size_t nb = (size_t)ceil_div(T, DSP_TOKENS);
    return align_up((nb > 0 ? nb : 1) * (size_t)E * sizeof(int32_t), 256);
}

// T entries (tokens, or k*n_tokens assignments of a top-k layer) over the rows of n_tokens tokens
static int dispatch_checked(const char *who, const void *x, const int32_t *expert_idx, const int32_t *replicas, int T,
                            int n_tokens, int d, int E, int slot_capacity, int max_slots, int dtype, int32_t *counts,
                            int32_t *kept, int32_t *expert_offset, int32_t *slot_offset, int32_t *perm, int32_t *inv,
                            int32_t *row_token, void *x_perm, void *ws, size_t ws_bytes, void *stream,
                            bool static_scratch = false)
{
    MOE_REQUIRE(T >= 0 && d > 0 && E > 0 && slot_capacity >= 1 && max_slots >= 0, MOE_ERR_INVALID_ARG,
                "%s: T=%d d=%d E=%d slot_capacity=%d max_slots=%d out of range", who, T, d, E, slot_capacity,
                max_slots);
    MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_ERR_INVALID_ARG, "%s: unknown dtype %d", who, dtype);
    MOE_REQUIRE(E <= MOE_MAX_EXPERTS, MOE_ERR_UNSUPPORTED, "%s: E=%d exceeds %d", who, E, MOE_MAX_EXPERTS);
    MOE_REQUIRE(counts && kept && expert_offset && (T == 0 || (expert_idx && perm && inv)), MOE_ERR_INVALID_ARG,
                "%s: null output or id pointer", who);
    MOE_REQUIRE((x == nullptr) == (x_perm == nullptr), MOE_ERR_INVALID_ARG,
                "%s: x and x_perm must both be given or both be NULL", who);
    MOE_REQUIRE(!slot_offset || max_slots >= E, MOE_ERR_INVALID_ARG, "%s: max_slots=%d smaller than E=%d", who,
                max_slots, E);
    size_t esz = dtype == MOE_F32 ? 4 : 2;
    MOE_REQUIRE(((size_t)d * esz) % 16 == 0, MOE_ERR_INVALID_ARG, "%s: row size %zu bytes is not a multiple of 16",
                who, (size_t)d * esz);
    MOE_REQUIRE(aligned16(x) && aligned16(x_perm), MOE_ERR_INVALID_ARG, "%s: x / x_perm misaligned", who);
    if (static_scratch) {
        MOE_REQUIRE(moe_dispatch_workspace_bytes(T, E) <= DSP_STATIC_BYTES, MOE_ERR_UNSUPPORTED,
                    "%s: ceil(T/1024)*E = %zu table entries exceed the %zu of the static scratch array "
                    "(use moe_dispatch with a workspace)",
                    who, moe_dispatch_workspace_bytes(T, E) / sizeof(int32_t), DSP_STATIC_BYTES / sizeof(int32_t));
        ws = static_scratch_of_current_device(who);
        if (!ws) return MOE_ERR_HIP;
    } else {
        MOE_REQUIRE(ws && ws_bytes >= moe_dispatch_workspace_bytes(T, E), MOE_ERR_WORKSPACE,
                    "%s: workspace of %zu bytes needed, %zu given", who, moe_dispatch_workspace_bytes(T, E), ws_bytes);
    }
    hipStream_t st = (hipStream_t)stream;
    int nb = ceil_div(T, DSP_TOKENS);
    int32_t *block_hist = (int32_t *)ws;
    if (nb > 0) {
        hipLaunchKernelGGL(dispatch_hist_kernel, dim3(nb), dim3(DSP_THREADS), 0, st, expert_idx, T, E, block_hist);
        MOE_CHECK_LAUNCH(who);
    }
    {
        int nbits = 0;
        while ((1 << nbits) < E) ++nbits;
        hipLaunchKernelGGL(dispatch_permute_kernel<0>, dim3(nb > 0 ? nb : 1), dim3(DSP_THREADS), 0, st, expert_idx,
                           replicas, T, E, nbits, slot_capacity, nb, max_slots, block_hist, counts, kept,
                           expert_offset, slot_offset, perm, inv, n_tokens > 0 ? n_tokens : 1, row_token, PlanArgs{});
        MOE_CHECK_LAUNCH(who);
        if (x && nb > 0) {
            int vec_per_row = (int)((size_t)d * esz / 16);
            int grid = ceil_div(T, GATHER_ROWS);
            hipLaunchKernelGGL(dispatch_gather_kernel, dim3(grid), dim3(DSP_THREADS), 0, st, (const uint4 *)x, perm,
                               T, n_tokens, vec_per_row, (uint4 *)x_perm);
            MOE_CHECK_LAUNCH(who);
        }
    }
    return MOE_OK;
}

extern "C" int moe_dispatch(const void *x, const int32_t *expert_idx, const int32_t *replicas, int T, int d,
                            int E, int slot_capacity, int max_slots, int dtype, int32_t *counts,
                            int32_t *kept, int32_t *expert_offset, int32_t *slot_offset, int32_t *perm,
                            int32_t *inv, void *x_perm, void *ws, size_t ws_bytes, void *stream)
{
    return dispatch_checked("moe_dispatch", x, expert_idx, replicas, T, T, d, E, slot_capacity, max_slots, dtype,
                            counts, kept, expert_offset, slot_offset, perm, inv, nullptr, x_perm, ws, ws_bytes, stream);
}

extern "C" int moe_dispatch_topk(const void *x, const int32_t *expert_idx, const int32_t *replicas, int T, int k,
                                 int d, int E, int slot_capacity, int max_slots, int dtype, int32_t *counts,
                                 int32_t *kept, int32_t *expert_offset, int32_t *slot_offset, int32_t *perm,
                                 int32_t *inv, int32_t *row_token, void *x_perm, void *ws, size_t ws_bytes,
                                 void *stream)
{
    MOE_REQUIRE(T >= 0 && k >= 1 && k <= MOE_MAX_TOPK && (long long)T * k <= 0x7fffffffLL, MOE_ERR_INVALID_ARG,
                "moe_dispatch_topk: T=%d k=%d out of range (k <= %d, T*k < 2^31)", T, k, MOE_MAX_TOPK);
    MOE_REQUIRE(T == 0 || row_token, MOE_ERR_INVALID_ARG, "moe_dispatch_topk: null row_token");
    return dispatch_checked("moe_dispatch_topk", x, expert_idx, replicas, T * k, T, d, E, slot_capacity, max_slots,
                            dtype, counts, kept, expert_offset, slot_offset, perm, inv, row_token, x_perm, ws, ws_bytes,
                            stream);
}

extern "C" int moe_dispatch_static(const void *x, const int32_t *expert_idx, const int32_t *replicas, int T, int d,
                                   int E, int slot_capacity, int max_slots, int dtype, int32_t *counts,
                                   int32_t *kept, int32_t *expert_offset, int32_t *slot_offset, int32_t *perm,
                                   int32_t *inv, void *x_perm, void *stream)
{
    return dispatch_checked("moe_dispatch_static", x, expert_idx, replicas, T, T, d, E, slot_capacity, max_slots,
                            dtype, counts, kept, expert_offset, slot_offset, perm, inv, nullptr, x_perm, nullptr, 0,
                            stream, true);
}
