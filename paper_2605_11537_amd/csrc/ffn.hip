// moe_expert_ffn: grouped expert FFN over experts and their replica slots, and
// moe_pack_weights: one-time re-layout of static expert weights for the matrix-core kernels.
//
//   worklist  one workgroup turns the device-side slot tables into a list of row tiles
//             (expert, first row, end row); a slot of more than 64 rows gives several tiles,
//             so the replicas of a hot expert and the tiles inside a replica all run side by
//             side.  In the "experts" schedule there is one item per logical expert instead
//             and the kernel walks its rows 64 at a time.
//   gemm1     h = relu(x_perm * W1[e])   per (row tile, 128-column tile)
//   gemm2     y_perm = h * W2[e]
// At large batch the list cuts every slot into pieces of 256 rows instead and both products run on
// the persistent 256 x 256 tile kernel (gemm_dense_bf16.h); the 128-column kernel is then not launched.
// At small batch with short slots the 128-column kernel reads the slot tables itself (no list kernel).
// Grids are sized for the worst case on the host (rows and slots are only known on the
// device); workgroups beyond the list exit at once.  Workgroup ids are remapped so that the
// column tiles of one row tile, which share the token rows, run on one XCD.
#include "gemm_bf16.h"
#include "gemm_dense_bf16.h"

namespace moe {

constexpr int FFN_BM = 64;    // rows per tile (fp32 path; short tile of the bf16 path)
constexpr int FFN_BM_TALL = 128;  // bf16 path: a slot is cut into tiles of up to 128 rows
constexpr int FFN_BN = 128;   // columns per workgroup (bf16 path)
constexpr int FFN_BK = 128;   // k chunk of the bf16 path, tiles of up to 64 rows
constexpr int FFN_BK_TALL = 64;   // k chunk for tiles of 65..128 rows
constexpr int FFN_GROUP = 8;             // row tiles per chunk of the grouped order

struct __attribute__((aligned(16))) WorkItem {
    int expert, row_begin, row_end;
    int reuse;   // 1: other tiles read the same expert's weights (keep them in L2); 0: read-once stream
};

// ------------------------------------------------------------------ weight packing
// 16-byte piece (((e*(N/32) + n/32)*(K/8) + k/8)*32 + n%32) = in[e][8*(k/8) .. +7][n]
__global__ __launch_bounds__(256) void pack_weights_kernel(const bf16_t *__restrict__ in, int K, int N,
                                                           uint4 *__restrict__ out)
{
    const int e = blockIdx.z, kg = blockIdx.y;
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n >= N) return;
    const bf16_t *src = in + ((size_t)e * K + (size_t)kg * 8) * N + n;
    uint32_t v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        v[j] = (uint32_t)src[(size_t)(2 * j) * N] | ((uint32_t)src[(size_t)(2 * j + 1) * N] << 16);
    out[(((size_t)e * (N / 32) + (n >> 5)) * (K / 8) + kg) * 32 + (n & 31)] = make_uint4(v[0], v[1], v[2], v[3]);
}

// ------------------------------------------------------------------ work list
// dense != 0 (slot schedule only): every slot's rows go, 256 at a time, to the list of the 256 x 256 tile
// kernel (it skips the row blocks a shorter last piece does not have) and the 128-column kernel gets
// nothing.  (Leaving it the last pieces of up to 64 rows, the weight-streaming case, was 3.5 % slower on
// the extreme-skew workload: a second, HBM-bound launch after an MFMA-bound one instead of one mixed one.)
// n_items = {row tiles, group size of the grouped order, dense tiles}.
__global__ __launch_bounds__(1024) void ffn_worklist_kernel(const int32_t *__restrict__ slot_offset,
                                                            const int32_t *__restrict__ slot_expert,
                                                            const int32_t *__restrict__ n_slots_p, int max_slots,
                                                            int max_items, int schedule, int tile_rows, int E,
                                                            int dense, int max_dense, WorkItem *__restrict__ items,
                                                            DenseTile *__restrict__ dtiles,
                                                            int32_t *__restrict__ n_items)
{
    __shared__ int wave_sums[16];
    __shared__ int total;
    __shared__ int n_distinct;
    if (threadIdx.x == 0) n_distinct = 0;
    __syncthreads();
    int P = n_slots_p[0];
    if (P > max_slots) P = max_slots;
    int base = 0, dbase = 0;
    for (int p0 = 0; p0 < P; p0 += 1024) {
        int p = p0 + threadIdx.x;
        int cnt = 0, nd = 0, e = -1, r0 = 0, r1 = 0, reuse = 0;
        if (p < P) {
            e = slot_expert[p];
            r0 = slot_offset[p];
            if (schedule == MOE_SCHEDULE_SLOTS) {
                r1 = slot_offset[p + 1];
                const int n = r1 > r0 ? r1 - r0 : 0;
                if (dense) nd = (n + DENSE_BM - 1) / DENSE_BM;
                const int covered = nd * DENSE_BM < n ? nd * DENSE_BM : n;
                cnt = (n - covered + tile_rows - 1) / tile_rows;
                reuse = cnt + nd > 1 || (p > 0 && slot_expert[p - 1] == e) || (p + 1 < P && slot_expert[p + 1] == e);
            } else if (p == 0 || slot_expert[p - 1] != e) {
                int q = p + 1;
                while (q < P && slot_expert[q] == e) ++q;
                r1 = slot_offset[q];
                cnt = r1 > r0 ? 1 : 0;
                reuse = r1 - r0 > tile_rows;
            }
            if (e < 0 || e >= E) cnt = nd = 0;   // never index weights with a bad id
            // experts that own at least one tile (slots of an expert are adjacent)
            if (cnt > 0 && (p == 0 || slot_expert[p - 1] != e)) atomicAdd(&n_distinct, 1);
        }
        int off = base + block_scan_excl_1024(cnt, wave_sums, &total);
        const int total_items = total;
        int doff = dbase + block_scan_excl_1024(nd, wave_sums, &total);
        const int total_dense = total;
        const int covered = nd * DENSE_BM < r1 - r0 ? nd * DENSE_BM : r1 - r0;
        for (int i = 0; i < nd; ++i) {
            if (doff + i < max_dense) {
                DenseTile t;
                t.expert = e;
                t.row_begin = r0 + i * DENSE_BM;
                t.row_end = t.row_begin + DENSE_BM < r1 ? t.row_begin + DENSE_BM : r1;
                dtiles[doff + i] = t;
            }
        }
        for (int i = 0; i < cnt; ++i) {
            if (off + i < max_items) {
                WorkItem it;
                it.expert = e;
                it.reuse = reuse;
                if (schedule == MOE_SCHEDULE_SLOTS) {
                    it.row_begin = r0 + covered + i * tile_rows;
                    it.row_end = it.row_begin + tile_rows < r1 ? it.row_begin + tile_rows : r1;
                } else {
                    it.row_begin = r0;
                    it.row_end = r1;
                }
                items[off + i] = it;
            }
        }
        base += total_items;
        dbase += total_dense;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        int n = base < max_items ? base : max_items;
        n_items[0] = n;
        // two or more row tiles per expert on average: the weights are re-read from cache by many
        // tiles, so use the chunked, column-tile-major order (see grouped_tile_of); otherwise the
        // weight stream binds, every tile costs the same, and contiguous ranges balance exactly
        n_items[1] = (n_distinct > 0 && n >= 2 * n_distinct) ? FFN_GROUP : 0;
        n_items[2] = dbase < max_dense ? dbase : max_dense;
    }
}

// ------------------------------------------------------------------ bf16 256 x 256 tiles (long row stretches)
template <bool RELU>
__global__ __launch_bounds__(GEMM_THREADS, 1) void ffn_dense_bf16_kernel(
    const bf16_t *__restrict__ A, const int32_t *__restrict__ row_index, int n_src_rows,
    const bf16_t *__restrict__ Wp, int K, int N, const DenseTile *__restrict__ tiles,
    const int32_t *__restrict__ n_tiles, bf16_t *__restrict__ C)
{
    __shared__ __attribute__((aligned(16))) uint4 smem[DENSE_LDS_BYTES / 16];
    dense_tiles_bf16<RELU>(A, row_index, n_src_rows, Wp, K, N, tiles, n_tiles[0], C, smem);
}

// ------------------------------------------------------------------ bf16 grouped GEMM
// Two tile heights.  Up to 64 rows: 2 row blocks per wavefront, k chunks of 128 -- the
// weight-streaming shape.  65..128 rows (TALL builds only): 4 row blocks per wavefront, so a weight
// byte fetched from L2/HBM feeds twice the rows.  The build without the tall tile walks a work item
// 64 rows at a time.  (Three or four workgroups per CU instead of two, tried with a k chunk of 64 to
// fit the registers, changed the HBM-bound launches by under 1%: two it stays.)
template <bool RELU, bool TALL>
__global__ __launch_bounds__(GEMM_THREADS, 2) void ffn_gemm_bf16_kernel(
    const bf16_t *__restrict__ A, const int32_t *__restrict__ row_index, int n_src_rows,
    const bf16_t *__restrict__ Wp, int K, int N, int E, const WorkItem *__restrict__ items,
    const int32_t *__restrict__ n_items, const int32_t *__restrict__ slot_offset,
    const int32_t *__restrict__ slot_expert, const int32_t *__restrict__ n_slots_p, int max_slots, int schedule,
    int max_rows, bf16_t *__restrict__ C)
{
    constexpr int TM = TALL ? FFN_BM_TALL : FFN_BM;          // rows per pass over a work item
    constexpr int MBT = TM / 32;
    constexpr int LDC = FFN_BN + 8;
    constexpr int S0 = gemm_lds_elems<2, FFN_BK>(), S1 = TALL ? gemm_lds_elems<4, FFN_BK_TALL>() : 0, S2 = TM * LDC;
    __shared__ __attribute__((aligned(16))) bf16_t lds[(S0 > S1 ? S0 : S1) > S2 ? (S0 > S1 ? S0 : S1) : S2];
    const int n_nt = N / FFN_BN;
    int item, nt;
    WorkItem it;
    if (items) {
        if (!grouped_tile_of(blockIdx.x, n_items[0], n_nt, n_items[1], item, nt)) return;
        it = items[item];
    } else {
        // No list: one work item per slot (per expert in the experts schedule), read straight from the
        // slot tables; a range longer than the tile is walked by the loop below.  Saves the list kernel
        // where slots are short anyway; the 8 contiguous XCD ranges are taken over all slots.
        int P = n_slots_p[0];
        if (P > max_slots) P = max_slots;
        const int lid = xcd_remap(blockIdx.x, P * n_nt);
        if (lid < 0) return;
        item = lid / n_nt;
        nt = lid - item * n_nt;
        const int e = slot_expert[item];
        it.expert = e;
        it.row_begin = slot_offset[item];
        const bool after_same = item > 0 && slot_expert[item - 1] == e;
        int last = item;
        if (schedule == MOE_SCHEDULE_EXPERTS) {
            if (after_same) return;                       // the expert's first slot walks all its rows
            while (last + 1 < P && slot_expert[last + 1] == e) ++last;
        }
        it.row_end = slot_offset[last + 1];
        it.reuse = it.row_end - it.row_begin > TM || (schedule == MOE_SCHEDULE_SLOTS &&
                                                     (after_same || (item + 1 < P && slot_expert[item + 1] == e)));
    }
    if (it.expert < 0 || it.expert >= E || it.row_begin < 0) return;  // never index weights with a bad id
    const bf16_t *Bp = Wp + (size_t)it.expert * K * N;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int row_end = it.row_end < max_rows ? it.row_end : max_rows;
    for (int r0 = it.row_begin; r0 < row_end; r0 += TM) {
        const int nrows = row_end - r0 < TM ? row_end - r0 : TM;
        const bf16_t *a0 = row_index ? A : A + (size_t)r0 * K;
        const int32_t *ri = row_index ? row_index + r0 : nullptr;
        f32x16_t acc[MBT][1];
        zero_acc<MBT, 1>(acc);
        if (!TALL || nrows <= FFN_BM) {
            f32x16_t(&acc2)[2][1] = reinterpret_cast<f32x16_t(&)[2][1]>(acc);
            if (it.reuse)
                gemm_tile_bf16<2, 1, FFN_BK, false>(a0, K, nrows, Bp, nt * FFN_BN, K, lds, acc2, ri, n_src_rows);
            else
                gemm_tile_bf16<2, 1, FFN_BK, true>(a0, K, nrows, Bp, nt * FFN_BN, K, lds, acc2, ri, n_src_rows);
        } else if constexpr (TALL) {
            if (it.reuse)
                gemm_tile_bf16<4, 1, FFN_BK_TALL, false>(a0, K, nrows, Bp, nt * FFN_BN, K, lds, acc, ri, n_src_rows);
            else
                gemm_tile_bf16<4, 1, FFN_BK_TALL, true>(a0, K, nrows, Bp, nt * FFN_BN, K, lds, acc, ri, n_src_rows);
        }
        // Epilogue through LDS: an accumulator lane holds single columns of 16 different rows,
        // and 2-byte stores that cover a quarter of a cache line each are slow.  The tile is
        // transposed in LDS (the A buffers are free after the last barrier of the product) and
        // leaves as 16-byte stores, 16 consecutive lanes writing the 256 contiguous bytes of a row.
#pragma unroll
        for (int mb = 0; mb < MBT; ++mb)
            if (mb * 32 < nrows) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float val = acc[mb][0][v];
                    if (RELU) val = val > 0.f ? val : 0.f;
                    lds[(mb * 32 + acc_row(v, lane)) * LDC + w * 32 + (lane & 31)] = f32_to_bf16(val);
                }
            }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < TM * (FFN_BN / 8) / GEMM_THREADS; ++i) {
            int p = threadIdx.x + i * GEMM_THREADS;
            int r = p / (FFN_BN / 8), c8 = p % (FFN_BN / 8);
            if (r < nrows)
                *reinterpret_cast<uint4 *>(C + (size_t)(r0 + r) * N + nt * FFN_BN + c8 * 8) =
                    *reinterpret_cast<const uint4 *>(lds + r * LDC + c8 * 8);
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------ fp32 grouped GEMM (plain weights)
// 64x64 tile, 256 threads, 4x4 outputs per thread, k ascending.
template <bool RELU>
__global__ __launch_bounds__(256) void ffn_gemm_f32_kernel(const float *__restrict__ A, const float *__restrict__ W,
                                                           const int32_t *__restrict__ row_index, int n_src_rows,
                                                           int K, int N, int E,
                                                           const WorkItem *__restrict__ items,
                                                           const int32_t *__restrict__ n_items, int max_rows,
                                                           float *__restrict__ C)
{
    __shared__ float As[16][64 + 4];
    __shared__ float Bs[16][64];
    const int n_nt = N / 64;
    const int item = blockIdx.x / n_nt, nt = blockIdx.x - item * n_nt;
    if (item >= n_items[0]) return;
    const WorkItem it = items[item];
    if (it.expert < 0 || it.expert >= E || it.row_begin < 0) return;
    const float *B = W + (size_t)it.expert * K * N + nt * 64;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int row_end = it.row_end < max_rows ? it.row_end : max_rows;
    for (int r0 = it.row_begin; r0 < row_end; r0 += FFN_BM) {
        const int nrows = row_end - r0 < FFN_BM ? row_end - r0 : FFN_BM;
        float acc[4][4] = {};
        // this thread's pieces of a 16-deep chunk: 4 consecutive k of token row r, 4 consecutive columns of
        // weight row kb.  The next chunk is fetched into registers while the current one is multiplied, so a
        // chunk costs its arithmetic and not a memory round trip.
        const int r = threadIdx.x >> 2, kq = (threadIdx.x & 3) * 4;
        const int kb = threadIdx.x >> 4, nb = (threadIdx.x & 15) * 4;
        const float *a_src = nullptr;
        if (r < nrows) {
            const int src = row_index ? row_index[r0 + r] : r0 + r;
            if (src >= 0 && src < n_src_rows) a_src = A + (size_t)src * K + kq;
        }
        auto fetch = [&](int k0, float4 &av, float4 &bv) {
            av = a_src ? *reinterpret_cast<const float4 *>(a_src + k0) : make_float4(0.f, 0.f, 0.f, 0.f);
            bv = *reinterpret_cast<const float4 *>(B + (size_t)(k0 + kb) * N + nb);
        };
        float4 av, bv;
        fetch(0, av, bv);
        for (int k0 = 0; k0 < K; k0 += 16) {
            As[kq + 0][r] = av.x;
            As[kq + 1][r] = av.y;
            As[kq + 2][r] = av.z;
            As[kq + 3][r] = av.w;
            *reinterpret_cast<float4 *>(&Bs[kb][nb]) = bv;
            __syncthreads();
            if (k0 + 16 < K) fetch(k0 + 16, av, bv);
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                float a[4], b[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
                for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
            }
            __syncthreads();
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int orow = ty * 4 + i;
            if (orow < nrows) {
                float4 o;
                o.x = RELU ? fmaxf(acc[i][0], 0.f) : acc[i][0];
                o.y = RELU ? fmaxf(acc[i][1], 0.f) : acc[i][1];
                o.z = RELU ? fmaxf(acc[i][2], 0.f) : acc[i][2];
                o.w = RELU ? fmaxf(acc[i][3], 0.f) : acc[i][3];
                *reinterpret_cast<float4 *>(C + (size_t)(r0 + orow) * N + nt * 64 + tx * 4) = o;
            }
        }
    }
}

static inline int ffn_max_items(int max_rows, int max_slots) { return max_slots + max_rows / FFN_BM + 1; }
// every dense tile but the last of a slot has 256 rows
static inline int ffn_max_dense(int max_rows, int max_slots) { return max_rows / DENSE_BM + max_slots + 1; }

// The 256 x 256 tile pays off when slots are long: it is launched when the rows could fill slots of
// 64 and more on average, the matrix sizes fit its tiling, and the batch can fill the chip.
static inline bool ffn_use_dense(int max_rows, int max_slots, int K, int N, int schedule)
{
    return schedule == MOE_SCHEDULE_SLOTS && N % DENSE_BN == 0 && K % DENSE_BK == 0 && K >= DENSE_MIN_K &&
           (long long)max_rows >= 64LL * max_slots && max_rows >= 4096;
}

}  // namespace moe

using namespace moe;

extern "C" size_t moe_packed_weights_bytes(int E, int K, int N, int dtype)
{
    if (E <= 0 || K <= 0 || N <= 0 || dtype != MOE_BF16) return 0;
    return (size_t)E * K * N * 2;
}

extern "C" int moe_pack_weights(const void *w, int E, int K, int N, int dtype, void *w_packed, void *stream)
{
    MOE_REQUIRE(E > 0 && K > 0 && N > 0, MOE_ERR_INVALID_ARG, "moe_pack_weights: E=%d K=%d N=%d out of range", E, K, N);
    MOE_REQUIRE(dtype == MOE_BF16, MOE_ERR_UNSUPPORTED, "moe_pack_weights: only MOE_BF16 weights are packed");
    MOE_REQUIRE(K % 8 == 0 && N % 32 == 0, MOE_ERR_INVALID_ARG,
                "moe_pack_weights: K=%d must be a multiple of 8 and N=%d of 32", K, N);
    MOE_REQUIRE(E <= 65535 && K / 8 <= 65535, MOE_ERR_UNSUPPORTED, "moe_pack_weights: E or K too large");
    MOE_REQUIRE(w && w_packed && w != w_packed, MOE_ERR_INVALID_ARG, "moe_pack_weights: null or aliased pointer");
    MOE_REQUIRE(aligned16(w_packed), MOE_ERR_INVALID_ARG, "moe_pack_weights: output misaligned");
    hipLaunchKernelGGL(pack_weights_kernel, dim3(ceil_div(N, 256), K / 8, E), dim3(256), 0, (hipStream_t)stream,
                       (const bf16_t *)w, K, N, (uint4 *)w_packed);
    MOE_CHECK_LAUNCH("moe_pack_weights");
    return MOE_OK;
}

extern "C" size_t moe_expert_ffn_workspace_bytes(int max_rows, int max_slots, int d, int F, int dtype)
{
    if (max_rows < 0 || max_slots <= 0 || d <= 0 || F <= 0) return 0;
    size_t esz = dtype == MOE_F32 ? 4 : 2;
    size_t h = align_up((size_t)(max_rows > 0 ? max_rows : 1) * F * esz, 256);
    size_t items = align_up((size_t)ffn_max_items(max_rows, max_slots) * sizeof(WorkItem), 256);
    size_t dense = align_up((size_t)ffn_max_dense(max_rows, max_slots) * sizeof(DenseTile), 256);
    return h + items + dense + 256;
}

// n_x_rows: rows of the matrix x_perm points to -- max_rows, or with row_index any number (the
// indices are checked against it)
static int expert_ffn_checked(const void *x_perm, int n_x_rows, const int32_t *row_index, const void *w1,
                              const void *w2, int weight_layout, const int32_t *slot_offset,
                              const int32_t *slot_expert, const int32_t *n_slots, int max_rows, int max_slots, int E,
                              int d, int F, int dtype, int schedule, void *y_perm, void *ws, size_t ws_bytes,
                              void *stream, void *const *timing_events = nullptr)
{
    MOE_REQUIRE(max_rows >= 0 && max_slots > 0 && E > 0 && d > 0 && F > 0, MOE_ERR_INVALID_ARG,
                "moe_expert_ffn: max_rows=%d max_slots=%d E=%d d=%d F=%d out of range", max_rows, max_slots, E, d,
                F);
    MOE_REQUIRE(dtype == MOE_F32 || dtype == MOE_BF16, MOE_ERR_INVALID_ARG, "moe_expert_ffn: unknown dtype %d", dtype);
    MOE_REQUIRE(schedule == MOE_SCHEDULE_SLOTS || schedule == MOE_SCHEDULE_EXPERTS, MOE_ERR_INVALID_ARG,
                "moe_expert_ffn: unknown schedule %d", schedule);
    MOE_REQUIRE(weight_layout == MOE_LAYOUT_PLAIN || weight_layout == MOE_LAYOUT_PACKED, MOE_ERR_INVALID_ARG,
                "moe_expert_ffn: unknown weight layout %d", weight_layout);
    MOE_REQUIRE(max_slots <= MOE_MAX_SLOTS, MOE_ERR_UNSUPPORTED, "moe_expert_ffn: max_slots=%d exceeds %d",
                max_slots, MOE_MAX_SLOTS);
    if (dtype == MOE_BF16) {
        MOE_REQUIRE(weight_layout == MOE_LAYOUT_PACKED, MOE_ERR_UNSUPPORTED,
                    "moe_expert_ffn: bf16 weights must be packed with moe_pack_weights");
        MOE_REQUIRE(d % FFN_BN == 0 && F % FFN_BN == 0, MOE_ERR_UNSUPPORTED,
                    "moe_expert_ffn: bf16 path needs d and F multiples of %d (d=%d F=%d)", FFN_BN, d, F);
    } else {
        MOE_REQUIRE(weight_layout == MOE_LAYOUT_PLAIN, MOE_ERR_UNSUPPORTED,
                    "moe_expert_ffn: fp32 weights are taken in the plain layout");
        MOE_REQUIRE(d % 64 == 0 && F % 64 == 0, MOE_ERR_UNSUPPORTED,
                    "moe_expert_ffn: fp32 path needs d and F multiples of 64 (d=%d F=%d)", d, F);
    }
    if (max_rows == 0) return MOE_OK;   // an empty batch: nothing to read or write, pointers are not looked at
    MOE_REQUIRE(x_perm && w1 && w2 && slot_offset && slot_expert && n_slots && y_perm, MOE_ERR_INVALID_ARG,
                "moe_expert_ffn: null pointer");
    MOE_REQUIRE(aligned16(x_perm) && aligned16(w1) && aligned16(w2) && aligned16(y_perm), MOE_ERR_INVALID_ARG,
                "moe_expert_ffn: tensor misaligned");
    size_t need = moe_expert_ffn_workspace_bytes(max_rows, max_slots, d, F, dtype);
    MOE_REQUIRE(ws && aligned16(ws) && ws_bytes >= need, MOE_ERR_WORKSPACE,
                "moe_expert_ffn: workspace of %zu bytes needed, %zu given", need, ws_bytes);

    hipStream_t st = (hipStream_t)stream;
    size_t esz = dtype == MOE_F32 ? 4 : 2;
    char *p = (char *)ws;
    void *h = p;
    p += align_up((size_t)max_rows * F * esz, 256);
    WorkItem *items = (WorkItem *)p;
    int max_items = ffn_max_items(max_rows, max_slots);
    p += align_up((size_t)max_items * sizeof(WorkItem), 256);
    DenseTile *dtiles = (DenseTile *)p;
    const int max_dense = ffn_max_dense(max_rows, max_slots);
    p += align_up((size_t)max_dense * sizeof(DenseTile), 256);
    int32_t *n_items = (int32_t *)p;

    // both products must take the dense route or neither: the lists split the rows once
    const bool dense = dtype == MOE_BF16 && ffn_use_dense(max_rows, max_slots, d, F, schedule) &&
                       ffn_use_dense(max_rows, max_slots, F, d, schedule);
    // Without the dense kernel (small batches, short slots on average, shapes outside its tiling, the
    // experts schedule) the 128-column kernel cuts work items 128 rows high and picks the tile height per
    // item; with it, the 128-column kernel is not launched at all.
    const bool tall = dtype == MOE_BF16 && !dense;
    const int tile_rows = tall ? FFN_BM_TALL : FFN_BM;
    // Slots that hold 64 rows on average at most are one tile each, give or take: the 128-column kernel
    // then reads the slot tables itself and the list kernel (a launch of ~5 us in front of the first
    // product) is skipped.  Long slots without the dense kernel keep the list: it cuts them into tiles
    // that run side by side.
    const bool listless = dtype == MOE_BF16 && !dense && (long long)max_rows <= 64LL * max_slots;
    if (!listless) {
        hipLaunchKernelGGL(ffn_worklist_kernel, dim3(1), dim3(1024), 0, st, slot_offset, slot_expert, n_slots,
                           max_slots, max_items, schedule, tile_rows, E, dense ? 1 : 0, max_dense, items, dtiles,
                           n_items);
        MOE_CHECK_LAUNCH("moe_expert_ffn/worklist");
    }
    const WorkItem *list = listless ? nullptr : items;
    // upper bounds of the 128-column kernel's list: with the dense kernel on, a slot leaves it one piece at most
    int grid_items = schedule != MOE_SCHEDULE_SLOTS ? (max_slots < max_items ? max_slots : max_items)
                     : (dense || listless)          ? max_slots
                                                    : max_slots + max_rows / tile_rows + 1;
    // measurement only (moe_expert_ffn_timed): events recorded before, between and after the two products
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    if (timing_events)
        for (int i = 0; i < 3; ++i) ev[i] = (hipEvent_t)timing_events[i];
    if (ev[0]) (void)hipEventRecord(ev[0], st);
    if (dtype == MOE_BF16) {
        // worst case of both orders: chunks of FFN_GROUP items, rounded up to 8 chunks
        size_t gi = align_up((size_t)ceil_div(grid_items, FFN_GROUP), 8) * FFN_GROUP;
        int g1 = (int)(gi * (F / FFN_BN));
        int g2 = (int)(gi * (d / FFN_BN));
        int n_cu = 0;
        if (dense) {
            int dev = 0;
            MOE_REQUIRE(hipGetDevice(&dev) == hipSuccess &&
                            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
                            n_cu >= 8,
                        MOE_ERR_HIP, "moe_expert_ffn: cannot read the compute unit count");
            n_cu -= n_cu % 8;   // one persistent workgroup per CU, the same number on every XCD
            hipLaunchKernelGGL(ffn_dense_bf16_kernel<true>, dim3(n_cu), dim3(GEMM_THREADS), 0, st,
                               (const bf16_t *)x_perm, row_index, n_x_rows, (const bf16_t *)w1, d, F, dtiles,
                               n_items + 2, (bf16_t *)h);
            MOE_CHECK_LAUNCH("moe_expert_ffn/dense gemm1");
        }
        if (dense) {
            // the dense kernel took every row
        } else if (tall)
            hipLaunchKernelGGL((ffn_gemm_bf16_kernel<true, true>), dim3(g1), dim3(GEMM_THREADS), 0, st,
                               (const bf16_t *)x_perm, row_index, n_x_rows, (const bf16_t *)w1, d, F, E, list,
                               n_items, slot_offset, slot_expert, n_slots, max_slots, schedule, max_rows,
                               (bf16_t *)h);
        else
            hipLaunchKernelGGL((ffn_gemm_bf16_kernel<true, false>), dim3(g1), dim3(GEMM_THREADS), 0,
                               st, (const bf16_t *)x_perm, row_index, n_x_rows, (const bf16_t *)w1, d, F, E, list,
                               n_items, slot_offset, slot_expert, n_slots, max_slots, schedule, max_rows,
                               (bf16_t *)h);
        MOE_CHECK_LAUNCH("moe_expert_ffn/gemm1");
        if (ev[1]) (void)hipEventRecord(ev[1], st);
        if (dense) {
            hipLaunchKernelGGL(ffn_dense_bf16_kernel<false>, dim3(n_cu), dim3(GEMM_THREADS), 0, st,
                               (const bf16_t *)h, (const int32_t *)nullptr, max_rows, (const bf16_t *)w2, F, d, dtiles,
                               n_items + 2, (bf16_t *)y_perm);
            MOE_CHECK_LAUNCH("moe_expert_ffn/dense gemm2");
        }
        if (dense) {
        } else if (tall)
            hipLaunchKernelGGL((ffn_gemm_bf16_kernel<false, true>), dim3(g2), dim3(GEMM_THREADS), 0, st,
                               (const bf16_t *)h, (const int32_t *)nullptr, max_rows, (const bf16_t *)w2, F, d, E,
                               list, n_items, slot_offset, slot_expert, n_slots, max_slots, schedule, max_rows,
                               (bf16_t *)y_perm);
        else
            hipLaunchKernelGGL((ffn_gemm_bf16_kernel<false, false>), dim3(g2), dim3(GEMM_THREADS), 0,
                               st, (const bf16_t *)h, (const int32_t *)nullptr, max_rows, (const bf16_t *)w2, F, d, E,
                               list, n_items, slot_offset, slot_expert, n_slots, max_slots, schedule, max_rows,
                               (bf16_t *)y_perm);
        MOE_CHECK_LAUNCH("moe_expert_ffn/gemm2");
    } else {
        int g1 = grid_items * (F / 64), g2 = grid_items * (d / 64);
        hipLaunchKernelGGL(ffn_gemm_f32_kernel<true>, dim3(g1), dim3(256), 0, st, (const float *)x_perm,
                           (const float *)w1, row_index, n_x_rows, d, F, E, items, n_items, max_rows, (float *)h);
        MOE_CHECK_LAUNCH("moe_expert_ffn/gemm1");
        if (ev[1]) (void)hipEventRecord(ev[1], st);
        hipLaunchKernelGGL(ffn_gemm_f32_kernel<false>, dim3(g2), dim3(256), 0, st, (const float *)h,
                           (const float *)w2, (const int32_t *)nullptr, max_rows, F, d, E, items, n_items, max_rows,
                           (float *)y_perm);
        MOE_CHECK_LAUNCH("moe_expert_ffn/gemm2");
    }
    if (ev[2]) (void)hipEventRecord(ev[2], st);
    return MOE_OK;
}

extern "C" int moe_expert_ffn(const void *x_perm, const int32_t *row_index, const void *w1, const void *w2,
                              int weight_layout,
                              const int32_t *slot_offset, const int32_t *slot_expert, const int32_t *n_slots,
                              int max_rows, int max_slots, int E, int d, int F, int dtype, int schedule,
                              void *y_perm, void *ws, size_t ws_bytes, void *stream)
{
    return expert_ffn_checked(x_perm, max_rows, row_index, w1, w2, weight_layout, slot_offset, slot_expert, n_slots,
                              max_rows, max_slots, E, d, F, dtype, schedule, y_perm, ws, ws_bytes, stream);
}

extern "C" int moe_expert_ffn_rows(const void *x, int n_x_rows, const int32_t *row_index, const void *w1,
                                   const void *w2, int weight_layout, const int32_t *slot_offset,
                                   const int32_t *slot_expert, const int32_t *n_slots, int max_rows, int max_slots,
                                   int E, int d, int F, int dtype, int schedule, void *y_perm, void *ws,
                                   size_t ws_bytes, void *stream)
{
    MOE_REQUIRE(n_x_rows >= 0 && (max_rows == 0 || (row_index && n_x_rows > 0)), MOE_ERR_INVALID_ARG,
                "moe_expert_ffn_rows: n_x_rows=%d out of range or null row_index", n_x_rows);
    return expert_ffn_checked(x, n_x_rows, row_index, w1, w2, weight_layout, slot_offset, slot_expert, n_slots,
                              max_rows, max_slots, E, d, F, dtype, schedule, y_perm, ws, ws_bytes, stream);
}

extern "C" int moe_expert_ffn_timed(const void *x, int n_x_rows, const int32_t *row_index, const void *w1,
                                    const void *w2, int weight_layout, const int32_t *slot_offset,
                                    const int32_t *slot_expert, const int32_t *n_slots, int max_rows, int max_slots,
                                    int E, int d, int F, int dtype, int schedule, void *y_perm, void *ws,
                                    size_t ws_bytes, void *stream, void *ev_before, void *ev_between, void *ev_after)
{
    MOE_REQUIRE(n_x_rows >= 0 && (row_index || n_x_rows == max_rows), MOE_ERR_INVALID_ARG,
                "moe_expert_ffn_timed: n_x_rows=%d must equal max_rows=%d without row_index", n_x_rows, max_rows);
    void *const evs[3] = {ev_before, ev_between, ev_after};
    return expert_ffn_checked(x, n_x_rows, row_index, w1, w2, weight_layout, slot_offset, slot_expert, n_slots,
                              max_rows, max_slots, E, d, F, dtype, schedule, y_perm, ws, ws_bytes, stream, evs);
}
