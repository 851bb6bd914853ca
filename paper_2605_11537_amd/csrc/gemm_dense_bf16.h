// Compute-bound bf16 tile product for gfx950: 256 rows x 256 columns per workgroup, used by the
// expert FFN for row tiles of more than 128 tokens (long slots of hot experts at large batch).
//
// Why a second tile shape.  A workgroup tile of R rows x C columns moves (R + C) * 2 bytes per
// k through the CU's vector memory path and does R * C * 2 flops with them.  The matrix cores of one
// CU retire 4096 flop per clock; the vector memory path delivers about 64 bytes per clock.  A
// 128 x 128 tile therefore needs all 64 bytes per clock to keep the matrix cores busy; 256 x 256
// needs half of that.  The four wavefronts form a 2 x 2 grid, each owns 128 x 128 outputs =
// 16 accumulator blocks = 256 registers, so one workgroup lives on a CU (one wavefront per SIMD).
//
// Data path.  Both operands go global -> LDS directly (global_load_lds, 16 bytes per lane, no
// register round trip) into a ring of NS = 4 stages of 32 k each (128 KB: three stages, 48 KB of
// weights, in flight per CU -- the ring depth is what a tile that streams its weights from HBM runs on).  A stage holds 16 token units and 16
// weight units of 1 KB; a unit is what one wavefront-wide load writes (64 lanes x 16 bytes, in lane
// order):
//   weight unit (strip s, step ks): the 1 KB of the packed weight image that IS the matrix-core
//       fragment of 32 columns x 16 k -- lane l later reads piece l back, conflict free;
//   token unit u: rows 16u..16u+15 of the tile x 4 k-groups of 8 (64 contiguous bytes per row).
//       Row r's k-group g sits at piece 4r + (g ^ (r >> 2) ^ (r & 3)); this XOR spreads the 16
//       lanes that the LDS serves per clock over all banks when a fragment (32 rows x 16 k) is read.
// One wavefront with no partner on its SIMD must hide everything itself: the LDS reads of the next
// fragments and the global->LDS loads of a later stage are placed by hand between the matrix
// instructions (each occupies the pipe for 32 clocks but issues in 4).  LDS reads are inline
// assembly: the compiler cannot tell which LDS bytes an in-flight global->LDS load will write and
// would wait for every outstanding load before any LDS read it can see.  The waits are explicit:
// vector memory operations complete in issue order, so "at most P outstanding" means every load
// older than the newest P has landed.
//
// The kernel is persistent: the row ranges are dealt to the XCDs in turn, and the workgroups of an XCD
// walk its tiles round robin.  The loads of the next tile's first stages are issued during
// the last stages of the current one, and each wavefront converts and stores its own 128 x 128 part
// through a private LDS strip, so the epilogue has no workgroup barrier.  The matrix instruction is
// fed (weights, tokens), i.e. it computes the transposed block: a lane then holds 4 consecutive
// output columns of one token, which pack into one 8-byte LDS write.
#pragma once
#include "gemm_bf16.h"
#include <type_traits>

namespace moe {

constexpr int DENSE_BM = 256, DENSE_BN = 256, DENSE_BK = 32;
constexpr int DENSE_NS = 4;                                   // stages in the ring
constexpr int DENSE_STAGE = 32 * 64;                          // 16-byte pieces per stage
constexpr int DENSE_LDE = 64 + 8;                             // epilogue strip (32 rows x 64 columns) row stride, elements
constexpr int DENSE_IDX_OFFSET = DENSE_NS * DENSE_STAGE * 16 + 4 * 32 * DENSE_LDE * 2;   // 256 gathered row numbers
constexpr int DENSE_LDS_BYTES = DENSE_IDX_OFFSET + 256 * 4;
constexpr int DENSE_MIN_K = 256;                              // the pipeline needs a few stages per tile

struct DenseTile {
    int expert, row_begin, row_end;
};

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glb_void_t;
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

#define MOE_DS_READ128(dst, addr, off) asm volatile("ds_read_b128 %0, %1 offset:" #off : "=v"(dst) : "v"(addr))
#define MOE_DS_WRITE64(addr, val, off)                                                                               \
    do {                                                                                                             \
        asm volatile("ds_write_b64 %0, %1 offset:" #off ::"v"(addr), "v"(val) : "memory");                           \
        __builtin_amdgcn_sched_barrier(0); /* keeps the conversions of later groups from piling up in registers */   \
    } while (0)
// the registers are operands so that no use of them can move above the wait
#define MOE_WAIT_LGKM0_8(a)                                                                                          \
    asm volatile("s_waitcnt lgkmcnt(0)"                                                                              \
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]))
#define MOE_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n)&15) | (((n) >> 4) << 14))
#define MOE_SB() __builtin_amdgcn_sched_barrier(0)
// wait until at most base + extra operations are outstanding; extra is 0, 8, 16, 24 or 32 (the wait takes an immediate)
#define MOE_VMCNT_PLUS(base, extra)                                                                                  \
    do {                                                                                                             \
        if ((extra) == 0) MOE_VMCNT(base);                                                                           \
        else if ((extra) == 8) MOE_VMCNT((base) + 8);                                                                \
        else if ((extra) == 16) MOE_VMCNT((base) + 16);                                                              \
        else if ((extra) == 24) MOE_VMCNT((base) + 24);                                                              \
        else MOE_VMCNT((base) + 32);                                                                                 \
    } while (0)

// A: token rows (row-major, K contiguous); row_idx (optional): tile row r reads A[row_idx[row_begin + r]].
// Wp: packed weights of all experts (K x N each).  tiles[0..n_tiles): row ranges of at most 256 rows,
// every column tile of N / 256 is computed for each.  C: row-major output (rows x N).
template <bool RELU>
__device__ __forceinline__ void dense_tiles_bf16(const bf16_t *__restrict__ A, const int32_t *__restrict__ row_idx,
                                                 int n_src_rows, const bf16_t *__restrict__ Wp, int K, int N,
                                                 const DenseTile *__restrict__ tiles, int n_items,
                                                 bf16_t *__restrict__ C, uint4 *smem)
{
    constexpr int NS = DENSE_NS, STAGE = DENSE_STAGE, BK = DENSE_BK, LDE = DENSE_LDE;
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 1, wn = w & 1;
    const int n_nt = N / DENSE_BN;
    const int nk = K / BK, KG = K >> 3;
    // This workgroup's tiles.  Row ranges are dealt to the 8 XCDs in turn (range i to XCD i % 8, with all
    // its column tiles, which share the token rows in that L2); tiles differ in cost by their row count
    // and long runs of one kind follow each other in the list, so dealing mixes them evenly.  The
    // workgroups of an XCD take its tiles round robin.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3, per_xcd = gridDim.x >> 3;
    const int t_end = n_items > xcd ? ((n_items - xcd + 7) >> 3) * n_nt : 0;
    int lin = local;                   // position in this XCD's sequence of tiles
    if (lin >= t_end) return;

    const unsigned lds0 = (unsigned)(unsigned long)(lds_void_t *)smem;
    const int r16 = lane & 15;
    unsigned a_addr[2], b_addr[2];     // byte addresses of this lane's fragment pieces in stage 0, per 16-deep step
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int kg = 2 * ks + (lane >> 5);
        a_addr[ks] = lds0 + 16u * ((wm * 2 + ((lane & 31) >> 4)) * 64 + r16 * 4 + (kg ^ (r16 >> 2) ^ (r16 & 3)));
        b_addr[ks] = lds0 + 16u * ((16 + wn * 8 + ks) * 64 + lane);
    }
    // what this lane loads: token row (lane >> 2) of units 4w..4w+3, k-group by the swizzle; weight units 4w..4w+3
    const int ld_r = lane >> 2;
    const int ld_kg = (lane & 3) ^ (ld_r >> 2) ^ (ld_r & 3);
    const bf16_t *a_src[4];
    const uint4 *b_src[4];
    int row0, nrows, nt;
    auto tile_rows = [&](int t, int &item, int &r0, int &n, int &ntile) {
        const int q = t / n_nt;
        ntile = t - q * n_nt;
        item = q * 8 + xcd;
        const DenseTile tl = tiles[item];
        r0 = tl.row_begin;
        n = tl.row_end - tl.row_begin;
        return tl.expert;
    };
    auto local_row = [&](int i, int n) {
        int row = 16 * (w * 4 + i) + ld_r;
        return row < n ? row : n - 1;                // padded rows re-read the last valid row
    };
    auto set_sources = [&](int expert, const int (&src_row)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a_src[i] = A + (size_t)src_row[i] * K + ld_kg * 8;
            const int u = w * 4 + i, strip = u >> 1, ks = u & 1;
            b_src[i] = reinterpret_cast<const uint4 *>(Wp + (size_t)expert * K * N) +
                       ((size_t)(nt * 8 + strip) * KG + ks * 2) * 32 + lane;
        }
    };
    auto checked = [&](int v) { return (v >= 0 && v < n_src_rows) ? v : 0; };   // a bad index reads row 0
    auto issue = [&](int kc, int buf) {
        uint4 *base = smem + buf * STAGE + (w * 4) * 64;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_global_load_lds((glb_void_t *)(a_src[i] + kc * BK), (lds_void_t *)(base + i * 64), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_global_load_lds((glb_void_t *)(b_src[i] + (size_t)kc * 4 * 32),
                                             (lds_void_t *)(base + 16 * 64 + i * 64), 16, 0, 0);
    };

    int expert;
    {
        int item;
        expert = tile_rows(lin, item, row0, nrows, nt);
        int src_row[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = row0 + local_row(i, nrows);
            src_row[i] = row_idx ? checked(row_idx[r]) : r;
        }
        set_sources(expert, src_row);
    }
    int buf = 0;                       // ring position of the current tile's stage 0
    int prev_stores = 0;               // stores of the previous tile's epilogue, younger than this tile's first loads
#pragma unroll
    for (int s = 0; s < NS; ++s) issue(s, s);

    u32x4_t fx[8], fy[8];              // fragments of the two 16-deep steps: [0..3] token row blocks, [4..7] weight strips
#pragma unroll
    for (int i = 0; i < 8; ++i) fx[i] = fy[i] = (u32x4_t){0u, 0u, 0u, 0u};   // blocks a wavefront does not own are never read
#define MOE_MF(f, mb, nb)                                                                                            \
    if (mb < MYB)                                                                                                    \
    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, f[4 + nb]),                   \
                                                          __builtin_bit_cast(bf16x8_t, f[mb]), acc[mb][nb], 0, 0, 0)
    while (true) {
        const int next = lin + per_xcd;
        const bool has_next = next < t_end;
        int n_item, n_row0 = 0, n_nrows = 1, n_nt_ = 0, n_expert = 0;
        if (has_next) n_expert = tile_rows(next, n_item, n_row0, n_nrows, n_nt_);
        const int cur_row0 = row0, cur_nrows = nrows, cur_nt = nt;
        // Row blocks of 32 are dealt to the two wavefront rows in turn (block 2*mb + wm), so a tile with few
        // rows still splits evenly.  Blocks past the tile's rows are skipped -- matrix instructions, fragment
        // reads and stores: the tile body is compiled once per number of blocks this wavefront owns.
        const int my_blocks = (((cur_nrows + 31) >> 5) - wm + 1) >> 1;
        auto run_tile = [&](auto myb_c) {
        constexpr int MYB = decltype(myb_c)::value;
        f32x16_t acc[4][4];
        zero_acc<4, 4>(acc);
        {
            // stage 0 landed: everything but the NS-1 younger stages -- and the stores of the previous
            // tile's epilogue, which are younger still
            MOE_VMCNT_PLUS((NS - 1) * 8, prev_stores);
            __builtin_amdgcn_s_barrier();
            const unsigned a = a_addr[0] + buf * (STAGE * 16), b = b_addr[0] + buf * (STAGE * 16);
            if (0 < MYB) MOE_DS_READ128(fx[0], a, 0); if (1 < MYB) MOE_DS_READ128(fx[1], a, 4096); if (2 < MYB) MOE_DS_READ128(fx[2], a, 8192); if (3 < MYB) MOE_DS_READ128(fx[3], a, 12288);
            MOE_DS_READ128(fx[4], b, 0); MOE_DS_READ128(fx[5], b, 2048); MOE_DS_READ128(fx[6], b, 4096); MOE_DS_READ128(fx[7], b, 6144);
            MOE_WAIT_LGKM0_8(fx);
        }
        for (int kc = 0; kc < nk; ++kc) {
            {   // first 16-deep step of the stage; fetch the fragments of the second
                const unsigned a = a_addr[1] + buf * (STAGE * 16), b = b_addr[1] + buf * (STAGE * 16);
                MOE_MF(fx, 0, 0); if (0 < MYB) MOE_DS_READ128(fy[0], a, 0); MOE_SB();
                MOE_MF(fx, 0, 1); MOE_DS_READ128(fy[4], b, 0); MOE_SB();
                MOE_MF(fx, 0, 2); MOE_DS_READ128(fy[5], b, 2048); MOE_SB();
                MOE_MF(fx, 0, 3); MOE_DS_READ128(fy[6], b, 4096); MOE_SB();
                MOE_MF(fx, 1, 0); MOE_DS_READ128(fy[7], b, 6144); MOE_SB();
                MOE_MF(fx, 1, 1); if (1 < MYB) MOE_DS_READ128(fy[1], a, 4096); MOE_SB();
                MOE_MF(fx, 1, 2); if (2 < MYB) MOE_DS_READ128(fy[2], a, 8192); MOE_SB();
                MOE_MF(fx, 1, 3); if (3 < MYB) MOE_DS_READ128(fy[3], a, 12288); MOE_SB();
                MOE_MF(fx, 2, 0); MOE_MF(fx, 2, 1); MOE_MF(fx, 2, 2); MOE_MF(fx, 2, 3);
                MOE_MF(fx, 3, 0); MOE_MF(fx, 3, 1); MOE_MF(fx, 3, 2); MOE_MF(fx, 3, 3); MOE_SB();
            }
            // the loads issued below belong to the next tile from stage nk on: switch the sources first
            if (kc + NS == nk && has_next) {
                int src_row[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) src_row[i] = n_row0 + local_row(i, n_nrows);
                if (row_idx) {
                    // this wavefront's 64 row numbers were put into LDS by its own load at kc = 0, which is
                    // older than loads the counted waits have since seen land
                    const unsigned ia = lds0 + DENSE_IDX_OFFSET + (w * 64 + ld_r) * 4;
                    asm volatile("ds_read_b32 %0, %4\n\tds_read_b32 %1, %4 offset:64\n\tds_read_b32 %2, %4 offset:128\n\t"
                                 "ds_read_b32 %3, %4 offset:192\n\ts_waitcnt lgkmcnt(0)"
                                 : "=&v"(src_row[0]), "=&v"(src_row[1]), "=&v"(src_row[2]), "=&v"(src_row[3])
                                 : "v"(ia)
                                 : "memory");
#pragma unroll
                    for (int i = 0; i < 4; ++i) src_row[i] = checked(src_row[i]);
                }
                row0 = n_row0; nrows = n_nrows; nt = n_nt_;
                set_sources(n_expert, src_row);
            }
            MOE_WAIT_LGKM0_8(fy);
            // stage kc+1 landed (this wavefront's part); the barrier makes that true for all four and
            // tells that everyone has read stage kc, whose buffer is refilled below.  Stages up to NS-1
            // of a tile were issued before the previous epilogue's stores.
            if (kc + 2 > NS) MOE_VMCNT((NS - 2) * 8);
            else MOE_VMCNT_PLUS((NS - 2) * 8, prev_stores);
            __builtin_amdgcn_s_barrier();
            MOE_SB();
            {
                if (kc == 0 && has_next && row_idx) {
                    // row numbers of the next tile's tokens, 64 per wavefront, straight into LDS.  Issued
                    // BEFORE this stage's loads: the counted waits assume the newest operations are stage loads.
                    int r = w * 64 + lane;
                    r = r < n_nrows ? r : n_nrows - 1;
                    __builtin_amdgcn_global_load_lds((glb_void_t *)(row_idx + n_row0 + r),
                                                     (lds_void_t *)((char *)smem + DENSE_IDX_OFFSET + w * 256), 4, 0, 0);
                }
                int nx = kc + NS;                  // stage to load into the buffer just freed
                if (nx >= nk) nx = has_next ? nx - nk : nk - 1;    // past the last tile: harmless re-read
                uint4 *base = smem + buf * STAGE + (w * 4) * 64;
                buf = buf + 1 == NS ? 0 : buf + 1;
                const unsigned a = a_addr[0] + buf * (STAGE * 16), b = b_addr[0] + buf * (STAGE * 16);
#define MOE_LA(i) __builtin_amdgcn_global_load_lds((glb_void_t *)(a_src[i] + nx * BK), (lds_void_t *)(base + i * 64), 16, 0, 0)
#define MOE_LB(i) __builtin_amdgcn_global_load_lds((glb_void_t *)(b_src[i] + (size_t)nx * 4 * 32), (lds_void_t *)(base + 16 * 64 + i * 64), 16, 0, 0)
                MOE_MF(fy, 0, 0); MOE_LA(0); MOE_SB();
                MOE_MF(fy, 0, 1); MOE_LA(1); MOE_SB();
                MOE_MF(fy, 0, 2); MOE_LA(2); MOE_SB();
                MOE_MF(fy, 0, 3); MOE_LA(3); MOE_SB();
                MOE_MF(fy, 1, 0); MOE_LB(0); MOE_SB();
                MOE_MF(fy, 1, 1); MOE_LB(1); MOE_SB();
                MOE_MF(fy, 1, 2); MOE_LB(2); MOE_SB();
                MOE_MF(fy, 1, 3); MOE_LB(3); MOE_SB();
                MOE_MF(fy, 2, 0); if (0 < MYB) MOE_DS_READ128(fx[0], a, 0); MOE_SB();
                MOE_MF(fy, 2, 1); MOE_DS_READ128(fx[4], b, 0); MOE_SB();
                MOE_MF(fy, 2, 2); MOE_DS_READ128(fx[5], b, 2048); MOE_SB();
                MOE_MF(fy, 2, 3); MOE_DS_READ128(fx[6], b, 4096); MOE_SB();
                MOE_MF(fy, 3, 0); MOE_DS_READ128(fx[7], b, 6144); MOE_SB();
                MOE_MF(fy, 3, 1); if (1 < MYB) MOE_DS_READ128(fx[1], a, 4096); MOE_SB();
                MOE_MF(fy, 3, 2); if (2 < MYB) MOE_DS_READ128(fx[2], a, 8192); MOE_SB();
                MOE_MF(fy, 3, 3); if (3 < MYB) MOE_DS_READ128(fx[3], a, 12288); MOE_SB();
#undef MOE_LA
#undef MOE_LB
            }
            MOE_WAIT_LGKM0_8(fx);
        }
        // epilogue: this wavefront's 128 x 128 part, 32 token rows x 64 columns at a time through its own
        // LDS strip (transposes lane-per-column into 16-byte row pieces)
        const unsigned strip = lds0 + NS * STAGE * 16 + w * (32 * LDE * 2);
        const unsigned wr_addr = strip + ((lane & 31) * LDE + 4 * (lane >> 5)) * 2;
        const unsigned rd_addr = strip + ((lane >> 3) * LDE + (lane & 7) * 8) * 2;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
            if (mb >= MYB) continue;
            typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
            typedef float f32x2_t __attribute__((ext_vector_type(2)));
// volatile asm: an ordinary max here is hoisted by the compiler onto the whole accumulator array right
// after the k loop, which needs 256 more registers and spills
#define MOE_RELU_BITS(f) ({ float r_; asm volatile("v_max_i32 %0, 0, %1" : "=v"(r_) : "v"((float)(f))); r_; })
#define MOE_PK(nb, q)                                                                                                \
    ({                                                                                                               \
        f32x2_t lo = {acc[mb][nb][4 * q], acc[mb][nb][4 * q + 1]}, hi = {acc[mb][nb][4 * q + 2], acc[mb][nb][4 * q + 3]}; \
        if (RELU) { /* as signed integers: anything with the sign bit set becomes +0 */                             \
            lo.x = MOE_RELU_BITS(lo.x); lo.y = MOE_RELU_BITS(lo.y); hi.x = MOE_RELU_BITS(hi.x); hi.y = MOE_RELU_BITS(hi.y); \
        }                                                                                                            \
        uint2 pk;                                                                                                    \
        pk.x = __builtin_bit_cast(unsigned, __builtin_convertvector(lo, bf16x2_t));                                  \
        pk.y = __builtin_bit_cast(unsigned, __builtin_convertvector(hi, bf16x2_t));                                  \
        pk;                                                                                                          \
    })
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                {
                    uint2 v;   // block nb, group q -> columns (nb%2)*32 + 8q + 4*(lane/32) .. +3 of token row lane%32
                    v = MOE_PK(2 * half, 0); MOE_DS_WRITE64(wr_addr, v, 0);       v = MOE_PK(2 * half, 1); MOE_DS_WRITE64(wr_addr, v, 16);
                    v = MOE_PK(2 * half, 2); MOE_DS_WRITE64(wr_addr, v, 32);      v = MOE_PK(2 * half, 3); MOE_DS_WRITE64(wr_addr, v, 48);
                    v = MOE_PK(2 * half + 1, 0); MOE_DS_WRITE64(wr_addr, v, 64);  v = MOE_PK(2 * half + 1, 1); MOE_DS_WRITE64(wr_addr, v, 80);
                    v = MOE_PK(2 * half + 1, 2); MOE_DS_WRITE64(wr_addr, v, 96);  v = MOE_PK(2 * half + 1, 3); MOE_DS_WRITE64(wr_addr, v, 112);
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                u32x4_t o[4];      // rows 8i + lane/8 of the strip: row stride 8 * LDE * 2 = 1152 bytes
                MOE_DS_READ128(o[0], rd_addr, 0);    MOE_DS_READ128(o[1], rd_addr, 1152);
                MOE_DS_READ128(o[2], rd_addr, 2304); MOE_DS_READ128(o[3], rd_addr, 3456);
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(o[0]), "+v"(o[1]), "+v"(o[2]), "+v"(o[3])::"memory");
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int gr = (2 * mb + wm) * 32 + i * 8 + (lane >> 3);
                    // always 8 stores per block, so the counted waits of the next tile hold: rows past the
                    // tile rewrite its last row with the same values (the clamped loads duplicated it)
                    const int sr = gr < cur_nrows ? gr : cur_nrows - 1;
                    *reinterpret_cast<u32x4_t *>(C + (size_t)(cur_row0 + sr) * N + cur_nt * DENSE_BN + wn * 128 + half * 64 +
                                                 (lane & 7) * 8) = o[i];
                }
            }
#undef MOE_PK
#undef MOE_RELU_BITS
        }
        };   // run_tile
        switch (my_blocks) {
        case 0: run_tile(std::integral_constant<int, 0>{}); break;
        case 1: run_tile(std::integral_constant<int, 1>{}); break;
        case 2: run_tile(std::integral_constant<int, 2>{}); break;
        case 3: run_tile(std::integral_constant<int, 3>{}); break;
        default: run_tile(std::integral_constant<int, 4>{}); break;
        }
        if (!has_next) break;
        lin = next;
        prev_stores = 8 * my_blocks;
    }
#undef MOE_MF
    MOE_VMCNT(0);
}

}  // namespace moe
