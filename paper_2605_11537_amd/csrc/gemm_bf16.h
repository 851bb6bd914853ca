// bf16 matrix-core tile product for gfx950, shared by the expert FFN, the router and the SRU
// projections.
//
//   C[BM x BN] (fp32 accumulators) += A[rows, K] (row-major bf16, k contiguous) * B[K, N]
//
// B is read from the packed image (see moe_pack_weights): columns are grouped in strips of
// 32; inside a strip, for every group of 8 consecutive k, the 32 columns follow each other
// with their 8 k-values contiguous (16 bytes).  uint4 index of (k/8 = g, column n):
//     ((n/32) * (K/8) + g) * 32 + n%32
// The B operand of v_mfma_f32_32x32x16_bf16 wants, per lane, 8 consecutive k of one column
// (lanes 0-31: k 0-7, lanes 32-63: k 8-15 of the 16-deep step): in this image that is ONE
// 16-byte load per lane, the 64 lanes of a wavefront reading 1 KB of consecutive memory, and
// a wavefront walking down K reads one strip front to back.  Weights therefore stream from
// HBM straight into registers exactly once per workgroup, in DRAM-page order, and never
// pass through LDS.
//
// One workgroup = 4 wavefronts arranged WM x WN (WN = 4 / WM).  Wavefront (wm, wn) owns MB row
// blocks of 32 rows (rows (wm*MB + mb)*32 ..) and NB column strips (columns
// n0 + (wn*NB + nb)*32 ..): MB*NB accumulators of 16 VGPRs.  WM = 1 is the weight-streaming
// shape (every weight byte is loaded by exactly one wavefront); WM = 2 doubles the rows per
// weight byte for compute-bound tiles.
// The A rows (tokens) are shared by the four wavefronts and staged through LDS in BK-wide k
// chunks, double buffered; the global loads of chunk i+1 (A and B) are issued before the
// matrix instructions of chunk i, B registers ping-pong between two sets so nothing is
// copied.
#pragma once
#include "common.h"

namespace moe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int GEMM_THREADS = 256;

template <int MB, int BK, int WM = 1>
constexpr int gemm_lds_elems()
{
    return 2 * WM * MB * 32 * (BK + 8);   // row stride BK+8 elements keeps the b128 reads conflict free
}

// Row of accumulator register v (0..15) of a 32x32 block for this lane; its column is lane & 31.
__device__ __forceinline__ int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// A: pointer to row 0 of the tile (already offset by the tile's first row); rows >= nrows read as 0.
// row_idx (optional, already offset to the tile's first row): tile row r is read from
//   A + row_idx[r]*lda instead of A + r*lda (fused gather of token rows).
// Bp: packed matrix (K x N) of this tile's expert; n0 = first column of the tile (multiple of 32).
// K must be a multiple of BK.
// STREAM_B: the B operand is read exactly once in the whole launch (expert weights): load it
// with the non-temporal hint so the stream does not evict the activations the other operand
// and the epilogue keep in cache.  (Measured on the 604 MB weight stream of a 128-expert
// layer: 120 -> 110 us for the first FFN product, 111 -> 101 us for the second.)
template <int MB, int NB, int BK, bool STREAM_B = false, int WM = 1>
__device__ __forceinline__ void gemm_tile_bf16(const bf16_t *__restrict__ A, int lda, int nrows,
                                               const bf16_t *__restrict__ Bp, int n0, int K,
                                               bf16_t *__restrict__ lds, f32x16_t (&acc)[MB][NB],
                                               const int32_t *__restrict__ row_idx = nullptr, int n_src_rows = 0)
{
    constexpr int LDA = BK + 8;
    constexpr int KS = BK / 16;                       // 16-deep MFMA steps per chunk
    constexpr int WN = 4 / WM;
    constexpr int BM = WM * MB * 32;                  // rows of the workgroup tile
    constexpr int PIECES = BM * (BK / 8);             // 16-byte pieces of one A chunk
    constexpr int A_PER_THREAD = PIECES / GEMM_THREADS;
    constexpr int ROW_STEP = GEMM_THREADS / (BK / 8);
    static_assert(PIECES % GEMM_THREADS == 0, "A chunk must split evenly over the workgroup");
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = w / WN, wn = w % WN;
    const int nk = K / BK;
    const int KG = K >> 3;
    uint4 a_reg[A_PER_THREAD];
    uint4 b0[KS][NB], b1[KS][NB];
    const int a_col = tid % (BK / 8);
    const int a_row = tid / (BK / 8);
    const uint4 *b_base = reinterpret_cast<const uint4 *>(Bp) + (size_t)((n0 >> 5) + wn * NB) * KG * 32 + lane;

    const bf16_t *a_src[A_PER_THREAD];   // this thread's rows stay the same for every k chunk
    bool a_ok[A_PER_THREAD];             // rows past the tile, or an index outside the source, read as 0
#pragma unroll
    for (int i = 0; i < A_PER_THREAD; ++i) {
        int r = a_row + i * ROW_STEP;
        a_ok[i] = r < nrows;
        int src_row = r;
        if (row_idx && a_ok[i]) {
            src_row = row_idx[r];
            a_ok[i] = src_row >= 0 && src_row < n_src_rows;
        }
        a_src[i] = A + (size_t)(a_ok[i] ? src_row : 0) * lda + a_col * 8;
    }
    auto load_a = [&](int kc) {
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i)
            a_reg[i] = a_ok[i] ? *reinterpret_cast<const uint4 *>(a_src[i] + kc * BK) : make_uint4(0, 0, 0, 0);
    };
    auto store_a = [&](int buf) {
        bf16_t *dst = lds + buf * (BM * LDA);
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i)
            *reinterpret_cast<uint4 *>(dst + (a_row + i * ROW_STEP) * LDA + a_col * 8) = a_reg[i];
    };
    auto load_b = [&](int kc, uint4(&b)[KS][NB]) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const uint4 *p = b_base + ((size_t)nb * KG + kc * (BK / 8) + ks * 2) * 32;
                if (STREAM_B) {
                    typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
                    u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
                    b[ks][nb] = make_uint4(v.x, v.y, v.z, v.w);
                } else {
                    b[ks][nb] = *p;
                }
            }
    };
    auto compute = [&](int kc, const uint4(&b)[KS][NB]) {
        const bf16_t *src = lds + (kc & 1) * (BM * LDA) + (wm * MB * 32 + (lane & 31)) * LDA + (lane >> 5) * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                uint4 av = *reinterpret_cast<const uint4 *>(src + mb * 32 * LDA + ks * 16);
                bf16x8_t a = __builtin_bit_cast(bf16x8_t, av);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8_t, b[ks][nb]),
                                                                          acc[mb][nb], 0, 0, 0);
            }
        }
    };
    // one pipeline stage: fetch chunk kc+1 into `nxt`, multiply chunk kc out of `cur`
    auto stage = [&](int kc, const uint4(&cur)[KS][NB], uint4(&nxt)[KS][NB]) {
        const bool more = kc + 1 < nk;
        if (more) {
            load_a(kc + 1);
            load_b(kc + 1, nxt);
        }
        // keep the prefetch where it is: left alone, the scheduler sinks these loads below the
        // matrix instructions to save registers, and every chunk then waits a full memory round trip
        __builtin_amdgcn_sched_barrier(0);
        compute(kc, cur);
        if (more) store_a((kc + 1) & 1);
        __syncthreads();
    };

    load_a(0);
    load_b(0, b0);
    store_a(0);
    __syncthreads();
    int kc = 0;
    for (; kc + 1 < nk; kc += 2) {
        stage(kc, b0, b1);
        stage(kc + 1, b1, b0);
    }
    if (kc < nk) stage(kc, b0, b1);
}

template <int MB, int NB>
__device__ __forceinline__ void zero_acc(f32x16_t (&acc)[MB][NB])
{
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;
}

}  // namespace moe
