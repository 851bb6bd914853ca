// bf16 matrix-core tile product for gfx950, shared by the expert FFN, the router and the SRU
// projections.
//
//   C[BM x BN] (fp32 accumulators) += A[rows, K] (row-major bf16, k contiguous)
//                                   * B (packed bf16: element ((k/8)*N + n)*8 + k%8 = B[k][n])
//
// One workgroup = 4 wavefronts.  Wavefront w owns NB column blocks of 32 (columns
// n0 + (w*NB + nb)*32 ..) and all MB row blocks of 32, i.e. MB*NB v_mfma_f32_32x32x16_bf16
// accumulators.  The B operand of that instruction wants, per lane, 8 consecutive k of one
// column: in the packed layout that is one 16-byte load, 32 lanes reading 512 contiguous
// bytes, so weights stream from HBM straight into registers exactly once per workgroup and
// never pass through LDS.  The A rows (tokens) are shared by the four wavefronts and staged
// through LDS in 64-wide k chunks, double buffered, with the next chunk's global loads (A and
// B) issued before the current chunk's matrix instructions.
#pragma once
#include "common.h"

namespace moe {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int GEMM_THREADS = 256;
constexpr int GEMM_BK = 64;
constexpr int GEMM_LDA = GEMM_BK + 8;  // LDS row stride in elements: 144 B keeps b128 reads conflict free

template <int MB>
constexpr int gemm_lds_elems()
{
    return 2 * MB * 32 * GEMM_LDA;
}

// Row of accumulator register v (0..15) of a 32x32 block for this lane; its column is lane & 31.
__device__ __forceinline__ int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// A: pointer to row 0 of the tile (already offset by the tile's first row); rows >= nrows read as 0.
// Bp: packed matrix of this tile's expert; N = its column count; n0 = first column of the tile.
template <int MB, int NB>
__device__ __forceinline__ void gemm_tile_bf16(const bf16_t *__restrict__ A, int lda, int nrows,
                                               const bf16_t *__restrict__ Bp, int N, int n0, int K,
                                               bf16_t *__restrict__ lds, f32x16_t (&acc)[MB][NB])
{
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nk = K / GEMM_BK;
    // A staging: chunk of MB*32 rows x 64 k = MB*256 16-byte pieces, MB per thread
    uint4 a_reg[MB];
    uint4 b_cur[4][NB], b_nxt[4][NB];
    const int a_col = tid & 7;            // 16-byte piece within the 128-byte chunk row
    const int a_row = tid >> 3;           // + i*32
    const uint4 *b_base = reinterpret_cast<const uint4 *>(Bp) + (size_t)(lane >> 5) * N + n0 + w * NB * 32 + (lane & 31);

    auto load_a = [&](int kc) {
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            int r = a_row + i * 32;
            a_reg[i] = r < nrows ? *reinterpret_cast<const uint4 *>(A + (size_t)r * lda + kc * GEMM_BK + a_col * 8)
                                 : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_a = [&](int buf) {
        bf16_t *dst = lds + buf * (MB * 32 * GEMM_LDA);
#pragma unroll
        for (int i = 0; i < MB; ++i)
            *reinterpret_cast<uint4 *>(dst + (a_row + i * 32) * GEMM_LDA + a_col * 8) = a_reg[i];
    };
    auto load_b = [&](int kc, uint4(&b)[4][NB]) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) b[ks][nb] = b_base[(size_t)(kc * 8 + ks * 2) * N + nb * 32];
    };

    load_a(0);
    load_b(0, b_cur);
    store_a(0);
    __syncthreads();
    for (int kc = 0; kc < nk; ++kc) {
        const bool more = kc + 1 < nk;
        if (more) {
            load_a(kc + 1);
            load_b(kc + 1, b_nxt);
        }
        const bf16_t *src = lds + (kc & 1) * (MB * 32 * GEMM_LDA) + (lane & 31) * GEMM_LDA + (lane >> 5) * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                uint4 av = *reinterpret_cast<const uint4 *>(src + mb * 32 * GEMM_LDA + ks * 16);
                bf16x8_t a = __builtin_bit_cast(bf16x8_t, av);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        a, __builtin_bit_cast(bf16x8_t, b_cur[ks][nb]), acc[mb][nb], 0, 0, 0);
            }
        }
        if (more) {
            store_a((kc + 1) & 1);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) b_cur[ks][nb] = b_nxt[ks][nb];
        }
        __syncthreads();
    }
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
