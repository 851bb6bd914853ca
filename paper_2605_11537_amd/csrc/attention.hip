// Sparsemax self-attention over the states of the last SRU layer (the predictor's "sparse
// attention": Methodology; SRU subsection, last paragraph).  Per sequence of L positions and
// n features:
//     s[t, j] = <h_t, h_j> / sqrt(n),   a[t, :] = sparsemax(s[t, :]),   z_t = h_t + sum_j a[t, j] h_j
// with sparsemax(s) = max(s - tau, 0), tau such that the entries sum to one (the Euclidean
// projection onto the simplex).  z is stored in bf16 and goes to the predictor's head.
//
// One workgroup = 32 consecutive positions of one sequence.
//   1. scores on the matrix cores: the 32 query rows sit in LDS; a key row of h is already the
//      operand fragment the matrix instruction wants (8 consecutive features per lane), so keys are
//      read straight from global memory (the sequence's states stay in L2 for its 16 workgroups);
//      the 32 x L fp32 score tile is kept in LDS.
//   2. sparsemax per row, one wavefront per 4 rows, each lane holding L/64 scores: tau by Michelot's
//      fixed point (tau = (sum of the entries above tau - 1) / their count, until the set is stable),
//      which ends at exactly the support the sorting definition gives.
//   3. the context sum_j a[t, j] h_j on the matrix cores: the contraction runs over positions, so the
//      state operand must have 8 consecutive positions of one feature per lane -- a small kernel first
//      writes, per sequence, the packed image of its states as a (positions x features) matrix (the
//      layout moe_pack_weights gives weights: a wavefront's fragment load is 1 KB of consecutive memory).
//      The weights go back into the score tile and are read from there
//      as the other operand, rounded to bf16 (relative error 2^-9 per weight, the size of the bf16
//      rounding of z itself).  On the vector units the same sum is 16384 multiply-adds per lane and took
//      three times as long as everything else in the kernel.
#include "gemm_bf16.h"
#include "route.h"

namespace moe {

constexpr int ATT_QT = 32;           // query rows per workgroup
constexpr int ATT_MAX_L = 1024;      // positions per sequence the LDS score tile holds
constexpr int ATT_MAX_N = 256;       // features per state
constexpr int ATT_WAVES = 8;         // wavefronts per workgroup (two per SIMD)
constexpr int ATT_THREADS = ATT_WAVES * 64;
constexpr int ATT_LDS_S = ATT_MAX_L + 4;

// Wavefront-wide reductions on the data-parallel-primitive path (a cross-lane operand of an ordinary
// vector instruction) instead of LDS-routed shuffles: sparsemax does a dozen of them per row, one
// after the other.  Four steps fold a row of 16 lanes (quad swaps, then rotations by 4 and 8); the
// four row results are read as scalars and added.  Every lane gets the result.
template <class Op>
__device__ __forceinline__ float wave_reduce_f(float v, Op op)
{
    auto dpp = [](float x, int ctrl) {
        switch (ctrl) {
        case 0: return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, false));
        case 1: return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xf, 0xf, false));
        case 2: return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x124, 0xf, 0xf, false));
        default: return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x128, 0xf, 0xf, false));
        }
    };
    v = op(v, dpp(v, 0));    // lane ^ 1
    v = op(v, dpp(v, 1));    // lane ^ 2
    v = op(v, dpp(v, 2));    // the quad 4 lanes away in the row of 16
    v = op(v, dpp(v, 3));    // the half row 8 lanes away
    const int b = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return op(op(r0, r1), op(r2, r3));
}
__device__ __forceinline__ float wave_sum_f(float v) { return wave_reduce_f(v, [](float a, float b) { return a + b; }); }
__device__ __forceinline__ float wave_max_f(float v) { return wave_reduce_f(v, [](float a, float b) { return fmaxf(a, b); }); }

__global__ __launch_bounds__(ATT_THREADS, 1) void sru_attention_kernel(const bf16_t *__restrict__ h,
                                                                        const bf16_t *__restrict__ hp, int L, int Lp,
                                                                        int n, bf16_t *__restrict__ z)
{
    __shared__ __attribute__((aligned(16))) float s_lds[ATT_QT * ATT_LDS_S];
    __shared__ __attribute__((aligned(16))) bf16_t q_lds[ATT_QT * (ATT_MAX_N + 8)];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    // Workgroup i runs on XCD i % 8; all query blocks of a sequence read the same keys and packed states,
    // so whole sequences go to one XCD (sequence b to XCD b % 8) when their number allows: an XCD's L2 then
    // holds 1/8 of the states instead of cycling through all of them.
    int seq, qblk;
    {
        const int nqb = (L + ATT_QT - 1) / ATT_QT, nseq = gridDim.x / nqb;
        if (nseq % 8 == 0) {
            const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
            seq = xcd + 8 * (slot / nqb);
            qblk = slot % nqb;
        } else {
            seq = blockIdx.x / nqb;
            qblk = blockIdx.x % nqb;
        }
    }
    const int q0 = qblk * ATT_QT;
    const bf16_t *hs = h + (size_t)seq * L * n;
    const int ldq = n + 8;
    // query rows (positions past the sequence end repeat its last row; they are never stored)
    for (int p = tid; p < ATT_QT * (n / 8); p += ATT_THREADS) {
        const int r = p / (n / 8), c8 = p % (n / 8);
        const int t = q0 + r < L ? q0 + r : L - 1;
        *reinterpret_cast<uint4 *>(q_lds + r * ldq + c8 * 8) = *reinterpret_cast<const uint4 *>(hs + (size_t)t * n + c8 * 8);
    }
    __syncthreads();
    // 1. scores: wavefront w takes key blocks w, w+8, ...
    const float scale = rsqrtf((float)n);
    const int n_kb = (L + 31) / 32;
    {
        // the key fragments of a block are all requested at once, and those of the wavefront's next block
        // before the current block's matrix instructions: one exposed round trip per wavefront, not per block
        constexpr int NKS = ATT_MAX_N / 16;
        uint4 kf[2][NKS];
        auto load_keys = [&](int kb, int buf) {
            const int key = kb * 32 + (lane & 31);
            const bf16_t *krow = hs + (size_t)(key < L ? key : L - 1) * n + (lane >> 5) * 8;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                if (ks * 16 < n) kf[buf][ks] = *reinterpret_cast<const uint4 *>(krow + ks * 16);
        };
        auto score_block = [&](int kb, int buf) {
            f32x16_t acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
            const int key = kb * 32 + (lane & 31);
            const bf16_t *qrow = q_lds + (lane & 31) * ldq + (lane >> 5) * 8;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                if (ks * 16 < n) {
                    const uint4 a = *reinterpret_cast<const uint4 *>(qrow + ks * 16);
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                                  __builtin_bit_cast(bf16x8_t, kf[buf][ks]), acc, 0, 0, 0);
                }
#pragma unroll
            for (int v = 0; v < 16; ++v) s_lds[acc_row(v, lane) * ATT_LDS_S + key] = acc[v] * scale;
        };
        if (w < n_kb) load_keys(w, 0);
        for (int kb = w; kb < n_kb; kb += 2 * ATT_WAVES) {
            if (kb + ATT_WAVES < n_kb) load_keys(kb + ATT_WAVES, 1);
            __builtin_amdgcn_sched_barrier(0);
            score_block(kb, 0);
            if (kb + ATT_WAVES < n_kb) {
                if (kb + 2 * ATT_WAVES < n_kb) load_keys(kb + 2 * ATT_WAVES, 0);
                __builtin_amdgcn_sched_barrier(0);
                score_block(kb + ATT_WAVES, 1);
            }
        }
    }
    __syncthreads();
    // 2. + 3. one wavefront per 4 rows
    constexpr int PER = ATT_MAX_L / 64;
    const int n_chunks = (L + 63) / 64;
    for (int rr = 0; rr < ATT_QT / ATT_WAVES; ++rr) {
        const int r = w * (ATT_QT / ATT_WAVES) + rr;
        const int t = q0 + r;
        if (t >= L) {                      // wave-uniform; the matrix product below reads all 32 weight rows
            for (int j = lane; j < Lp; j += 64) s_lds[r * ATT_LDS_S + j] = 0.f;
            continue;
        }
        float zr[PER];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int j = i * 64 + lane;
            zr[i] = (i < n_chunks && j < L) ? s_lds[r * ATT_LDS_S + j] : -INFINITY;
            mx = fmaxf(mx, zr[i]);
        }
        mx = wave_max_f(mx);
        // shift by the row maximum (sparsemax is shift invariant): the sums below stay small
        // counts are kept as floats (exact up to 2^24) so that one reduction serves sums and counts alike
        float sum = 0.f, cnt = 0.f;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            zr[i] -= mx;                    // -inf stays -inf
            if (zr[i] > -INFINITY) {
                sum += zr[i];
                cnt += 1.f;
            }
        }
        sum = wave_sum_f(sum);
        cnt = wave_sum_f(cnt);
        float tau = (sum - 1.f) / cnt;
        for (;;) {
            float s2 = 0.f, c2 = 0.f;
#pragma unroll
            for (int i = 0; i < PER; ++i)
                if (zr[i] > tau) {
                    s2 += zr[i];
                    c2 += 1.f;
                }
            s2 = wave_sum_f(s2);
            c2 = wave_sum_f(c2);
            if (c2 >= cnt) break;           // the set above tau did not shrink: tau is final (and the loop ends)
            cnt = c2;                       // never 0: the maximum (0 after the shift) stays above tau < 0
            tau = (s2 - 1.f) / c2;
        }
        // the weights go back into the row of the score tile (positions past the sequence get 0)
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (i < n_chunks && i * 64 + lane < Lp) s_lds[r * ATT_LDS_S + i * 64 + lane] = zr[i] > tau ? zr[i] - tau : 0.f;
    }
    __syncthreads();   // every row's weights are in the score tile
    // 3. context on the matrix cores: wavefront w owns feature block w (32 features; and w + 8) of all
    // 32 rows; per step of 16 positions one weight fragment (from the score tile, rounded to bf16) and one
    // fragment of the packed states per block.
    {
        // packed image of this sequence's states as a (positions x features) matrix, positions >= L zero:
        // a wavefront's fragment load is 1 KB of consecutive memory
        const uint4 *hps = reinterpret_cast<const uint4 *>(hp) + (size_t)seq * (n / 32) * (Lp / 8) * 32;
        f32x16_t acc[2];
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[0][v] = acc[1][v] = 0.f;
        // wavefront w owns feature blocks w and w + ATT_WAVES (32 features each)
        const int fb0 = w;
        const bool have[2] = {fb0 * 32 < n, (fb0 + ATT_WAVES) * 32 < n};      // wave-uniform
        const float *arow = s_lds + (lane & 31) * ATT_LDS_S + (lane >> 5) * 8;
        const uint4 *b0 = hps + ((size_t)fb0 * (Lp / 8) + (lane >> 5)) * 32 + (lane & 31);
        const uint4 *b1 = b0 + (size_t)ATT_WAVES * (Lp / 8) * 32;
        // the state fragments of 8 steps (128 positions) are requested together, the next batch before the
        // current batch's matrix instructions; fetched one step at a time, every step waited a round trip
        constexpr int CB = 8;
        uint4 sf[2][CB][2];
        auto load_states = [&](int j0, int buf) {
#pragma unroll
            for (int u = 0; u < CB; ++u) {
                const int j = j0 + u * 16;
                sf[buf][u][0] = have[0] && j < Lp ? b0[(size_t)(j >> 3) * 32] : make_uint4(0, 0, 0, 0);
                sf[buf][u][1] = have[1] && j < Lp ? b1[(size_t)(j >> 3) * 32] : make_uint4(0, 0, 0, 0);
            }
        };
        auto context_batch = [&](int j0, int buf) {
#pragma unroll
            for (int u = 0; u < CB; ++u) {
                const int j = j0 + u * 16;
                if (j < Lp) {                                          // wave-uniform
                    const float4 a_lo = *reinterpret_cast<const float4 *>(arow + j);
                    const float4 a_hi = *reinterpret_cast<const float4 *>(arow + j + 4);
                    uint4 af;
                    af.x = pack_bf16x2(a_lo.x, a_lo.y);
                    af.y = pack_bf16x2(a_lo.z, a_lo.w);
                    af.z = pack_bf16x2(a_hi.x, a_hi.y);
                    af.w = pack_bf16x2(a_hi.z, a_hi.w);
                    if (have[0])
                        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, af),
                                                                         __builtin_bit_cast(bf16x8_t, sf[buf][u][0]),
                                                                         acc[0], 0, 0, 0);
                    if (have[1])
                        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, af),
                                                                         __builtin_bit_cast(bf16x8_t, sf[buf][u][1]),
                                                                         acc[1], 0, 0, 0);
                }
            }
        };
        load_states(0, 0);
        for (int j0 = 0; j0 < Lp; j0 += 2 * CB * 16) {
            if (j0 + CB * 16 < Lp) load_states(j0 + CB * 16, 1);
            __builtin_amdgcn_sched_barrier(0);
            context_batch(j0, 0);
            if (j0 + CB * 16 < Lp) {
                if (j0 + 2 * CB * 16 < Lp) load_states(j0 + 2 * CB * 16, 0);
                __builtin_amdgcn_sched_barrier(0);
                context_batch(j0 + CB * 16, 1);
            }
        }
#pragma unroll
        for (int k = 0; k < 2; ++k)
            if (have[k]) {
                const int f = (fb0 + k * ATT_WAVES) * 32 + (lane & 31);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = acc_row(v, lane);
                    if (q0 + r < L)
                        z[((size_t)seq * L + q0 + r) * n + f] = f32_to_bf16(bf16_to_f32(q_lds[r * ldq + f]) + acc[k][v]);
                }
            }
    }
}

// h [B*L, n] -> per sequence the packed image of the (Lp x n) matrix of its states (positions past L are
// zero): 16-byte piece ((f / 32) * (Lp / 8) + t / 8) * 32 + f % 32 holds h[8 (t / 8) .. + 7][f]
__global__ __launch_bounds__(256) void sru_pack_states_kernel(const bf16_t *__restrict__ h, int L, int Lp, int n,
                                                              uint4 *__restrict__ hp)
{
    const int per_seq = (n / 32) * (Lp / 8) * 32;
    const int p = blockIdx.x * 256 + threadIdx.x, seq = blockIdx.y;
    if (p >= per_seq) return;
    const int c = p & 31, kg = (p >> 5) % (Lp / 8), strip = (p >> 5) / (Lp / 8);
    const bf16_t *src = h + ((size_t)seq * L + kg * 8) * n + strip * 32 + c;
    uint32_t v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = kg * 8 + 2 * i;
        const uint32_t lo = t < L ? src[(size_t)(2 * i) * n] : 0, hi = t + 1 < L ? src[(size_t)(2 * i + 1) * n] : 0;
        v[i] = lo | (hi << 16);
    }
    hp[(size_t)seq * per_seq + p] = make_uint4(v[0], v[1], v[2], v[3]);
}

size_t sru_attention_ws_bytes(int B, int L, int n) { return align_up((size_t)(B > 0 ? B : 1) * n * align_up((size_t)L, 16) * 2, 256); }

int sru_attention_launch(const void *h, int B, int L, int n, void *z, void *ht_ws, hipStream_t st, const char *who)
{
    MOE_REQUIRE(L <= ATT_MAX_L && n <= ATT_MAX_N && n % 64 == 0, MOE_ERR_UNSUPPORTED,
                "%s: sparsemax attention is built for L <= %d and n_hidden <= %d (multiple of 64); got L=%d n_hidden=%d", who,
                ATT_MAX_L, ATT_MAX_N, L, n);
    if (B == 0) return MOE_OK;
    const int Lp = (int)align_up((size_t)L, 16);
    hipLaunchKernelGGL(sru_pack_states_kernel, dim3(ceil_div((n / 32) * (Lp / 8) * 32, 256), B), dim3(256), 0, st,
                       (const bf16_t *)h, L, Lp, n, (uint4 *)ht_ws);
    MOE_CHECK_LAUNCH(who);
    hipLaunchKernelGGL(sru_attention_kernel, dim3(ceil_div(L, ATT_QT) * B), dim3(ATT_THREADS), 0, st, (const bf16_t *)h,
                       (const bf16_t *)ht_ws, L, Lp, n, (bf16_t *)z);
    MOE_CHECK_LAUNCH(who);
    return MOE_OK;
}

}  // namespace moe
