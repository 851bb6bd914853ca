// sru_predict: SRU stack + linear head + argmax, the expert predictor.
//
// Per layer: (1) the concatenated weight [n_in, k*n_h] is re-laid into the packed image the MFMA B
// operand wants (small, into the workspace; skipped when the weights arrive packed, see
// sru_weights.w_layout); (2) one matrix-core product U = X * [W | W_f | W_r | (W_h)] for all B*L
// tokens at once (the part of the SRU that is parallel over time); (3) the recurrence.  The gates
// depend on the input only, so c_t = f_t c_{t-1} + (1-f_t) x'_t is a linear recurrence in c: a
// workgroup takes a few channels of one sequence and cuts the time axis into 64 chunks; every thread
// first composes its chunk into (A, B) with c_out = A c_in + B, the 64 chunk maps of a channel are
// composed by a scan, and each thread then re-runs its chunk from its true carry-in and writes h_t.
// For sequences of up to 512 positions steps (2) and (3) are one kernel per layer with the projections
// kept in LDS (sru_layer_fused_kernel below); the two-kernel form (sru_proj_kernel, sru_scan_kernel)
// serves longer sequences.  The head is a router-shaped product + argmax and reuses the router's kernel.
#include "gemm_bf16.h"
#include "route.h"

namespace moe {

constexpr int SRU_CHUNKS = 64;     // time chunks per sequence
constexpr int SRU_CHANNELS = 16;   // channels per workgroup (SRU_CHUNKS * SRU_CHANNELS = 1024 threads)

// U[T, N] (fp32) = X[T, K] (bf16) * packed W
__global__ __launch_bounds__(GEMM_THREADS) void sru_proj_kernel(const bf16_t *__restrict__ X,
                                                                const bf16_t *__restrict__ Wp, int T, int K, int N,
                                                                float *__restrict__ U)
{
    __shared__ __attribute__((aligned(16))) bf16_t lds[gemm_lds_elems<2, 64>()];
    const int n_nt = N / 128;
    const int mt = blockIdx.x / n_nt, nt = blockIdx.x - mt * n_nt;
    const int row0 = mt * 64;
    const int nrows = T - row0 < 64 ? T - row0 : 64;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    f32x16_t acc[2][1];
    zero_acc<2, 1>(acc);
    gemm_tile_bf16<2, 1, 64>(X + (size_t)row0 * K, K, nrows, Wp, nt * 128, K, lds, acc);
    const int col = nt * 128 + w * 32 + (lane & 31);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int r = mb * 32 + acc_row(v, lane);
            if (r < nrows) U[(size_t)(row0 + r) * N + col] = acc[mb][0][v];
        }
}

// binary32 with the hardware exponential: a few ulp, far inside the bf16 rounding of h
__device__ __forceinline__ float sigmoidf_(float v) { return 1.f / (1.f + __expf(-v)); }
__device__ __forceinline__ float tanhf_(float v)
{
    float a = fminf(fabsf(v), 15.f);
    float t = 1.f - 2.f / (1.f + __expf(2.f * a));
    return copysignf(t, v);
}

// grid (n_h/16, B); block = 16 channels x 64 time chunks.  Phase 1: every thread composes its
// chunk into (A, B) with c_out = A*c_in + B.  Phase 2: one wavefront per channel composes the 64
// chunk maps by a scan.  Phase 3: every thread re-runs its chunk from its true carry-in and writes h_t.
// CL > 0: a chunk holds at most CL steps and the thread keeps all its inputs in registers -- every load of
// the kernel is issued up front, one memory round trip instead of four (U was written by other XCDs a
// moment ago, so each exposed round trip is a miss in this XCD's L2).  CL = 0: any chunk length, the
// inputs are streamed twice.
template <int CL>
__global__ __launch_bounds__(SRU_CHUNKS * SRU_CHANNELS) void sru_scan_kernel(
    const float *__restrict__ U, const bf16_t *__restrict__ x_in, int L, int n_h, int k,
    const float *__restrict__ b_f, const float *__restrict__ b_r, bf16_t *__restrict__ h_out)
{
    __shared__ float carry_a[SRU_CHUNKS][SRU_CHANNELS], carry_b[SRU_CHUNKS][SRU_CHANNELS];
    const int ch = threadIdx.x & (SRU_CHANNELS - 1), q = threadIdx.x / SRU_CHANNELS;
    const int j = blockIdx.x * SRU_CHANNELS + ch;
    const int b = blockIdx.y;
    const int ncol = k * n_h;
    const int cl = (L + SRU_CHUNKS - 1) / SRU_CHUNKS;
    const int t0 = q * cl < L ? q * cl : L, t1 = (t0 + cl < L) ? t0 + cl : L;
    const float bf = b_f ? b_f[j] : 0.f, br = b_r ? b_r[j] : 0.f;
    const float *u = U + (size_t)b * L * ncol + j;
    const bf16_t *xi = x_in + (size_t)b * L * n_h + j;   // only read when k == 3 (n_in == n_h)
    bf16_t *ho = h_out + (size_t)b * L * n_h + j;

    constexpr int NR = CL > 0 ? CL : 1;
    float ux[NR], uf[NR], ur[NR], uh[NR];
    if (CL > 0) {
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            const int t = t0 + i;
            const bool ok = t < t1;
            const float *ut = u + (size_t)(ok ? t : t0) * ncol;
            ux[i] = ok ? ut[0] : 0.f;
            uf[i] = ok ? ut[n_h] : 0.f;
            ur[i] = ok ? ut[2 * n_h] : 0.f;
            uh[i] = !ok ? 0.f : (k == 4 ? ut[3 * n_h] : bf16_to_f32(xi[(size_t)t * n_h]));
        }
    }

    float a = 1.f, c = 0.f;
    if (CL > 0) {
#pragma unroll
        for (int i = 0; i < NR; ++i)
            if (t0 + i < t1) {
                const float f = sigmoidf_(uf[i] + bf);
                uf[i] = f;                               // the gate itself from here on
                a *= f;
                c = f * c + (1.f - f) * ux[i];
            }
    } else {
#pragma unroll 4
        for (int t = t0; t < t1; ++t) {
            const float *ut = u + (size_t)t * ncol;
            float f = sigmoidf_(ut[n_h] + bf);
            a *= f;
            c = f * c + (1.f - f) * ut[0];
        }
    }
    carry_a[q][ch] = a;
    carry_b[q][ch] = c;
    __syncthreads();
    // Carry-in of every chunk, in place (carry_b[p] <- state entering chunk p): the 64 chunk maps
    // c -> a c + b of a channel are composed by an inclusive scan across the 64 lanes of one wavefront
    // (wavefront w takes channel w; six doubling steps instead of a serial chain of 64 LDS round trips,
    // which was ~40 % of this kernel's time)
    {
        const int lane = threadIdx.x & 63, sc = threadIdx.x >> 6;      // lane = chunk, sc = channel
        float pa = carry_a[lane][sc], pb = carry_b[lane][sc];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const float qa = __shfl_up(pa, o, 64), qb = __shfl_up(pb, o, 64);   // the map of the chunks before
            if (lane >= o) {
                pb = pa * qb + pb;       // (this) o (earlier): c -> pa (qa c + qb) + pb
                pa = pa * qa;
            }
        }
        // state after chunks 0..lane from c = 0 is pb; chunk lane + 1 starts from it
        const float into_next = pb;
        const float mine = __shfl_up(into_next, 1, 64);
        __syncthreads();                 // every (a, b) has been read before any carry is overwritten
        carry_b[lane][sc] = lane == 0 ? 0.f : mine;
    }
    __syncthreads();
    c = carry_b[q][ch];

    if (CL > 0) {
#pragma unroll
        for (int i = 0; i < NR; ++i)
            if (t0 + i < t1) {
                const float f = uf[i];
                const float r = sigmoidf_(ur[i] + br);
                c = f * c + (1.f - f) * ux[i];
                ho[(size_t)(t0 + i) * n_h] = f32_to_bf16(r * tanhf_(c) + (1.f - r) * uh[i]);
            }
        return;
    }
#pragma unroll 4
    for (int t = t0; t < t1; ++t) {
        const float *ut = u + (size_t)t * ncol;
        float f = sigmoidf_(ut[n_h] + bf);
        float r = sigmoidf_(ut[2 * n_h] + br);
        c = f * c + (1.f - f) * ut[0];
        float hw = k == 4 ? ut[3 * n_h] : bf16_to_f32(xi[(size_t)t * n_h]);
        ho[(size_t)t * n_h] = f32_to_bf16(r * tanhf_(c) + (1.f - r) * hw);
    }
}

// ------------------------------------------------------------------ one SRU layer in one kernel (L <= 512)
// Workgroup (channel block cb of 8 channels, sequence b): the projections of ITS 8 channels for all L
// positions -- 32 columns of [W | W_f | W_r | (W_h)], one matrix-core column block, gathered from the packed
// image piece by piece -- land in LDS (L x 32 binary32), and the recurrence runs from there: time chunks
// x 8 channels (64 chunks), chunk maps composed by a doubling scan across the chunks, every chunk re-run from its true
// carry-in.  The projections never go to memory (the two-kernel form writes and re-reads 3-4 binary32
// values per position and channel, and its scan was bound by what one CU can fetch), there is one launch per
// layer instead of two, and B * n_h / 8 workgroups cover the chip at 8 sequences x 256 channels.
// The token rows reach the matrix cores without a workgroup barrier (whole lines from memory, a
// wavefront-private LDS transposition, see below).
constexpr int FUS_CH = 8;              // channels per workgroup
constexpr int FUS_THREADS = 512;       // 8 wavefronts: 2 per SIMD, so one's loads fly under the other's work
constexpr int FUS_CHUNKS = FUS_THREADS / FUS_CH;   // 64 time chunks per sequence
constexpr int FUS_MAX_L = 512;
constexpr int FUS_CL = FUS_MAX_L / FUS_CHUNKS;     // steps per chunk at most
constexpr int FUS_LDU = 33;            // row stride of the LDS tile, binary32 elements
constexpr int FUS_KC = 64;             // k per register buffer

template <int NRB>                     // 32-row blocks per wavefront: L <= 256 * NRB
__global__ __launch_bounds__(FUS_THREADS, 1) void sru_layer_fused_kernel(const bf16_t *__restrict__ X,
                                                                         const bf16_t *__restrict__ Wp, int L, int K,
                                                                         int n_h, int kgates,
                                                                         const float *__restrict__ b_f,
                                                                         const float *__restrict__ b_r,
                                                                         bf16_t *__restrict__ h_out)
{
    // the L x 32 tile of projections; during the product, the wavefronts' staging pieces for the token rows
    constexpr int TILE_FLOATS = FUS_MAX_L * FUS_LDU, STAGE_FLOATS = (FUS_THREADS / 64) * NRB * 32 * (FUS_KC + 8) / 2;
    __shared__ __attribute__((aligned(16))) float u_lds[TILE_FLOATS > STAGE_FLOATS ? TILE_FLOATS : STAGE_FLOATS];
    __shared__ float car_a[2][FUS_CHUNKS][FUS_CH], car_b[2][FUS_CHUNKS][FUS_CH];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    // Workgroup i runs on XCD i % 8.  All channel blocks of a sequence read the same token rows, written a
    // moment ago by other XCDs: with whole sequences per XCD (sequence b on XCD b % 8, when their number
    // allows) an XCD's L2 fetches 1/8 of the rows instead of all of them.
    int cb, b;
    {
        const int ncb = n_h / FUS_CH, nseq = gridDim.x / ncb;
        if (nseq % 8 == 0) {
            const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
            b = xcd + 8 * (slot / ncb);
            cb = slot % ncb;
        } else {
            b = blockIdx.x / ncb;
            cb = blockIdx.x % ncb;
        }
    }
    const int KG = K >> 3;
    // recurrence roles: thread = (chunk q, channel ch)
    const int ch = tid & (FUS_CH - 1), q = tid / FUS_CH;
    const int j = cb * FUS_CH + ch;
    const int cl = (L + FUS_CHUNKS - 1) / FUS_CHUNKS;
    const int t0 = q * cl < L ? q * cl : L, t1 = t0 + cl < L ? t0 + cl : L;
    // highway input when the widths are equal (K == n_h): fetched now, used at the very end
    float hwv[FUS_CL];
    if (kgates == 3) {
        const bf16_t *xi = X + (size_t)b * L * K + j;
#pragma unroll
        for (int i = 0; i < FUS_CL; ++i) hwv[i] = t0 + i < t1 ? bf16_to_f32(xi[(size_t)(t0 + i) * K]) : 0.f;
    }
    // ---- projections: U[t][c], c = gate * 8 + channel
    {
        // Token rows: a wavefront fetches its own row blocks in whole 128-byte lines (8 lanes per row, 8 rows
        // per load), turns them into A fragments through a private piece of LDS (row stride 72 elements, no
        // barrier: LDS operations of one wavefront execute in order), three register buffers deep.  A lane
        // loading its fragment straight from memory touches 32 bytes of 32 different lines per load, and
        // the kernel was bound by those transactions.
        constexpr int LDA = FUS_KC + 8;
        bf16_t *stage = reinterpret_cast<bf16_t *>(u_lds) + (size_t)w * (NRB * 32 * LDA);
        const int r = lane & 31, kh = lane >> 5;
        const int lrow = lane >> 3, lpiece = lane & 7;
        const bf16_t *a_ptr[NRB][4];
        bool a_ok[NRB][4];
#pragma unroll
        for (int i = 0; i < NRB; ++i)
#pragma unroll
            for (int sb = 0; sb < 4; ++sb) {
                const int t = (w + 8 * i) * 32 + sb * 8 + lrow;   // row blocks dealt to the eight wavefronts in turn
                a_ok[i][sb] = t < L;
                a_ptr[i][sb] = X + ((size_t)b * L + (a_ok[i][sb] ? t : 0)) * K + lpiece * 8;
            }
        const int gate = r >> 3, chn = r & 7;
        const bool b_ok = gate < kgates;
        const int col = (b_ok ? gate : 0) * n_h + cb * FUS_CH + chn;
        const uint4 *b_ptr = reinterpret_cast<const uint4 *>(Wp) + ((size_t)(col >> 5) * KG + kh) * 32 + (col & 31);
        f32x16_t acc[NRB][1];
        zero_acc<NRB, 1>(acc);
        constexpr int KS = FUS_KC / 16;
        uint4 ga[3][NRB][4], fb[3][KS];
        auto load = [&](int kc, int buf) {
            const int k0 = kc * FUS_KC;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                fb[buf][ks] = b_ok ? b_ptr[(size_t)((k0 >> 3) + ks * 2) * 32] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < NRB; ++i)
#pragma unroll
                for (int sb = 0; sb < 4; ++sb)
                    ga[buf][i][sb] =
                        a_ok[i][sb] ? *reinterpret_cast<const uint4 *>(a_ptr[i][sb] + k0) : make_uint4(0, 0, 0, 0);
        };
        auto compute = [&](int buf) {
#pragma unroll
            for (int i = 0; i < NRB; ++i)
#pragma unroll
                for (int sb = 0; sb < 4; ++sb)
                    *reinterpret_cast<uint4 *>(stage + (i * 32 + sb * 8 + lrow) * LDA + lpiece * 8) = ga[buf][i][sb];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int i = 0; i < NRB; ++i) {
                    const uint4 av = *reinterpret_cast<const uint4 *>(stage + (i * 32 + r) * LDA + ks * 16 + kh * 8);
                    acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, av),
                                                                        __builtin_bit_cast(bf16x8_t, fb[buf][ks]),
                                                                        acc[i][0], 0, 0, 0);
                }
        };
        const int nkc = K / FUS_KC;
        load(0, 0);
        if (nkc > 1) load(1, 1);
        for (int kc = 0; kc < nkc; kc += 3) {
            if (kc + 2 < nkc) load(kc + 2, 2);
            __builtin_amdgcn_sched_barrier(0);
            compute(0);
            if (kc + 1 < nkc) {
                if (kc + 3 < nkc) load(kc + 3, 0);
                __builtin_amdgcn_sched_barrier(0);
                compute(1);
            }
            if (kc + 2 < nkc) {
                if (kc + 4 < nkc) load(kc + 4, 1);
                __builtin_amdgcn_sched_barrier(0);
                compute(2);
            }
        }
        __syncthreads();           // the staging pieces alias the tile written next
#pragma unroll
        for (int i = 0; i < NRB; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = (w + 8 * i) * 32 + acc_row(v, lane);
                if (t < FUS_MAX_L) u_lds[t * FUS_LDU + r] = acc[i][0][v];
            }
    }
    __syncthreads();

    // ---- recurrence
    const float bf = b_f ? b_f[j] : 0.f, br = b_r ? b_r[j] : 0.f;
    float a = 1.f, c = 0.f;
#pragma unroll
    for (int i = 0; i < FUS_CL; ++i)
        if (t0 + i < t1) {
            float *ut = u_lds + (t0 + i) * FUS_LDU;
            const float f = sigmoidf_(ut[FUS_CH + ch] + bf);
            ut[FUS_CH + ch] = f;                           // the gate itself from here on
            a *= f;
            c = f * c + (1.f - f) * ut[ch];
        }
    // inclusive doubling scan of the chunk maps c -> a c + b over the chunks of a channel
    int cur = 0;
#pragma unroll
    for (int o = 1; o < FUS_CHUNKS; o <<= 1) {
        car_a[cur][q][ch] = a;
        car_b[cur][q][ch] = c;
        __syncthreads();
        if (q >= o) {
            const float qa = car_a[cur][q - o][ch], qb = car_b[cur][q - o][ch];
            c = a * qb + c;                                // (this) after (earlier)
            a = a * qa;
        }
        cur ^= 1;
    }
    car_b[cur][q][ch] = c;                                 // state after chunks 0..q, starting from 0
    __syncthreads();
    c = q > 0 ? car_b[cur][q - 1][ch] : 0.f;

    bf16_t *ho = h_out + (size_t)b * L * n_h + j;
#pragma unroll
    for (int i = 0; i < FUS_CL; ++i)
        if (t0 + i < t1) {
            const float *ut = u_lds + (t0 + i) * FUS_LDU;
            const float f = ut[FUS_CH + ch];
            const float r = sigmoidf_(ut[2 * FUS_CH + ch] + br);
            c = f * c + (1.f - f) * ut[ch];
            const float hw = kgates == 4 ? ut[3 * FUS_CH + ch] : hwv[i];
            ho[(size_t)(t0 + i) * n_h] = f32_to_bf16(r * tanhf_(c) + (1.f - r) * hw);
        }
}

struct SruWs {
    size_t u, h0, h1, wp, rws, prob, ht, total;
};

static SruWs sru_ws_layout(const sru_weights *w, int B, int L)
{
    SruWs s;
    size_t T = (size_t)B * L;
    if (T == 0) T = 1;
    int wide = w->n_in > w->n_hidden ? w->n_in : w->n_hidden;
    size_t off = 0;
    s.u = off;
    off += align_up(T * 4 * (size_t)w->n_hidden * sizeof(float), 256);
    s.h0 = off;
    off += align_up(T * (size_t)w->n_hidden * 2, 256);
    s.h1 = off;
    off += align_up(T * (size_t)w->n_hidden * 2, 256);
    s.wp = off;
    off += align_up((size_t)wide * 4 * w->n_hidden * 2, 256);
    s.rws = off;
    off += route_ws_bytes(w->n_hidden, w->n_out, MOE_BF16);
    s.prob = off;
    off += align_up(T * sizeof(float), 256);
    s.ht = off;
    if (w->attention) off += sru_attention_ws_bytes(B, L, w->n_hidden);
    s.total = off;
    return s;
}

static int sru_check(const sru_weights *w, int B, int L, int dtype)
{
    MOE_REQUIRE(w, MOE_ERR_INVALID_ARG, "sru_predict: null weights");
    MOE_REQUIRE(B >= 0 && L > 0 && w->n_layers > 0 && w->n_in > 0 && w->n_hidden > 0 && w->n_out > 0,
                MOE_ERR_INVALID_ARG, "sru_predict: B=%d L=%d layers=%d n_in=%d n_hidden=%d n_out=%d out of range", B, L,
                w->n_layers, w->n_in, w->n_hidden, w->n_out);
    MOE_REQUIRE((long long)B * L <= 0x7fffffffLL / 4096, MOE_ERR_UNSUPPORTED, "sru_predict: B*L too large");
    MOE_REQUIRE(dtype == MOE_BF16, MOE_ERR_UNSUPPORTED, "sru_predict: only MOE_BF16 is built");
    MOE_REQUIRE(w->n_in % 64 == 0 && w->n_hidden % 128 == 0, MOE_ERR_UNSUPPORTED,
                "sru_predict: n_in=%d must be a multiple of 64 and n_hidden=%d of 128", w->n_in, w->n_hidden);
    MOE_REQUIRE(w->n_out <= MOE_MAX_EXPERTS && w->n_out % 8 == 0, MOE_ERR_UNSUPPORTED,
                "sru_predict: n_out=%d must be a multiple of 8 and at most %d", w->n_out, MOE_MAX_EXPERTS);
    MOE_REQUIRE(B <= 65535, MOE_ERR_UNSUPPORTED, "sru_predict: B=%d exceeds 65535", B);
    MOE_REQUIRE(w->w_layout == MOE_LAYOUT_PLAIN || w->w_layout == MOE_LAYOUT_PACKED, MOE_ERR_INVALID_ARG,
                "sru_predict: unknown weight layout %d", w->w_layout);
    MOE_REQUIRE(w->attention == 0 || w->attention == 1, MOE_ERR_INVALID_ARG, "sru_predict: attention must be 0 or 1");
    MOE_REQUIRE(!w->attention || (L <= 1024 && w->n_hidden <= 256), MOE_ERR_UNSUPPORTED,
                "sru_predict: sparsemax attention needs L <= 1024 and n_hidden <= 256 (L=%d n_hidden=%d)", L,
                w->n_hidden);
    MOE_REQUIRE(w->w_layout == MOE_LAYOUT_PLAIN ||
                    ((w->n_out == 128 || w->n_out == 256) && w->n_hidden % 128 == 0),
                MOE_ERR_UNSUPPORTED, "sru_predict: packed weights need n_out = 128 or 256");
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" size_t sru_predict_workspace_bytes(const sru_weights *w, int B, int L, int dtype)
{
    if (sru_check(w, B, L, dtype) != MOE_OK) return 0;
    return sru_ws_layout(w, B, L).total;
}

extern "C" int sru_predict(const void *emb, const sru_weights *w, int B, int L, int dtype, int32_t *pred_idx,
                           float *logits_opt, void *ws, size_t ws_bytes, void *stream)
{
    int rc = sru_check(w, B, L, dtype);
    if (rc != MOE_OK) return rc;
    MOE_REQUIRE(w->w_cat && w->w_head, MOE_ERR_INVALID_ARG, "sru_predict: null weight table");
    for (int l = 0; l < w->n_layers; ++l)
        MOE_REQUIRE(w->w_cat[l] && aligned16(w->w_cat[l]), MOE_ERR_INVALID_ARG,
                    "sru_predict: w_cat[%d] null or misaligned", l);
    if (B == 0) return MOE_OK;
    MOE_REQUIRE(emb && pred_idx && aligned16(emb), MOE_ERR_INVALID_ARG, "sru_predict: null or misaligned pointer");
    SruWs lay = sru_ws_layout(w, B, L);
    MOE_REQUIRE(ws && aligned16(ws) && ws_bytes >= lay.total, MOE_ERR_WORKSPACE,
                "sru_predict: workspace of %zu bytes needed, %zu given", lay.total, ws_bytes);
    hipStream_t st = (hipStream_t)stream;
    char *base = (char *)ws;
    float *U = (float *)(base + lay.u);
    bf16_t *hbuf[2] = {(bf16_t *)(base + lay.h0), (bf16_t *)(base + lay.h1)};
    void *wp = base + lay.wp;
    const int T = B * L, n_h = w->n_hidden;
    // a packed head is only usable by the matrix-core head kernel; otherwise the head stays plain
    const int head_layout = w->w_layout;
    const bf16_t *cur = (const bf16_t *)emb;
    int nin = w->n_in;
    for (int l = 0; l < w->n_layers; ++l) {
        int k = nin == n_h ? 3 : 4;
        int ncol = k * n_h;
        const void *wl = w->w_cat[l];
        if (w->w_layout == MOE_LAYOUT_PLAIN) {
            rc = pack_matrix_launch(w->w_cat[l], nin, ncol, wp, st, "sru_predict/pack");
            if (rc != MOE_OK) return rc;
            wl = wp;
        }
        bf16_t *out = hbuf[l & 1];
        if (L <= FUS_MAX_L) {
            // the whole layer in one kernel
            auto fused = L <= 256 ? sru_layer_fused_kernel<1> : sru_layer_fused_kernel<2>;
            hipLaunchKernelGGL(fused, dim3((n_h / FUS_CH) * B), dim3(FUS_THREADS), 0, st, cur, (const bf16_t *)wl, L, nin, n_h, k,
                               w->b_f ? w->b_f[l] : nullptr, w->b_r ? w->b_r[l] : nullptr, out);
            MOE_CHECK_LAUNCH("sru_predict/layer");
            cur = out;
            nin = n_h;
            continue;
        }
        hipLaunchKernelGGL(sru_proj_kernel, dim3(ceil_div(T, 64) * (ncol / 128)), dim3(GEMM_THREADS), 0, st, cur,
                           (const bf16_t *)wl, T, nin, ncol, U);
        MOE_CHECK_LAUNCH("sru_predict/proj");
        const int chunk_len = ceil_div(L, SRU_CHUNKS);
        auto scan = chunk_len <= 8 ? sru_scan_kernel<8> : chunk_len <= 16 ? sru_scan_kernel<16> : sru_scan_kernel<0>;
        hipLaunchKernelGGL(scan, dim3(n_h / SRU_CHANNELS, B), dim3(SRU_CHUNKS * SRU_CHANNELS), 0, st, U, cur, L,
                           n_h, k,
                           w->b_f ? w->b_f[l] : nullptr, w->b_r ? w->b_r[l] : nullptr, out);
        MOE_CHECK_LAUNCH("sru_predict/scan");
        cur = out;
        nin = n_h;
    }
    if (w->attention) {
        bf16_t *zbuf = hbuf[w->n_layers & 1];      // the buffer the last layer did not write
        rc = sru_attention_launch(cur, B, L, n_h, zbuf, base + lay.ht, st, "sru_predict/attention");
        if (rc != MOE_OK) return rc;
        cur = zbuf;
    }
    return route_launch(cur, w->w_head, head_layout, w->b_head, T, n_h, w->n_out, MOE_BF16, 1, 0, pred_idx, (float *)(base + lay.prob),
                        logits_opt, base + lay.rws, st, "sru_predict/head");
}
