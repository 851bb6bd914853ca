// Router for large batches (bf16, E = 256): the packed router matrix stays in registers.
//
// At 16384 tokens and more the router is bound by what each workgroup re-reads: the tile kernel in
// route.hip fetches the whole packed router matrix (d x 256 bf16 = 393 KB at d = 768) from L2 for every
// 32- or 64-token tile, four bytes of it for every byte of tokens.  Here a workgroup is persistent: its four
// wavefronts (one per SIMD, 512 registers each) load the matrix ONCE -- wavefront w keeps the two 32-column
// strips 2w, 2w+1 for all of K, d/2 registers per lane, each piece already the matrix-core B fragment of
// the packed image -- and then walks token tiles of 32 rows.  Only the tokens stream: HBM -> LDS by direct
// global->LDS loads into a ring of NS stages of 32 rows x 256 k (16 KB), four loads of 1 KB per wavefront
// and stage, running NS-1 stages (6 stages = 96 KB per CU) ahead of the matrix instructions, which is what
// it takes to keep HBM busy from 256 CUs.  Fragment reads are inline assembly with counted waits: the
// compiler cannot tell which LDS bytes an in-flight global->LDS load will write and would wait for all of
// them before any LDS access it can see (the epilogue's LDS accesses are assembly for the same reason).
//
// LDS layout of a stage: unit (row group rg of 16 rows, k block kb of 32) is the 1 KB one wavefront-wide
// load writes, at byte (kb*2 + rg)*1024; inside it row r's k-group g (8 k) is piece 4r + (g ^ (r>>2) ^ (r&3)),
// which spreads the 16 lanes the LDS serves per clock over all banks when a 32 x 16 fragment is read.
//
// Epilogue: the tile's 32 x 256 logits (+ bias) go through an LDS tile; 8 threads per row reduce them (row
// maximum, then in a second pass the sum of exponentials and the first index that holds the maximum), top-k
// by repeated selection.  One wavefront per SIMD has nobody to hide that arithmetic behind, and a wavefront-
// wide vector instruction occupies the issue port for 4 clocks (16 for an exponential), so done between two
// products it costs more than the product itself.  With top-1 routing at d = 768 the epilogue of tile i is
// therefore cut into pieces of a few instructions that are issued between the matrix instructions of tile
// i + 1 (each holds the matrix pipe for 32 clocks and the issue port for 4); the LDS reads of a piece are
// counted into the fragment reads' in-order waits.
#pragma once
#include "gemm_dense_bf16.h"
#include <utility>

namespace moe {

constexpr int RR_E = 256, RR_BM = 32, RR_BKS = 256, RR_NS = 7;
constexpr int RR_MIN_T = 16384;      // below this the tile kernel's many small workgroups win
constexpr int RR_STAGE_BYTES = RR_BM * RR_BKS * 2;
constexpr int RR_LDL = RR_E + 32;      // rows 32 banks apart: two rows x 8 threads x 16 bytes cover all 64 banks
constexpr int RR_LDS_BYTES = RR_NS * RR_STAGE_BYTES + 32 * RR_LDL * 4;

__device__ __forceinline__ void rr_argmax_merge(float &v, int &i, float ov, int oi)
{
    if (ov > v || (ov == v && oi < i)) {
        v = ov;
        i = oi;
    }
}

// LDS accesses with the offset as an immediate: one address register for all of them (a computed address
// per access is loop invariant, and the compiler keeps every one of them in a register across the tiles)
template <int OFF>
__device__ __forceinline__ void rr_ds_write32(unsigned addr, float val)
{
    asm volatile("ds_write_b32 %0, %1 offset:%2" ::"v"(addr), "v"(val), "n"(OFF) : "memory");
}
template <int OFF>
__device__ __forceinline__ void rr_ds_read32(float &dst, unsigned addr)
{
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
template <int OFF>
__device__ __forceinline__ void rr_ds_read128(u32x4_t &dst, unsigned addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
#define RR_LGKM0() asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory")

// value of the partner lane in three exchange steps that together connect the 8 lanes of a group (lanes
// 8g .. 8g+7): lane ^ 1, lane ^ 2 inside quads, then the mirror image inside the half row (lane 7 - i of the
// group, which lies in the other quad).  Data-parallel-primitive moves: no LDS round trip.
template <int STEP>
__device__ __forceinline__ int rr_dpp8(int x)
{
    if (STEP == 0) return __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xf, 0xf, false);
    if (STEP == 1) return __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xf, 0xf, false);
    return __builtin_amdgcn_update_dpp(0, x, 0x141, 0xf, 0xf, false);
}
__device__ __forceinline__ void rr_argmax_over8(float &v, int &i)
{
#define RR_AM(S)                                                                  \
    {                                                                             \
        const float ov = __builtin_bit_cast(float, rr_dpp8<S>(__builtin_bit_cast(int, v))); \
        const int oi = rr_dpp8<S>(i);                                             \
        rr_argmax_merge(v, i, ov, oi);                                            \
    }
    RR_AM(0) RR_AM(1) RR_AM(2)
#undef RR_AM
}
__device__ __forceinline__ float rr_sum_over8(float v)
{
    v += __builtin_bit_cast(float, rr_dpp8<0>(__builtin_bit_cast(int, v)));
    v += __builtin_bit_cast(float, rr_dpp8<1>(__builtin_bit_cast(int, v)));
    v += __builtin_bit_cast(float, rr_dpp8<2>(__builtin_bit_cast(int, v)));
    return v;
}

template <class F, int... I>
__device__ __forceinline__ void rr_static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void rr_static_for(F &&f)
{
    rr_static_for_impl(f, std::make_integer_sequence<int, N>{});
}

constexpr int RR_B_IN_ACC = 56;        // pieces of the resident matrix kept in accumulation registers (4 each)
constexpr float RR_LOG2E = 1.4426950408889634f;

// 16-deep steps after whose second matrix instruction the overlapped epilogue issues its LDS reads (2 of 16
// bytes per slot); the step after such a slot must allow those 2 reads to be outstanding on top of its own
// two fragment reads.  Pass 1 (row maximum): chunks at steps 0, 2, 4, 6; pass 2 (sum, index): 10, 16, 22, 28.
__host__ __device__ constexpr bool rr_read_slot(int s)
{
    return s == 0 || s == 2 || s == 4 || s == 6 || s == 10 || s == 16 || s == 22 || s == 28;
}

// KSTEPS = d / 16 (a multiple of 16).  TOPK: the call wants more than one choice per token (extra selection
// passes, epilogue not overlapped).  Grid: any number of workgroups; workgroup g takes tiles g, g + grid, ...
template <int KSTEPS, bool TOPK>
__global__ __launch_bounds__(GEMM_THREADS, 1) void route_resident_kernel(
    const bf16_t *__restrict__ x, const bf16_t *__restrict__ wr_packed, const float *__restrict__ bias, int T,
    int top_k, int renormalize, int32_t *__restrict__ idx, float *__restrict__ prob, float *__restrict__ logits_opt)
{
    constexpr int D = KSTEPS * 16, NST = D / RR_BKS, NS = RR_NS, KG = D / 8, LDL = RR_LDL;
    constexpr bool OVERLAP = !TOPK && KSTEPS >= 36;     // the schedule of pieces below needs 36 steps per tile
    static_assert(KSTEPS % 16 == 0, "d must be a multiple of 256");
    static_assert(D / RR_BKS + 1 <= RR_NS - 2, "the first tile's stages must all be among the prologue's");
    __shared__ __attribute__((aligned(16))) char smem[RR_LDS_BYTES];
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_tiles = (T + RR_BM - 1) / RR_BM;
    const int first = blockIdx.x, step = gridDim.x;
    if (first >= n_tiles) return;
    const int n_my = (n_tiles - first + step - 1) / step;
    const int G = n_my * NST;                       // stages this workgroup walks

    // ---- token stream.  Wavefront w loads, per stage, row group w & 1 (16 rows) x k blocks 4*(w>>1) .. +3:
    // 256 contiguous bytes of each of its rows; this lane fetches row ld_r, k-group ld_kg of each block.
    const int ld_r = lane >> 2, ld_kg = (lane & 3) ^ (ld_r >> 2) ^ (ld_r & 3);
    int is_tile = 0, is_st = 0, is_buf = 0, is_g = 0;      // cursor of the next stage to issue
    auto row_ptr = [&](int tile_no) {
        int row = (first + tile_no * step) * RR_BM + (w & 1) * 16 + ld_r;
        row = row < T ? row : T - 1;                       // rows past the batch re-read its last row
        return x + (size_t)row * D + (w >> 1) * 128 + ld_kg * 8;
    };
    const bf16_t *is_src = row_ptr(0);
    auto issue = [&]() {
        // past the last stage: a harmless re-read of the last one keeps the counted waits uniform
        const bf16_t *src = is_src + is_st * RR_BKS;
        char *dst = smem + is_buf * RR_STAGE_BYTES + ((w >> 1) * 8 + (w & 1)) * 1024;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            __builtin_amdgcn_global_load_lds((glb_void_t *)(src + j * 32), (lds_void_t *)(dst + j * 2048), 16, 0, 0);
        is_buf = is_buf + 1 == NS ? 0 : is_buf + 1;
        if (++is_g < G) {
            if (++is_st == NST) {
                is_st = 0;
                is_src = row_ptr(++is_tile);
            }
        }
    };

    // the first stages of the token stream go out before the matrix loads, so that they are under way while
    // the 393 KB of the matrix arrive
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue();
    asm volatile("" ::: "memory");      // the loads below stay below (the first tile's wait counts on that order)
    MOE_SB();
    // ---- the router matrix, resident: strips 2w, 2w+1, all of K
    u32x4_t b[KSTEPS][2];
    {
        const u32x4_t *b_base = reinterpret_cast<const u32x4_t *>(wr_packed) + (size_t)(w * 2) * KG * 32 + lane;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) b[ks][nb] = b_base[((size_t)nb * KG + ks * 2) * 32];
    }
    // No wait here: the first tile's matrix instructions start as the pieces arrive (the compiler waits for
    // each piece before its first use; vector memory loads return in order).

    float bia[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) bia[nb] = bias ? bias[(w * 2 + nb) * 32 + (lane & 31)] : 0.f;

    const unsigned lds0 = (unsigned)(unsigned long)(lds_void_t *)smem;
    const int r16 = lane & 15, sw = (r16 >> 2) ^ (r16 & 3);
    unsigned a_addr[2];                 // fragment piece of this lane in stage buffer 0, even / odd 16-deep step
#pragma unroll
    for (int o = 0; o < 2; ++o)
        a_addr[o] = lds0 + 16u * ((((lane & 31) >> 4)) * 64 + r16 * 4 + ((2 * o + (lane >> 5)) ^ sw));
    const unsigned tile0 = lds0 + NS * RR_STAGE_BYTES;
    // epilogue addresses: accumulator register v of block nb holds row acc_row(v, lane), column (2w+nb)*32 + lane%32
    const unsigned wr_base = tile0 + 4u * ((4 * (lane >> 5)) * LDL + w * 64 + (lane & 31));
    const int er = tid >> 3, sub = tid & 7;
    const unsigned rd_base = tile0 + 4u * (er * LDL + 4 * sub);

    // ---- epilogue pieces.  Thread (er, sub) owns the 32 logits of row er at columns 4*sub + 32g + t (g < 8,
    // t < 4), read 8 at a time as two 16-byte pieces (chunk c: g = 2c, 2c + 1; lv[4u + t] = column
    // 4*sub + 64c + 32u + t).  State of the tile whose logits are in the LDS tile:
    u32x4_t lq0, lq1;                   // the chunk's 8 logits as they arrive from LDS
    float e_max = 0.f, e_msc = 0.f, e_z = 0.f;
    int e_bi = 0, e_row = 0;
    bool e_live = false;
    auto ep_col = [&](int c, int j) { return 4 * sub + 64 * c + 32 * (j >> 2) + (j & 3); };
    auto ep_read = [&](auto C) {
        constexpr int c = decltype(C)::value;
        rr_ds_read128<256 * c>(lq0, rd_base);
        rr_ds_read128<256 * c + 128>(lq1, rd_base);
    };
    auto lvf = [&](int j) { return __builtin_bit_cast(float, j < 4 ? lq0[j & 3] : lq1[j & 3]); };
    // the values requested by ep_read may be used from here on (the caller has waited for them)
    auto ep_arrived = [&]() {
        asm volatile("" : "+v"(lq0), "+v"(lq1));
    };
    auto ep_wait = [&]() {
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(lq0), "+v"(lq1));
    };
    auto ep_max = [&](auto C) {          // pass 1: running row maximum (and the logits themselves, if asked for)
        constexpr int c = decltype(C)::value;
        const float m0 = fmaxf(fmaxf(lvf(0), lvf(1)), fmaxf(lvf(2), lvf(3)));
        const float m1 = fmaxf(fmaxf(lvf(4), lvf(5)), fmaxf(lvf(6), lvf(7)));
        e_max = c == 0 ? fmaxf(m0, m1) : fmaxf(e_max, fmaxf(m0, m1));
        if (logits_opt && e_live) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
                *reinterpret_cast<float4 *>(logits_opt + (size_t)e_row * RR_E + ep_col(c, 4 * u)) =
                    make_float4(lvf(4 * u), lvf(4 * u + 1), lvf(4 * u + 2), lvf(4 * u + 3));
        }
    };
    auto ep_mid = [&]() {                // the row maximum over the 8 threads of the row
#pragma unroll
        for (int stp = 0; stp < 3; ++stp) {
            const int o = stp == 0 ? rr_dpp8<0>(__builtin_bit_cast(int, e_max))
                          : stp == 1 ? rr_dpp8<1>(__builtin_bit_cast(int, e_max))
                                     : rr_dpp8<2>(__builtin_bit_cast(int, e_max));
            e_max = fmaxf(e_max, __builtin_bit_cast(float, o));
        }
        e_msc = e_max * RR_LOG2E;
        e_z = 0.f;
        e_bi = 0x3fffffff;
    };
    // pass 2, logit 7 - Q of chunk c (the 8 threads of a row take their columns in descending order over the
    // whole pass, so a thread's last match is its lowest column; the lowest of the 8 is taken in ep_end):
    // sum of exp(l - max) as exp2(l*log2e - max*log2e), and the index of a logit equal to the maximum
    auto ep_sum = [&](auto C, auto Q) {
        constexpr int c = decltype(C)::value, j = 7 - decltype(Q)::value;
        e_z += __builtin_amdgcn_exp2f(fmaf(lvf(j), RR_LOG2E, -e_msc));
        e_bi = lvf(j) == e_max ? 64 * c + 32 * (j >> 2) + (j & 3) : e_bi;      // the column without its 4*sub
    };
    auto ep_end = [&]() {
        e_z = rr_sum_over8(e_z);
        e_bi += 4 * sub;
#pragma unroll
        for (int stp = 0; stp < 3; ++stp) {
            const int o = stp == 0 ? rr_dpp8<0>(e_bi) : stp == 1 ? rr_dpp8<1>(e_bi) : rr_dpp8<2>(e_bi);
            e_bi = o < e_bi ? o : e_bi;
        }
        if (sub == 0 && e_live) {
            idx[e_row] = e_bi;
            prob[e_row] = 1.f / e_z;
        }
    };
    // the whole epilogue in one go (not overlapped)
    auto ep_all = [&]() {
        rr_static_for<4>([&](auto C) {
            ep_read(C);
            ep_wait();
            ep_max(C);
        });
        ep_mid();
        rr_static_for<4>([&](auto CC) {
            std::integral_constant<int, 3 - decltype(CC)::value> C;
            ep_read(C);
            ep_wait();
            rr_static_for<8>([&](auto Q) { ep_sum(C, Q); });
        });
        ep_end();
        if constexpr (TOPK) {
            // choice j: the largest logit after choice j-1 in the order (logit descending, id ascending)
            float pv = e_max, wsum = 1.f / e_z;
            int pi = e_bi;
            for (int j = 1; j < top_k; ++j) {
                float v = -INFINITY;
                int vi = 0x7fffffff;
                rr_static_for<4>([&](auto C) {
                    constexpr int c = decltype(C)::value;
                    ep_read(C);
                    ep_wait();
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        const float t = lvf(q);
                        const int col = ep_col(c, q);
                        if (t < pv || (t == pv && col > pi)) rr_argmax_merge(v, vi, t, col);
                    }
                });
                rr_argmax_over8(v, vi);
                const float cw = __builtin_amdgcn_exp2f(fmaf(v, RR_LOG2E, -e_msc)) / e_z;
                wsum += cw;
                if (sub == 0 && e_live) {
                    idx[(size_t)j * T + e_row] = vi;
                    prob[(size_t)j * T + e_row] = cw;
                }
                pv = v;
                pi = vi;
            }
            if (renormalize && sub == 0 && e_live) {
                // the weights written above divided by their sum (this thread reads back what it wrote itself)
                for (int j = 0; j < top_k; ++j) prob[(size_t)j * T + e_row] = prob[(size_t)j * T + e_row] / wsum;
            }
        }
    };
    // The piece that follows matrix instruction H (0, 1) of 16-deep step S of the next tile's product: at most
    // about 28 clocks of issue each, the time the instruction before it keeps the matrix pipe busy.  Reads are
    // issued after the second instruction of the steps rr_read_slot() names and are usable two steps later.
    auto ep_slot = [&](auto SS, auto HH) {
        constexpr int S = decltype(SS)::value, H = decltype(HH)::value, M = 2 * S + H;
        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        using I2 = std::integral_constant<int, 2>;
        using I3 = std::integral_constant<int, 3>;
        if constexpr (M == 1) ep_read(I0{});
        if constexpr (M == 5) { ep_arrived(); ep_max(I0{}); ep_read(I1{}); }
        if constexpr (M == 9) { ep_arrived(); ep_max(I1{}); ep_read(I2{}); }
        if constexpr (M == 13) { ep_arrived(); ep_max(I2{}); ep_read(I3{}); }
        if constexpr (M == 17) { ep_arrived(); ep_max(I3{}); }
        if constexpr (M == 19) ep_mid();
        if constexpr (S >= 10 && S < 34) {
            // chunk 3 - cc: read after step 10 + 6cc, its 8 logits after the 8 matrix instructions from the
            // second of step 12 + 6cc on
            constexpr int cc = (S - 10) / 6, r = 2 * ((S - 10) % 6) + H;     // r = 0 .. 11 inside the chunk's 6 steps
            std::integral_constant<int, 3 - cc> C;
            if constexpr (r == 1) ep_read(C);
            if constexpr (r == 5) ep_arrived();
            if constexpr (r >= 5 && r < 12) ep_sum(C, std::integral_constant<int, r - 5>{});
        }
        if constexpr (S >= 16 && S < 40 && (S - 10) % 6 == 0 && H == 0) {
            // the eighth logit of the previous chunk, just before the next chunk's read replaces it
            constexpr int cc = (S - 16) / 6;
            ep_sum(std::integral_constant<int, 3 - cc>{}, std::integral_constant<int, 7>{});
        }
        if constexpr (M == 2 * 34 + 1) ep_end();
        MOE_SB();
    };

    int buf = 0;
    u32x4_t f0, f1, f2, f3;             // token fragments of four consecutive 16-deep steps (three reads in flight)
    f32x16_t acc[1][2];
// The matrix instruction as assembly, so that the resident piece is named where it lives: through the
// builtin, the register allocator treats accumulation registers as spill space and moves every piece into an
// ordinary register before its use (4 moves + wait states per matrix instruction, on the issue port that the
// overlapped epilogue needs).  Piece p = 2*step + block sits in accumulation registers when p < RR_B_IN_ACC,
// else in ordinary ones.  The first step of a tile takes a zero accumulator as an immediate.  What the
// compiler cannot see through the assembly is handled by hand: between two uses of one accumulator lies the
// other accumulator's instruction (32 clocks, the result is complete), and rr_after_product() covers the
// wait states before ordinary instructions may read the results.
#define RR_MF(f, nb, KS)                                                                                           \
    {                                                                                                              \
        constexpr int p_ = 2 * (KS) + nb;                                                                          \
        if constexpr ((KS) == 0) {                                                                                 \
            if constexpr (p_ < RR_B_IN_ACC)                                                                        \
                asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=a"(acc[0][nb]) : "v"(f), "a"(b[KS][nb])); \
            else                                                                                                   \
                asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=a"(acc[0][nb]) : "v"(f), "v"(b[KS][nb])); \
        } else {                                                                                                   \
            if constexpr (p_ < RR_B_IN_ACC)                                                                        \
                asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[0][nb]) : "v"(f), "a"(b[KS][nb])); \
            else                                                                                                   \
                asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc[0][nb]) : "v"(f), "v"(b[KS][nb])); \
        }                                                                                                          \
    }
// One 16-deep step out of `cur`; the fragment three steps on is requested into `far` (the register of the
// step before this one, free again), and `nxt`, requested two steps ago, must have arrived: LDS reads return
// in order, so "at most two outstanding" means exactly that -- four when the epilogue piece after the
// previous step has put 2 reads of its own behind them.
#define RR_STEP(cur, nxt, far, SI, faddr, off)                                                                     \
    {                                                                                                              \
        constexpr int s_ = st * 16 + SI;                                                                           \
        RR_MF(cur, 0, s_); MOE_DS_READ128(far, faddr, off); MOE_SB();                                              \
        if constexpr (EPI) ep_slot(std::integral_constant<int, s_>{}, std::integral_constant<int, 0>{});           \
        RR_MF(cur, 1, s_); MOE_SB();                                                                               \
        asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(nxt) : "n"((EPI && s_ > 0 && rr_read_slot(s_ - 1)) ? 4 : 2)); \
        if constexpr (EPI) ep_slot(std::integral_constant<int, s_>{}, std::integral_constant<int, 1>{});           \
    }
    // the product of one tile; EPI: the epilogue of the previous tile rides along
    auto product = [&](auto EPI_, bool very_first) {
        constexpr bool EPI = decltype(EPI_)::value;
        rr_static_for<NST>([&](auto ST) {
            constexpr int st = decltype(ST)::value;
            // Stages up to the one after this have landed: issued so far are the stages up to g + NS - 2, so
            // at most NS - 3 stages (4 loads each) may still be outstanding.  The barrier makes that true for
            // all four wavefronts and tells that everyone is done with the previous stage, whose buffer the
            // load issued next refills.
            // The very first tile differs: its NS - 1 stages went out BEFORE the 2 * KSTEPS loads of the matrix
            // (and the two of the bias), so "at most 2 * KSTEPS outstanding" (63 is the counter's range) already
            // says that all of them have landed, and its later stages need no wait of their own.
            if (very_first) {
                if (st == 0) MOE_VMCNT(2 * KSTEPS < 63 ? 2 * KSTEPS : 63);
            } else {
                MOE_VMCNT(4 * (NS - 3));
            }
            __builtin_amdgcn_s_barrier();
            MOE_SB();
            issue();
            MOE_SB();
            const unsigned ae = a_addr[0] + buf * RR_STAGE_BYTES, ao = a_addr[1] + buf * RR_STAGE_BYTES;
            const int nbuf = buf + 1 == NS ? 0 : buf + 1;
            const unsigned ne = a_addr[0] + nbuf * RR_STAGE_BYTES, no = a_addr[1] + nbuf * RR_STAGE_BYTES;
            if (st == 0 && very_first) {    // nothing was prefetched
                MOE_DS_READ128(f0, ae, 0);
                MOE_DS_READ128(f1, ao, 0);
                MOE_DS_READ128(f2, ae, 2048);
                asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(f0));
            }
            // step s reads out of f(s % 4) and requests step s + 3 into f((s + 3) % 4)
            RR_STEP(f0, f1, f3, 0, ao, 2048);
            RR_STEP(f1, f2, f0, 1, ae, 4096);
            RR_STEP(f2, f3, f1, 2, ao, 4096);
            RR_STEP(f3, f0, f2, 3, ae, 6144);
            RR_STEP(f0, f1, f3, 4, ao, 6144);
            RR_STEP(f1, f2, f0, 5, ae, 8192);
            RR_STEP(f2, f3, f1, 6, ao, 8192);
            RR_STEP(f3, f0, f2, 7, ae, 10240);
            RR_STEP(f0, f1, f3, 8, ao, 10240);
            RR_STEP(f1, f2, f0, 9, ae, 12288);
            RR_STEP(f2, f3, f1, 10, ao, 12288);
            RR_STEP(f3, f0, f2, 11, ae, 14336);
            RR_STEP(f0, f1, f3, 12, ao, 14336);
            // the first three fragments of the next stage (landed, see above)
            RR_STEP(f1, f2, f0, 13, ne, 0);
            RR_STEP(f2, f3, f1, 14, no, 0);
            RR_STEP(f3, f0, f2, 15, ne, 2048);
            buf = nbuf;
        });
        // the three fragment reads still in flight belong to the next tile (or to nobody after the last one);
        // they have to land before the LDS waits of what follows count anything
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f0), "+v"(f1), "+v"(f2));
        // wait states between the last matrix instructions and ordinary reads of their results (the compiler
        // inserts them for its own matrix instructions; it does not look into assembly)
        asm volatile("s_nop 15\n\ts_nop 15" : "+a"(acc[0][0]), "+a"(acc[0][1]));
    };

    for (int i = 0; i < n_my; ++i) {
        const int row0 = (first + i * step) * RR_BM;
        const int nrows = T - row0 < RR_BM ? T - row0 : RR_BM;
        if (OVERLAP && i > 0) product(std::true_type{}, false);
        else product(std::false_type{}, i == 0);
        // every wavefront is done reading the previous tile's logits
        __builtin_amdgcn_s_barrier();
        MOE_SB();
        rr_static_for<32>([&](auto I) {
            constexpr int nb = decltype(I)::value >> 4, v = decltype(I)::value & 15;
            rr_ds_write32<4 * ((8 * (v >> 2) + (v & 3)) * LDL + nb * 32)>(wr_base, acc[0][nb][v] + bia[nb]);
        });
        RR_LGKM0();
        e_row = row0 + er;
        e_live = er < nrows;
        if (!OVERLAP) {
            __builtin_amdgcn_s_barrier();
            MOE_SB();
            ep_all();
        }
        // (overlapped: the first barrier of the next product makes the logits visible to their readers)
    }
    if (OVERLAP) {
        __builtin_amdgcn_s_barrier();
        MOE_SB();
        ep_all();
    }
#undef RR_STEP
#undef RR_MF
    MOE_VMCNT(0);
}

}  // namespace moe
