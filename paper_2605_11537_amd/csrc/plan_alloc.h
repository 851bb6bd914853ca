// Pieces of replica_plan shared by its own kernels and by the fused small-batch front end:
// the ballot-aggregated LDS histogram of ids and the integer allocation run by one wavefront.
#pragma once
#include "common.h"

namespace moe {

constexpr int PLAN_THREADS = 1024;
constexpr int PLAN_BATCH = 8;  // ids fetched per thread before any of them is counted

// One lane of the row of 16 to another on the data-parallel-primitive path (no trip through LDS):
// lane ^ 1, lane ^ 2, the lane 4 further, the lane 8 further (rotations inside the row).
template <int STEP>
__device__ __forceinline__ int row_exchange(int x)
{
    if (STEP == 0) return __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xf, 0xf, false);
    if (STEP == 1) return __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xf, 0xf, false);
    if (STEP == 2) return __builtin_amdgcn_update_dpp(0, x, 0x124, 0xf, 0xf, false);
    return __builtin_amdgcn_update_dpp(0, x, 0x128, 0xf, 0xf, false);
}

template <int STEP>
__device__ __forceinline__ long long row_exchange_ll(long long v)
{
    const unsigned lo = (unsigned)row_exchange<STEP>((int)(unsigned)v);
    const unsigned hi = (unsigned)row_exchange<STEP>((int)(unsigned)((unsigned long long)v >> 32));
    return (long long)(((unsigned long long)hi << 32) | lo);
}

// sum over the wavefront (all 64 lanes active), result in every lane: rows of 16 folded by lane
// exchanges, the four row sums added as scalars
__device__ __forceinline__ long long wave_sum_ll(long long v)
{
    v += row_exchange_ll<0>(v);
    v += row_exchange_ll<1>(v);
    v += row_exchange_ll<2>(v);
    v += row_exchange_ll<3>(v);
    long long t = 0;
#pragma unroll
    for (int row = 0; row < 4; ++row) {
        const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, 16 * row);
        const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)((unsigned long long)v >> 32), 16 * row);
        t += (long long)(((unsigned long long)hi << 32) | lo);
    }
    return t;
}

constexpr int PLAN_BLOCK_TOKENS = PLAN_THREADS * PLAN_BATCH;   // ids per workgroup of the partial pass

// ballot-aggregated LDS histogram of ids [t_begin, t_end)
__device__ __forceinline__ void plan_histogram(const int32_t *__restrict__ idx, int t_begin, int t_end, int E,
                                               int nbits, int *hist)
{
    const int tid = threadIdx.x, lane = tid & 63;
    for (int t0 = t_begin; t0 < t_end; t0 += PLAN_THREADS * PLAN_BATCH) {
        int eb[PLAN_BATCH];
#pragma unroll
        for (int u = 0; u < PLAN_BATCH; ++u) {
            int t = t0 + u * PLAN_THREADS + tid;
            eb[u] = t < t_end ? idx[t] : -1;
        }
#pragma unroll
        for (int u = 0; u < PLAN_BATCH; ++u) {
            int e = eb[u];
            bool valid = e >= 0 && e < E;
            unsigned long long mask = __ballot(valid);
            if (mask == 0) continue;
            for (int b = 0; b < nbits; ++b) {
                bool bit = (e >> b) & 1;
                unsigned long long bal = __ballot(bit);
                mask &= bit ? bal : ~bal;
            }
            if (valid && (mask & ((1ull << lane) - 1ull)) == 0) atomicAdd(&hist[e], __popcll(mask));
        }
    }
}

// Load per slot n / r as a binary64 quotient.  The order of two such quotients is the exact order of the
// fractions: the division is correctly rounded, so equal fractions give equal quotients, and different
// ones differ by at least 1 / (r r') > ulp(n / r) as long as n r' < 2^52 (n < 2^31, r <= 2^13 here).
__device__ __forceinline__ double load_per_slot(int n, int r) { return (double)n / (double)r; }

// candidate (ok, oe) against the best so far: the larger load per slot wins, the lower expert id among
// equals; e < 0 = no candidate
__device__ __forceinline__ void most_loaded_merge(double &bk, int &be, double ok, int oe)
{
    if (oe >= 0 && (be < 0 || ok > bk || (ok == bk && oe < be))) {
        bk = ok;
        be = oe;
    }
}

template <int STEP>
__device__ __forceinline__ double row_exchange_f64(double v)
{
    return __builtin_bit_cast(double, row_exchange_ll<STEP>(__builtin_bit_cast(long long, v)));
}

// The allocation of Algorithm 1 with the budget cap, run by ONE wavefront entirely in registers (lane l
// owns experts l, l+64, ...; sums and arg-max searches are wavefront reductions, so the one-by-one
// hand-out of the slots left by the floors needs no barrier).  hist: counts per expert (LDS), n_ids: their
// sum at most.
// Writes rep[e] (LDS) and, with write_tables, the replicas / plan_counts tables.
template <int PLAN_PER_LANE>
__device__ __forceinline__ void plan_allocate_wave(const int *hist, int *rep, int n_ids, int E, int R, int C,
                                                   int policy, int32_t *__restrict__ replicas,
                                                   int32_t *__restrict__ plan_counts, bool write_tables = true)
{
    const int lane = threadIdx.x & 63;
    int n[PLAN_PER_LANE], r[PLAN_PER_LANE];
    long long want[PLAN_PER_LANE];
    long long dsum = 0;
#pragma unroll
    for (int i = 0; i < PLAN_PER_LANE; ++i) {
        int e = lane + i * WAVE;
        n[i] = e < E ? hist[e] : 0;
        // ceil(n / C) - 1 (n, C < 2^31: the sum fits 32 bits unsigned, a 64-bit division is a long routine)
        long long w = (long long)(((unsigned)n[i] + (unsigned)C - 1u) / (unsigned)C) - 1;
        want[i] = (e < E && w > 0) ? w : 0;
        r[i] = 1;
        dsum += want[i];
    }
    const long long D = wave_sum_ll(dsum);
    if (D <= (long long)R) {
#pragma unroll
        for (int i = 0; i < PLAN_PER_LANE; ++i) r[i] += (int)want[i];
    } else {
        long long left = R;
        if (policy == 0) {
            long long used = 0;
            const bool narrow = (unsigned long long)R * (unsigned long long)D < (1ull << 32);   // uniform
#pragma unroll
            for (int i = 0; i < PLAN_PER_LANE; ++i) {
                long long extra = narrow ? (long long)(((unsigned)R * (unsigned)want[i]) / (unsigned)D)
                                         : (long long)R * want[i] / D;
                r[i] += (int)extra;
                used += extra;
            }
            left -= wave_sum_ll(used);
        } else {
            for (;;) {
                long long nw = 0;
#pragma unroll
                for (int i = 0; i < PLAN_PER_LANE; ++i) nw += (long long)r[i] - 1 < want[i];
                nw = wave_sum_ll(nw);
                if (nw == 0) break;
                long long q = left / nw;
                if (q == 0) break;
                long long given = 0;
#pragma unroll
                for (int i = 0; i < PLAN_PER_LANE; ++i) {
                    long long unmet = want[i] - ((long long)r[i] - 1);
                    if (unmet > 0) {
                        long long g = q < unmet ? q : unmet;
                        r[i] += (int)g;
                        given += g;
                    }
                }
                left -= wave_sum_ll(given);
            }
        }
        // the slots still left go one at a time to the most loaded expert per slot.  A dependent chain of
        // up to R steps on one wavefront: rows of 16 lanes are folded by lane exchanges, the four rows as
        // scalars (shuffles routed through LDS and cross products made each step ~2000 cycles)
        if (n_ids < (1 << 24)) {
            // Counts below 2^24: load per slot and expert id in ONE 64-bit integer, so a fold step is an
            // unsigned maximum.  q = floor(RN(n 2^28 / r)) is monotone in n / r, equal for equal fractions,
            // and different fractions differ by 2^28 / (r r') >= 4 (r <= 2^13), so the order of the q is the
            // exact order of the fractions; the low 10 bits hold 1023 - id (lower id wins among equals);
            // 0 = no candidate (an open expert has n > C >= 1, so its q is positive).
            auto slot_key = [&](int i) -> unsigned long long {
                const bool open = (long long)r[i] - 1 < want[i];
                const unsigned long long q = (unsigned long long)((double)n[i] * 268435456.0 / (double)r[i]);
                return open ? (q << 10) | (unsigned long long)(1023 - (lane + i * WAVE)) : 0ull;
            };
            auto umax = [](unsigned long long a, unsigned long long b) { return a > b ? a : b; };
            unsigned long long key[PLAN_PER_LANE];
#pragma unroll
            for (int i = 0; i < PLAN_PER_LANE; ++i) key[i] = slot_key(i);
            while (left > 0) {
                unsigned long long bk = 0ull;
#pragma unroll
                for (int i = 0; i < PLAN_PER_LANE; ++i) bk = umax(bk, key[i]);
                bk = umax(bk, (unsigned long long)row_exchange_ll<0>((long long)bk));
                bk = umax(bk, (unsigned long long)row_exchange_ll<1>((long long)bk));
                bk = umax(bk, (unsigned long long)row_exchange_ll<2>((long long)bk));
                bk = umax(bk, (unsigned long long)row_exchange_ll<3>((long long)bk));
                unsigned long long sk = 0ull;
#pragma unroll
                for (int row = 0; row < 4; ++row) {
                    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)bk, 16 * row);
                    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(bk >> 32), 16 * row);
                    sk = umax(sk, ((unsigned long long)hi << 32) | lo);
                }
                if (sk == 0ull) break;
                const int be = 1023 - (int)(sk & 1023ull);
#pragma unroll
                for (int i = 0; i < PLAN_PER_LANE; ++i)
                    if (be == lane + i * WAVE) {
                        r[i] += 1;
                        key[i] = slot_key(i);
                    }
                left -= 1;
            }
        } else {
        double key[PLAN_PER_LANE];
#pragma unroll
        for (int i = 0; i < PLAN_PER_LANE; ++i) key[i] = load_per_slot(n[i], r[i]);
        while (left > 0) {
            double bk = 0.0;
            int be = -1;
#pragma unroll
            for (int i = 0; i < PLAN_PER_LANE; ++i) {
                const bool open = (long long)r[i] - 1 < want[i];
                most_loaded_merge(bk, be, key[i], open ? lane + i * WAVE : -1);   // ascending ids inside a lane
            }
            most_loaded_merge(bk, be, row_exchange_f64<0>(bk), row_exchange<0>(be));
            most_loaded_merge(bk, be, row_exchange_f64<1>(bk), row_exchange<1>(be));
            most_loaded_merge(bk, be, row_exchange_f64<2>(bk), row_exchange<2>(be));
            most_loaded_merge(bk, be, row_exchange_f64<3>(bk), row_exchange<3>(be));
            {
                const long long kb = __builtin_bit_cast(long long, bk);
                double sk = 0.0;
                int se = -1;
#pragma unroll
                for (int row = 0; row < 4; ++row) {
                    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)kb, 16 * row);
                    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)((unsigned long long)kb >> 32), 16 * row);
                    most_loaded_merge(sk, se, __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo),
                                      __builtin_amdgcn_readlane(be, 16 * row));
                }
                be = se;
            }
            if (be < 0) break;
#pragma unroll
            for (int i = 0; i < PLAN_PER_LANE; ++i)
                if (be == lane + i * WAVE) {
                    r[i] += 1;
                    key[i] = load_per_slot(n[i], r[i]);
                }
            left -= 1;
        }
        }
    }
#pragma unroll
    for (int i = 0; i < PLAN_PER_LANE; ++i) {
        int e = lane + i * WAVE;
        if (e < E) {
            rep[e] = r[i];
            if (write_tables) {
                replicas[e] = r[i];
                plan_counts[e] = n[i];
            }
        }
    }
}

}  // namespace moe
