// Measurement kernels (not part of the method): what this memory system and these matrix cores deliver to
// kernels shaped like the library's own, so that a roofline fraction can be quoted against a measured
// ceiling beside the nominal one.
//
//   moe_measure_stream_read   every workgroup streams its share of a buffer with 16-byte loads (plain or
//                             non-temporal), as the weight-streaming GEMM tiles do; nothing is stored
//                             but one word per workgroup.  With one workgroup per compute unit or fewer,
//                             each keeps 128 KB in flight (the rate of a unit's load path)
//   moe_measure_mfma_bf16     one workgroup of 4 wavefronts per CU, each wavefront 4 x 4 accumulator blocks
//                             (256 registers) of v_mfma_f32_32x32x16_bf16 -- the instruction mix of the
//                             256 x 256 tile kernel -- with operands that change every step, either held in
//                             registers or re-read from LDS as that kernel reads them; no global memory
//                             traffic inside the loop
#include "gemm_bf16.h"

namespace moe {

typedef unsigned meas_u32x4_t __attribute__((ext_vector_type(4)));

template <bool NT, int U>
__global__ __launch_bounds__(256) void measure_stream_read_kernel(const meas_u32x4_t *__restrict__ buf, size_t n_vec,
                                                                  unsigned *__restrict__ sink)
{
    // contiguous region per workgroup, walked front to back U x 4 KB (256 lanes x 16 bytes) at a time, U loads in flight
    const size_t per = (n_vec + gridDim.x - 1) / gridDim.x;
    const size_t begin = per * blockIdx.x, end = begin + per < n_vec ? begin + per : n_vec;
    meas_u32x4_t acc = {0u, 0u, 0u, 0u};
    size_t i = begin + threadIdx.x;
    for (; i + 256 * (U - 1) < end; i += 256 * U) {
        meas_u32x4_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = NT ? __builtin_nontemporal_load(buf + i + 256 * u) : buf[i + 256 * u];
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    for (; i < end; i += 256) acc ^= NT ? __builtin_nontemporal_load(buf + i) : buf[i];
    const unsigned r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (r == 0x9e3779b9u) sink[blockIdx.x] = r;     // practically never true: the loads cannot be dropped
}

template <bool FROM_LDS>
__global__ __launch_bounds__(GEMM_THREADS, 1) void measure_mfma_bf16_kernel(int iters, float *__restrict__ sink)
{
    __shared__ __attribute__((aligned(16))) meas_u32x4_t frags[2][8][64];   // two steps x (4 row + 4 column fragments)
    const int lane = threadIdx.x & 63;
    // bf16 values of magnitude around 1 with mixed signs and mantissas (what real operands look like to the
    // multipliers), different per lane, fragment and step
    unsigned s = 0x1234567u + threadIdx.x * 2654435761u + blockIdx.x * 40503u;
    auto rnd = [&]() {
        s = s * 1664525u + 1013904223u;
        const unsigned lo = 0x3f00u | ((s >> 9) & 0x80ffu), hi = 0x3f00u | ((s >> 17) & 0x80ffu);
        return lo | (hi << 16);
    };
    meas_u32x4_t f[2][8];
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            f[st][i] = (meas_u32x4_t){rnd(), rnd(), rnd(), rnd()};
            if (threadIdx.x < 64) frags[st][i][lane] = f[st][i];
        }
    __syncthreads();
    f32x16_t acc[4][4];
    zero_acc<4, 4>(acc);
    meas_u32x4_t g[2][8];               // fragments of the current and of the next step
#pragma unroll
    for (int i = 0; i < 8; ++i) g[0][i] = FROM_LDS ? frags[0][i][lane] : f[0][i];
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            // the next step's fragments are requested before this step's matrix instructions, as the tile kernel does
#pragma unroll
            for (int i = 0; i < 8; ++i) g[st ^ 1][i] = FROM_LDS ? frags[st ^ 1][i][lane] : f[st ^ 1][i];
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                for (int nb = 0; nb < 4; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, g[st][4 + nb]),
                                                                          __builtin_bit_cast(bf16x8_t, g[st][mb]),
                                                                          acc[mb][nb], 0, 0, 0);
            if (!FROM_LDS) {
                // new operand bits every step without touching memory: rotate the words of every fragment
#pragma unroll
                for (int i = 0; i < 8; ++i) f[st][i] = (meas_u32x4_t){f[st][i].y, f[st][i].z, f[st][i].w, f[st][i].x};
            }
        }
    }
    float r = 0.f;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) r += acc[mb][nb][v];
    if (r == 12345.678f) sink[blockIdx.x * GEMM_THREADS + threadIdx.x] = r;
}

static int cu_count()
{
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return 0;
    return n;
}

}  // namespace moe

using namespace moe;

extern "C" int moe_measure_stream_read(const void *buf, size_t bytes, int nontemporal, int n_workgroups, void *sink,
                                       void *stream)
{
    MOE_REQUIRE(buf && sink && aligned16(buf) && bytes >= 16 && bytes % 16 == 0, MOE_ERR_INVALID_ARG,
                "moe_measure_stream_read: buffer missing, misaligned or not a multiple of 16 bytes");
    MOE_REQUIRE(nontemporal == 0 || nontemporal == 1, MOE_ERR_INVALID_ARG, "moe_measure_stream_read: flag must be 0 or 1");
    const int n_cu = cu_count();
    MOE_REQUIRE(n_cu > 0, MOE_ERR_HIP, "moe_measure_stream_read: cannot read the compute unit count");
    MOE_REQUIRE(n_workgroups >= 0 && n_workgroups <= n_cu * 8, MOE_ERR_INVALID_ARG,
                "moe_measure_stream_read: n_workgroups=%d outside 0..%d", n_workgroups, n_cu * 8);
    const int grid = n_workgroups > 0 ? n_workgroups : n_cu * 8;      // sink holds a word per workgroup
    // one workgroup per compute unit at most: 32 loads (128 KB per workgroup) in flight, so that the rate shown is
    // what the unit's load path gives and not what 16 KB in flight wait for; the whole chip: 4 loads, 8 workgroups per unit
    const bool deep = n_workgroups > 0 && n_workgroups <= n_cu;
    auto kern = deep ? (nontemporal ? measure_stream_read_kernel<true, 32> : measure_stream_read_kernel<false, 32>)
                     : (nontemporal ? measure_stream_read_kernel<true, 4> : measure_stream_read_kernel<false, 4>);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const meas_u32x4_t *)buf, bytes / 16,
                       (unsigned *)sink);
    MOE_CHECK_LAUNCH("moe_measure_stream_read");
    return MOE_OK;
}

extern "C" size_t moe_measure_sink_bytes(void)
{
    const int n_cu = cu_count();
    return (size_t)(n_cu > 0 ? n_cu : 1024) * GEMM_THREADS * 8 * sizeof(float);
}

extern "C" size_t moe_measure_mfma_bf16_flops(int iters)
{
    const int n_cu = cu_count();
    if (iters <= 0 || n_cu <= 0) return 0;
    // per workgroup and iteration: 2 steps x 4 wavefronts x 16 instructions of 32 x 32 x 16 multiply-adds
    return (size_t)n_cu * (size_t)iters * 2 * 4 * 16 * (2ull * 32 * 32 * 16);
}

extern "C" int moe_measure_mfma_bf16(int iters, int from_lds, void *sink, void *stream)
{
    MOE_REQUIRE(iters > 0 && iters <= (1 << 24) && sink, MOE_ERR_INVALID_ARG, "moe_measure_mfma_bf16: iters=%d or sink", iters);
    MOE_REQUIRE(from_lds == 0 || from_lds == 1, MOE_ERR_INVALID_ARG, "moe_measure_mfma_bf16: flag must be 0 or 1");
    const int n_cu = cu_count();
    MOE_REQUIRE(n_cu > 0, MOE_ERR_HIP, "moe_measure_mfma_bf16: cannot read the compute unit count");
    if (from_lds)
        hipLaunchKernelGGL(measure_mfma_bf16_kernel<true>, dim3(n_cu), dim3(GEMM_THREADS), 0, (hipStream_t)stream, iters,
                           (float *)sink);
    else
        hipLaunchKernelGGL(measure_mfma_bf16_kernel<false>, dim3(n_cu), dim3(GEMM_THREADS), 0, (hipStream_t)stream, iters,
                           (float *)sink);
    MOE_CHECK_LAUNCH("moe_measure_mfma_bf16");
    return MOE_OK;
}
