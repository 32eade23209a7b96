// Two measuring sticks for benchmarks: what the matrix cores and HBM of THIS chip sustain with
// nothing else in the way.  They are not part of the method; a benchmark runs them beside the
// layer so that a roofline fraction against the data-sheet peak can be read next to the fraction
// of what is reachable (sustained clocks under MFMA load are well below the peak clock).
#include "moe_internal.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 512;        // 8 wavefronts, two per SIMD, as in the large-tile expert kernels
constexpr int kChains = 8;           // independent accumulators per wavefront

// Register-only v_mfma_f32_32x32x16_bf16 stream: `iters` rounds of kChains independent MFMAs.
// `random_operands` != 0 feeds the multipliers pseudo-random values in (-1, 1) that change from
// one MFMA to the next (the power such data draws is what sets the sustained clock of real
// kernels); 0 feeds small constants (the issue-rate ceiling).
__global__ __launch_bounds__(kThreads) void k_ceiling_mfma(int iters, int random_operands, float *sink)
{
    bf16x8 a[4], b[4];
    uint32_t h = (threadIdx.x + 1u) * 0x9e3779b9u + blockIdx.x * 0x85ebca6bu;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            h = h * 1664525u + 1013904223u;
            const float ra = random_operands ? (float)(int)(h >> 8 & 0xffff) * (1.f / 32768.f) - 1.f : (float)((threadIdx.x + i) & 3);
            h = h * 1664525u + 1013904223u;
            const float rb = random_operands ? (float)(int)(h >> 8 & 0xffff) * (1.f / 32768.f) - 1.f : (float)((threadIdx.x >> 2) & 1);
            a[j][i] = (__bf16)ra;
            b[j][i] = (__bf16)rb;
        }
    f32x16 acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c & 3], b[(c + (c >> 2)) & 3], acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[c][r];
    if (s == 123456.789f) sink[0] = s;   // keeps the chains alive; practically never true
}

// Plain streaming read: 16 bytes per lane, consecutive lanes on consecutive addresses, grid-stride.
__global__ __launch_bounds__(256) void k_ceiling_stream(const uint4 *__restrict__ buf, size_t n16, float *sink)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint32_t s = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        const uint4 v = buf[i];
        s += v.x ^ v.y ^ v.z ^ v.w;
    }
    if (s == 0x12345678u) sink[0] = 1.f;   // keeps the loads alive; practically never true
}

}  // namespace

double ceiling_mfma_flops(int blocks, int iters) { return (double)blocks * (kThreads / 64) * (double)iters * kChains * 2.0 * 32 * 32 * 16; }

hipError_t launch_ceiling_mfma(int blocks, int iters, int random_operands, float *sink, hipStream_t st)
{
    hipLaunchKernelGGL(k_ceiling_mfma, dim3(blocks), dim3(kThreads), 0, st, iters, random_operands, sink);
    return hipGetLastError();
}

hipError_t launch_ceiling_stream(const void *buf, size_t bytes, float *sink, hipStream_t st)
{
    hipLaunchKernelGGL(k_ceiling_stream, dim3(8192), dim3(256), 0, st, (const uint4 *)buf, bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace emoe
