// Measuring sticks for benchmarks: what the matrix cores and HBM of THIS chip sustain with
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

// The weight stream of the large-tile expert kernels with everything else taken away: a workgroup (one per
// compute unit: the LDS it declares leaves room for no second one) walks a tile of 256 rows in steps of 128
// bytes per row, four wavefronts copying 8 pieces of 1 KB each (8 rows x 128 B, global -> LDS) per step into
// a 2-deep ring, waiting only for the older step.  Same pieces, same instruction, same row stride as the
// kernels' weight loaders; no token rows, no multiply, no barrier.
template <bool kNt>
__global__ __launch_bounds__(256) void k_ceiling_tile_stream(const char *buf, size_t row_bytes, int steps)
{
    __shared__ __attribute__((aligned(1024))) char ring[128 * 1024];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const char *tile = buf + (size_t)blockIdx.x * 256 * row_bytes;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)ring;
    uint32_t off[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) off[i] = (uint32_t)((wave * 8 + i) * 8 + (lane >> 3)) * (uint32_t)row_bytes + (lane & 7) * 16;
    auto issue = [&](int s) {
        const char *b = tile + (size_t)s * 128;
        const uint32_t stage = lds0 + (s & 1) * 32768;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t dst = stage + (wave * 8 + i) * 1024;
            if (kNt) asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(dst), "v"(off[i]), "s"(b) : "memory", "m0");
            else     asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(off[i]), "s"(b) : "memory", "m0");
        }
    };
    if (steps > 0) issue(0);
    for (int s = 0; s < steps; ++s) {
        if (s + 1 < steps) {
            issue(s + 1);
            __builtin_amdgcn_s_waitcnt((8 & 15) | ((8 >> 4) << 14) | (7 << 4) | (15 << 8));   // vmcnt(8): step s has landed
        } else {
            __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));                             // vmcnt(0)
        }
    }
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

hipError_t launch_ceiling_tile_stream(const void *buf, int n_tiles, size_t row_bytes, int non_temporal, hipStream_t st)
{
    const int steps = (int)(row_bytes / 128);
    if (non_temporal) hipLaunchKernelGGL((k_ceiling_tile_stream<true>), dim3(n_tiles), dim3(256), 0, st, (const char *)buf, row_bytes, steps);
    else              hipLaunchKernelGGL((k_ceiling_tile_stream<false>), dim3(n_tiles), dim3(256), 0, st, (const char *)buf, row_bytes, steps);
    return hipGetLastError();
}

}  // namespace emoe
