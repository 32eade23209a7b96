// Un-permute and weighted combine: out[t] = sum_j w[t,j] * y[inv[t,j]].
//
// The sum runs over the token's assignments in selection order (routed experts
// first, then the shared experts with weight 1), skipping experts that live on
// another rank (inv == -1); accumulation is fp32 with a single final rounding, so
// the result does not depend on which physical slot an expert occupies -- the
// property the paper's remapping needs (Sec. 3.2, "Virtual Expert Management":
// kernels see the same logical layout whatever the physical placement).
// A token with no local assignment gets a zero row (partial sum for the
// cross-rank reduction of expert parallelism, Sec. 2.1).
//
// A workgroup owns one token and every gridDim.y-th run of 256 16-byte column chunks of its row, so
// that every y row and the out row are read / written fully coalesced; gridDim.y > 1 spreads a
// decode-sized batch over the chip.
#include "moe_internal.h"

namespace emoe {
namespace {

constexpr int kMaxKK = 36;  // top_k <= 32 plus <= 4 shared experts

template <typename T> struct Chunk;
template <> struct Chunk<uint16_t> { static constexpr int n = 8; };  // 8 bf16 = 16 B
template <> struct Chunk<float> { static constexpr int n = 4; };     // 4 fp32 = 16 B

// kChunks: 0 = few tokens (see below), else the column chunks a thread works on at once
template <typename T, int kChunks>
__global__ __launch_bounds__(256) void k_combine(Pass p)
{
    constexpr int C = Chunk<T>::n;
    __shared__ int32_t rows[kMaxKK];
    __shared__ float wts[kMaxKK];
    __shared__ int32_t n_local;
    const int t = blockIdx.x;
    if (threadIdx.x < 64) {   // first wavefront: the token's local assignments, compacted, still in selection order
        const int j = threadIdx.x;
        int r = -1;
        float wv = 0.f;
        if (j < p.kk) {
            r = p.inv[(size_t)t * p.kk + j];
            wv = j < p.k ? p.w[(size_t)t * p.k + j] : 1.0f;
        }
        const unsigned long long m = __ballot(r >= 0);
        if (r >= 0) {
            const int at = __popcll(m & ((1ull << j) - 1ull));
            rows[at] = r;
            wts[at] = wv;
        }
        if (j == 0) n_local = __popcll(m);
    }
    __syncthreads();
    const int n = n_local;
    const T *y = (const T *)p.y;
    T *out = (T *)p.out + (size_t)t * p.H;
    const int stride = gridDim.y * 256 * C;
    if (kChunks == 0) {
        // few tokens: the rows of four assignments are requested before any is added (the loads are
        // independent, only the additions are ordered), since there is no other workgroup to hide them
        for (int c = (blockIdx.y * 256 + threadIdx.x) * C; c < p.H; c += stride) {
            float acc[C];
#pragma unroll
            for (int i = 0; i < C; ++i) acc[i] = 0.f;
            for (int j0 = 0; j0 < n; j0 += 4) {
                uint4 raw[4];
                float wj[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    // past the last local assignment: weight 0 times zeros (nothing is read)
                    raw[u] = make_uint4(0, 0, 0, 0);
                    if (j0 + u < n) raw[u] = *(const uint4 *)(y + (size_t)rows[j0 + u] * p.H + c);
                    wj[u] = j0 + u < n ? wts[j0 + u] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const T *v = (const T *)&raw[u];
#pragma unroll
                    for (int i = 0; i < C; ++i) acc[i] = fmaf(wj[u], load_f32<T>(v, i), acc[i]);
                }
            }
            uint4 o;
            T *ov = (T *)&o;
#pragma unroll
            for (int i = 0; i < C; ++i) store_f32<T>(ov, i, acc[i]);
            *(uint4 *)(out + c) = o;
        }
    } else {
        // many tokens: a thread works on all (up to four) of its column chunks at once, so that as many loads of
        // a row are in flight per thread (a token has one or two local assignments when the experts are spread
        // over ranks, and the other workgroups of the compute unit do not cover the latency alone)
        constexpr int U = kChunks > 0 ? kChunks : 1;
        for (int c0 = (blockIdx.y * 256 + threadIdx.x) * C; c0 < p.H; c0 += U * stride) {
            float acc[U][C];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < C; ++i) acc[u][i] = 0.f;
            for (int j = 0; j < n; ++j) {
                const T *yr = y + (size_t)rows[j] * p.H;
                const float wj = wts[j];
                uint4 raw[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    raw[u] = make_uint4(0, 0, 0, 0);
                    if (c0 + u * stride < p.H) raw[u] = *(const uint4 *)(yr + c0 + u * stride);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const T *v = (const T *)&raw[u];
#pragma unroll
                    for (int i = 0; i < C; ++i) acc[u][i] = fmaf(wj, load_f32<T>(v, i), acc[u][i]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (c0 + u * stride >= p.H) continue;
                uint4 o;
                T *ov = (T *)&o;
#pragma unroll
                for (int i = 0; i < C; ++i) store_f32<T>(ov, i, acc[u][i]);
                *(uint4 *)(out + c0 + u * stride) = o;
            }
        }
    }
}

struct MapChunk { int32_t v[256]; };

__global__ void k_write_map(int32_t *dst, MapChunk c, int n)
{
    const int i = threadIdx.x;
    if (i < n) dst[i] = c.v[i];
}

// Plain device-to-device copy, 16 bytes per lane, grid-stride: the grid size is the caller's
// throttle on how much HBM bandwidth a background slot fill may take from the forwards.
__global__ __launch_bounds__(256) void k_copy16(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

hipError_t launch_copy(void *dst, const void *src, size_t bytes, int blocks, hipStream_t st)
{
    hipLaunchKernelGGL(k_copy16, dim3(blocks), dim3(256), 0, st, (uint4 *)dst, (const uint4 *)src, bytes / 16);
    return hipGetLastError();
}

hipError_t launch_combine(const Pass &p, hipStream_t st)
{
    // a row is shared out over several workgroups only while there are too few tokens to fill the chip
    const int per = 256 * (p.act_bf16 ? 8 : 4);
    const int ny = p.T >= 1024 ? 1 : (p.H + per - 1) / per;
    const bool few = p.T < 1024;
    const bool wide = p.H > per;       // a thread has several chunks of the row
    if (p.act_bf16) {
        if (few)       hipLaunchKernelGGL((k_combine<uint16_t, 0>), dim3(p.T, ny), dim3(256), 0, st, p);
        else if (wide) hipLaunchKernelGGL((k_combine<uint16_t, 4>), dim3(p.T, ny), dim3(256), 0, st, p);
        else           hipLaunchKernelGGL((k_combine<uint16_t, 1>), dim3(p.T, ny), dim3(256), 0, st, p);
    } else {
        if (few)       hipLaunchKernelGGL((k_combine<float, 0>), dim3(p.T, ny), dim3(256), 0, st, p);
        else if (wide) hipLaunchKernelGGL((k_combine<float, 4>), dim3(p.T, ny), dim3(256), 0, st, p);
        else           hipLaunchKernelGGL((k_combine<float, 1>), dim3(p.T, ny), dim3(256), 0, st, p);
    }
    return hipGetLastError();
}

// The table travels as a kernel argument (captured at launch time), so the host
// array may be reused as soon as this returns and the write is ordered on `st`
// like any other kernel; no staging buffer, no memcpy node.
hipError_t launch_write_map(int32_t *dst, const int32_t *host_vals, int n, hipStream_t st)
{
    for (int o = 0; o < n; o += 256) {
        MapChunk c;
        const int m = n - o < 256 ? n - o : 256;
        for (int i = 0; i < 256; ++i) c.v[i] = i < m ? host_vals[o + i] : -1;
        hipLaunchKernelGGL(k_write_map, dim3(1), dim3(256), 0, st, dst + o, c, m);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace emoe
