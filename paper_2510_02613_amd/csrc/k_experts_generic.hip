// Plain grouped expert FFN kernels (fp32 FMA, LDS tiled).  They serve the fp32
// layer and act as the debugging path for bf16 layers; the fast path for bf16 is
// the MFMA kernels.
//
// Per weight slot s and its grouped rows r (Sec. 2.1 of the paper: the selected
// experts process the token; under expert parallelism only the resident ones):
//     GEMM-1   g = x_r . W13[s][0:I]^T,  u = x_r . W13[s][I:2I]^T,  h_r = silu(g) * u
//     GEMM-2   y_r = h_r . W2[s]^T
// x rows are gathered through perm[] while the A tile is staged, so the permuted
// activation matrix is never materialised.  The slot index comes from the M-tile
// list, which was built from the active expert map: weights are only ever
// addressed as pool + slot * stride.
#include "moe_internal.h"

namespace emoe {
namespace {

constexpr int kBM = kGenericTileRows;  // 32
constexpr int kBN = 64;
constexpr int kBK = 32;
constexpr int kThreads = 256;

template <typename T, bool kFirst>
__global__ __launch_bounds__(kThreads) void k_expert_gemm_generic(Pass p)
{
    const int tile = blockIdx.y;
    if (tile >= *p.n_tiles) return;
    const MTile mt = p.tiles[tile];
    const int K = kFirst ? p.H : p.I;   // contraction length
    const int N = kFirst ? p.I : p.H;   // output columns
    const int n0 = blockIdx.x * kBN;

    __shared__ float As[kBM][kBK + 1];
    __shared__ float Bs[kBN][kBK + 1];
    __shared__ float Bu[kFirst ? kBN : 1][kBK + 1];
    __shared__ int32_t src_row[kBM];

    const int tid = threadIdx.x;
    if (tid < kBM) {
        int r = min(tid, mt.rows - 1);  // rows past the group's end re-read its last row
        src_row[tid] = kFirst ? p.perm[mt.row_begin + r] : (mt.row_begin + r);
    }
    const T *A = (const T *)(kFirst ? p.x : p.h);
    const T *W = (const T *)(kFirst ? p.w13 : p.w2) + (size_t)mt.slot * (kFirst ? 2 : 1) * p.I * p.H;
    const int ty = tid >> 4, tx = tid & 15;
    float acc[2][4] = {}, acu[2][4] = {};
    __syncthreads();

    for (int k0 = 0; k0 < K; k0 += kBK) {
        for (int idx = tid; idx < kBM * kBK; idx += kThreads) {
            int r = idx / kBK, kc = idx % kBK;
            As[r][kc] = (k0 + kc < K) ? load_f32<T>(A, (size_t)src_row[r] * K + k0 + kc) : 0.f;
        }
        for (int idx = tid; idx < kBN * kBK; idx += kThreads) {
            int n = idx / kBK, kc = idx % kBK;
            bool ok = (n0 + n < N) && (k0 + kc < K);
            Bs[n][kc] = ok ? load_f32<T>(W, (size_t)(n0 + n) * K + k0 + kc) : 0.f;
            if (kFirst) Bu[n][kc] = ok ? load_f32<T>(W, (size_t)(p.I + n0 + n) * K + k0 + kc) : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int kc = 0; kc < kBK; ++kc) {
            float a0 = As[ty * 2][kc], a1 = As[ty * 2 + 1][kc];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float b = Bs[tx * 4 + j][kc];
                acc[0][j] = fmaf(a0, b, acc[0][j]);
                acc[1][j] = fmaf(a1, b, acc[1][j]);
                if (kFirst) {
                    float u = Bu[tx * 4 + j][kc];
                    acu[0][j] = fmaf(a0, u, acu[0][j]);
                    acu[1][j] = fmaf(a1, u, acu[1][j]);
                }
            }
        }
        __syncthreads();
    }
    T *O = (T *)(kFirst ? p.h : p.y);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = ty * 2 + i;
        if (r >= mt.rows) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float v = acc[i][j];
            if (kFirst) v = v / (1.f + expf(-v)) * acu[i][j];
            store_f32<T>(O, (size_t)(mt.row_begin + r) * N + n, v);
        }
    }
}

// test mode: every expert is the identity, y_r = x[perm[r]]
template <typename T>
__global__ __launch_bounds__(256) void k_identity_experts(Pass p)
{
    const int r = blockIdx.x;
    if (r >= p.offs[p.S]) return;
    const T *x = (const T *)p.x + (size_t)p.perm[r] * p.H;
    T *y = (T *)p.y + (size_t)r * p.H;
    for (int c = threadIdx.x; c < p.H; c += 256) y[c] = x[c];
}

}  // namespace

hipError_t launch_experts_generic(const Pass &p, int which, hipStream_t st)
{
    dim3 block(kThreads);
    dim3 g1((p.I + kBN - 1) / kBN, p.max_tiles), g2((p.H + kBN - 1) / kBN, p.max_tiles);
    if (p.act_bf16) {
        if (which == 0) hipLaunchKernelGGL((k_expert_gemm_generic<uint16_t, true>), g1, block, 0, st, p);
        else            hipLaunchKernelGGL((k_expert_gemm_generic<uint16_t, false>), g2, block, 0, st, p);
    } else {
        if (which == 0) hipLaunchKernelGGL((k_expert_gemm_generic<float, true>), g1, block, 0, st, p);
        else            hipLaunchKernelGGL((k_expert_gemm_generic<float, false>), g2, block, 0, st, p);
    }
    return hipGetLastError();
}

hipError_t launch_identity_experts(const Pass &p, hipStream_t st)
{
    const int rows = p.T * p.kk;  // upper bound of grouped rows; extra blocks exit
    if (p.act_bf16) hipLaunchKernelGGL((k_identity_experts<uint16_t>), dim3(rows), dim3(256), 0, st, p);
    else            hipLaunchKernelGGL((k_identity_experts<float>), dim3(rows), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace emoe
