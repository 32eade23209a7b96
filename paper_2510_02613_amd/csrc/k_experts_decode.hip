// Weight-streaming expert kernels for decode-sized batches (bf16).
//
// With a few tokens per step most resident experts receive 0-4 rows (the
// memory-bound regime of the layer of Sec. 2.1 of the paper under expert
// parallelism): the work is reading every ACTIVE expert's weights once, and the
// right measure is HBM bandwidth.  Slots without rows are never touched -- the
// tile list, built from the active expert map (Sec. 3.2 / 4.6: placement is data,
// not layout), only names slots that have rows.
//
// One wavefront owns a block of weight rows of one M-tile (<= 16 grouped rows) and
// walks the whole contraction: GEMM-1 takes 16 gate rows and the 16 matching up rows
// (so silu(g)*u is formed in registers), GEMM-2 takes 16 consecutive W2 rows.  Weights
// and token rows go straight from global memory into MFMA operand layout, as in
// the gate kernel: for a K-chunk of 128, lane (n = l%16, q = l/16) reads the 32 k
// {jj*32 + q*8 + i} of row n with four 16-byte loads issued back to back, so every
// row contributes a contiguous 256-byte run per chunk.  v_mfma_f32_16x16x32_bf16
// with the weights as first operand gives lane (j = l%16, q) the outputs of token
// j for weight rows 4q..4q+3: one 8-byte store.  The next chunk's loads are in
// flight during the current chunk's MFMAs; with 4 wavefronts per SIMD that keeps
// more than 128 KB per compute unit on its way from HBM.
#include "moe_internal.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 64;    // one wavefront per workgroup: tasks are dealt to compute units one by one, which
                                // balances a grid that is only about one round of the chip deep
constexpr int kTileRows = 16;   // grouped rows per M-tile (one MFMA N dimension)
constexpr int kWRows = 32;      // weight rows per wavefront

struct Run { uint4 v[4]; };     // a lane's 32 k of one row of a 128-wide K chunk

__device__ __forceinline__ void load_run(Run &r, const uint16_t *row, int k0, int q, int K)
{
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        const int k = k0 + jj * 32 + q * 8;
        r.v[jj] = (k < K) ? *(const uint4 *)(row + k) : make_uint4(0, 0, 0, 0);  // K % 8 == 0
    }
}

constexpr int kBlocks2 = 1;   // 16-row weight blocks per wavefront in GEMM-2: its contraction is short (I), and
                              // twice as many, half as long tasks keep more of the chip streaming to the end

template <bool kFirst>
__global__ __launch_bounds__(kThreads) void k_expert_decode(Pass p)
{
    const int K = kFirst ? p.H : p.I;
    const int N = kFirst ? p.I : p.H;                       // output columns
    constexpr bool kTwo = kFirst || kBlocks2 == 2;          // two weight rows per lane
    constexpr int COLS = kFirst ? kWRows / 2 : 16 * kBlocks2;   // output columns per wavefront
    const int groups = (N + COLS - 1) / COLS;               // wavefront tasks per M-tile
    const int lane = threadIdx.x;
    const int task = blockIdx.x;
    const int tile = task / groups;
    if (tile >= *p.n_tiles) return;
    const MTile mt = p.tiles[tile];
    const int n0 = (task % groups) * COLS;
    const int n = lane & 15, q = lane >> 4;

    const uint16_t *W = (const uint16_t *)(kFirst ? p.w13 : p.w2) + (size_t)mt.slot * (kFirst ? 2 : 1) * (size_t)p.I * p.H;
    // two weight rows per lane: (gate, up) of one h column, or two W2 rows 16 apart
    const int ra = min(n0 + n, N - 1);
    const int rb = kFirst ? p.I + ra : min(n0 + 16 + n, N - 1);
    const uint16_t *wa = W + (size_t)ra * K, *wb = W + (size_t)rb * K;
    // token row of this lane (rows past the tile's end re-read its last row; their outputs are dropped)
    const int tr = mt.row_begin + min(n, mt.rows - 1);
    const uint16_t *xr = (const uint16_t *)(kFirst ? p.x : p.h) + (size_t)(kFirst ? p.perm[tr] : tr) * K;

    f32x4 acc_a = {0.f, 0.f, 0.f, 0.f}, acc_b = {0.f, 0.f, 0.f, 0.f};
    Run ca, cb, cx, na, nb, nx;
    load_run(ca, wa, 0, q, K);
    if (kTwo) load_run(cb, wb, 0, q, K);
    load_run(cx, xr, 0, q, K);
    for (int k0 = 0; k0 < K; k0 += 128) {
        if (k0 + 128 < K) {
            load_run(na, wa, k0 + 128, q, K);
            if (kTwo) load_run(nb, wb, k0 + 128, q, K);
            load_run(nx, xr, k0 + 128, q, K);
        }
        __builtin_amdgcn_sched_barrier(0);  // the prefetch must be issued before this chunk's MFMAs, not after
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            acc_a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&ca.v[jj], *(bf16x8 *)&cx.v[jj], acc_a, 0, 0, 0);
            if (kTwo) acc_b = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&cb.v[jj], *(bf16x8 *)&cx.v[jj], acc_b, 0, 0, 0);
        }
        ca = na; cb = nb; cx = nx;
    }

    // lane holds token n, weight rows 4q..4q+3 of each of its two row blocks
    if (n >= mt.rows) return;
    uint16_t *O = (uint16_t *)(kFirst ? p.h : p.y) + (size_t)(mt.row_begin + n) * N;
    auto pack = [](float a, float b, float c, float d) {
        return make_uint2((uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16),
                          (uint32_t)f32_to_bf16(c) | ((uint32_t)f32_to_bf16(d) << 16));
    };
    if (kFirst) {
        const int col = n0 + 4 * q;
        if (col < N) {
            float h[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) h[r] = silu_mul(acc_a[r], acc_b[r]);
            *(uint2 *)(O + col) = pack(h[0], h[1], h[2], h[3]);
        }
    } else {
        const int c0 = n0 + 4 * q, c1 = n0 + 16 + 4 * q;
        if (c0 < N) *(uint2 *)(O + c0) = pack(acc_a[0], acc_a[1], acc_a[2], acc_a[3]);
        if (kTwo && c1 < N) *(uint2 *)(O + c1) = pack(acc_b[0], acc_b[1], acc_b[2], acc_b[3]);
    }
}

}  // namespace

int decode_tile_rows() { return kTileRows; }

hipError_t launch_experts_decode(const Pass &p, int which, hipStream_t st)
{
    if (which == 0) {
        const int groups = (p.I + kWRows / 2 - 1) / (kWRows / 2);
        const int blocks = p.max_tiles * groups;
        hipLaunchKernelGGL((k_expert_decode<true>), dim3(blocks), dim3(kThreads), 0, st, p);
    } else {
        const int groups = (p.H + 16 * kBlocks2 - 1) / (16 * kBlocks2);
        const int blocks = p.max_tiles * groups;
        hipLaunchKernelGGL((k_expert_decode<false>), dim3(blocks), dim3(kThreads), 0, st, p);
    }
    return hipGetLastError();
}

}  // namespace emoe
