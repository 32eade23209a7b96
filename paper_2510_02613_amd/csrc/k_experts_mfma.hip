// Grouped SwiGLU expert GEMMs on the gfx950 matrix cores (bf16 in, fp32 accumulate).
//
// The computation is the expert FFN of the layer the paper describes in Sec. 2.1,
// applied slot by slot to the grouped rows; which weights a group uses is read from
// the M-tile list (built from the active expert map), so a re-placement of experts
// (virtual expert management, Sec. 3.2; vpage-remap, Sec. 4.6) changes nothing here
// but the slot number.
//
//   GEMM-1  h[r, i] = silu(x_r . Wg[i]) * (x_r . Wu[i])     K = H, gathers x through perm
//   GEMM-2  y[r, n] = h_r . W2[n]                           K = I
//
// Tiling.  One workgroup (4 wavefronts, 2x2) owns BM grouped rows x BN weight rows
// and walks K in steps of 64.  Both operands are K-contiguous in memory, so a tile
// row is one 128-byte line; tiles are staged global -> registers -> LDS with the
// next K-step's loads in flight during the current step's MFMAs (double buffered
// LDS, one barrier per step).  LDS rows are 128 bytes with the 16-byte chunk index
// XOR-ed by (row & 7), which makes both the 16-byte staging writes and the 16-byte
// operand reads conflict free.
//
// MFMA.  v_mfma_f32_32x32x16_bf16 with the WEIGHT rows as the first operand and the
// token rows as the second: lane l then holds, for token (l % 32), weight rows
// 8*(r/4) + 4*(l/32) + (r%4), r = 0..15 -- four consecutive output columns per
// register quad, stored as one 8-byte packet.  For GEMM-1 a wavefront's first half
// of weight sub-tiles are gate rows and the second half the matching up rows, so
// silu(g) * u is formed in registers and only h is written.
//
// Scheduling.  The grid is one-dimensional and sized from an upper bound of the
// tile count; the real count is read from device memory (no host sync).  Workgroup
// ids are dealt round-robin to the 8 XCDs by the hardware, so id b is remapped to
// (b % 8) * ceil(n/8) + b / 8: each XCD walks a contiguous range of the tile list,
// N-tiles fastest, so the M-tiles of one expert run on one XCD at about the same
// time and its weights cross HBM -> L2 once.
#include "moe_internal.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;        // K step (bf16 elements): one 128-byte line per tile row
constexpr int kThreads = 256;  // 4 wavefronts
constexpr int kXcds = 8;

__device__ __forceinline__ int swz(int row, int chunk) { return row * 8 + (chunk ^ (row & 7)); }  // in 16-byte units

template <int BM, int BN, bool kFirst>
__global__ __launch_bounds__(kThreads, 2) void k_expert_gemm_mfma(Pass p)
{
    static_assert(BM % 64 == 0 && BN % 64 == 0, "2x2 wavefronts of 32x32 MFMA tiles");
    constexpr int WN = BN / 2, WM = BM / 2;   // wavefront tile: WN weight rows x WM token rows
    constexpr int TN = WN / 32, TM = WM / 32;
    constexpr int PW = BN / 32, PX = BM / 32; // staging passes (32 rows each)
    constexpr int BNO = kFirst ? BN / 2 : BN; // output columns per tile

    const int K = kFirst ? p.H : p.I;
    const int N = kFirst ? p.I : p.H;          // output columns
    const int n_ntiles = (N + BNO - 1) / BNO;

    // XCD-aware tile id
    const int total = *p.n_tiles * n_ntiles;
    const int per_xcd = (total + kXcds - 1) / kXcds;
    const int b = blockIdx.x;
    if (b / kXcds >= per_xcd) return;
    const int lid = (b % kXcds) * per_xcd + b / kXcds;
    if (lid >= total) return;
    const MTile mt = p.tiles[lid / n_ntiles];
    const int n0 = (lid % n_ntiles) * BNO;

    __shared__ uint4 lds[2][(BN + BM) * 8];  // per buffer: W tile rows then X tile rows, 8 chunks per row
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wn = wave & 1, wm = wave >> 1;

    // ---- staging addresses: thread -> (row = pass*32 + tid/8, chunk = tid%8) ----
    const int srow = tid >> 3, schunk = tid & 7;
    const uint16_t *W = (const uint16_t *)(kFirst ? p.w13 : p.w2) + (size_t)mt.slot * (kFirst ? 2 : 1) * (size_t)p.I * p.H;
    const uint16_t *A = (const uint16_t *)(kFirst ? p.x : p.h);
    const uint16_t *wptr[PW];
    const uint16_t *xptr[PX];
#pragma unroll
    for (int i = 0; i < PW; ++i) {
        const int r = i * 32 + srow;  // row inside the W tile
        int g;                        // global weight row
        if (kFirst) g = (r < BN / 2) ? min(n0 + r, N - 1) : p.I + min(n0 + r - BN / 2, N - 1);
        else        g = min(n0 + r, N - 1);
        wptr[i] = W + (size_t)g * K + schunk * 8;
    }
#pragma unroll
    for (int i = 0; i < PX; ++i) {
        const int r = min(i * 32 + srow, mt.rows - 1);  // rows past the group's end re-read its last row
        const int src = kFirst ? p.perm[mt.row_begin + r] : mt.row_begin + r;
        xptr[i] = A + (size_t)src * K + schunk * 8;
    }

    uint4 wreg[PW], xreg[PX];
    auto load_global = [&](int k0) {
        const bool ok = k0 + schunk * 8 < K;  // K is a multiple of 8: a chunk is all in or all out
#pragma unroll
        for (int i = 0; i < PW; ++i) wreg[i] = ok ? *(const uint4 *)(wptr[i] + k0) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < PX; ++i) xreg[i] = ok ? *(const uint4 *)(xptr[i] + k0) : make_uint4(0, 0, 0, 0);
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < PW; ++i) lds[buf][swz(i * 32 + srow, schunk)] = wreg[i];
#pragma unroll
        for (int i = 0; i < PX; ++i) lds[buf][BN * 8 + swz(i * 32 + srow, schunk)] = xreg[i];
    };

    f32x16 acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int c = 0; c < TM; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][c][r] = 0.f;

    // LDS row of this lane inside each operand sub-tile
    int wrow[TN], xrow[TM];
#pragma unroll
    for (int a = 0; a < TN; ++a) {
        if (kFirst) wrow[a] = (a / (TN / 2)) * (BN / 2) + wn * (WN / 2) + (a % (TN / 2)) * 32 + (lane & 31);
        else        wrow[a] = wn * WN + a * 32 + (lane & 31);
    }
#pragma unroll
    for (int c = 0; c < TM; ++c) xrow[c] = wm * WM + c * 32 + (lane & 31);
    const int khalf = lane >> 5;  // which 8 of the 16 k of one MFMA this lane feeds

    const int KT = (K + kBK - 1) / kBK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_global((kt + 1) * kBK);
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
            bf16x8 wf[TN], xf[TM];
            const int chunk = ks * 2 + khalf;
#pragma unroll
            for (int a = 0; a < TN; ++a) { uint4 v = lds[buf][swz(wrow[a], chunk)]; wf[a] = *(bf16x8 *)&v; }
#pragma unroll
            for (int c = 0; c < TM; ++c) { uint4 v = lds[buf][BN * 8 + swz(xrow[c], chunk)]; xf[c] = *(bf16x8 *)&v; }
#pragma unroll
            for (int a = 0; a < TN; ++a)
#pragma unroll
                for (int c = 0; c < TM; ++c)
                    acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[a], xf[c], acc[a][c], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane owns token (l%32) and 4 consecutive output columns per register quad ----
    uint16_t *O = (uint16_t *)(kFirst ? p.h : p.y);
    constexpr int TNO = kFirst ? TN / 2 : TN;  // output sub-tiles along N per wavefront
#pragma unroll
    for (int c = 0; c < TM; ++c) {
        const int m = wm * WM + c * 32 + (lane & 31);
        if (m >= mt.rows) continue;
        uint16_t *orow = O + (size_t)(mt.row_begin + m) * N;
#pragma unroll
        for (int a = 0; a < TNO; ++a) {
            const int ncol = n0 + (kFirst ? wn * (WN / 2) : wn * WN) + a * 32;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = ncol + q * 8 + khalf * 4;
                if (n >= N) continue;
                uint16_t v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float g = acc[a][c][q * 4 + e];
                    if (kFirst) {
                        const float u = acc[a + TN / 2][c][q * 4 + e];
                        g = silu_mul(g, u);
                    }
                    v[e] = f32_to_bf16(g);
                }
                *(uint2 *)(orow + n) = make_uint2((uint32_t)v[0] | ((uint32_t)v[1] << 16), (uint32_t)v[2] | ((uint32_t)v[3] << 16));
            }
        }
    }
}

}  // namespace

int mfma_tile_rows() { return 128; }

hipError_t launch_experts_mfma(const Pass &p, int which, hipStream_t st)
{
    constexpr int BM = 128, BN = 128;
    if (which == 0) {
        const int nt = (p.I + BN / 2 - 1) / (BN / 2);
        const int grid = (p.max_tiles * nt + kXcds - 1) / kXcds * kXcds;
        hipLaunchKernelGGL((k_expert_gemm_mfma<BM, BN, true>), dim3(grid), dim3(kThreads), 0, st, p);
    } else {
        const int nt = (p.H + BN - 1) / BN;
        const int grid = (p.max_tiles * nt + kXcds - 1) / kXcds * kXcds;
        hipLaunchKernelGGL((k_expert_gemm_mfma<BM, BN, false>), dim3(grid), dim3(kThreads), 0, st, p);
    }
    return hipGetLastError();
}

}  // namespace emoe
