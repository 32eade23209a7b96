// Large-tile grouped SwiGLU expert GEMMs for prefill-sized groups (bf16, K % 32 == 0).
//
// Same computation as the 4-wavefront kernels (the expert FFN of Sec. 2.1 of the
// paper over slot-grouped rows, weights addressed by slot so that a re-placement of
// experts -- Sec. 3.2 / 4.6 -- costs nothing here); what changes is the tile shape
// and the staging, chosen for three facts of this chip and this workload:
//
//  * Every expert's weights are used by only ~256 rows, so the layer streams all
//    resident weights from HBM once per pass: the kernel must keep HBM busy.  A
//    compute unit has to hold ~48 KB of weight bytes in flight to cover HBM latency
//    at full bandwidth; the K loop therefore runs a 4-deep ring of 32 KB stages
//    (K-step 32) and only ever waits for the OLDEST stage.
//  * A compute unit pulls ~64 B/clk from L2 but retires 4096 bf16 flops/clk, so a
//    tile must reuse staged bytes >= 64 times: 256 token rows x 256 weight rows
//    gives 128 (a 128 x 128 tile gives exactly 64 and is bandwidth bound).
//  * Groups are ragged (tokens per expert are binomial): the tile list carries
//    chunks of <= 256 rows balanced in units of 32, and a wavefront only multiplies
//    the 32-row token tiles that exist.
//
// Workgroup: 8 wavefronts as 2 (token) x 4 (weight).  Wavefront (wm, wn) owns weight
// rows [wn*64, wn*64+64) and token tiles wm, wm+2, wm+4, wm+6 (interleaved so that a
// ragged tile count splits evenly): 2 x 4 accumulators of 32x32 = 128 registers, two
// wavefronts per SIMD so that one's LDS waits hide under the other's MFMAs.
//
// Staging: global_load_lds_dwordx4 -- global memory straight into LDS, 16 bytes per
// lane, no VGPR round trip, no ds_write.  One instruction fills 16 rows x 64 bytes;
// lane i supplies row i/4 and lands in 16-byte slot i%4, so it FETCHES chunk
// (i%4) ^ ((row>>1)&3): the XOR swizzle that keeps the 16-byte operand reads
// conflict free is applied on the global side.
//
// GEMM-1 packs every 32-row MFMA weight tile as 16 gate rows followed by the 16
// matching up rows; in the 32x32 accumulator layout a lane then holds gate value r
// and up value r+8 of the same (token, column), so silu(g)*u needs no shuffles.
//
// Epilogue: every wavefront transposes its accumulators through a private LDS
// region (row stride = row bytes + 8, conflict free for the 8-byte writes) and
// writes whole contiguous row segments, so global stores are full cache lines.
#include "moe_internal.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBK = 32;                    // K-step: 64 bytes per tile row
constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kBN = 256;                   // weight rows per workgroup
constexpr int kMaxTT = 8;                  // token tiles (32 rows) per workgroup
constexpr int kBM = kMaxTT * 32;           // 256
constexpr int kRows = kBN + kBM;           // LDS rows per stage
constexpr int kStageBytes = kRows * 64;    // 32 KB
constexpr int kStages = 4;
constexpr int kPieces = kRows / 16;        // 1 KB pieces (16 rows) per stage = 32
constexpr int kPiecesPerWave = kPieces / kWaves;  // 4: two weight pieces, two token pieces
constexpr int kXcds = 8;
constexpr int kTC = kMaxTT / 2;            // token tiles per wavefront
constexpr int kWT = 2;                     // weight tiles per wavefront
constexpr int kEpiStride1 = 2 * kWT * 16 + 8;   // GEMM-1: 32 h columns per wavefront, bytes per staged row
constexpr int kEpiStride2 = 2 * kWT * 32 + 8;   // GEMM-2: 64 y columns per wavefront
constexpr int kLdsBytes = (kStages * kStageBytes > kWaves * kTC * 32 * kEpiStride2) ? kStages * kStageBytes : kWaves * kTC * 32 * kEpiStride2;
static_assert(kTC == 4, "the dispatch on token tiles per wavefront below lists cases 0..4");
static_assert(kLdsBytes <= 160 * 1024, "LDS budget");

// Everything one wavefront needs for its K loop.
struct WaveCtx {
    const uint16_t *wbase, *abase;        // slot's weight matrix, activation matrix
    uint32_t off[kPiecesPerWave];         // this lane's byte offset (from the matrix base) of each piece it stages, k = 0
    uint32_t woff[kBK / 16], xoff[kBK / 16];  // LDS byte offsets (inside a stage) of this lane's operand rows per sub-step
    int wave, lane, wm, wn, n_tt;
};

// LDS byte address of a __shared__ object (LDS pointers are 32-bit offsets in address space 3).
__device__ __forceinline__ uint32_t lds_addr(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

// Direct global -> LDS copy of one 1 KB piece: lane i's 16 bytes land at m0_base + 16*i.
// The global address is a wave-uniform base (SGPR pair) plus this lane's 32-bit byte offset.
// Issued as inline assembly on purpose: the compiler's wait-count insertion would otherwise
// hold every later LDS read until these loads (which belong to a LATER stage) have returned.
// Completion is awaited explicitly (wait_stages) before the stage's barrier.
__device__ __forceinline__ void dma_piece(const void *base, uint32_t byte_off, uint32_t lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_byte_addr), "v"(byte_off), "s"(base) : "memory", "m0");
}

// Stage the K-step that starts at element k0 into the ring slot at stage_addr: every
// wavefront copies its 4 pieces (w, w+8 : weight rows; w+16, w+24 : token rows).
__device__ __forceinline__ void issue_stage(const WaveCtx &c, uint32_t stage_addr, int k0)
{
    const uint16_t *wb = c.wbase + k0, *ab = c.abase + k0;
#pragma unroll
    for (int i = 0; i < kPiecesPerWave; ++i) {
        const int pb = c.wave + i * kWaves;
        dma_piece(i < kPiecesPerWave / 2 ? wb : ab, c.off[i], stage_addr + pb * 1024);
    }
}

// Wait until at most `pending` of this wavefront's staged K-steps are still in flight.
template <int pending>
__device__ __forceinline__ void wait_stages()
{
    // s_waitcnt simm16: vmcnt = bits [3:0] and [15:14], expcnt [6:4] = 7, lgkmcnt [11:8] = 15 (no wait)
    constexpr int n = pending * kPiecesPerWave;
    static_assert(n < 64, "vmcnt has 6 bits");
    __builtin_amdgcn_s_waitcnt((n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8));
}

// One K-step (32 k) of this wavefront: NTC token tiles x 2 weight tiles.  The 2 x NTC
// (sub-step, token tile) pairs run as one software pipeline: the token operand of pair s+2 and
// the weight operands of the next sub-step are requested from LDS before the MFMAs of pair s.
template <int NTC>
__device__ __forceinline__ void multiply_stage(const WaveCtx &c, const char *stage, f32x16 (&acc)[kWT][kTC])
{
    if constexpr (NTC > 0) {
        const char *Ws = stage, *Xs = stage + kBN * 64;
        constexpr int KS = kBK / 16, STEPS = KS * NTC, D = 2;
        bf16x8 wf[2][kWT], xf[D + 1];
        auto fetch_w = [&](int ks) {
#pragma unroll
            for (int a = 0; a < kWT; ++a) {
                const uint4 v = *(const uint4 *)(Ws + c.woff[ks] + a * 32 * 64);
                wf[ks & 1][a] = *(const bf16x8 *)&v;
            }
        };
        auto fetch_x = [&](int step) {
            const int ks = step / NTC, t = step % NTC;
            const uint4 v = *(const uint4 *)(Xs + c.xoff[ks] + t * 64 * 64);
            xf[step % (D + 1)] = *(const bf16x8 *)&v;
        };
        fetch_w(0);
#pragma unroll
        for (int s0 = 0; s0 < D && s0 < STEPS; ++s0) fetch_x(s0);
#pragma unroll
        for (int step = 0; step < STEPS; ++step) {
            const int ks = step / NTC, t = step % NTC;
            if (t == 0 && ks + 1 < KS) fetch_w(ks + 1);
            if (step + D < STEPS) fetch_x(step + D);
#pragma unroll
            for (int a = 0; a < kWT; ++a)
                acc[a][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ks & 1][a], xf[step % (D + 1)], acc[a][t], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);  // keep the written order: the prefetch depth is the register budget
        }
    }
}

template <int NTC>
__device__ __forceinline__ void k_loop(const WaveCtx &c, const char *ring, int KT, f32x16 (&acc)[kWT][kTC])
{
    const uint32_t a0 = lds_addr(ring);
    // the caller issued stages 0 .. kStages-2 (those that exist)
    for (int kt = 0; kt < KT; ++kt) {
        // stage kt must have landed: allow the kStages-2 younger ones to stay in flight
        if (kt + kStages - 2 < KT) wait_stages<kStages - 2>();
        else                       wait_stages<0>();
        __syncthreads();  // everyone's share of stage kt is in LDS; everyone is done reading stage kt-1
        if (kt + kStages - 1 < KT) issue_stage(c, a0 + ((kt + kStages - 1) % kStages) * kStageBytes, (kt + kStages - 1) * kBK);
        multiply_stage<NTC>(c, ring + (kt % kStages) * kStageBytes, acc);
    }
}

template <bool kFirst, int NTC>
__device__ __forceinline__ void wave_body(const Pass &p, const WaveCtx &c, const MTile &mt, int n0, int N, int KT, char *ring)
{
    f32x16 acc[kWT][kTC];
#pragma unroll
    for (int a = 0; a < kWT; ++a)
#pragma unroll
        for (int t = 0; t < kTC; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][t][r] = 0.f;
    k_loop<NTC>(c, ring, KT, acc);
    __syncthreads();  // all operand reads are done: the ring becomes the epilogue staging area

    // ---- epilogue: accumulators -> private LDS region [token row][column] -> coalesced rows ----
    constexpr int COLS = kFirst ? kWT * 16 : kWT * 32;      // output columns of this wavefront
    constexpr int STRIDE = kFirst ? kEpiStride1 : kEpiStride2;
    char *mine = ring + c.wave * (kTC * 32 * kEpiStride2);
    const int l31 = c.lane & 31, khalf = c.lane >> 5;
#pragma unroll
    for (int t = 0; t < NTC; ++t) {
        char *row = mine + (t * 32 + l31) * STRIDE;
#pragma unroll
        for (int a = 0; a < kWT; ++a) {
            constexpr int Q = kFirst ? 2 : 4;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                uint16_t v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float g = acc[a][t][q * 4 + e];
                    if (kFirst) {
                        const float u = acc[a][t][(q + 2) * 4 + e];
                        g = g / (1.f + __expf(-g)) * u;
                    }
                    v[e] = f32_to_bf16(g);
                }
                const int col = a * (kFirst ? 16 : 32) + q * 8 + khalf * 4;
                *(uint2 *)(row + col * 2) = make_uint2((uint32_t)v[0] | ((uint32_t)v[1] << 16), (uint32_t)v[2] | ((uint32_t)v[3] << 16));
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // copy out: 8 bytes per lane, LPR lanes per row, 64/LPR rows per instruction
    constexpr int LPR = COLS / 4;
    constexpr int RPI = 64 / LPR;
    uint16_t *O = (uint16_t *)(kFirst ? p.h : p.y);
    const int ncol0 = n0 + c.wn * COLS;
    const int lr = c.lane / LPR, lc = (c.lane % LPR) * 4;
#pragma unroll
    for (int t = 0; t < NTC; ++t) {
#pragma unroll
        for (int r0 = 0; r0 < 32; r0 += RPI) {
            const int rr = r0 + lr;                       // row inside the token tile
            const int m = (2 * t + c.wm) * 32 + rr;       // row inside the chunk
            const uint2 v = *(const uint2 *)(mine + (t * 32 + rr) * STRIDE + lc * 2);
            if (m < mt.rows && ncol0 + lc < N)
                *(uint2 *)(O + (size_t)(mt.row_begin + m) * N + ncol0 + lc) = v;
        }
    }
}

template <bool kFirst>
__global__ __launch_bounds__(kThreads, 1) void k_expert_gemm_mfma8(Pass p)
{
    const int K = kFirst ? p.H : p.I;
    const int N = kFirst ? p.I : p.H;                  // output columns
    constexpr int BNO = kFirst ? kBN / 2 : kBN;        // output columns per workgroup
    const int n_ntiles = (N + BNO - 1) / BNO;

    const int total = *p.n_tiles * n_ntiles;
    const int per_xcd = (total + kXcds - 1) / kXcds;
    const int b = blockIdx.x;
    if (b / kXcds >= per_xcd) return;
    const int lid = (b % kXcds) * per_xcd + b / kXcds;
    if (lid >= total) return;
    const MTile mt = p.tiles[lid / n_ntiles];
    const int n0 = (lid % n_ntiles) * BNO;

    __shared__ __attribute__((aligned(1024))) char ring[kLdsBytes];
    WaveCtx c;
    c.lane = threadIdx.x & 63;
    c.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    c.wn = c.wave & 3;
    c.wm = c.wave >> 2;
    c.n_tt = (mt.rows + 31) >> 5;                      // token tiles that exist

    // ---- staging plan ----
    const uint16_t *W = (const uint16_t *)(kFirst ? p.w13 : p.w2) + (size_t)mt.slot * (kFirst ? 2 : 1) * (size_t)p.I * p.H;
    const uint16_t *A = (const uint16_t *)(kFirst ? p.x : p.h);
    c.wbase = W;
    c.abase = A;
#pragma unroll
    for (int i = 0; i < kPiecesPerWave; ++i) {
        const int pb = c.wave + i * kWaves;            // piece: LDS rows pb*16 .. +16 of the stage
        const int row = pb * 16 + (c.lane >> 2);
        const int chunk = (c.lane & 3) ^ ((row >> 1) & 3);
        if (i < kPiecesPerWave / 2) {                  // weight rows
            int g;
            if (kFirst) {
                const int tile = row >> 5, within = row & 31;
                const int col = min(n0 + tile * 16 + (within & 15), N - 1);
                g = (within < 16) ? col : p.I + col;
            } else {
                g = min(n0 + row, N - 1);
            }
            c.off[i] = ((uint32_t)g * K + chunk * 8) * 2;
        } else {                                       // token rows (rows past the chunk re-read its last row)
            const int r = min(row - kBN, mt.rows - 1);
            const int s = kFirst ? p.perm[mt.row_begin + r] : mt.row_begin + r;
            c.off[i] = ((uint32_t)s * K + chunk * 8) * 2;
        }
    }
    {   // operand rows of this lane: weight row wn*64 + l31 (+32a), token row wm*32 + l31 (+64t)
        const int l31 = c.lane & 31, khalf = c.lane >> 5;
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
            const int chunk = ks * 2 + khalf;
            const int wr = c.wn * kWT * 32 + l31, xr = c.wm * 32 + l31;
            c.woff[ks] = wr * 64 + ((chunk ^ ((wr >> 1) & 3)) << 4);
            c.xoff[ks] = xr * 64 + ((chunk ^ ((xr >> 1) & 3)) << 4);
        }
    }

    const int KT = K / kBK;
    const uint32_t a0 = lds_addr(ring);
#pragma unroll
    for (int s = 0; s < kStages - 1; ++s)
        if (s < KT) issue_stage(c, a0 + s * kStageBytes, s * kBK);
    // token tiles this wavefront multiplies: wm, wm+2, ... < n_tt.  The whole rest of the
    // wavefront's work is specialised on that count so that its K loop is straight-line code.
    const int ntc = (c.n_tt - c.wm + 1) >> 1;
    switch (ntc) {
    case 4: wave_body<kFirst, 4>(p, c, mt, n0, N, KT, ring); break;
    case 3: wave_body<kFirst, 3>(p, c, mt, n0, N, KT, ring); break;
    case 2: wave_body<kFirst, 2>(p, c, mt, n0, N, KT, ring); break;
    case 1: wave_body<kFirst, 1>(p, c, mt, n0, N, KT, ring); break;
    default: wave_body<kFirst, 0>(p, c, mt, n0, N, KT, ring); break;
    }
}

}  // namespace

int mfma8_tile_rows() { return kBM; }

// usable when both contraction lengths are whole K-steps (direct-to-LDS loads cannot zero fill)
bool mfma8_supports(const Pass &p) { return p.act_bf16 && p.H % kBK == 0 && p.I % kBK == 0; }

hipError_t launch_experts_mfma8(const Pass &p, int which, hipStream_t st)
{
    if (which == 0) {
        const int nt = (p.I + kBN / 2 - 1) / (kBN / 2);
        const int grid = (p.max_tiles * nt + kXcds - 1) / kXcds * kXcds;
        hipLaunchKernelGGL((k_expert_gemm_mfma8<true>), dim3(grid), dim3(kThreads), 0, st, p);
    } else {
        const int nt = (p.H + kBN - 1) / kBN;
        const int grid = (p.max_tiles * nt + kXcds - 1) / kXcds * kXcds;
        hipLaunchKernelGGL((k_expert_gemm_mfma8<false>), dim3(grid), dim3(kThreads), 0, st, p);
    }
    return hipGetLastError();
}

}  // namespace emoe
