// Large-tile grouped SwiGLU expert GEMMs for prefill-sized groups (bf16, H and I multiples of 64).
//
// Same computation as the 4-wavefront kernels (the expert FFN of Sec. 2.1 of the
// paper over slot-grouped rows, weights addressed by slot so that a re-placement of
// experts -- Sec. 3.2 / 4.6 -- costs nothing here); what changes is the tile shape
// and the staging, chosen for three facts of this chip and this workload:
//
//  * Every expert's weights are used by only ~256 rows, so the layer streams all
//    resident weights from HBM once per pass: the kernel must keep HBM busy.  A
//    compute unit has to hold ~48 KB of weight bytes in flight to cover HBM latency
//    at full bandwidth, and whole 128-byte lines travel much faster than half lines
//    (also out of L2: a copy instruction that touches 16 half lines costs the issuing
//    wavefront twice one that touches 8 whole lines).  Both operands therefore travel
//    in steps of 64 k -- one full line per row: 32 KB of weight rows, up to 40 KB of
//    token rows per step -- through a 2-deep ring each (144 of the 160 KB of LDS: a
//    third weight step does not fit beside two token steps), with their own loader
//    wavefronts.  The weight step is issued half way through a K-step's multiply,
//    between two rounds of token copies (see k_loop: a compute unit returns copies in
//    issue order).
//  * A compute unit pulls ~64 B/clk from L2 but retires 4096 bf16 flops/clk, so a
//    tile must reuse staged bytes >= 64 times: up to 320 token rows x 256 weight
//    rows gives 114-142 (a 128 x 128 tile gives exactly 64 and is bandwidth bound).
//    Measured, staged bytes are the scarce resource of this kernel: a group's weights
//    should be staged once, and token rows that do not exist not at all.
//  * Groups are ragged (tokens per expert are binomial): the tile list carries
//    chunks of <= 320 rows balanced in units of 32 (one chunk for all but the
//    largest groups), token rows that do not exist are neither staged nor multiplied.
//
// Workgroup: 8 wavefronts as 2 (token) x 4 (weight).  Wavefront (wm, wn) owns weight
// rows [wn*64, wn*64+64) and token tiles wm, wm+2, ... (interleaved so that a ragged
// tile count splits evenly): up to 2 x 5 accumulators of 32x32 = 160 registers, two
// wavefronts per SIMD so that one's LDS waits hide under the other's MFMAs.
//
// Staging: global_load_lds_dwordx4 -- global memory straight into LDS, 16 bytes per
// lane, no VGPR round trip, no ds_write.  One instruction fills 1 KB: 8 rows of
// 128 bytes (token rows or weight rows); lane i lands in 16-byte slot i of the
// piece, so it FETCHES the chunk that belongs there: the XOR swizzle that keeps the
// 16-byte operand reads conflict free is applied on the global side.
//
// GEMM-1 packs every 32-row MFMA weight tile as 16 gate rows followed by the 16
// matching up rows; in the 32x32 accumulator layout a lane then holds gate value r
// and up value r+8 of the same (token, column), so silu(g)*u needs no shuffles.
//
// Epilogue: every wavefront transposes its accumulators through a private LDS
// region (row stride = row bytes + 16: rows stay 16-byte aligned for the copy out, the
// 8-byte writes meet two to a bank) and writes whole contiguous row segments, 16 bytes
// per lane, so global stores are full cache lines.  The epilogue is instruction bound
// (3 us of a workgroup): 16-byte rather than 8-byte copies out halve its longest loop.
#include "moe_internal.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;                    // K-step: 128 bytes per tile row, one whole cache line, for both operands
constexpr int kThreads = 512;
constexpr int kWaves = 8;
constexpr int kBN = 256;                   // weight rows per workgroup
constexpr int kMaxTT = 10;                 // token tiles (32 rows) per workgroup
constexpr int kBM = kMaxTT * 32;           // 320: a whole group with its ragged tail in the usual case
constexpr int kBKW = 64;                   // weight K-step: 128 bytes per row = one whole cache line
constexpr int kWStage = kBN * kBKW * 2;    // 32 KB of weight rows per weight step
constexpr int kXStage = kBM * kBK * 2;     // 40 KB of token rows per K-step
#ifdef EMOE_TIMING_W3
constexpr int kNW = 3;                     // TIMING ONLY: a third weight stage, two steps in flight (see kXBase)
#else
constexpr int kNW = 2;                     // weight ring depth: one step multiplied, one in flight
#endif
constexpr int kNX = 2;                     // token ring depth
constexpr int kWPieces = kWStage / 1024 / 4;   // 8: 1 KB pieces (8 rows x 128 B) per weight-loader wavefront per weight step
constexpr int kXPieces = kXStage / 1024 / 4;   // 10: 1 KB pieces (8 rows x 128 B) per token-loader wavefront per K-step
#ifdef EMOE_TIMING_W3
constexpr int kXBase = kNW * kWStage - 16384;   // the token stages overlap the third weight stage (it does not fit beside them): garbage results
#else
constexpr int kXBase = kNW * kWStage;      // the token ring follows the weight ring
#endif
constexpr int kRingBytes = kXBase + kNX * kXStage;
constexpr int kXcds = 8;
constexpr int kMaxPartialSets = 256;        // partial-sum sets the workspace has room for: one round of a 256-unit chip
constexpr int kTC = kMaxTT / 2;            // token tiles per wavefront
constexpr int kWT = 2;                     // weight tiles per wavefront
constexpr int kEpiStride1 = 2 * kWT * 16 + 16;  // GEMM-1: 32 h columns per wavefront, bytes per staged row (rows stay 16-byte aligned)
constexpr int kEpiStride2 = 2 * kWT * 32 + 16;  // GEMM-2: 64 y columns per wavefront
constexpr int kEpiBytes = 32 * kEpiStride2;     // one token tile of one wavefront
constexpr int kLdsBytes = kRingBytes;
static_assert(kWaves * kEpiBytes <= kRingBytes, "epilogue staging reuses the ring");
static_assert(kTC == 5, "the dispatch on token tiles per wavefront below lists cases 0..5");
static_assert(kLdsBytes <= 160 * 1024, "LDS budget");

// Everything one wavefront needs for its K loop.
struct WaveCtx {
    const uint16_t *wbase, *abase;        // slot's weight matrix, activation matrix
    uint32_t off[kXPieces > kWPieces ? kXPieces : kWPieces];               // this lane's byte offset (from the matrix base) of each piece it stages, k = 0
    uint32_t woff[kBKW / 16], xoff[kBK / 16]; // LDS byte offsets (inside a stage) of this lane's operand rows per sub-step
    int wave, lane, wm, wn, n_tt;
    uint32_t wkb;                         // EMOE_TIMING_KMAJOR: elements between the k-blocks of a slot
    bool stream_w;                        // this tile's weight rows are read by no other tile: copy them non-temporally
    int xlive;                            // token-loader wavefronts: how many of their pieces hold rows that exist
};

// 16-byte slot swizzle of a 128-byte tile row: slot = chunk ^ swz8(row).  An LDS read of 16 bytes
// per lane is served 16 lanes at a time over 64 four-byte banks (256 bytes, i.e. 2 rows): the
// 16 consecutive rows a half-wavefront reads for one MFMA operand must therefore hit 16 distinct
// 16-byte bank groups.  Row bits (1, 2, 0^3) do that.
__device__ __forceinline__ int swz8(int row) { return ((row >> 1) & 3) | (((row ^ (row >> 3)) & 1) << 2); }

// LDS byte address of a __shared__ object (LDS pointers are 32-bit offsets in address space 3).
__device__ __forceinline__ uint32_t lds_addr(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

// Direct global -> LDS copy of one 1 KB piece: lane i's 16 bytes land at m0_base + 16*i.
// The global address is a wave-uniform base (SGPR pair) plus this lane's 32-bit byte offset.
// Issued as inline assembly on purpose: the compiler's wait-count insertion would otherwise
// hold every later LDS read until these loads (which belong to a LATER stage) have returned.
// Completion is awaited explicitly (wait_loads) before the step's barrier.
// kStream: the line is marked non-temporal -- read once and not worth a place in L2.  Used for the weight
// rows of a slot whose rows are a single chunk (no other tile reads them): the weight stream then does not
// push out what is read again -- the chunk's token rows (once per N-slice), h between the two GEMMs, and the
// rows y that the combine kernel reads back right after.  A slot with several chunks keeps the default
// policy, so that the later chunks find the weights in L2.
template <bool kStream>
__device__ __forceinline__ void dma_piece(const void *base, uint32_t byte_off, uint32_t lds_byte_addr)
{
    if (kStream) asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_byte_addr), "v"(byte_off), "s"(base) : "memory", "m0");
    else         asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_byte_addr), "v"(byte_off), "s"(base) : "memory", "m0");
}

// Loader roles: wavefronts 0-3 stream the weight rows (8 pieces each per K-step), wavefronts 4-7
// the token rows (up to 10 pieces each per K-step, only those whose rows exist).  The two kinds go
// out at different moments of a K-step (see k_loop), which one wavefront issuing both could not do
// without making the token copies wait for the weight copies ahead of them: a wavefront's loads
// complete in order.
__device__ __forceinline__ void issue_step(const WaveCtx &c, uint32_t slot_addr, int k0)
{
    // Timing-only builds (results are garbage): leave out the weight copies, the token copies or (below) the
    // multiply, to time what is left; EMOE_TIMING_W3 and EMOE_TIMING_KMAJOR time a third weight stage and a
    // k-block-major pool without building either.  Off unless the build defines the macro.
#ifdef EMOE_TIMING_NO_W
    if (c.wave < 4) return;
#endif
#ifdef EMOE_TIMING_NO_X
    if (c.wave >= 4) return;
#endif
    if (c.wave < 4) {
#ifdef EMOE_TIMING_KMAJOR
        const uint16_t *b = c.wbase + (size_t)(k0 / kBKW) * c.wkb;   // TIMING ONLY: the pool read as if it were [K/64][rows][64]
#else
        const uint16_t *b = c.wbase + k0;
#endif
        if (c.stream_w) {
#pragma unroll
            for (int i = 0; i < kWPieces; ++i) dma_piece<true>(b, c.off[i], slot_addr + (c.wave * kWPieces + i) * 1024);
        } else {
#pragma unroll
            for (int i = 0; i < kWPieces; ++i) dma_piece<false>(b, c.off[i], slot_addr + (c.wave * kWPieces + i) * 1024);
        }
    } else {
        const uint16_t *b = c.abase + k0;
#pragma unroll
        for (int i = 0; i < kXPieces; ++i)
            if (i < c.xlive) dma_piece<false>(b, c.off[i], slot_addr + ((c.wave & 3) + 4 * i) * 1024);
    }
}

// Orders this wavefront's own LDS traffic (writes before, reads after) WITHOUT waiting for its
// global stores: LDS instructions of one wavefront execute in order, so all that is needed is
// that the compiler keeps the order and that outstanding LDS operations have retired.  (A
// release/acquire fence here would also drain the vector-memory counter, i.e. stall every token
// tile of the epilogue on the round trip of the previous tile's stores.)
__device__ __forceinline__ void wave_lds_sync()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
}

// Wait until at most n of this wavefront's loads are still in flight (they complete in order).
template <int n>
__device__ __forceinline__ void wait_loads()
{
    // s_waitcnt simm16: vmcnt = bits [3:0] and [15:14], expcnt [6:4] = 7, lgkmcnt [11:8] = 15 (no wait)
    static_assert(n < 64, "vmcnt has 6 bits");
    __builtin_amdgcn_s_waitcnt((n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8));
}

// One K-step (64 k) of this wavefront: NTC token tiles x 2 weight tiles x 4 sub-steps of 16 k.  The
// (sub-step, token tile) pairs run as one software pipeline: the token operand of pair s+2 and the
// weight operands of the next sub-step are requested from LDS before the MFMAs of pair s.  `mid` is
// called once, half way through.
template <int NTC, typename Mid>
__device__ __forceinline__ void multiply_stage(const WaveCtx &c, const char *Ws, const char *Xs, f32x16 (&acc)[kWT][kTC], Mid mid)
{
#ifdef EMOE_TIMING_NO_MUL
    mid();
    return;
#endif
    if constexpr (NTC > 0) {
        constexpr int KS = kBK / 16, STEPS = KS * NTC, D = 2;
        bf16x8 wf[2][kWT], xf[D + 1];
        auto fetch_w = [&](int ks) {
#pragma unroll
            for (int a = 0; a < kWT; ++a) {
                const uint4 v = *(const uint4 *)(Ws + c.woff[ks] + a * 32 * 128);
                wf[ks & 1][a] = *(const bf16x8 *)&v;
            }
        };
        auto fetch_x = [&](int step) {
            const int ks = step / NTC, t = step % NTC;
            const uint4 v = *(const uint4 *)(Xs + c.xoff[ks] + t * 64 * 128);
            xf[step % (D + 1)] = *(const bf16x8 *)&v;
        };
        fetch_w(0);
#pragma unroll
        for (int s0 = 0; s0 < D && s0 < STEPS; ++s0) fetch_x(s0);
#pragma unroll
        for (int step = 0; step < STEPS; ++step) {
            const int ks = step / NTC, t = step % NTC;
            if (step == STEPS / 2) mid();
            if (t == 0 && ks + 1 < KS) fetch_w(ks + 1);
            if (step + D < STEPS) fetch_x(step + D);
#pragma unroll
            for (int a = 0; a < kWT; ++a)
                acc[a][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ks & 1][a], xf[step % (D + 1)], acc[a][t], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);  // keep the written order: the prefetch depth is the register budget
        }
    } else {
        mid();
    }
}

template <int NTC>
__device__ __forceinline__ void k_loop(const WaveCtx &c, const char *ring, int KT, f32x16 (&acc)[kWT][kTC])
{
    // KT K-steps of 64.  Both rings are two deep: step kt+1 is copied while step kt is multiplied.  The
    // caller issued step 0.  Token copies go out right after the barrier, the weight copies half way
    // through the multiply: a compute unit returns copies in issue order, and token copies (L2 hits)
    // issued just behind a burst of weight copies would wait out that burst's HBM latency.
    const bool wloader = c.wave < 4;
    const uint32_t wring = lds_addr(ring), xring = wring + kXBase;
    int slot = 0;
#ifdef EMOE_TIMING_W3
    // TIMING ONLY: weight step kt+2 goes out half way through step kt (the caller issued steps 0 and 1)
    int ws = 0;
    for (int kt = 0; kt < KT; ++kt) {
        const bool more = kt + 1 < KT;
        if (wloader && more) wait_loads<kWPieces>(); else wait_loads<0>();   // step kt has landed; kt+1 may be in flight
        __syncthreads();
        if (!wloader && more) issue_step(c, xring + (slot ^ 1) * kXStage, (kt + 1) * kBK);
        const int w2 = ws == 0 ? 2 : ws - 1;    // stage of step kt+2 = stage of step kt-1
        multiply_stage<NTC>(c, ring + ws * kWStage, ring + kXBase + slot * kXStage, acc,
                            [&]() { if (wloader && kt + 2 < KT) issue_step(c, wring + w2 * kWStage, (kt + 2) * kBKW); });
        slot ^= 1;
        ws = ws == 2 ? 0 : ws + 1;
    }
#else
    for (int kt = 0; kt < KT; ++kt) {
        wait_loads<0>();   // this wavefront's share of step kt has landed (nothing younger is in flight)
        __syncthreads();   // everyone's share of step kt is in LDS; everyone is done reading step kt-1
        const bool more = kt + 1 < KT;
        if (!wloader && more) issue_step(c, xring + (slot ^ 1) * kXStage, (kt + 1) * kBK);
        multiply_stage<NTC>(c, ring + slot * kWStage, ring + kXBase + slot * kXStage, acc,
                            [&]() { if (wloader && more) issue_step(c, wring + (slot ^ 1) * kWStage, (kt + 1) * kBKW); });
        slot ^= 1;
    }
#endif
}

// Partial sums of a tile whose contraction is shared out over several workgroups (the tail of a
// launch, see the kernel): floats per set, and where a wavefront's accumulator registers go.
constexpr int kPartialFloats = kWaves * kWT * kTC * 16 * 64;   // 81920 = 320 KB
__device__ __forceinline__ float *partial_at(float *set, int wave, int a, int t, int r4, int lane)
{
    return set + ((((wave * kWT + a) * kTC + t) * 4 + r4) * 64 + lane) * 4;   // 16 bytes per lane, 1 KB per instruction
}

// Epilogue of one token tile of a wavefront: accumulators (token tile t of the wavefront, its kWT weight
// tiles) -> the wavefront's private LDS region [token row][column] -> coalesced rows of h (with SwiGLU) or y.
template <bool kFirst>
__device__ __forceinline__ void emit_token_tile(const Pass &p, const WaveCtx &c, const MTile &mt, int n0, int N, char *ring, int t,
                                                const f32x16 (&v)[kWT])
{
    constexpr int COLS = kFirst ? kWT * 16 : kWT * 32;      // output columns of this wavefront
    constexpr int STRIDE = kFirst ? kEpiStride1 : kEpiStride2;
    char *mine = ring + c.wave * kEpiBytes;
    const int l31 = c.lane & 31, khalf = c.lane >> 5;
    constexpr int LPR = COLS / 8;                           // copy out: 16 bytes per lane, LPR lanes per row,
    constexpr int RPI = 64 / LPR;                           // 64/LPR rows per instruction
    static_assert(STRIDE % 16 == 0 && kEpiBytes % 16 == 0 && 32 % RPI == 0, "16-byte reads of the staged rows");
    uint16_t *O = (uint16_t *)(kFirst ? p.h : p.y);
    const int ncol0 = n0 + c.wn * COLS;
    const int lr = c.lane / LPR, lc = (c.lane % LPR) * 8;
    char *row = mine + l31 * STRIDE;
#pragma unroll
    for (int a = 0; a < kWT; ++a) {
        constexpr int Q = kFirst ? 2 : 4;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            uint16_t o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float g = v[a][q * 4 + e];
                if (kFirst) {
                    const float u = v[a][(q + 2) * 4 + e];
                    g = silu_mul(g, u);
                }
                o[e] = f32_to_bf16(g);
            }
            const int col = a * (kFirst ? 16 : 32) + q * 8 + khalf * 4;
            *(uint2 *)(row + col * 2) = make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16), (uint32_t)o[2] | ((uint32_t)o[3] << 16));
        }
    }
    wave_lds_sync();
#pragma unroll
    for (int r0 = 0; r0 < 32; r0 += RPI) {
        const int rr = r0 + lr;                       // row inside the token tile
        const int m = (2 * t + c.wm) * 32 + rr;       // row inside the chunk
        const uint4 w = *(const uint4 *)(mine + rr * STRIDE + lc * 2);
        if (m < mt.rows && ncol0 + lc < N)   // N is a multiple of 64: the lane's 8 columns exist together
            *(uint4 *)(O + (size_t)(mt.row_begin + m) * N + ncol0 + lc) = w;
    }
    wave_lds_sync();  // the region is rewritten by the next token tile
}

// kPhase 0: a whole tile.  1: the partial sums of one of n_parts K ranges of a tile, left in
// p.partials (phase 2, sum_body below, adds them up).
// (Letting the last of a tile's workgroups to finish do the adding, in the same launch, was
// measured and is slower: the device-wide fence it needs costs more than the third launch.)
template <bool kFirst, int NTC, int kPhase>
__device__ __forceinline__ void wave_body(const Pass &p, const WaveCtx &c, const MTile &mt, int n0, int N, int KT, char *ring,
                                          float *tile_sets, int part)
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
    if (kPhase == 1) {
        float *mine = tile_sets + (size_t)part * kPartialFloats;
#pragma unroll
        for (int a = 0; a < kWT; ++a)
#pragma unroll
            for (int t = 0; t < NTC; ++t)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    float4 v = make_float4(acc[a][t][r4 * 4], acc[a][t][r4 * 4 + 1], acc[a][t][r4 * 4 + 2], acc[a][t][r4 * 4 + 3]);
                    *(float4 *)partial_at(mine, c.wave, a, t, r4, c.lane) = v;
                }
        return;
    }
#pragma unroll
    for (int t = 0; t < NTC; ++t) {
        f32x16 v[kWT];
#pragma unroll
        for (int a = 0; a < kWT; ++a) v[a] = acc[a][t];
        emit_token_tile<kFirst>(p, c, mt, n0, N, ring, t, v);
    }
}

// Phase 2: the sum of a tile's partial sums, in K order, for token tile t of this wavefront, then the
// same epilogue as a whole tile.  The sets of four parts are requested together (32 loads of 16 bytes
// per lane in flight: the launch is one round of the chip, its length is that of one workgroup) and
// added one after the other.
template <bool kFirst>
__device__ __forceinline__ void sum_body(const Pass &p, const WaveCtx &c, const MTile &mt, int n0, int N, char *ring,
                                         float *tile_sets, int n_parts, int t)
{
    f32x16 s[kWT];
#pragma unroll
    for (int a = 0; a < kWT; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[a][r] = 0.f;
    for (int q0 = 0; q0 < n_parts; q0 += 4) {
        float4 v[4][kWT][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (q0 + u >= n_parts) continue;               // uniform
            float *set = tile_sets + (size_t)(q0 + u) * kPartialFloats;
#pragma unroll
            for (int a = 0; a < kWT; ++a)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) v[u][a][r4] = *(const float4 *)partial_at(set, c.wave, a, t, r4, c.lane);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (q0 + u >= n_parts) continue;
#pragma unroll
            for (int a = 0; a < kWT; ++a)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    s[a][r4 * 4] += v[u][a][r4].x; s[a][r4 * 4 + 1] += v[u][a][r4].y;
                    s[a][r4 * 4 + 2] += v[u][a][r4].z; s[a][r4 * 4 + 3] += v[u][a][r4].w;
                }
        }
    }
    emit_token_tile<kFirst>(p, c, mt, n0, N, ring, t, s);
}

template <bool kFirst, int kPhase>
__global__ __launch_bounds__(kThreads, 1) void k_expert_gemm_mfma8(Pass p)
{
    const int K = kFirst ? p.H : p.I;
    const int N = kFirst ? p.I : p.H;                  // output columns
    constexpr int BNO = kFirst ? kBN / 2 : kBN;        // output columns per workgroup

    // Work is dealt to the 8 XCDs in UNITS: a tile (chunk) of the size-ordered list with a run of its
    // N-slices.  The unit list of this GEMM was written by the bookkeeping kernel in rows of 8 -- entry
    // 8 i + x is the i-th unit of XCD x, largest tiles first on every XCD, loads equal to within one unit,
    // the tiles of one slot one behind the other on one XCD -- and workgroup ids are dealt round-robin to
    // the XCDs by the hardware, so workgroup b works for XCD b % 8 and takes that XCD's units in order,
    // the N-slices of a unit on consecutive workgroups (they share the tile's token rows in that XCD's L2).
    const UnitHdr hdr = p.unit_hdr[kFirst ? 0 : 1];
    const int spp = hdr.spp;                           // N-slices per unit

    // The tail of the launch.  Workgroups run in rounds of one per compute unit; with long
    // contractions a launch is only a few rounds deep, and a last round that fills a fraction of the
    // chip costs a whole round.  When the launch allows it (p.k_split), the workgroups of that last
    // round are run separately: each tile's contraction is shared out over n_parts workgroups
    // (phase 1, partial sums to p.partials), which a third launch adds up in K order (phase 2).  The
    // split is a function of the unit list alone, so all three launches agree on it.
    const int rows_total = hdr.n_rows;                 // rows of 8 workgroups, holes at the ends of the columns included
    const int rows_round = min(p.n_cus, kMaxPartialSets) / kXcds;
    int tail_rows = 0, n_parts = 1;
    if (p.k_split && rows_total >= rows_round) {
        const int tr = rows_total % rows_round;
        int parts = tr ? rows_round / tr : 1;
        parts = min(parts, min(8, K / kBKW / 8));       // eight weight steps or more per part
        if (parts >= 2) { tail_rows = tr; n_parts = parts; }
    }
    const int head_blocks = (rows_total - tail_rows) * kXcds;
    int b, part = 0;
    if (kPhase == 0) {
        b = blockIdx.x;
        if (b >= head_blocks) return;
    } else if (kPhase == 1) {
        const int tail_blocks = tail_rows * kXcds;
        if (tail_blocks == 0) return;
        part = blockIdx.x / tail_blocks;
        if (part >= n_parts) return;
        b = head_blocks + blockIdx.x % tail_blocks;     // consecutive workgroups keep their XCDs (tail_blocks is a multiple of 8)
    } else {
        if ((int)blockIdx.x >= tail_rows * kXcds) return;
        b = head_blocks + blockIdx.x;
    }
    float *tile_sets = kPhase == 0 ? nullptr : p.partials + (size_t)((b - head_blocks) * n_parts) * kPartialFloats;
    const int j = b / kXcds;
    const MUnit un = p.units[kFirst ? 0 : 1][(j / spp) * kXcds + b % kXcds];
    if (un.rows == 0) return;                          // a hole at the end of this XCD's column
    MTile mt;
    mt.slot = un.slot; mt.row_begin = un.row_begin; mt.rows = un.rows; mt.single = un.info & 1;
    const int n0 = ((un.info >> 1) + j % spp) * BNO;

    __shared__ __attribute__((aligned(1024))) char ring[kPhase == 2 ? kWaves * kEpiBytes : kLdsBytes];   // phase 2 only stages its epilogue
    WaveCtx c;
    c.lane = threadIdx.x & 63;
    c.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    c.wn = c.wave & 3;
    c.wm = c.wave >> 2;
    c.n_tt = (mt.rows + 31) >> 5;                      // token tiles that exist
    c.stream_w = mt.single != 0;                       // the slot's rows are one chunk: nobody else reads these weights (known from the tile itself: no further lookup before the first weight copies)
    c.xlive = c.wave < 4 ? 0 : min(kXPieces, c.n_tt);  // pieces w, w+4, ... < 4*n_tt (8 rows each)

    // ---- staging plan ----
    // this workgroup's K range: everything, or (phase 1) weight steps [w0, w1) of the tile
    const int wsteps = K / kBKW;
    const int w0 = kPhase == 1 ? (int)((long long)part * wsteps / n_parts) : 0;
    const int w1 = kPhase == 1 ? (int)((long long)(part + 1) * wsteps / n_parts) : wsteps;
    const uint16_t *W = (const uint16_t *)(kFirst ? p.w13 : p.w2) + (size_t)mt.slot * (kFirst ? 2 : 1) * (size_t)p.I * p.H;
    const uint16_t *A = (const uint16_t *)(kFirst ? p.x : p.h);
#ifdef EMOE_TIMING_KMAJOR
    c.wkb = (uint32_t)(kFirst ? 2 * p.I : p.H) * kBKW;
    c.wbase = W + (size_t)w0 * c.wkb;
#else
    c.wbase = W + w0 * kBKW;      // rows are K-contiguous: the piece offsets below are relative to the range's first k
#endif
    c.abase = A + w0 * kBKW;
    if (c.wave < 4) {
#pragma unroll
        for (int i = 0; i < kWPieces; ++i) {
            // weight piece: rows [8*pc, 8*pc+8) of the weight tile, 128 bytes each
            const int pc = c.wave * kWPieces + i;
            const int row = pc * 8 + (c.lane >> 3);
            const int chunk = (c.lane & 7) ^ swz8(row);
            int g;
            if (kFirst) {
                const int tile = row >> 5, within = row & 31;
                const int col = min(n0 + tile * 16 + (within & 15), N - 1);
                g = (within < 16) ? col : p.I + col;
            } else {
                g = min(n0 + row, N - 1);
            }
#ifdef EMOE_TIMING_KMAJOR
            // the workgroup's 256 weight rows as one contiguous 32 KB block per k-block (stays inside the slot)
            (void)g; (void)chunk;
            c.off[i] = ((uint32_t)min((n0 / BNO) * kBN + row, (kFirst ? 2 * p.I : p.H) - 1) * kBKW + (c.lane & 7) * 8) * 2;
#else
            c.off[i] = ((uint32_t)g * K + chunk * 8) * 2;
#endif
        }
    } else {
#pragma unroll
        for (int i = 0; i < kXPieces; ++i) {
            // token piece: rows [8*pc, 8*pc+8) of the token tile, 128 bytes each (rows past the chunk re-read its last row)
            const int pc = (c.wave & 3) + 4 * i;   // interleaved over the 4 loaders so that live pieces are shared evenly
            const int row = pc * 8 + (c.lane >> 3);
            const int chunk = (c.lane & 7) ^ swz8(row);
            const int r = min(row, mt.rows - 1);
            const int sr = kFirst ? p.perm[mt.row_begin + r] : mt.row_begin + r;
            c.off[i] = ((uint32_t)sr * K + chunk * 8) * 2;
        }
    }
    {   // operand rows of this lane: weight row wn*64 + l31 (+32a), token row wm*32 + l31 (+64t)
        const int l31 = c.lane & 31, khalf = c.lane >> 5;
        const int wr = c.wn * kWT * 32 + l31, xr = c.wm * 32 + l31;
#pragma unroll
        for (int ks = 0; ks < kBKW / 16; ++ks) c.woff[ks] = wr * 128 + (((ks * 2 + khalf) ^ swz8(wr)) << 4);
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) c.xoff[ks] = xr * 128 + (((ks * 2 + khalf) ^ swz8(xr)) << 4);
    }

    const int KT = w1 - w0;
    if (kPhase != 2) {
        const uint32_t wring = lds_addr(ring), xring = wring + kXBase;
        if (KT > 0) issue_step(c, c.wave < 4 ? wring : xring, 0);
#ifdef EMOE_TIMING_W3
        if (KT > 1 && c.wave < 4) issue_step(c, wring + kWStage, kBKW);
#endif
    }
    // token tiles this wavefront multiplies: wm, wm+2, ... < n_tt.  The whole rest of the
    // wavefront's work is specialised on that count so that its K loop is straight-line code.
    const int ntc = (c.n_tt - c.wm + 1) >> 1;
    if constexpr (kPhase == 2) {
        // phase 2 is spread over the token tiles too: a workgroup adds up one per wavefront
        if ((int)blockIdx.y < ntc) sum_body<kFirst>(p, c, mt, n0, N, ring, tile_sets, n_parts, (int)blockIdx.y);
    } else {
        switch (ntc) {
        case 5: wave_body<kFirst, 5, kPhase>(p, c, mt, n0, N, KT, ring, tile_sets, part); break;
        case 4: wave_body<kFirst, 4, kPhase>(p, c, mt, n0, N, KT, ring, tile_sets, part); break;
        case 3: wave_body<kFirst, 3, kPhase>(p, c, mt, n0, N, KT, ring, tile_sets, part); break;
        case 2: wave_body<kFirst, 2, kPhase>(p, c, mt, n0, N, KT, ring, tile_sets, part); break;
        case 1: wave_body<kFirst, 1, kPhase>(p, c, mt, n0, N, KT, ring, tile_sets, part); break;
        default: wave_body<kFirst, 0, kPhase>(p, c, mt, n0, N, KT, ring, tile_sets, part); break;
        }
    }
}

}  // namespace

int mfma8_tile_rows() { return kBM; }

// usable when both contraction lengths are whole K-steps (direct-to-LDS loads cannot zero fill)
// Whole K-steps only (the copies cannot zero fill), and the copies address their rows with 32-bit byte
// offsets from the matrix base: x by token index, h by grouped row, a slot's weights by weight row.
bool mfma8_supports(const Pass &p)
{
    const size_t lim = (size_t)1 << 32;
    return p.act_bf16 && p.H % kBKW == 0 && p.I % kBKW == 0 &&
           (size_t)p.T * p.H * 2 < lim && (size_t)p.T * p.kk * p.I * 2 < lim && (size_t)2 * p.I * p.H * 2 < lim;
}

size_t mfma8_partial_bytes() { return (size_t)kMaxPartialSets * kPartialFloats * sizeof(float); }

int mfma8_n_slices(int H, int I, int which) { return which == 0 ? (I + kBN / 2 - 1) / (kBN / 2) : (H + kBN - 1) / kBN; }

// Rows of 8 workgroups a launch provides (and unit rows x N-slices per unit its unit list has room for):
// every tile's N-slices, dealt evenly (rounded up to whole units), plus kUnitSlack units per column for columns
// of unequal length when the tiles of a slot are kept on one XCD.
int mfma8_grid_rows(int max_tiles, int n_slices) { return (max_tiles * n_slices + kXcds - 1) / kXcds + (kUnitSlack + 1) * n_slices; }

hipError_t launch_experts_mfma8(const Pass &p0, int which, hipStream_t st)
{
    // compute units of the CURRENT device (looked up once per device: a process may drive several)
    static int cus_of[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    int cus = dev >= 0 && dev < 64 ? cus_of[dev] : 0;
    if (cus == 0) {
        int n = 0;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        cus = n >= kXcds ? n : kXcds;
        if (dev >= 0 && dev < 64) cus_of[dev] = cus;
    }
    Pass p = p0;
    p.n_cus = cus;
    // sharing out the contraction of the last round's tiles pays when a tile is long: 64 weight steps or more
    const int K = which == 0 ? p.H : p.I;
    p.k_split = p.partials != nullptr && K / kBKW >= 64;
    if (!p.units[0] || !p.unit_hdr) return hipErrorInvalidValue;   // the bookkeeping kernel must have been asked for unit lists
    const int nt = p.n_slices[which];
    const int grid = mfma8_grid_rows(p.max_tiles, nt) * kXcds;
    const int round_blocks = (cus < kMaxPartialSets ? cus : kMaxPartialSets) / kXcds * kXcds;
    if (which == 0) {
        hipLaunchKernelGGL((k_expert_gemm_mfma8<true, 0>), dim3(grid), dim3(kThreads), 0, st, p);
        if (p.k_split) {
            hipLaunchKernelGGL((k_expert_gemm_mfma8<true, 1>), dim3(round_blocks), dim3(kThreads), 0, st, p);
            hipLaunchKernelGGL((k_expert_gemm_mfma8<true, 2>), dim3(round_blocks / 2, kTC), dim3(kThreads), 0, st, p);
        }
    } else {
        hipLaunchKernelGGL((k_expert_gemm_mfma8<false, 0>), dim3(grid), dim3(kThreads), 0, st, p);
        if (p.k_split) {
            hipLaunchKernelGGL((k_expert_gemm_mfma8<false, 1>), dim3(round_blocks), dim3(kThreads), 0, st, p);
            hipLaunchKernelGGL((k_expert_gemm_mfma8<false, 2>), dim3(round_blocks / 2, kTC), dim3(kThreads), 0, st, p);
        }
    }
    return hipGetLastError();
}

}  // namespace emoe
