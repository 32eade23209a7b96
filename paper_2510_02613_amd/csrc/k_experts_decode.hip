// Weight-streaming expert kernels for decode-sized batches (bf16).
//
// With a few tokens per step most resident experts receive 0-4 rows (the
// memory-bound regime of the layer of Sec. 2.1 of the paper under expert
// parallelism): the work is reading every ACTIVE expert's weights once, and the
// right measure is HBM bandwidth.  Slots without rows are never touched -- the
// tile list, built from the active expert map (Sec. 3.2 / 4.6: placement is data,
// not layout), only names slots that have rows.
//
// A task is a block of weight rows of one M-tile (<= 16 grouped rows): GEMM-1 takes 16
// gate rows and the 16 matching up rows (so silu(g)*u is formed in registers), GEMM-2
// 32 consecutive W2 rows.  A task is one workgroup of four wavefronts, each walking a
// quarter of the contraction.  Weights and token rows go straight from global memory
// into MFMA operand layout, as in the gate kernel: for a K-chunk of 128, lane
// (n = l%16, q = l/16) reads the 32 k {jj*32 + q*8 + i} of row n with four 16-byte
// loads issued back to back, so every row contributes a contiguous 256-byte run per
// chunk.  v_mfma_f32_16x16x32_bf16 with the weights as first operand gives lane
// (j = l%16, q) the outputs of token j for weight rows 4q..4q+3: one 8-byte store.
// The next chunk's loads are in flight during the current chunk's MFMAs; with 4
// wavefronts per SIMD that keeps more than 128 KB per compute unit on its way from HBM.
#include "moe_internal.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 64;    // a wavefront; a workgroup is one task: the kSplit wavefronts that share its contraction
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

constexpr int kBlocks2 = 2;   // 16-row weight blocks per task in GEMM-2
// Wavefronts that share a task's contraction: each takes a contiguous quarter of the K-chunks, the first adds
// the four sums in K order (through LDS) and stores.  A wavefront's stream is latency bound (one chunk in
// flight), so a launch ends with a tail as long as one task in which ever fewer wavefronts stream; with four
// wavefronts per task that tail is a quarter as long, and the tasks of a launch (several rounds of the chip's
// wavefront slots in GEMM-2) are dealt to the compute units in finer pieces.  Measured on the DeepSeek-V3-shaped
// rank with 64 tokens: GEMM-1 291 -> 277 us, GEMM-2 161 -> 140 us (2 or 8 wavefronts per task: slower).
constexpr int kSplit1 = 4;
constexpr int kSplit2 = 4;

// Self-derived tiles (GEMM-1 of passes with at most 64 tokens and 64 slots whose selection kernel left per-block
// slot masks): with so few tokens the offsets / permutation / tile-list kernel is pure latency in front of the
// weight stream, and everything a GEMM-1 workgroup needs from it follows from 4 count bytes per slot.  So that
// kernel is not launched: every wavefront adds up the counts itself (lane s = slot s), finds the slot and chunk
// of its tile with a wavefront scan, and reads its rows' tokens off the slot's block masks; workgroup 0 of the
// same launch writes the tables that GEMM-2, the combine and the workspace view read, while the others stream.
constexpr int kSelfMaxSlots = 64, kSelfMaxBlocks = 4;

// position of the r-th (0-based) set bit of m; m has more than r bits set
__device__ __forceinline__ int nth_set_bit(unsigned long long m, int r)
{
    int pos = 0;
#pragma unroll
    for (int w = 32; w >= 1; w >>= 1) {
        const int cnt = __popcll(m & ((1ull << w) - 1ull));
        if (r >= cnt) { r -= cnt; m >>= w; pos += w; }
    }
    return pos;
}

// the count bytes of slot s that exist (blocks past nb hold nothing defined)
__device__ __forceinline__ uint32_t self_counts(const Pass &p, int s, int nb)
{
    const uint32_t w = *(const uint32_t *)(p.blk_cnt + (size_t)s * fused_row_stride(nb));
    return nb >= 4 ? w : w & ((1u << (8 * nb)) - 1u);
}

// Workgroup 0: counts, offsets, tile list (slot order, chunks of kTileRows), permutation and its inverse --
// the tables of the bookkeeping kernels, for the few-token case.  256 threads.
__device__ void self_tables(const Pass &p)
{
    __shared__ int32_t s_cb[kSelfMaxSlots][kSelfMaxBlocks];   // rows of slot s in block b
    __shared__ int32_t s_off[kSelfMaxSlots];
    const int tid = threadIdx.x, S = p.S, nb = (p.T + kFusedTokens - 1) / kFusedTokens;
    if (tid < S) {
        const uint32_t w = self_counts(p, tid, nb);
#pragma unroll
        for (int b = 0; b < kSelfMaxBlocks; ++b) s_cb[tid][b] = (int)((w >> (8 * b)) & 0xffu);
    }
    __syncthreads();
    if (tid == 0) {
        int row = 0, tl = 0;
        for (int s = 0; s < S; ++s) {
            const int c = s_cb[s][0] + s_cb[s][1] + s_cb[s][2] + s_cb[s][3];
            const int nt = (c + kTileRows - 1) / kTileRows;
            p.counts[s] = c;
            p.offs[s] = row;
            s_off[s] = row;
            for (int i = 0; i < nt; ++i, ++tl)
                if (tl < p.max_tiles) {
                    MTile mt;
                    mt.slot = s; mt.row_begin = row + i * kTileRows; mt.rows = min(kTileRows, c - i * kTileRows); mt.single = nt == 1;
                    p.tiles[tl] = mt;
                }
            row += c;
        }
        p.offs[S] = row;
        *p.n_tiles = min(tl, p.max_tiles);
    }
    __syncthreads();
    for (int a = tid; a < p.T * p.kk; a += blockDim.x) {
        const int sr = p.slot_rank[a];
        int row = -1;
        if (sr >= 0) {
            const int slot = sr >> 12, rank = sr & 0xfff, t = a / p.kk, b = t / kFusedTokens;
            row = s_off[slot] + rank;
            for (int b2 = 0; b2 < b; ++b2) row += s_cb[slot][b2];
            p.perm[row] = t;
        }
        p.inv[a] = row;
    }
}

template <bool kFirst, bool kSelf = false>
__global__ __launch_bounds__(kFirst ? kThreads * kSplit1 : kThreads * kSplit2) void k_expert_decode(Pass p)
{
    static_assert(!kSelf || kFirst, "only GEMM-1 derives its tiles itself");
    constexpr int NS = kFirst ? kSplit1 : kSplit2;                // wavefronts of this workgroup (one task)
    const int K = kFirst ? p.H : p.I;
    const int N = kFirst ? p.I : p.H;                       // output columns
    constexpr bool kTwo = kFirst || kBlocks2 == 2;          // two weight rows per lane
    constexpr int COLS = kFirst ? kWRows / 2 : 16 * kBlocks2;   // output columns per wavefront
    const int groups = (N + COLS - 1) / COLS;               // wavefront tasks per M-tile
    const int lane = threadIdx.x & 63;
    const int ks = NS > 1 ? (int)(threadIdx.x >> 6) : 0;    // which part of the contraction
    int task = blockIdx.x;
    if (kSelf) {
        if (task == 0) { self_tables(p); return; }
        task -= 1;
    }
    const int tile = task / groups;
    const int n = lane & 15, q = lane >> 4;
    MTile mt;
    int self_token = 0;                                     // kSelf: the token of this lane's row
    if (kSelf) {
        const int nb = (p.T + kFusedTokens - 1) / kFusedTokens, stride = fused_row_stride(nb);
        // lane s: rows and tiles of slot s, then inclusive sums over the slots (rows in the high half)
        int c = 0;
        if (lane < p.S) c = (int)__builtin_amdgcn_sad_u8(self_counts(p, lane, nb), 0u, 0u);
        const int nt = (c + kTileRows - 1) / kTileRows;
        int incl = (c << 16) | nt;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off, 64);
            if (lane >= off) incl += o;
        }
        const unsigned long long owners = __ballot((incl & 0xffff) > tile);
        if (owners == 0) return;                            // past the last tile (the same in every wavefront)
        const int s = __ffsll((long long)owners) - 1;
        const int before = __shfl(incl - ((c << 16) | nt), s, 64), cs = __shfl(c, s, 64);
        const int chunk = tile - (before & 0xffff);
        mt.slot = s;
        mt.row_begin = (before >> 16) + chunk * kTileRows;
        mt.rows = min(kTileRows, cs - chunk * kTileRows);
        mt.single = cs <= kTileRows;
        // the slot's tokens, ascending: bit t of the block masks side by side
        unsigned long long m = 0;
        for (int b = 0; b < nb; ++b) m |= (unsigned long long)((uint32_t)p.blk_hist[(size_t)s * stride + b] & 0xffffu) << (16 * b);
        self_token = nth_set_bit(m, chunk * kTileRows + min(n, mt.rows - 1));
    } else {
        if (tile >= *p.n_tiles) return;
        mt = p.tiles[tile];
    }
    const int n0 = (task % groups) * COLS;

    const uint16_t *W = (const uint16_t *)(kFirst ? p.w13 : p.w2) + (size_t)mt.slot * (kFirst ? 2 : 1) * (size_t)p.I * p.H;
    // two weight rows per lane: (gate, up) of one h column, or two W2 rows 16 apart
    const int ra = min(n0 + n, N - 1);
    const int rb = kFirst ? p.I + ra : min(n0 + 16 + n, N - 1);
    const uint16_t *wa = W + (size_t)ra * K, *wb = W + (size_t)rb * K;
    // token row of this lane (rows past the tile's end re-read its last row; their outputs are dropped)
    const int tr = mt.row_begin + min(n, mt.rows - 1);
    const uint16_t *xr = (const uint16_t *)(kFirst ? p.x : p.h) + (size_t)(kSelf ? self_token : kFirst ? p.perm[tr] : tr) * K;

    // this wavefront's K-chunks: [kbeg, kend)
    const int chunks = (K + 127) >> 7, per = (chunks + NS - 1) / NS;
    const int kbeg = min(ks * per, chunks) * 128, kend = min(min((ks + 1) * per, chunks) * 128, K), kstep = 128;
    f32x4 acc_a = {0.f, 0.f, 0.f, 0.f}, acc_b = {0.f, 0.f, 0.f, 0.f};
    Run ca, cb, cx, na, nb, nx;
    load_run(ca, wa, kbeg, q, K);
    if (kTwo) load_run(cb, wb, kbeg, q, K);
    load_run(cx, xr, kbeg, q, K);
    for (int k0 = kbeg; k0 < kend; k0 += kstep) {
        if (k0 + kstep < kend) {
            load_run(na, wa, k0 + kstep, q, K);
            if (kTwo) load_run(nb, wb, k0 + kstep, q, K);
            load_run(nx, xr, k0 + kstep, q, K);
        }
        __builtin_amdgcn_sched_barrier(0);  // the prefetch must be issued before this chunk's MFMAs, not after
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            acc_a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&ca.v[jj], *(bf16x8 *)&cx.v[jj], acc_a, 0, 0, 0);
            if (kTwo) acc_b = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&cb.v[jj], *(bf16x8 *)&cx.v[jj], acc_b, 0, 0, 0);
        }
        ca = na; cb = nb; cx = nx;
    }

    if constexpr (NS > 1) {   // the parts' sums, added in K order by the first wavefront
        __shared__ f32x4 part[NS - 1 > 0 ? NS - 1 : 1][kTwo ? 2 : 1][64];
        if (ks > 0) { part[ks - 1][0][lane] = acc_a; if (kTwo) part[ks - 1][kTwo ? 1 : 0][lane] = acc_b; }
        __syncthreads();
        if (ks > 0) return;
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) {
            const f32x4 a = part[s][0][lane];
            acc_a[0] += a[0]; acc_a[1] += a[1]; acc_a[2] += a[2]; acc_a[3] += a[3];
            if (kTwo) { const f32x4 b = part[s][kTwo ? 1 : 0][lane]; acc_b[0] += b[0]; acc_b[1] += b[1]; acc_b[2] += b[2]; acc_b[3] += b[3]; }
        }
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

// GEMM-1 can derive its tiles itself when the selection kernel left per-block masks for at most 4 blocks and 64 slots
bool decode_self_tiles(const Pass &p)
{
    return p.fused_hist && p.S <= kSelfMaxSlots && p.T <= kSelfMaxBlocks * kFusedTokens && kSplit1 * kThreads >= 64;
}

hipError_t launch_experts_decode(const Pass &p, int which, hipStream_t st)
{
    if (which == 0) {
        const int groups = (p.I + kWRows / 2 - 1) / (kWRows / 2);
        const int blocks = p.max_tiles * groups;
        if (p.self_tiles) hipLaunchKernelGGL((k_expert_decode<true, true>), dim3(blocks + 1), dim3(kThreads * kSplit1), 0, st, p);
        else              hipLaunchKernelGGL((k_expert_decode<true>), dim3(blocks), dim3(kThreads * kSplit1), 0, st, p);
    } else {
        const int groups = (p.H + 16 * kBlocks2 - 1) / (16 * kBlocks2);
        const int blocks = p.max_tiles * groups;
        hipLaunchKernelGGL((k_expert_decode<false>), dim3(blocks), dim3(kThreads * kSplit2), 0, st, p);
    }
    return hipGetLastError();
}

}  // namespace emoe
