// Routing bookkeeping between the gate and the expert GEMMs.
//
// Every (token, selected expert) pair whose expert is resident on this rank
// becomes one row of a slot-grouped activation matrix.  "Resident" is decided by
// the expert map: the paper's virtual expert management (Sec. 3.2; vpage-remap,
// Sec. 4.6 / App. D) lets the expert placement change without moving weights, so
// the kernels here translate logical expert ids to physical weight slots on every
// pass and never assume a placement.
//
//   k_slot_hist  per block of 1024 assignments: slot lookup, LDS histogram, and the
//                rank of every assignment among the block's earlier assignments to
//                the same slot (deterministic: token order): lane scan inside a
//                wavefront, wavefronts take turns on the LDS counts.
//   k_slot_scan  one block: per-slot running sum over the blocks, exclusive prefix
//                sum over slots (LDS scan), and the M-tile list for the GEMMs.
//   k_slot_place row = offsets[slot] + block base + rank; perm[row] = token,
//                inv[assignment] = row (or -1 when the expert is not local).
//
// Rows of one slot end up ordered by (token, selection position); nothing depends
// on atomics ordering, so two passes over the same input give the same layout.
#include "moe_internal.h"
#include "wave_ops.h"

namespace emoe {
namespace {

constexpr int kThreads = 256;               // scan and place kernels
constexpr int kHistThreads = kAssignPerBlock;  // one thread per assignment, 16 wavefronts

// slot of assignment a (token a / kk, column a % kk), or -1 when it is not this rank's
__device__ __forceinline__ int slot_of(const Pass &p, int a)
{
    if (a >= p.T * p.kk) return -1;
    const int t = a / p.kk, j = a - t * p.kk;
    if (j < p.k) {
        // ids come from the gate, or from the caller when the routing is given: an id outside
        // [0, E) is an assignment that does not exist
        const int id = p.ids[(size_t)t * p.k + j];
        if ((unsigned)id >= (unsigned)p.E) return -1;
        const int m = p.map[id];
        if (m >= -1) return m;
        // replicated expert: -2 - m is where its copy list (count R >= 2, then R slots) starts behind
        // the E + n_shared entries; token t uses copy t mod R
        const int32_t *copies = p.map + p.E + p.n_shared + (-2 - m);
        return copies[1 + t % copies[0]];
    }
    if (t >= p.shared_begin && t < p.shared_end) return p.map[p.E + (j - p.k)];
    return -1;
}

constexpr int kHistWaves = kHistThreads / 64;
constexpr int kPerWaveSlots = 512;   // up to this many slots every wavefront has its own row of counts in LDS

// LDS ints rank_in_block needs for S slots: hist[S], and below kPerWaveSlots one more row per wavefront
__host__ __device__ constexpr size_t rank_lds_ints(int S) { return (size_t)S * (S <= kPerWaveSlots ? 1 + kHistWaves : 1); }

// Rank of this thread's assignment among the earlier assignments of the block with the same slot
// (thread order), and the block's rows per slot in hist[S] (LDS, written here).
__device__ __forceinline__ int rank_in_block(int slot, int32_t *hist, int S)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // The lanes of this wavefront with the same slot, found bit by bit of the slot number (a ballot per
    // bit, each lane keeping the side it is on); from that mask the rank among the earlier lanes and
    // whether a later lane has the slot too.
    unsigned long long peers = __ballot(slot >= 0);
    for (int b = 0; (S - 1) >> b; ++b) {
        const bool bit = (slot >> b) & 1;
        const unsigned long long ones = __ballot(bit);
        peers &= bit ? ones : ~ones;
    }
    const int rank0 = __popcll(peers & ((1ull << lane) - 1ull));
    int rank = slot >= 0 ? rank0 : 0;
    const bool last = ((peers >> lane) >> 1) == 0ull;
    if (S <= kPerWaveSlots) {
        // every wavefront leaves its rows per slot in its own row of counts (the last lane of a slot
        // knows the total), then the rows are turned into running sums over the wavefronts
        int32_t *cnt = hist + S;                      // [kHistWaves][S]
        for (int i = tid; i < kHistWaves * S; i += kHistThreads) cnt[i] = 0;
        __syncthreads();
        if (slot >= 0 && last) cnt[wave * S + slot] = rank + 1;
        __syncthreads();
        for (int s = tid; s < S; s += kHistThreads) {
            int run = 0;
#pragma unroll
            for (int w = 0; w < kHistWaves; ++w) {
                const int c = cnt[w * S + s];
                cnt[w * S + s] = run;
                run += c;
            }
            hist[s] = run;
        }
        __syncthreads();
        if (slot >= 0) rank += cnt[wave * S + slot];
        return rank;
    }
    for (int s = tid; s < S; s += kHistThreads) hist[s] = 0;
    __syncthreads();
    // wavefronts take turns in order: read the slot's running count, then add this wavefront's rows
    for (int w = 0; w < kHistWaves; ++w) {
        if (wave == w && slot >= 0) {
            rank += hist[slot];
        }
        __syncthreads();
        if (wave == w && slot >= 0) atomicAdd(&hist[slot], 1);
        __syncthreads();
    }
    return rank;
}

// A block's word per slot: rows of the slot in the block (<= 1024) in the low 16 bits, and above them
// the thread (= assignment of the block) that is the block's first for the slot.
__global__ __launch_bounds__(kHistThreads) void k_slot_hist(Pass p)
{
    extern __shared__ int32_t hist[];   // [S] rows per slot seen so far in this block, the ranking's rows, then first[S]
    const int tid = threadIdx.x;
    const int a = blockIdx.x * kHistThreads + tid;
    const int slot = slot_of(p, a);
    const int rank = rank_in_block(slot, hist, p.S);
    int32_t *first = hist + rank_lds_ints(p.S);
    if (slot >= 0 && rank == 0) first[slot] = tid;     // one writer per slot with rows; slots without rows are not read
    if (a < p.T * p.kk) p.slot_rank[a] = slot >= 0 ? ((slot << 12) | rank) : -1;
    __syncthreads();
    for (int s = tid; s < p.S; s += kHistThreads) {
        const int c = hist[s];
        p.blk_hist[(size_t)blockIdx.x * p.S + s] = c ? (c | (first[s] << 16)) : 0;
    }
}

// exclusive scan of v over the NT threads of the block (v is per-thread), returns the
// exclusive prefix; *total receives the block sum.  scratch: NT/64 ints of LDS.
template <int NT = kThreads>
__device__ __forceinline__ int block_exclusive_scan(int v, int32_t *scratch, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int o = __shfl_up(incl, off, 64);
        if (lane >= off) incl += o;
    }
    if (lane == 63) scratch[wave] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
        int s = scratch[w];
        if (w < wave) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + incl - v;
}

// The M-tiles of one slot: its c rows split into nt nearly equal chunks (multiples of 32 rows, or of
// tile_rows when that is smaller) so that no chunk is a sliver.
__device__ __forceinline__ void emit_tiles(const Pass &p, int s, int c, int nt, int row_off, int tile_off, int tile_rows, MTile *dst)
{
    const int gran = tile_rows < 32 ? tile_rows : 32;
    const int per = nt ? min(tile_rows, ((c + nt - 1) / nt + gran - 1) / gran * gran) : 0;
    for (int i = 0; i < nt; ++i) {
        const int idx = tile_off + i;
        if (idx < p.max_tiles) {
            MTile mt;
            mt.slot = s;
            mt.row_begin = row_off + i * per;
            mt.rows = max(0, min(per, c - i * per));
            mt.single = nt == 1;
            dst[idx] = mt;
        }
    }
}

constexpr int kSortMax = 2048;   // tile lists up to this long can be ordered by size (staged in LDS)
constexpr int kSizeBins = 12;    // size classes: 32-row token tiles of a chunk, capped

constexpr int kMaxSlots = 2048;  // n_slots <= 2047

// exclusive scan of a 64-bit value over the NT threads of the block (two 32-bit counters side by side)
template <int NT>
__device__ __forceinline__ unsigned long long block_exclusive_scan_u64(unsigned long long v, unsigned long long *scratch, unsigned long long *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const unsigned long long o = __shfl_up(incl, off, 64);
        if (lane >= off) incl += o;
    }
    if (lane == 63) scratch[wave] = incl;
    __syncthreads();
    unsigned long long base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
        const unsigned long long x = scratch[w];
        if (w < wave) base += x;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return base + incl - v;
}

// Rows per slot, row offsets and the M-tile list, written by one workgroup of NT threads from
//   cnt[s]   (LDS) rows per slot
//   fkey[s]  (LDS) first assignment of the slot's group, INT_MAX without rows
// staging: the tile list is left ordered by size class, largest first (longest-processing-time-first:
// the tail of a launch that is only a few rounds of the chip deep then consists of the cheapest
// tiles), and within a class by the FIRST ASSIGNMENT of the slot's group (the lowest token-and-position
// that was routed to it), chunks of a group in row order.  Neither key depends on which slot a group's
// expert sits in, so the order -- and with it which tiles the large-tile kernels run in their split
// last round -- is the same under every placement of the same experts.  Otherwise: slot order.
// The keys are all different, so a tile's place in the order is the number of tiles with a smaller key:
// counted directly (n^2 / NT comparisons per thread out of LDS, n <= kSortMax and a few hundred in
// practice), which is one pass instead of the chain of scans a counting sort needs.
template <int NT>
__device__ void offsets_and_tiles(const Pass &p, int tile_rows, bool staging, const int32_t *cnt, const int32_t *fkey)
{
    __shared__ unsigned long long scratch[NT / 64];
    __shared__ MTile staged[kSortMax];
    __shared__ unsigned long long skey[kSortMax];
    __shared__ int32_t scratch_pos[NT];      // places of the tiles of a short list (fewer than NT tiles)
    const int tid = threadIdx.x;
    const int S = p.S;
    // one scan over the slots for both offsets: rows in the high half, tiles in the low half
    unsigned long long carry = 0;
    for (int s0 = 0; s0 < S; s0 += NT) {
        const int s = s0 + tid;
        const int c = s < S ? cnt[s] : 0;
        const int nt = (c + tile_rows - 1) / tile_rows;
        unsigned long long tot;
        const unsigned long long off = carry + block_exclusive_scan_u64<NT>(((unsigned long long)c << 32) | (unsigned)nt, scratch, &tot);
        if (s < S) {
            const int row_off = (int)(off >> 32), tile_off = (int)(off & 0xffffffffu);
            p.counts[s] = c;
            p.offs[s] = row_off;
            emit_tiles(p, s, c, nt, row_off, tile_off, tile_rows, staging ? staged : p.tiles);
            if (staging) {
                const int gran = tile_rows < 32 ? tile_rows : 32;
                const int per = nt ? min(tile_rows, ((c + nt - 1) / nt + gran - 1) / gran * gran) : 0;
                for (int i = 0; i < nt && tile_off + i < p.max_tiles; ++i) {
                    const int rows = max(0, min(per, c - i * per));
                    const int cls = min(kSizeBins - 1, (rows + 31) >> 5);
                    skey[tile_off + i] = ((unsigned long long)(kSizeBins - 1 - cls) << 48) | ((unsigned long long)(unsigned)fkey[s] << 16) | (unsigned)i;
                }
            }
        }
        carry += tot;
    }
    const int n_rows = (int)(carry >> 32);
    const int n = min((int)(carry & 0xffffffffu), p.max_tiles);
    if (tid == 0) {
        p.offs[S] = n_rows;
        *p.n_tiles = n;
    }
    if (!staging) return;
    __syncthreads();
    // a short list is shared out over all threads: `parts` threads per tile, each counting a range of the others
    const int parts = n > 0 && n < NT ? NT / n : 1;
    if (parts > 1) {
        int32_t *pos = (int32_t *)scratch_pos;
        for (int i = tid; i < n; i += NT) pos[i] = 0;
        __syncthreads();
        const int i = tid % n, part = tid / n;
        if (part < parts) {
            const int per = (n + parts - 1) / parts, j0 = part * per, j1 = min(n, j0 + per);
            const unsigned long long mine = skey[i];
            int cntl = 0;
            int j = j0;
            for (; j + 8 <= j1; j += 8) {
                unsigned long long k[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) k[u] = skey[j + u];
#pragma unroll
                for (int u = 0; u < 8; ++u) cntl += k[u] < mine;
            }
            for (; j < j1; ++j) cntl += skey[j] < mine;
            atomicAdd(&pos[i], cntl);
        }
        __syncthreads();
        for (int i2 = tid; i2 < n; i2 += NT) p.tiles[pos[i2]] = staged[i2];
        return;
    }
    for (int i = tid; i < n; i += NT) {
        const unsigned long long mine = skey[i];
        int pos = 0;
        int j = 0;
        for (; j + 8 <= n; j += 8) {
            unsigned long long k[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) k[u] = skey[j + u];
#pragma unroll
            for (int u = 0; u < 8; ++u) pos += k[u] < mine;
        }
        for (; j < n; ++j) pos += skey[j] < mine;
        p.tiles[pos] = staged[i];
    }
}

// sort_tiles != 0: a size-ordered tile list (lists longer than kSortMax stay in slot order).
__global__ __launch_bounds__(kThreads) void k_slot_scan(Pass p, int n_blocks, int tile_rows, int sort_tiles)
{
    __shared__ int32_t fkey[kMaxSlots];      // first assignment of the slot's group (INT_MAX: no rows)
    __shared__ int32_t cnt[kMaxSlots];       // rows per slot
    const int tid = threadIdx.x;
    const int S = p.S;
    // per slot: running sum over blocks (blk_hist becomes the block's exclusive base)
    for (int s = tid; s < S; s += kThreads) {
        int run = 0, key = 0x7fffffff;
        for (int b0 = 0; b0 < n_blocks; b0 += 16) {   // 16 loads in flight, then their running sum
            int c[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) c[i] = b0 + i < n_blocks ? p.blk_hist[(size_t)(b0 + i) * S + s] : 0;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (b0 + i < n_blocks) p.blk_hist[(size_t)(b0 + i) * S + s] = run;
                if (c[i] && key == 0x7fffffff) key = (b0 + i) * kAssignPerBlock + (c[i] >> 16);
                run += c[i] & 0xffff;
            }
        }
        cnt[s] = run;
        fkey[s] = key;
    }
    __syncthreads();
    offsets_and_tiles<kThreads>(p, tile_rows, sort_tiles && p.max_tiles <= kSortMax, cnt, fkey);
}

// Second and last kernel of the fused bookkeeping (after k_gate_select_hist).  Workgroup b < n_blocks
// places the assignments of tokens [16 b, 16 b + 16); workgroup n_blocks writes counts, offsets and the
// tile list.  Nobody waits for anybody: every workgroup adds up, for itself, the block masks of all
// slots (a wavefront per slot, 64 blocks per load, wavefront reductions) -- rows per slot in the whole
// pass and in the blocks before its own -- and scans the totals; at most 512 blocks x S words, out of L2.
// 64 registers at most: two workgroups of 16 wavefronts per compute unit, so that all workgroups of a pass of up to 8192
// tokens run at once (the tile list's workgroup is the last one of the grid)
__global__ __launch_bounds__(kFusedTokens * 64) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_scan_place(Pass p, int n_blocks, int tile_rows, int sort_tiles)
{
    constexpr int NT = kFusedTokens * 64;
    __shared__ int32_t total[kMaxSlots];   // rows per slot, then (placing workgroups) the slot's first row
    __shared__ int32_t base[kMaxSlots];    // rows of the slot in earlier blocks; the tile workgroup: the group's first-assignment key
    __shared__ int32_t scratch[NT / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = p.S, b = blockIdx.x;
    const bool tiles_wg = b == n_blocks;
    // Every workgroup of the launch adds up the rows per (slot, block) of the whole pass, so this loop is the
    // kernel.  The counts are bytes (at most 16 rows of a slot per block), blk_cnt [S][row_stride]: a quarter
    // wavefront owns a slot (four slots per wavefront and round), lane `sub` of the 16 the bytes of blocks
    // [sub lb, (sub + 1) lb); four counts are added by one v_sad_u8, the 16 partial sums meet in four row-wise
    // DPP steps -- for the four slots at once.  The next round's loads are issued before this round is counted.
    const int row_stride = fused_row_stride(n_blocks);     // bytes; a multiple of 64, blocks past n_blocks hold nothing defined
    const int lb = row_stride >> 4;                        // blocks (bytes) per lane: 4, 8, ... 32
    const int nw = lb >> 2;                                // words per lane: 1 .. 8
    const int sub = lane & 15, qrow = lane >> 4;
    // byte masks of this lane's words: blocks that exist, blocks before this workgroup's
    uint32_t mv[8], mb[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        mv[i] = mb[i] = 0u;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int blk = sub * lb + 4 * i + e;
            if (blk < n_blocks) mv[i] |= 0xffu << (8 * e);
            if (blk < b) mb[i] |= 0xffu << (8 * e);        // b <= n_blocks
        }
    }
    auto load_row = [&](int s0, uint32_t (&v)[8]) {
        const uint32_t *row = (const uint32_t *)(p.blk_cnt + (size_t)min(s0 + qrow, S - 1) * row_stride + sub * lb);
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (i < nw) v[i] = row[i];                     // uniform condition
    };
    uint32_t cur[8], nxt[8];
    if (wave * 4 < S) load_row(wave * 4, cur);
    for (int s0 = wave * 4; s0 < S; s0 += 4 * (NT / 64)) {
        const int s = s0 + qrow;
        const bool more = s0 + 4 * (NT / 64) < S;
        if (more) load_row(s0 + 4 * (NT / 64), nxt);
        uint32_t tot = 0u, before = 0u;
        int first = 0x7fffffff;                            // first block of this lane's with a row of the slot
#pragma unroll
        for (int i = 7; i >= 0; --i) {
            if (i >= nw) continue;                         // uniform
            const uint32_t w = cur[i] & mv[i];
            tot = __builtin_amdgcn_sad_u8(w, 0u, tot);
            before = __builtin_amdgcn_sad_u8(w & mb[i], 0u, before);
            if (tiles_wg && w) first = sub * lb + 4 * i + ((__ffs(w) - 1) >> 3);
        }
        // at most 8192 rows per slot on either side: no carry between the halves
        int both = (int)(tot | (before << 16));
#define STEP(CTRL) both += dpp_i32<CTRL, 0xf>(0, both);
        STEP(0x111) STEP(0x112) STEP(0x114) STEP(0x118)    // row_shr 1, 2, 4, 8: lane 15 of the row has the sum
#undef STEP
        if (tiles_wg) {
#define STEP(CTRL) { const int o = dpp_i32<CTRL, 0xf>(0x7fffffff, first); first = o < first ? o : first; }
            STEP(0x111) STEP(0x112) STEP(0x114) STEP(0x118)
#undef STEP
        }
        if (sub == 15 && s < S) {
            total[s] = both & 0xffff;
            int v = both >> 16;
            if (tiles_wg) {
                // the group's first assignment: its first block with a row, that block's lowest token, that row's position
                v = 0x7fffffff;
                if (first != 0x7fffffff) {
                    const uint32_t m = (uint32_t)p.blk_hist[(size_t)s * row_stride + first];
                    v = (((first * kFusedTokens + (__ffs(m & 0xffffu) - 1)) << 6) | (int)(m >> 16));
                }
            }
            base[s] = v;
        }
        if (more) {
#pragma unroll
            for (int i = 0; i < 8; ++i) cur[i] = nxt[i];
        }
    }
    __syncthreads();
    if (tiles_wg) {
        // four wavefronts carry on (the barriers below count the wavefronts still running): that keeps the
        // kernel's LDS at two workgroups per compute unit, so that the placing workgroups all run at once
        if (tid >= kThreads) return;
        offsets_and_tiles<kThreads>(p, tile_rows, sort_tiles && p.max_tiles <= kSortMax, total, base);
        return;
    }
    // exclusive scan of the totals: total[s] becomes the first grouped row of slot s
    int carry = 0;
    for (int s0 = 0; s0 < S; s0 += NT) {
        const int s = s0 + tid;
        const int c = s < S ? total[s] : 0;
        int tot;
        const int off = carry + block_exclusive_scan<NT>(c, scratch, &tot);
        if (s < S) total[s] = off;
        carry += tot;
    }
    __syncthreads();
    if (tid < kFusedTokens * p.kk) {
        const int t = b * kFusedTokens + tid / p.kk;
        if (t < p.T) {
            const int a = t * p.kk + tid % p.kk;
            const int sr = p.slot_rank[a];
            int row = -1;
            if (sr >= 0) {
                const int slot = sr >> 12, rank = sr & 0xfff;
                row = total[slot] + base[slot] + rank;
                p.perm[row] = t;
            }
            p.inv[a] = row;
        }
    }
}

__global__ __launch_bounds__(kThreads) void k_slot_place(Pass p)
{
    const int a = blockIdx.x * kThreads + threadIdx.x;
    if (a >= p.T * p.kk) return;
    const int sr = p.slot_rank[a];
    int row = -1;
    if (sr >= 0) {
        const int slot = sr >> 12, rank = sr & 0xfff;
        row = p.offs[slot] + p.blk_hist[(size_t)(a / kAssignPerBlock) * p.S + slot] + rank;
        p.perm[row] = a / p.kk;
    }
    p.inv[a] = row;
}

// The three steps in one workgroup, for passes with at most kAssignPerBlock assignments (decode-sized
// batches, where three launches cost more than the work): slot and in-block rank of every
// assignment, scan over the slots (offsets and tile list, kept in LDS for the placement), placement.
__global__ __launch_bounds__(kHistThreads) void k_permute_one_block(Pass p, int tile_rows)
{
    extern __shared__ int32_t sm[];     // the ranking's counts (hist[S] first), then offs[S]
    __shared__ int32_t scratch[kHistThreads / 64];
    const int S = p.S, tid = threadIdx.x;
    int32_t *hist = sm, *offs = sm + rank_lds_ints(S);
    const int slot = slot_of(p, tid);
    const int rank = rank_in_block(slot, hist, S);
    int row_carry = 0, tile_carry = 0;
    for (int s0 = 0; s0 < S; s0 += kHistThreads) {
        const int s = s0 + tid;
        const int c = s < S ? hist[s] : 0;
        const int nt = (c + tile_rows - 1) / tile_rows;
        int row_tot, tile_tot;
        const int row_off = row_carry + block_exclusive_scan<kHistThreads>(c, scratch, &row_tot);
        const int tile_off = tile_carry + block_exclusive_scan<kHistThreads>(nt, scratch, &tile_tot);
        if (s < S) {
            p.counts[s] = c;
            p.offs[s] = row_off;
            offs[s] = row_off;
            emit_tiles(p, s, c, nt, row_off, tile_off, tile_rows, p.tiles);
        }
        row_carry += row_tot;
        tile_carry += tile_tot;
    }
    if (tid == 0) {
        p.offs[S] = row_carry;
        *p.n_tiles = min(tile_carry, p.max_tiles);
    }
    __syncthreads();
    if (tid < p.T * p.kk) {
        int row = -1;
        if (slot >= 0) {
            row = offs[slot] + rank;
            p.perm[row] = tid / p.kk;
        }
        p.inv[tid] = row;
    }
}

}  // namespace

hipError_t launch_permute(const Pass &p, int tile_rows, bool sort_tiles, hipStream_t st)
{
    if (p.fused_hist) {   // the selection kernel has ranked the assignments already
        const int nb = (p.T + kFusedTokens - 1) / kFusedTokens;
        hipLaunchKernelGGL(k_scan_place, dim3(nb + 1), dim3(kFusedTokens * 64), 0, st, p, nb, tile_rows, sort_tiles ? 1 : 0);
        return hipGetLastError();
    }
    const int n_assign = p.T * p.kk;
    const int nb = (n_assign + kAssignPerBlock - 1) / kAssignPerBlock;   // histogram blocks
    const int nbp = (n_assign + kThreads - 1) / kThreads;                 // placement blocks
    const size_t one_block_lds = sizeof(int32_t) * (rank_lds_ints(p.S) + p.S);
    if (nb == 1 && !sort_tiles && one_block_lds <= 48 * 1024) {
        hipLaunchKernelGGL(k_permute_one_block, dim3(1), dim3(kHistThreads), one_block_lds, st, p, tile_rows);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(k_slot_hist, dim3(nb), dim3(kHistThreads), sizeof(int32_t) * (rank_lds_ints(p.S) + p.S), st, p);
    hipLaunchKernelGGL(k_slot_scan, dim3(1), dim3(kThreads), 0, st, p, nb, tile_rows, sort_tiles ? 1 : 0);
    hipLaunchKernelGGL(k_slot_place, dim3(nbp), dim3(kThreads), 0, st, p);
    return hipGetLastError();
}

}  // namespace emoe
