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
            mt.pad = 0;
            dst[idx] = mt;
        }
    }
}

constexpr int kSortMax = 2048;   // tile lists up to this long can be ordered by size (staged in LDS)
constexpr int kSizeBins = 12;    // size classes: 32-row token tiles of a chunk, capped (even, scanned in pairs)

constexpr int kMaxSlots = 2048;  // n_slots <= 2047

// sort_tiles != 0: the tile list is left ordered by size class, largest first (longest-processing-time-
// first: the tail of a launch that is only a few rounds of the chip deep then consists of the
// cheapest tiles), and within a class by the FIRST ASSIGNMENT of the slot's group (the lowest
// token-and-position that was routed to it), chunks of a group in row order.  Neither key depends on
// which slot a group's expert sits in, so the order -- and with it which tiles the large-tile kernels
// run in their split last round -- is the same under every placement of the same experts.  Lists
// longer than kSortMax stay in slot order.
__global__ __launch_bounds__(kThreads) void k_slot_scan(Pass p, int n_blocks, int tile_rows, int sort_tiles)
{
    __shared__ int32_t scratch[8];
    __shared__ MTile staged[kSortMax];
    __shared__ int32_t bin_cnt[kSizeBins][kThreads + 1];
    __shared__ int32_t fkey[kMaxSlots];      // first assignment of the slot's group (INT_MAX: no rows)
    __shared__ int32_t srank[kMaxSlots];     // position of the slot when slots are ordered by fkey
    __shared__ int32_t by_rank[kMaxSlots];   // tiles of the slot at that position, then their exclusive prefix sum
    const bool staging = sort_tiles && p.max_tiles <= kSortMax;
    const int tid = threadIdx.x;
    const int S = p.S;
    // 1. per slot: running sum over blocks (blk_hist becomes the block's exclusive base)
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
        p.counts[s] = run;
        fkey[s] = key;
    }
    __syncthreads();
    // 2. the order tiles are emitted in: slot order, or (size-ordered lists) the order of the groups' first assignments
    if (staging) {
        for (int s = tid; s < S; s += kThreads) {
            const int key = fkey[s];
            int r = 0;
            for (int o = 0; o < S; ++o) {
                const int ko = fkey[o];
                r += (ko < key) || (ko == key && o < s);   // keys of slots with rows are distinct; empty slots follow in slot order
            }
            srank[s] = r;
        }
    } else {
        for (int s = tid; s < S; s += kThreads) srank[s] = s;
    }
    __syncthreads();
    for (int s = tid; s < S; s += kThreads) by_rank[srank[s]] = (p.counts[s] + tile_rows - 1) / tile_rows;
    __syncthreads();
    // 3. exclusive scans in chunks of 256: row offsets over slots, tile offsets over positions
    int row_carry = 0, tile_carry = 0;
    for (int s0 = 0; s0 < S; s0 += kThreads) {
        const int s = s0 + tid;
        const int c = s < S ? p.counts[s] : 0;
        const int nt = s < S ? by_rank[s] : 0;
        int row_tot, tile_tot;
        const int row_off = row_carry + block_exclusive_scan(c, scratch, &row_tot);
        const int tile_off = tile_carry + block_exclusive_scan(nt, scratch, &tile_tot);
        if (s < S) p.offs[s] = row_off;
        __syncthreads();
        if (s < S) by_rank[s] = tile_off;          // position s: first tile of the slot that holds it
        row_carry += row_tot;
        tile_carry += tile_tot;
    }
    if (tid == 0) {
        p.offs[S] = row_carry;
        *p.n_tiles = min(tile_carry, p.max_tiles);
    }
    __syncthreads();
    for (int s = tid; s < S; s += kThreads) {
        const int c = p.counts[s];
        emit_tiles(p, s, c, (c + tile_rows - 1) / tile_rows, p.offs[s], by_rank[srank[s]], tile_rows, staging ? staged : p.tiles);
    }
    if (!staging) return;
    // 4. stable counting sort of the staged list by size class, descending.  Thread t owns the
    // contiguous index range [t*per_thread, (t+1)*per_thread): counts per (class, thread), an
    // exclusive scan over (class descending, thread ascending), then placement in index order.
    __syncthreads();
    const int n = min(tile_carry, p.max_tiles);
    const int per_thread = (n + kThreads - 1) / kThreads;
    const int i0 = min(n, tid * per_thread), i1 = min(n, i0 + per_thread);
    auto size_class = [](int rows) { return min(kSizeBins - 1, (rows + 31) >> 5); };
    int mine[kSizeBins];
#pragma unroll
    for (int b = 0; b < kSizeBins; ++b) mine[b] = 0;
    for (int i = i0; i < i1; ++i) {
        const int c = size_class(staged[i].rows);
#pragma unroll
        for (int b = 0; b < kSizeBins; ++b) mine[b] += (b == c);
    }
    // two classes per scan (16-bit fields: a field's total is at most kSortMax)
    int carry = 0;
#pragma unroll
    for (int b = kSizeBins - 1; b >= 1; b -= 2) {
        int tot;
        const int ex = block_exclusive_scan(mine[b] | (mine[b - 1] << 16), scratch, &tot);
        bin_cnt[b][tid] = carry + (ex & 0xffff);
        carry += tot & 0xffff;
        bin_cnt[b - 1][tid] = carry + (ex >> 16);
        carry += tot >> 16;
    }
    for (int i = i0; i < i1; ++i) {
        const MTile mt = staged[i];
        const int c = size_class(mt.rows);
        p.tiles[bin_cnt[c][tid]++] = mt;
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
