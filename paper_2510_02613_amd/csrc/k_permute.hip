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

// Units of one GEMM in list order: the tile at place q of the order, run r -> unit q runs + r (unit u works for
// XCD u mod 8).  `threads` threads starting at `first` take part.  src: the tiles; order[q]: index in src of the
// tile at place q (NULL: src is in order already).
__device__ void deal_units(const Pass &p, const MTile *src, const int32_t *order, int n, int which, int first, int threads)
{
    const int t = (int)threadIdx.x - first;
    const int ns = p.n_slices[which];
    const int runs = mfma8_runs(n, ns), spp = ns / runs;
    MUnit *units = p.units[which];
    const int n_units = min((n * runs + 7) / 8 * 8, p.unit_cap);
    for (int at = t; at < n * runs && at < p.unit_cap; at += threads) {
        const int q = at / runs, r = at - q * runs;
        const MTile mt = src[order ? order[q] : q];
        MUnit u;
        u.slot = mt.slot; u.row_begin = mt.row_begin; u.rows = mt.rows;
        u.info = ((r * spp) << 1) | (mt.single & 1);
        units[at] = u;
    }
    for (int at = n * runs + t; at < n_units; at += threads) {
        MUnit u;
        u.slot = 0; u.row_begin = 0; u.rows = 0; u.info = 0;
        units[at] = u;
    }
    if (t == 0) {
        UnitHdr h;
        h.n_rows = n_units / 8 * spp; h.spp = spp; h.n_units = n_units; h.runs = runs;
        p.unit_hdr[which] = h;
    }
}
template <int NT>
__device__ void deal_units_in_order(const Pass &p, const MTile *src, const int32_t *order, int n)
{
    deal_units(p, src, order, n, 0, 0, NT);
    deal_units(p, src, order, n, 1, 0, NT);
}
// exclusive scan of a 64-bit value over one HALF of the block's NT threads (threads [0, NT/2) and [NT/2, NT) scan
// separately, both halves call it together); scratch: NT/64 entries
template <int NT>
__device__ __forceinline__ unsigned long long half_exclusive_scan_u64(unsigned long long v, unsigned long long *scratch, unsigned long long *total)
{
    constexpr int HW = NT / 128;                            // wavefronts per half
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = wave / HW;
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
    for (int w = 0; w < HW; ++w) {
        const unsigned long long x = scratch[half * HW + w];
        if (half * HW + w < wave) base += x;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return base + incl - v;
}

// Units of both GEMMs with the tiles of a slot kept on one XCD (see offsets_and_tiles); all NT threads call it:
// the first half of them deals GEMM-1's units, the second half GEMM-2's, side by side.
//   src, order   the tiles and the order (order[q]: index in src of the tile at place q)
//   gq0[g]       first place of group g of ng (maximal runs of one slot in the order)
//   tmp          kSortMax ints of LDS (the pieces, a half per GEMM), scratch: the scans'
// A GEMM falls back to the plain deal (unit q runs + r to XCD u mod 8) when its pieces do not fit tmp or a column
// would outgrow what the launch provides.
template <int NT>
__device__ void deal_units_grouped(const Pass &p, const MTile *src, const int32_t *order, const int32_t *gq0,
                                   int ng, int n, int32_t *tmp_all, unsigned long long *scratch)
{
    constexpr int HT = NT / 2;
    __shared__ int32_t colF_all[2][8];   // units at the head of every column that belong to pieces
    __shared__ int32_t colC_all[2][8];   // whole single tiles a column has room for on top of them
    const int which = (int)threadIdx.x / HT, t = (int)threadIdx.x % HT;
    int32_t *tmp = tmp_all + which * (kSortMax / 2);
    int32_t *colF = colF_all[which];
    int32_t *cap = colC_all[which];
    const int ns = p.n_slices[which];
    const int runs = mfma8_runs(n, ns), spp = ns / runs;
    const int total = n * runs;
    const int target = (total + 7) / 8, limit = target + kUnitSlack;
    const int pm = max(2, target / 2);                     // largest piece
    MUnit *units = p.units[which];
    if (t < 8) colF[t] = 0;
    const bool ok = total <= kSortMax / 2 && runs <= 64;
    // pieces and single tiles per group -> each group's start in the two numberings (one scan, two counters)
    auto shape = [&](int g, int &m, int &np, int &singles) {
        m = (g + 1 < ng ? gq0[g + 1] : n) - gq0[g];
        np = 0; singles = 0;
        if (m == 1) { singles = 1; }
        else {
            np = (m + pm - 1) / pm;
            if (m - (np - 1) * pm == 1) { --np; singles = 1; }   // a last piece of one tile is a single tile
        }
    };
    unsigned long long carry = 0;
    for (int g0 = 0; g0 < ng; g0 += HT) {
        const int g = g0 + t;
        int m = 0, np = 0, singles = 0;
        if (g < ng) shape(g, m, np, singles);
        unsigned long long tot;
        const unsigned long long at = carry + half_exclusive_scan_u64<NT>(((unsigned long long)(np * runs) << 32) | (unsigned)(singles * runs), scratch, &tot);
        if (g < ng && ok) {
            const int k0 = (int)(at >> 32);
            for (int pi = 0; pi < np; ++pi) {
                const int size = min(pm, m - pi * pm);
                for (int r = 0; r < runs; ++r)              // first place in the order (11 bits) | tiles (11) | run (6)
                    tmp[k0 + pi * runs + r] = (gq0[g] + pi * pm) | (size << 11) | (r << 22);
            }
            // the group's single tile starts at this number among the single units (kept for the second pass)
        }
        carry += tot;
    }
    const int P = (int)(carry >> 32);
    int R = (int)(carry & 0xffffffffu);                     // single units (later: those dealt unit by unit)
    __syncthreads();
    // piece k sits in column k mod 8 behind the earlier pieces of that column
    if (ok) {
        for (int k = t; k < P; k += HT) {
            if (k + 8 >= P) {                                // the last piece of its column knows the column's length
                int at = 0;
                for (int j = k & 7; j < k; j += 8) at += (tmp[j] >> 11) & 0x7ff;
                colF[k & 7] = at + ((tmp[k] >> 11) & 0x7ff);
            }
        }
    }
    __syncthreads();
    int F[8], Fmax = 0;
#pragma unroll
    for (int x = 0; x < 8; ++x) { F[x] = colF[x]; Fmax = max(Fmax, F[x]); }
    const bool grouped = ok && Fmax <= limit;               // uniform over the half
    // Single tiles come in `runs` units each.  As long as whole tiles fit under the even column height, a tile's
    // runs stay in ONE column, one behind the other (its token rows are then fetched by one XCD): tile j of the
    // first NA single tiles goes to block level k -- the k-th tile on top of a column's pieces -- of the columns
    // that have room for it, level by level; what is left of the single tiles is dealt unit by unit as before.
    int capsum = 0, capmax = 0;
    {
        int U = R;
#pragma unroll
        for (int x = 0; x < 8; ++x) U += F[x];
        const int even = U / 8;
        if (t < 8) cap[t] = runs > 1 ? max(0, (even - colF[t]) / runs) : 0;   // kept in LDS: registers are scarce here
        __syncthreads();
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            capsum += cap[x];
            capmax = max(capmax, cap[x]);
        }
    }
    const int NA = min(R / runs, capsum);                   // single tiles kept whole
    auto belowA = [&](int k) { int c = 0;
#pragma unroll
        for (int x = 0; x < 8; ++x) c += min(cap[x], k);
        return c; };
    auto levelA = [&](int j) {                              // the largest k with belowA(k) <= j  (j < capsum)
        int lo = 0, hi = capmax + 1;
        while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (belowA(mid) <= j) lo = mid; else hi = mid; }
        return lo; };
    if (NA > 0) {                                           // column heights with the whole tiles on top of the pieces
        const int kL = levelA(NA - 1), lastn = NA - belowA(kL);
        int rank = 0;
        Fmax = 0;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            int used = min(cap[x], kL);
            if (cap[x] > kL) { if (rank < lastn) ++used; ++rank; }
            F[x] += used * runs;
            Fmax = max(Fmax, F[x]);
        }
    }
    R -= NA * runs;                                         // the single units that are dealt one by one
    // level of single unit i: the largest l with C(l) <= i, C(l) = sum over columns of max(0, l - F[x]) = single units below level l
    auto below = [&](int l) { int c = 0;
#pragma unroll
        for (int x = 0; x < 8; ++x) c += max(0, l - F[x]);
        return c; };
    auto level_of = [&](int i) {
        int lo = 0, hi = Fmax + (R + 7) / 8 + 1;               // C(lo) = 0 <= i < C(hi)
        while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (below(mid) <= i) lo = mid; else hi = mid; }
        return lo; };
    auto put = [&](int row, int x, const MTile &tl, int r) {
        MUnit u;
        u.slot = tl.slot; u.row_begin = tl.row_begin; u.rows = tl.rows;
        u.info = ((r * spp) << 1) | (tl.single & 1);
        units[(size_t)row * 8 + x] = u;
    };
    if (grouped) {
        for (int k = t; k < P; k += HT) {
            int at = 0;
            for (int j = k & 7; j < k; j += 8) at += (tmp[j] >> 11) & 0x7ff;
            const int w = tmp[k], q = w & 0x7ff, size = (w >> 11) & 0x7ff, r = (w >> 22) & 0x3f;
            for (int i = 0; i < size; ++i) put(at + i, k & 7, src[order[q + i]], r);
        }
        // column x ends where its single units end: one per level from F[x] to the last level, which only the
        // first `last_n` of the columns that reach it take part in
        const int l_last = R ? level_of(R - 1) : -1;
        const int last_n = R ? R - below(l_last) : 0;
        const int rows_used = R ? max(Fmax, l_last + 1) : Fmax;
        if (t < 8) {
            int fill = F[0];
#pragma unroll
            for (int x = 1; x < 8; ++x) if (t == x) fill = F[x];
            if (R && fill <= l_last) {
                int before = 0;
#pragma unroll
                for (int y = 0; y < 8; ++y) before += (y < t && F[y] <= l_last);
                fill = before < last_n ? l_last + 1 : l_last;
            }
            for (int row = fill; row < rows_used; ++row) {   // holes
                MUnit u;
                u.slot = 0; u.row_begin = 0; u.rows = 0; u.info = 0;
                units[(size_t)row * 8 + t] = u;
            }
        }
        if (t == 0) {
            UnitHdr h;
            h.n_rows = rows_used * spp; h.spp = spp; h.n_units = rows_used * 8; h.runs = runs;
            p.unit_hdr[which] = h;
        }
    }
    // single units, numbered group by group in the order (a group has at most one single tile), run by run
    unsigned long long carry2 = 0;
    for (int g0 = 0; g0 < ng; g0 += HT) {
        const int g = g0 + t;
        int m = 0, np = 0, has = 0;
        if (g < ng) shape(g, m, np, has);
        unsigned long long tot;
        const int i0 = (int)(carry2 + half_exclusive_scan_u64<NT>((unsigned long long)(has * runs), scratch, &tot));
        if (has && grouped) {
            const MTile tl = src[order[gq0[g] + m - 1]];      // the group's last tile
            const int j = i0 / runs;                         // its number among the single tiles
            if (j < NA) {                                    // whole: block level k of the rank-th column that reaches it
                const int k = levelA(j), rank = j - belowA(k);
                int x = 0, base = 0;
#pragma unroll
                for (int xx = 7; xx >= 0; --xx) {
                    int before = 0;
#pragma unroll
                    for (int y = 0; y < 8; ++y) before += (y < xx && cap[y] > k);
                    if (cap[xx] > k && before == rank) { x = xx; base = colF[xx]; }   // the column's pieces end there
                }
                for (int r = 0; r < runs; ++r) put(base + k * runs + r, x, tl, r);
            } else
            for (int r = 0; r < runs; ++r) {
                const int i = i0 - NA * runs + r, l = level_of(i);
                const int rank = i - below(l);
                int x = 0;
#pragma unroll
                for (int xx = 7; xx >= 0; --xx) {            // the rank-th column (ascending) that is no longer than l
                    int before = 0;
#pragma unroll
                    for (int y = 0; y < 8; ++y) before += (y < xx && F[y] <= l);
                    if (F[xx] <= l && before == rank) x = xx;
                }
                put(l, x, tl, r);
            }
        }
        carry2 += tot;
    }
    if (!grouped) deal_units(p, src, order, n, which, which * HT, HT);
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
    __shared__ int32_t tpos[kSortMax];       // a tile's place in the order
    __shared__ int32_t any_multi;            // some slot has several tiles
    const int tid = threadIdx.x;
    if (tid == 0) any_multi = 0;
    __syncthreads();
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
            if (nt > 1) any_multi = 1;
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
    __syncthreads();
    const bool multi = any_multi != 0;
    if (!staging) {
        if (p.units[0]) {   // a list too long to order: units straight from the slot-ordered list in global memory
            __threadfence();
            __syncthreads();
            deal_units_in_order<NT>(p, p.tiles, nullptr, n);
        }
        return;
    }
    __syncthreads();
    // a tile's place in the order: a short list is shared out over all threads (`parts` threads per tile,
    // each counting a range of the others)
    for (int i = tid; i < n; i += NT) tpos[i] = 0;
    __syncthreads();
    const int parts = n > 0 && n < NT ? NT / n : 1;
    for (int w = tid; w < n * parts; w += NT) {
        const int i = w % n, part = w / n;
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
        atomicAdd(&tpos[i], cntl);
    }
    __syncthreads();
    for (int i = tid; i < n; i += NT) p.tiles[tpos[i]] = staged[i];
    if (!p.units[0]) return;
    // ---- work units of the large-tile GEMMs ----
    int32_t *inv = (int32_t *)skey;                 // order -> staged index (the keys are no longer needed)
    __syncthreads();
    for (int i = tid; i < n; i += NT) inv[tpos[i]] = i;
    __syncthreads();
    // Keeping a slot's tiles on one XCD costs this workgroup -- the longest of the launch -- several more scans;
    // it pays when a tile's weights are tens of megabytes (measured: hidden x intermediate of 7168 x 2048 gains
    // 5 % in GEMM-2 and 5 % of the fetched bytes, 2048 x 768 gains nothing)
    if (!multi || (long long)p.H * p.I < (4ll << 20)) {
        deal_units_in_order<NT>(p, staged, inv, n);
        return;
    }
    // Some slot has several tiles: their weights are worth fetching once.  The tiles of one slot (of one size
    // class: they sit next to each other in the order) form a group; a group's units go to ONE XCD, one behind
    // the other at the head of that XCD's column, so that they run at the same time and the later ones find the
    // slot's weights in that XCD's L2.  Everything is closed form, no thread walks the list: groups are cut into
    // pieces of at most half a column, piece k goes to XCD k mod 8, and the single tiles then fill the columns up
    // level by level (a tile goes to the shortest columns first), in size order.
    int32_t *gq0 = inv + kSortMax;                  // group -> its first place in the order
    __shared__ int32_t n_groups;
    {   // groups: maximal runs of one slot in the order; compacted by a scan of the run starts
        int carry_g = 0;
        for (int q0 = 0; q0 < n; q0 += NT) {
            const int q = q0 + tid;
            const int start = q < n && (q == 0 || staged[inv[q]].slot != staged[inv[q - 1]].slot) ? 1 : 0;
            unsigned long long tot;
            const int at = carry_g + (int)block_exclusive_scan_u64<NT>((unsigned long long)start, scratch, &tot);
            if (start) gq0[at] = q;
            carry_g += (int)tot;
        }
        if (tid == 0) n_groups = carry_g;
    }
    __syncthreads();
    deal_units_grouped<NT>(p, staged, inv, gq0, n_groups, n, tpos, scratch);
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

// Second and last kernel of the fused bookkeeping (after k_gate_select_hist).  Workgroup 0 writes counts,
// offsets, the tile list and the unit lists; workgroup b + 1, b < n_blocks, places the assignments of tokens
// [16 b, 16 b + 16).  Nobody waits for anybody: every workgroup adds up, for itself, the block masks of all
// slots (a quarter wavefront per slot, row-wise reductions) -- rows per slot in the whole
// pass and in the blocks before its own -- and scans the totals; at most 512 blocks x S words, out of L2.
// 64 registers at most: two workgroups of 16 wavefronts per compute unit, 512 on the chip.  The tile list's
// workgroup is the longest of the launch (2 to 3 times a placing one) and therefore the first of the grid: at
// 8192 tokens the launch has 513 workgroups, and the one that has to wait for a place should be a short one
// (measured at 8192 tokens: the kernel 3 us shorter than with the tile list's workgroup last).
__global__ __launch_bounds__(kFusedTokens * 64) __attribute__((amdgpu_waves_per_eu(8, 8))) void k_scan_place(Pass p, int n_blocks, int tile_rows, int sort_tiles)
{
    constexpr int NT = kFusedTokens * 64;
    __shared__ int32_t total[kMaxSlots];   // rows per slot, then (placing workgroups) the slot's first row
    __shared__ int32_t base[kMaxSlots];    // rows of the slot in earlier blocks; the tile workgroup: the group's first-assignment key
    __shared__ int32_t scratch[NT / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = p.S;
    const bool tiles_wg = blockIdx.x == 0;
    const int b = tiles_wg ? n_blocks : (int)blockIdx.x - 1;
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
