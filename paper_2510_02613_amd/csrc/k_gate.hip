// Gating: logits, scores, (group limited) top-k, renormalised weights.
//
// The paper (Sec. 2.1) only says that a gating function picks a few experts per
// token; the rules implemented here are the two its evaluated model families use:
// softmax over all experts then top-k, and sigmoid scores with group-limited
// top-k (group score = sum of the group's two best), both with optional
// renormalisation over the k selected and a constant scale.
//
// One workgroup owns kTokens tokens.  Phase 1 accumulates their logits in fp32
// (activations and router rows staged through LDS in K-chunks).  Phase 2 gives
// each token to one 64-lane wavefront: scores live in LDS, every arg-max is a
// wavefront reduction over a 64-bit (score, inverted index) key, so ties go to
// the lower index exactly as the ordering rule demands.
#include <type_traits>

#include "moe_internal.h"
#include "wave_ops.h"

namespace emoe {

namespace {

constexpr int kTokens = 8;     // tokens per workgroup
constexpr int kThreads = 256;  // 4 wavefronts
constexpr int kET = 128;       // experts per logit tile
constexpr int kKC = 32;        // K chunk

// Monotone map float -> uint32 (larger float <-> larger integer).
__device__ __forceinline__ uint32_t orderable(float f)
{
    uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// key: larger = better score, and among equal scores the LOWER index
__device__ __forceinline__ unsigned long long make_key(float score, int idx)
{
    return ((unsigned long long)orderable(score) << 32) | (unsigned long long)(0xffffffffu - (uint32_t)idx);
}
__device__ __forceinline__ int key_index(unsigned long long key) { return (int)(0xffffffffu - (uint32_t)(key & 0xffffffffull)); }

// Phase 2 for one token, run by one wavefront.
//   lg   : LDS [E] logits in, scores out
//   cs   : LDS [E] selection scores (biased), destroyed (taken entries -> -inf)
// Returns the expert this lane holds (lane j < k: the j-th selected), which is also written to p.ids.
__device__ int select_token(const Pass &p, int t, float *lg, float *cs, int lane)
{
    const int E = p.E;
    const float NEG = -__builtin_huge_valf();
    // scores
    if (p.gate == MOE_GATE_SOFTMAX_TOPK) {
        float m = NEG;
        for (int e = lane; e < E; e += 64) m = fmaxf(m, lg[e]);
        m = wave_max_f32(m);
        float z = 0.f;
        for (int e = lane; e < E; e += 64) { float v = __expf(lg[e] - m); lg[e] = v; z += v; }   // hardware exp2: ~1e-7 relative, far inside the 1e-5 tie bar
        z = wave_sum_f32(z);
        for (int e = lane; e < E; e += 64) lg[e] = lg[e] / z;
    } else {
        for (int e = lane; e < E; e += 64) lg[e] = __builtin_amdgcn_rcpf(1.f + __expf(-lg[e]));   // hardware exp2 and reciprocal, ~1 ulp each
    }
    for (int e = lane; e < E; e += 64) cs[e] = lg[e] + (p.select_bias ? p.select_bias[e] : 0.f);
    wave_sync();
    // group limiting
    if (p.gate == MOE_GATE_SIGMOID_GROUP_TOPK && p.n_group > 1) {
        const int G = p.n_group, per = E / G;
        // L lanes share a group's experts (L a power of two, G * L <= 64): each finds the two largest
        // of its share, then the pairs are merged across the L lanes -- a group's score is the sum of
        // its two largest selection scores, which does not depend on the order they are found in
        int Lsh = 0;
        while ((2 * G) << Lsh <= 64) ++Lsh;
        const int L = 1 << Lsh;
        const int g = lane >> Lsh, sub = lane & (L - 1);
        float b1 = NEG, b2 = NEG;
        if (g < G) {
            for (int e = g * per + sub; e < (g + 1) * per; e += L) {
                const float v = cs[e];
                if (v > b1) { b2 = b1; b1 = v; } else if (v > b2) { b2 = v; }
            }
        }
        for (int d = 1; d < L; d <<= 1) {
            const float o1 = __shfl_xor(b1, d, 64), o2 = __shfl_xor(b2, d, 64);
            b2 = fmaxf(fminf(b1, o1), fmaxf(b2, o2));
            b1 = fmaxf(b1, o1);
        }
        // every lane of a group now holds the group's score.  The topk_group best groups are kept, the lower
        // index first among equal scores: a group's rank is the number of groups that come before it in that
        // order (the scores of all groups are read lane by lane), and it is kept when its rank is below topk_group
        const uint32_t mine = orderable((per > 1) ? b1 + b2 : b1);
        int rank = 0;
        for (int h = 0; h < G; ++h) {
            const uint32_t other = (uint32_t)__builtin_amdgcn_readlane((int)mine, h << Lsh);
            rank += (other > mine || (other == mine && h < g)) ? 1 : 0;
        }
        const unsigned long long keptmask = __ballot(g < G && rank < p.topk_group);   // bit g L: group g is kept
        const bool pow2 = (per & (per - 1)) == 0;
        const int psh = 31 - __clz(per);
        for (int e = lane; e < E; e += 64) {
            const int ge = pow2 ? e >> psh : e / per;
            if (!((keptmask >> (ge << Lsh)) & 1ull)) cs[e] = NEG;
        }
        wave_sync();
    }
    // top-k by repeated wavefront arg-max
    int my_id = 0;
    float my_s = 0.f;
    bool none = false;         // this lane's selection round found no candidate
    constexpr int kRegs = 8;   // up to 512 experts: the candidates live in registers, entry i of a lane is expert lane + 64 i
    if (E <= 64 * kRegs) {
        // NR = registers in use; the winners' scores are fetched once, after the last round.
        // Candidates are kept as order-preserving 32-bit integers (0 = taken or absent): a round is
        // a 32-bit wavefront maximum, and only when several lanes hold that maximum (equal scores)
        // a second reduction for the lowest expert index among them.
        auto rounds = [&](auto nr) {
            constexpr int NR = decltype(nr)::value;
            uint32_t c[NR];
#pragma unroll
            for (int i = 0; i < NR; ++i) {
                const float v = lane + 64 * i < E ? cs[lane + 64 * i] : NEG;
                c[i] = v != NEG ? orderable(v) : 0u;
            }
            for (int j = 0; j < p.k; ++j) {
                uint32_t best = 0u;
                int bi = 0;
#pragma unroll
                for (int i = 0; i < NR; ++i)
                    if (c[i] > best) { best = c[i]; bi = i; }    // strict: the lowest index among a lane's equal scores
                const uint32_t m = wave_max_u32(best);
                const unsigned long long holders = __ballot(best == m && m != 0u);
                int win;
                if (__popcll(holders) == 1) {
                    const int src = __ffsll((long long)holders) - 1;
                    win = src + 64 * __builtin_amdgcn_readlane(bi, src);
                } else {
                    win = wave_min_i32(best == m && m != 0u ? lane + 64 * bi : 0x7fffffff);
                    if (win == 0x7fffffff) win = -1;             // no candidate left
                }
                // fewer than k candidates (non-finite biases or activations): the slot keeps id 0 with
                // weight 0 (my_s is only fetched for a real winner), so that nothing is indexed by -1
                if (lane == j) { my_id = win < 0 ? 0 : win; none = win < 0; }
#pragma unroll
                for (int i = 0; i < NR; ++i)
                    if (lane + 64 * i == win) c[i] = 0u;
            }
        };
        if (E <= 128)      rounds(std::integral_constant<int, 2>{});
        else if (E <= 256) rounds(std::integral_constant<int, 4>{});
        else               rounds(std::integral_constant<int, kRegs>{});
        if (lane < p.k) my_s = none ? 0.f : lg[my_id];
    } else {
        for (int j = 0; j < p.k; ++j) {
            unsigned long long key = 0ull;
            for (int e = lane; e < E; e += 64) {
                float v = cs[e];
                if (v != NEG) { unsigned long long kk = make_key(v, e); key = kk > key ? kk : key; }
            }
            key = wave_max_u64(key);
            if (key == 0ull) continue;                     // no candidate left: id 0, weight 0 (wave-uniform)
            int win = key_index(key);
            if (lane == j) { my_id = win; my_s = lg[win]; }
            if (lane == (win & 63)) cs[win] = NEG;
            wave_sync();
        }
    }
    float sum = wave_sum_f32(lane < p.k ? my_s : 0.f);
    if (lane < p.k) {
        float wv = p.renormalize ? my_s / sum : my_s;
        p.ids[(size_t)t * p.k + lane] = my_id;
        p.w[(size_t)t * p.k + lane] = wv * p.routed_scale;
    }
    return my_id;
}

template <typename XT, typename WT>
__global__ __launch_bounds__(kThreads) void k_gate(Pass p)
{
    extern __shared__ float smem[];
    float *xs = smem;                        // [kTokens][kKC]
    float *ws = xs + kTokens * kKC;          // [kET][kKC+1]
    float *lg = ws + kET * (kKC + 1);        // [kTokens][E]
    float *cs = lg + kTokens * p.E;          // [4 waves][E]

    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * kTokens;
    const XT *x = (const XT *)p.x;
    const WT *wr = (const WT *)p.router_w;
    const int H = p.H, E = p.E;

    // phase 1: logits.  thread -> expert (tid % 128) of the tile, tokens (tid / 128) * 4 .. +4
    const int el = tid & (kET - 1);
    const int th = (tid >> 7) * (kTokens / 2);
    for (int e0 = 0; e0 < E; e0 += kET) {
        float acc[kTokens / 2];
#pragma unroll
        for (int i = 0; i < kTokens / 2; ++i) acc[i] = 0.f;
        for (int k0 = 0; k0 < H; k0 += kKC) {
            __syncthreads();
            {   // stage x chunk: kTokens*kKC = 256 values, one per thread
                int tt = tid / kKC, kc = tid % kKC;
                int t = t0 + tt, kx = k0 + kc;
                xs[tt * kKC + kc] = (t < p.T && kx < H) ? load_f32<XT>(x, (size_t)t * H + kx) : 0.f;
            }
            for (int idx = tid; idx < kET * kKC; idx += kThreads) {
                int er = idx / kKC, kc = idx % kKC;
                int e = e0 + er, kx = k0 + kc;
                ws[er * (kKC + 1) + kc] = (e < E && kx < H) ? load_f32<WT>(wr, (size_t)e * H + kx) : 0.f;
            }
            __syncthreads();
#pragma unroll 8
            for (int kc = 0; kc < kKC; ++kc) {
                float wv = ws[el * (kKC + 1) + kc];
#pragma unroll
                for (int i = 0; i < kTokens / 2; ++i) acc[i] = fmaf(xs[(th + i) * kKC + kc], wv, acc[i]);
            }
        }
        int e = e0 + el;
        if (e < E) {
            float b = p.logit_bias ? p.logit_bias[e] : 0.f;
#pragma unroll
            for (int i = 0; i < kTokens / 2; ++i) lg[(th + i) * E + e] = acc[i] + b;
        }
    }
    __syncthreads();

    // phase 2: one wavefront per token
    const int wave = tid >> 6, lane = tid & 63;
    for (int tt = wave; tt < kTokens; tt += 4) {
        int t = t0 + tt;
        if (t < p.T) select_token(p, t, lg + tt * E, cs + wave * E, lane);
    }
}


// ---------------------------------------------------------------------------------
// Matrix-core path for bf16 activations: a logits kernel and a selection kernel.
//
// k_gate_logits.  A workgroup owns 16*TT tokens x a block of experts and writes their
// fp32 logits to the workspace.  Both MFMA operands are read straight from global
// memory in operand layout (no LDS): for a K-chunk of 128, lane (n = l%16, q = l/16)
// reads 32 of the 128 k of row n, interleaved with the other three lanes of the row
// in units of 8, and feeds them to the matrix core 8 (bf16) or 1 (fp32) at a time.
// The contraction does not care which k a lane group carries as long as the router
// row and the token row use the same assignment, which they do.
//   bf16 router: v_mfma_f32_16x16x32_bf16, fp32 accumulate.
//   fp32 router: tokens widened to fp32 (exact), v_mfma_f32_16x16x4_f32: every
//                product is a true fp32 product ("fp32 gate").
// The next chunk's loads are issued before the current chunk's MFMAs.
// Two ways to split a workgroup's work over its 4 wavefronts:
//   expert split (KSPLIT = false): wavefront w owns ET expert tiles of the workgroup's
//       4*ET tiles; used when there are enough tokens to fill the chip;
//   K split (KSPLIT = true): all wavefronts own the same ET expert tiles and a quarter
//       of K each; partial sums meet in LDS and are added in wavefront order
//       (deterministic).  Used for decode-sized batches, where the router matrix
//       must be streamed by many workgroups at once.
//
// k_gate_select.  One wavefront per token: scores, group limiting, top-k, weights
// (select_token above).  Its reductions are latency chains, so it runs as many small
// workgroups as possible and lets occupancy hide them.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename WT> struct RouterRun;           // the lane's 32 k of one row
template <> struct RouterRun<uint16_t> { uint4 v[4]; };
template <> struct RouterRun<float> { uint4 v[8]; };

// Loads the lane's 32 elements of a 128-wide K chunk.  Element (jj, i) of the lane in k-group q
// is k0 + jj*32 + q*8 + i (jj < 4, i < 8): the four lanes of a row then read one contiguous
// 64-byte (bf16) or 128-byte (fp32) span per pair of load instructions.
template <typename WT>
__device__ __forceinline__ void load_run(RouterRun<WT> &r, const WT *row, int k0, int q, int kend)
{
    constexpr int per16 = 16 / sizeof(WT);  // elements per 16-byte load: 8 or 4
    constexpr int parts = 8 / per16;         // loads per 8 elements: 1 or 2
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        const int k = k0 + jj * 32 + q * 8;
        const bool ok = k < kend;  // kend % 8 == 0: the 8 elements are all in or all out
#pragma unroll
        for (int h = 0; h < parts; ++h)
            r.v[jj * parts + h] = ok ? *(const uint4 *)(row + k + h * per16) : make_uint4(0, 0, 0, 0);
    }
}

template <typename WT, int TT, int ET, bool KSPLIT>
__global__ __launch_bounds__(kThreads) void k_gate_logits(Pass p)
{
    __shared__ float part[KSPLIT ? 4 * TT * ET * 256 : 1];
    const int E = p.E, H = p.H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, q = lane >> 4;
    const int t0 = blockIdx.x * 16 * TT;
    const int et0 = KSPLIT ? blockIdx.y * ET : (blockIdx.y * 4 + wave) * ET;   // first expert tile of this wavefront
    if (!KSPLIT && et0 * 16 >= E) return;
    const uint16_t *x = (const uint16_t *)p.x;
    const WT *wr = (const WT *)p.router_w;
    // K range of this wavefront (whole chunks of 128)
    int kbeg = 0, kend = H;
    if (KSPLIT) {
        // workgroup z of gridDim.z takes an equal share of the chunks (its sums go to plane z of the
        // logits buffer), its wavefronts a quarter of that each
        const int chunks = (H + 127) / 128;
        const int c0 = (int)((long long)blockIdx.z * chunks / gridDim.z), c1 = (int)((long long)(blockIdx.z + 1) * chunks / gridDim.z);
        const int per = (c1 - c0 + 3) / 4;
        kbeg = min(H, min(c1, c0 + wave * per) * 128);
        kend = min(H, min(c1, c0 + (wave + 1) * per) * 128);
    }

    const uint16_t *xrow[TT];
    const WT *wrow[ET];
#pragma unroll
    for (int tb = 0; tb < TT; ++tb) xrow[tb] = x + (size_t)min(t0 + tb * 16 + n, p.T - 1) * H;
#pragma unroll
    for (int a = 0; a < ET; ++a) wrow[a] = wr + (size_t)min((et0 + a) * 16 + n, E - 1) * H;

    f32x4 acc[ET][TT];
#pragma unroll
    for (int a = 0; a < ET; ++a)
#pragma unroll
        for (int tb = 0; tb < TT; ++tb) acc[a][tb] = (f32x4){0.f, 0.f, 0.f, 0.f};

    RouterRun<uint16_t> xc[TT], xn[TT];
    RouterRun<WT> wc[ET], wn[ET];
    auto load_chunk = [&](int k0, RouterRun<uint16_t> *xd, RouterRun<WT> *wd) {
#pragma unroll
        for (int tb = 0; tb < TT; ++tb) load_run<uint16_t>(xd[tb], xrow[tb], k0, q, kend);
#pragma unroll
        for (int a = 0; a < ET; ++a) load_run<WT>(wd[a], wrow[a], k0, q, kend);
    };
    if (kbeg < kend) load_chunk(kbeg, xc, wc);
    for (int k0 = kbeg; k0 < kend; k0 += 128) {
        if (k0 + 128 < kend) load_chunk(k0 + 128, xn, wn);
        __builtin_amdgcn_sched_barrier(0);  // the prefetch must be issued before this chunk's MFMAs, not after
        if constexpr (sizeof(WT) == 2) {
#pragma unroll
            for (int a = 0; a < ET; ++a)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int tb = 0; tb < TT; ++tb)
                        acc[a][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(bf16x8 *)&wc[a].v[j], *(bf16x8 *)&xc[tb].v[j], acc[a][tb], 0, 0, 0);
        } else {
            float xf[TT][32];
#pragma unroll
            for (int tb = 0; tb < TT; ++tb)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t *u = (const uint32_t *)&xc[tb].v[j];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        xf[tb][j * 8 + 2 * e] = __uint_as_float(u[e] << 16);
                        xf[tb][j * 8 + 2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
                    }
                }
#pragma unroll
            for (int a = 0; a < ET; ++a) {
                const float *wf = (const float *)&wc[a].v[0];
#pragma unroll
                for (int e = 0; e < 32; ++e)
#pragma unroll
                    for (int tb = 0; tb < TT; ++tb)
                        acc[a][tb] = __builtin_amdgcn_mfma_f32_16x16x4f32(wf[e], xf[tb][e], acc[a][tb], 0, 0, 0);
            }
        }
#pragma unroll
        for (int tb = 0; tb < TT; ++tb) xc[tb] = xn[tb];
#pragma unroll
        for (int a = 0; a < ET; ++a) wc[a] = wn[a];
    }

    if (KSPLIT) {  // partial sums of the 4 K-quarters meet in LDS, added in wavefront order
#pragma unroll
        for (int a = 0; a < ET; ++a)
#pragma unroll
            for (int tb = 0; tb < TT; ++tb)
#pragma unroll
                for (int r = 0; r < 4; ++r) part[((wave * ET + a) * TT + tb) * 256 + r * 64 + lane] = acc[a][tb][r];
        __syncthreads();
        if (wave != 0) return;
#pragma unroll
        for (int a = 0; a < ET; ++a)
#pragma unroll
            for (int tb = 0; tb < TT; ++tb)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float s = 0.f;
#pragma unroll
                    for (int w = 0; w < 4; ++w) s += part[((w * ET + a) * TT + tb) * 256 + r * 64 + lane];
                    acc[a][tb][r] = s;
                }
    }
    // lane holds token n of each token tile, experts 4q + r of each of its expert tiles
    float *plane = p.logits + (size_t)blockIdx.z * p.T * E;
    const float *bias = blockIdx.z == 0 ? p.logit_bias : nullptr;   // added once
#pragma unroll
    for (int a = 0; a < ET; ++a)
#pragma unroll
        for (int tb = 0; tb < TT; ++tb) {
            const int t = t0 + tb * 16 + n;
            const int e = (et0 + a) * 16 + 4 * q;   // E may be any size: guard each of the 4
            if (t < p.T) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (e + r < E) plane[(size_t)t * E + e + r] = acc[a][tb][r] + (bias ? bias[e + r] : 0.f);
            }
        }
}

// LDS-tiled logits kernel for prefill-sized batches.  A workgroup owns 16*TBT tokens x 64*EBT
// experts; the token tile and the router tile of a K-step of 64 are staged once in LDS (global ->
// registers -> LDS, next step's loads in flight during this step's MFMAs) and shared by the four
// wavefronts, wavefront w taking expert tiles w*EBT .. of 16 experts each.  Tile rows are 128
// bytes with their 16-byte chunks XOR-swizzled so that the 16 rows a half-wavefront reads for one
// operand fall into 16 distinct bank groups.
// fp32 router weights are split on the fly into three bf16 planes hi + mid + lo (each the
// truncated top 8 mantissa bits of what is left: the split is exact), so that x . w is three bf16
// MFMAs whose products are all exact and whose sum is accumulated in fp32: the same products and
// the same accumulator width as an fp32 multiply-add chain.
__device__ __forceinline__ int gate_swz(int row) { return ((row >> 1) & 3) | (((row ^ (row >> 3)) & 1) << 2); }

template <typename WT, int TBT, int EBT>
__global__ __launch_bounds__(kThreads) void k_gate_logits_lds(Pass p)
{
    constexpr int P = sizeof(WT) == 2 ? 1 : 3;          // bf16 planes per router tile
    constexpr int TB = 16 * TBT, EB = 64 * EBT;
    constexpr int XCH = TB * 8, WCH = EB * 8;           // 16-byte chunks per tile (per plane)
    constexpr int XL = (XCH + kThreads - 1) / kThreads; // staging loads per thread
    constexpr int WL = WCH / kThreads * (P == 3 ? 2 : 1);   // fp32: 8 floats = 2 loads per 8-element chunk
    constexpr int WCL = WCH / kThreads;                 // 8-element chunks per thread
    __shared__ uint4 lds[2][XCH + P * WCH];
    const int E = p.E, H = p.H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = blockIdx.x * TB, e0 = blockIdx.y * EB;
    const uint16_t *x = (const uint16_t *)p.x;
    const WT *wr = (const WT *)p.router_w;

    uint4 xa[XL], wa[WL], xb[XL], wb[WL];   // two register stages: K-steps kt+1 and kt+2 are in flight
    auto load_global = [&](int k0, uint4 *xreg, uint4 *wreg) {
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int c = tid + i * kThreads, row = c >> 3, ch = c & 7;
            const int k = k0 + ch * 8;
            xreg[i] = (c < XCH && k < H) ? *(const uint4 *)(x + (size_t)min(t0 + row, p.T - 1) * H + k) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < WCL; ++i) {
            const int c = tid + i * kThreads, row = c >> 3, ch = c & 7;
            const int k = k0 + ch * 8;
            const WT *src = wr + (size_t)min(e0 + row, E - 1) * H + k;
            if constexpr (P == 1) {
                wreg[i] = (k < H) ? *(const uint4 *)src : make_uint4(0, 0, 0, 0);
            } else {
                wreg[2 * i] = (k < H) ? *(const uint4 *)src : make_uint4(0, 0, 0, 0);
                wreg[2 * i + 1] = (k < H) ? *(const uint4 *)(src + 4) : make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto store_lds = [&](int buf, const uint4 *xreg, const uint4 *wreg) {
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int c = tid + i * kThreads, row = c >> 3, ch = c & 7;
            if (c < XCH) lds[buf][row * 8 + (ch ^ gate_swz(row))] = xreg[i];
        }
#pragma unroll
        for (int i = 0; i < WCL; ++i) {
            const int c = tid + i * kThreads, row = c >> 3, ch = c & 7;
            const int at = XCH + row * 8 + (ch ^ gate_swz(row));
            if constexpr (P == 1) {
                lds[buf][at] = wreg[i];
            } else {
                const uint32_t *f = (const uint32_t *)&wreg[2 * i];   // 8 fp32 bit patterns
                uint32_t hi[8], mid[8], lo[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    hi[e] = f[e] & 0xffff0000u;
                    const float r1 = __uint_as_float(f[e]) - __uint_as_float(hi[e]);
                    mid[e] = __float_as_uint(r1) & 0xffff0000u;
                    const float r2 = r1 - __uint_as_float(mid[e]);
                    lo[e] = __float_as_uint(r2);   // at most 8 significant bits left: already a bf16 value
                }
                auto pack = [](const uint32_t *v) {
                    return make_uint4((v[0] >> 16) | v[1], (v[2] >> 16) | v[3], (v[4] >> 16) | v[5], (v[6] >> 16) | v[7]);
                };
                uint32_t lom[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) lom[e] = lo[e] & 0xffff0000u;
                lds[buf][at] = pack(hi);
                lds[buf][at + WCH] = pack(mid);
                lds[buf][at + 2 * WCH] = pack(lom);
            }
        }
    };

    f32x4 acc[EBT][TBT];
#pragma unroll
    for (int a = 0; a < EBT; ++a)
#pragma unroll
        for (int tb = 0; tb < TBT; ++tb) acc[a][tb] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const int n = lane & 15, q = lane >> 4;

    auto multiply = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int ch = ks * 4 + q;
            bf16x8 xf[TBT];
#pragma unroll
            for (int tb = 0; tb < TBT; ++tb) {
                const int row = tb * 16 + n;
                const uint4 v = lds[buf][row * 8 + (ch ^ gate_swz(row))];
                xf[tb] = *(const bf16x8 *)&v;
            }
#pragma unroll
            for (int a = 0; a < EBT; ++a) {
                const int row = (wave * EBT + a) * 16 + n;
#pragma unroll
                for (int pl = 0; pl < P; ++pl) {
                    const uint4 v = lds[buf][XCH + pl * WCH + row * 8 + (ch ^ gate_swz(row))];
                    const bf16x8 wf = *(const bf16x8 *)&v;
#pragma unroll
                    for (int tb = 0; tb < TBT; ++tb)
                        acc[a][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xf[tb], acc[a][tb], 0, 0, 0);
                }
            }
        }
    };
    // Loads past the end of K are predicated off (they return zeros), so the pipeline needs no tail code.
    const int KT = (H + 63) / 64;
    load_global(0, xa, wa);
    load_global(64, xb, wb);
    store_lds(0, xa, wa);
    load_global(128, xa, wa);
    __syncthreads();
    for (int kt = 0; kt < KT; kt += 2) {
        multiply(0);                          // K-step kt
        store_lds(1, xb, wb);                 // K-step kt+1 (loaded one whole iteration ago)
        load_global((kt + 3) * 64, xb, wb);
        __syncthreads();
        if (kt + 1 < KT) multiply(1);         // K-step kt+1
        store_lds(0, xa, wa);                 // K-step kt+2
        load_global((kt + 4) * 64, xa, wa);
        __syncthreads();
    }
    // lane holds token n of each token tile, experts 4q + r of each of its expert tiles
#pragma unroll
    for (int a = 0; a < EBT; ++a)
#pragma unroll
        for (int tb = 0; tb < TBT; ++tb) {
            const int t = t0 + tb * 16 + n;
            const int e = e0 + (wave * EBT + a) * 16 + 4 * q;
            if (t < p.T) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (e + r < E) p.logits[(size_t)t * E + e + r] = acc[a][tb][r] + (p.logit_bias ? p.logit_bias[e + r] : 0.f);
            }
        }
}

template <typename WT, int TBT, int EBT>
hipError_t launch_gate_logits_lds(const Pass &p, hipStream_t st)
{
    dim3 grid((p.T + 16 * TBT - 1) / (16 * TBT), (p.E + 64 * EBT - 1) / (64 * EBT));
    hipLaunchKernelGGL((k_gate_logits_lds<WT, TBT, EBT>), grid, dim3(kThreads), 0, st, p);
    return hipGetLastError();
}

__global__ __launch_bounds__(kThreads) void k_gate_select(Pass p)
{
    extern __shared__ float smem[];
    const int E = p.E;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *lg = smem + wave * 2 * E;         // [E] logits -> scores
    float *cs = lg + E;                       // [E] selection scores
    const int t = blockIdx.x * 4 + wave;
    if (t >= p.T) return;
    for (int e = lane; e < E; e += 64) {
        // partial sums of the K ranges: all planes are requested at once, then added in K order
        float part[kGatePlanes];
#pragma unroll
        for (int z = 0; z < kGatePlanes; ++z) part[z] = z < p.logit_planes ? p.logits[((size_t)z * p.T + t) * E + e] : 0.f;
        float v = part[0];
#pragma unroll
        for (int z = 1; z < kGatePlanes; ++z)
            if (z < p.logit_planes) v += part[z];
        lg[e] = v;
    }
    wave_sync();
    select_token(p, t, lg, cs, lane);
}

// The selection kernel with the first step of the routing bookkeeping fused in: a workgroup of 16
// wavefronts owns kFusedTokens = 16 consecutive tokens, one per wavefront.  After the selection every
// lane j < k + n_shared holds one assignment of its token; its slot is looked up in the expert table and
// the workgroup builds, per slot, the 16-bit mask of its tokens that have a row in the slot (a token's
// assignments go to distinct slots: distinct experts, one-to-one table), from which an assignment's rank
// among the block's earlier rows of the slot is a population count -- deterministic, token order.
// Word [slot][block] of blk_hist: the mask, and above it (bits 16..21) the selection position of the
// block's first row in the slot (with the token it makes the group's first-assignment key); byte
// [slot][block] of blk_cnt: the number of rows, i.e. of mask bits.
__global__ __launch_bounds__(kFusedTokens * 64) void k_gate_select_hist(Pass p, int n_blocks)
{
    extern __shared__ float smem[];
    const int E = p.E, S = p.S;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *lg = smem + wave * 2 * E;         // [E] logits -> scores
    float *cs = lg + E;                       // [E] selection scores
    uint32_t *blkmask = (uint32_t *)(smem + kFusedTokens * 2 * E);   // [S]
    for (int s = threadIdx.x; s < S; s += kFusedTokens * 64) blkmask[s] = 0u;
    const int t = blockIdx.x * kFusedTokens + wave;
    int slot = -1;
    if (t < p.T) {
        for (int e = lane; e < E; e += 64) {
            // partial sums of the K ranges: all planes are requested at once, then added in K order
            float part[kGatePlanes];
#pragma unroll
            for (int z = 0; z < kGatePlanes; ++z) part[z] = z < p.logit_planes ? p.logits[((size_t)z * p.T + t) * E + e] : 0.f;
            float v = part[0];
#pragma unroll
            for (int z = 1; z < kGatePlanes; ++z)
                if (z < p.logit_planes) v += part[z];
            lg[e] = v;
        }
        wave_sync();
        const int id = select_token(p, t, lg, cs, lane);
        if (lane < p.k) {
            const int m = p.map[id];
            if (m >= -1) {
                slot = m;
            } else {   // an expert with several copies: token t uses copy t mod R of the list behind the table's entries
                const int32_t *copies = p.map + p.E + p.n_shared + (-2 - m);
                slot = copies[1 + t % copies[0]];
            }
        } else if (lane < p.kk && t >= p.shared_begin && t < p.shared_end) {
            slot = p.map[p.E + (lane - p.k)];
        }
    }
    __syncthreads();
    if (slot >= 0) atomicOr(&blkmask[slot], 1u << wave);
    __syncthreads();
    int rank = 0;
    if (slot >= 0) {
        rank = __popc(blkmask[slot] & ((1u << wave) - 1u));
        if (rank == 0) atomicOr(&blkmask[slot], (uint32_t)lane << 16);   // one such lane per slot
    }
    if (t < p.T && lane < p.kk) p.slot_rank[(size_t)t * p.kk + lane] = slot >= 0 ? ((slot << 12) | rank) : -1;
    __syncthreads();
    for (int s = threadIdx.x; s < S; s += kFusedTokens * 64) {
        const uint32_t m = blkmask[s];
        p.blk_hist[(size_t)s * fused_row_stride(n_blocks) + blockIdx.x] = (int32_t)m;
        p.blk_cnt[(size_t)s * fused_row_stride(n_blocks) + blockIdx.x] = (uint8_t)__popc(m & 0xffffu);   // what the placing kernel adds up
    }
}

template <typename WT, int TT, int ET, bool KSPLIT>
hipError_t launch_gate_logits_t(const Pass &p, int planes, hipStream_t st)
{
    const int eb = (KSPLIT ? 1 : 4) * ET * 16;
    dim3 grid((p.T + 16 * TT - 1) / (16 * TT), (p.E + eb - 1) / eb, planes);
    hipLaunchKernelGGL((k_gate_logits<WT, TT, ET, KSPLIT>), grid, dim3(kThreads), 0, st, p);
    return hipGetLastError();
}

template <typename WT>
hipError_t launch_gate_mfma(const Pass &p0, hipStream_t st)
{
    Pass p = p0;
    int planes = 1;
    hipError_t e;
    // Up to a hundred or so tokens there are too few (token, expert) tiles for the LDS-tiled kernels: the
    // K-split kernel reads both operands straight into registers, 16 tokens x 16 experts per workgroup, and
    // shares the contraction out over its wavefronts and over workgroups.  (Without the direct-to-LDS
    // kernel -- H not a multiple of 64 -- it stays ahead until the router re-reads reach about 128 MB.)
    const size_t router_rereads = (size_t)((p.T + 15) / 16) * p.E * p.H * (p.router_bf16 ? 2 : 4);
    const bool small = gate_dma_supports(p) ? p.T <= 128 : (p.T <= 256 || router_rereads <= (size_t)128 << 20);
    if (!p.gate_tiled && small) {
        // 4 chunks of 128 (one per wavefront) or more per workgroup
        if (p.T <= 256) planes = min(kGatePlanes, max(1, (p.H + 127) / 128 / 4));
        e = launch_gate_logits_t<WT, 1, 1, true>(p, planes, st);
    }
    else if (gate_dma_supports(p))      e = launch_gate_logits_dma(p, &planes, st);    // LDS ring filled by direct copies
    else if (p.E > 64 && p.T >= 8192)   e = launch_gate_logits_lds<WT, 4, 2>(p, st);   // 64 tokens x 128 experts
    else                                e = launch_gate_logits_lds<WT, 2, 1>(p, st);   // 32 tokens x 64 experts
    if (e != hipSuccess) return e;
    p.logit_planes = planes;
    if (p.fused_hist) {
        const int nb = (p.T + kFusedTokens - 1) / kFusedTokens;
        const size_t smem = sizeof(float) * kFusedTokens * 2 * (size_t)p.E + sizeof(uint32_t) * p.S;
        if (smem > 64 * 1024) {
            e = hipFuncSetAttribute((const void *)k_gate_select_hist, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(k_gate_select_hist, dim3(nb), dim3(kFusedTokens * 64), smem, st, p, nb);
        return hipGetLastError();
    }
    const size_t smem = sizeof(float) * 4 * 2 * (size_t)p.E;
    hipLaunchKernelGGL(k_gate_select, dim3((p.T + 3) / 4), dim3(kThreads), smem, st, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gate(const Pass &p, hipStream_t st)
{
    if (p.act_bf16) return p.router_bf16 ? launch_gate_mfma<uint16_t>(p, st) : launch_gate_mfma<float>(p, st);
    const int blocks = (p.T + kTokens - 1) / kTokens;
    const size_t smem = sizeof(float) * (kTokens * kKC + kET * (kKC + 1) + (size_t)kTokens * p.E + 4 * (size_t)p.E);
    dim3 grid(blocks), block(kThreads);
    if (smem > 64 * 1024) {  // opt in to the large-LDS launch once per kernel variant is cheap enough
        hipError_t e = hipSuccess;
        if (p.act_bf16 && p.router_bf16) e = hipFuncSetAttribute((const void *)k_gate<uint16_t, uint16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        else if (p.act_bf16)             e = hipFuncSetAttribute((const void *)k_gate<uint16_t, float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        else if (p.router_bf16)          e = hipFuncSetAttribute((const void *)k_gate<float, uint16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        else                             e = hipFuncSetAttribute((const void *)k_gate<float, float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    if (p.act_bf16) {
        if (p.router_bf16) hipLaunchKernelGGL((k_gate<uint16_t, uint16_t>), grid, block, smem, st, p);
        else               hipLaunchKernelGGL((k_gate<uint16_t, float>), grid, block, smem, st, p);
    } else {
        if (p.router_bf16) hipLaunchKernelGGL((k_gate<float, uint16_t>), grid, block, smem, st, p);
        else               hipLaunchKernelGGL((k_gate<float, float>), grid, block, smem, st, p);
    }
    return hipGetLastError();
}

}  // namespace emoe
