// Gate logits for prefill-sized batches, staged by direct global -> LDS copies.
//
// logits[t, e] = sum_h x[t, h] * Wr[e, h] (+ logit_bias[e]) in fp32 -- step 1 of the gate of the
// layer of Sec. 2.1 of the paper; scores and the top-k selection follow in k_gate_select.
//
// The contraction is small (2*T*H*E flops); what costs is moving its operands into the compute
// units: a workgroup owns a tile of tokens x experts and walks K in steps of 64 through LDS rings
// filled by global_load_lds_dwordx4 (no register round trip), waiting only for the oldest step
// in flight.  The NW wavefronts form a WM x (NW/WM) grid: wavefront (wt, we) multiplies token
// tiles wt*TBT .. +TBT-1 (16 tokens each) with expert tiles we*EBT .. +EBT-1 (16 experts each),
// v_mfma_f32_16x16x32_bf16.
//
// * The bytes a workgroup pulls are (tokens + experts of its tile) * H: large tiles (up to 128
//   tokens x 256 experts) cut them, and the contraction is then split over gridDim.z workgroups
//   so that the chip stays full.  Split z writes its partial sums to plane z of the logits
//   buffer; the selection kernel adds the planes in order.
// * Issuing a copy instruction costs a wavefront on the order of a hundred cycles, during which
//   it multiplies nothing: the large tiles run on 8 wavefronts (two per SIMD, one issuing while
//   the other multiplies).
// * Accumulators go out through LDS as whole row segments (stored from registers, every
//   instruction would touch 16 rows of the plane, 64 bytes each: a third of the kernel's time).
//
// Rows are 128 bytes (bf16) or 256 bytes (fp32 router) with their 16-byte chunks XOR-swizzled on
// the global side of the copy, so that the 16 rows a quarter-wavefront reads for one operand fall
// into 16 distinct bank groups.  An fp32 router row is split when it is READ from LDS into three
// bf16 planes hi + mid + lo (each the truncated top 8 mantissa bits of what is left: the split is
// exact), so that x . w is three bf16 MFMAs whose products are all exact and whose sum is
// accumulated in fp32 -- the same products and the same accumulator width as an fp32 chain.
#include "moe_internal.h"

namespace emoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;   // K-step

__device__ __forceinline__ uint32_t lds_addr(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

// global -> LDS copy of one 1 KB piece: lane i's 16 bytes land at lds_byte_addr + 16*i.  Inline
// assembly on purpose: the compiler's wait-count insertion would otherwise hold every later LDS
// read until these copies (which belong to a LATER K-step) have landed.
__device__ __forceinline__ void dma_piece(const void *base, uint32_t byte_off, uint32_t lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_byte_addr), "v"(byte_off), "s"(base) : "memory", "m0");
}

template <int n>
__device__ __forceinline__ void wait_loads()
{
    static_assert(n >= 0 && n < 64, "vmcnt has 6 bits");
    __builtin_amdgcn_s_waitcnt((n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8));   // vmcnt only
}

// exact split of 8 fp32 values (two 16-byte loads) into three bf16 planes
__device__ __forceinline__ void split3(const uint4 &lo4, const uint4 &hi4, bf16x8 &ph, bf16x8 &pm, bf16x8 &pl)
{
    const uint32_t f[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
    uint32_t h[8], m[8], l[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        h[e] = f[e] & 0xffff0000u;
        const float r1 = __uint_as_float(f[e]) - __uint_as_float(h[e]);
        m[e] = __float_as_uint(r1) & 0xffff0000u;
        const float r2 = r1 - __uint_as_float(m[e]);
        l[e] = __float_as_uint(r2) & 0xffff0000u;   // at most 8 significant bits are left: already a bf16 value
    }
    auto pack = [](const uint32_t *v) {
        const uint4 u = make_uint4((v[0] >> 16) | v[1], (v[2] >> 16) | v[3], (v[4] >> 16) | v[5], (v[6] >> 16) | v[7]);
        return *(const bf16x8 *)&u;
    };
    ph = pack(h); pm = pack(m); pl = pack(l);
}

// NSW = 0: one ring of NS stages, a stage = the step's token rows + router rows, every wavefront
// copies its share of both.  NSW > 0: two rings -- NS stages of token rows, NSW of router rows;
// the first half of the wavefronts copies token rows, the second half router rows.  A
// wavefront's copies complete in order, so only with separate loaders can the token rows (each
// read once, from HBM, ~4 us away) be many steps ahead while the router rows (re-read by every
// workgroup, from L2) are one or two: LDS then holds mostly token rows in flight, which is what
// the HBM stream of x needs at large T * H.
template <typename WT, int TBT, int EBT, int NS, int NW, int WM, int NSW>
__global__ __launch_bounds__(NW * 64) void k_gate_logits_dma(Pass p)
{
    constexpr bool F32 = sizeof(WT) == 4;
    constexpr bool TWO = NSW > 0;
    constexpr int kWaves = NW, WE = NW / WM;
    constexpr int TB = 16 * TBT * WM, EB = 16 * EBT * WE;
    constexpr int XBYTES = TB * 128, WROW = F32 ? 256 : 128, WBYTES = EB * WROW, STAGE = XBYTES + WBYTES;
    constexpr int XP = XBYTES / 1024, WP = WBYTES / 1024;   // 1 KB pieces: 8 rows of 128 B, or 4 rows of 256 B
    constexpr int XPW = TWO ? XP / (NW / 2) : 0, WPW = TWO ? WP / (NW / 2) : 0;   // two rings: pieces per loader per K-step
    constexpr int PW = TWO ? (XPW > WPW ? XPW : WPW) : (XP + WP) / kWaves;        // pieces per wavefront per K-step
    static_assert(TWO || (XP + WP) % kWaves == 0, "pieces are dealt evenly to the wavefronts");
    static_assert(!TWO || (XP % (NW / 2) == 0 && WP % (NW / 2) == 0 && NSW >= 2), "pieces are dealt evenly to the loaders of a ring");
    static_assert(NS >= 2 && (NS - 2) * PW < 64, "load counter");
    constexpr int LDS = TWO ? NS * XBYTES + NSW * WBYTES : NS * STAGE;
    static_assert(LDS <= 160 * 1024, "rings fit LDS");
    __shared__ __attribute__((aligned(1024))) char ring[LDS];
    // single ring: stage s at s * STAGE, token rows first.  Two rings: token stages, then router stages.
    constexpr int XSTRIDE = TWO ? XBYTES : STAGE, WSTRIDE = TWO ? WBYTES : STAGE, WRING0 = TWO ? NS * XBYTES : XBYTES;

    const int E = p.E, H = p.H;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wt = wave / WE, we = wave % WE;
    const int t0 = blockIdx.x * TB, e0 = blockIdx.y * EB;
    // this workgroup's share of the K-steps
    const int kt0 = (int)((long long)blockIdx.z * (H / kBK) / gridDim.z), kt1 = (int)((long long)(blockIdx.z + 1) * (H / kBK) / gridDim.z);
    const char *xbase = (const char *)p.x;
    const char *wbase = (const char *)p.router_w;

    // ---- this lane's share of every K-step: its pieces, their global byte offsets at k = 0 ----
    const bool xloader = TWO && wave < NW / 2;
    uint32_t src[PW];
    uint32_t dst[PW];   // wave-uniform LDS offset of the piece inside its stage
    bool isx[PW];
#pragma unroll
    for (int i = 0; i < PW; ++i) {
        // single ring: piece wave + NW i of the XP + WP pieces of a stage.  Two rings: token piece
        // wave + (NW/2) i for the first half of the wavefronts, router piece likewise for the second.
        int pc = TWO ? (wave % (NW / 2)) + (NW / 2) * i : wave + kWaves * i;
        isx[i] = TWO ? xloader : pc < XP;
        if (!TWO && !isx[i]) pc -= XP;
        if (TWO && pc >= (xloader ? XP : WP)) pc = 0;       // never issued (i >= this ring's pieces per loader)
        if (isx[i]) {
            const int row = pc * 8 + (lane >> 3);
            const int chunk = (lane & 7) ^ ((row >> 1) & 7);
            src[i] = (uint32_t)min(t0 + row, p.T - 1) * (uint32_t)H * 2u + chunk * 16;
        } else if (!F32) {
            const int row = pc * 8 + (lane >> 3);
            const int chunk = (lane & 7) ^ ((row >> 1) & 7);
            src[i] = (uint32_t)min(e0 + row, E - 1) * (uint32_t)H * 2u + chunk * 16;
        } else {
            const int row = pc * 4 + (lane >> 4);
            const int chunk = (lane & 15) ^ (row & 15);
            src[i] = (uint32_t)min(e0 + row, E - 1) * (uint32_t)H * 4u + chunk * 16;
        }
        dst[i] = pc * 1024;
    }
    const uint32_t ring_a = lds_addr(ring);
    // copies of this wavefront for K-step kt into stage `slot` of the ring(s) it loads
    auto issue = [&](int kt, int slot) {
#pragma unroll
        for (int i = 0; i < PW; ++i) {
            if (TWO && i >= (xloader ? XPW : WPW)) continue;
            const char *b = isx[i] ? xbase + (size_t)kt * (kBK * 2) : wbase + (size_t)kt * (kBK * (F32 ? 4 : 2));
            const uint32_t stage = isx[i] ? slot * XSTRIDE : WRING0 + slot * WSTRIDE;
            dma_piece(b, src[i], ring_a + stage + __builtin_amdgcn_readfirstlane(dst[i]));
        }
    };

    // ---- operand reads: lane (n = l % 16, q = l / 16) holds k = 8q .. 8q+7 of row n of a 16-row tile ----
    const int n = lane & 15, q = lane >> 4;
    uint32_t xoff[2], woff[2][F32 ? 2 : 1];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int ch = ks * 4 + q;
        xoff[ks] = n * 128 + ((ch ^ ((n >> 1) & 7)) << 4);
        if (F32) {
            woff[ks][0] = n * 256 + (((2 * ch) ^ n) << 4);
            woff[ks][F32 ? 1 : 0] = n * 256 + (((2 * ch + 1) ^ n) << 4);
        } else {
            woff[ks][0] = xoff[ks];
        }
    }

    f32x4 acc[EBT][TBT];
#pragma unroll
    for (int a = 0; a < EBT; ++a)
#pragma unroll
        for (int tb = 0; tb < TBT; ++tb) acc[a][tb] = (f32x4){0.f, 0.f, 0.f, 0.f};

    auto multiply = [&](int xslot, int wslot) {
        const char *W = ring + WRING0 + wslot * WSTRIDE + we * EBT * 16 * WROW;
        const char *X = ring + xslot * XSTRIDE + wt * TBT * 16 * 128;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 xf[TBT];
#pragma unroll
            for (int tb = 0; tb < TBT; ++tb) {
                const uint4 v = *(const uint4 *)(X + xoff[ks] + tb * 16 * 128);
                xf[tb] = *(const bf16x8 *)&v;
            }
#pragma unroll
            for (int a = 0; a < EBT; ++a) {
                if constexpr (F32) {
                    const uint4 v0 = *(const uint4 *)(W + woff[ks][0] + a * 16 * WROW);
                    const uint4 v1 = *(const uint4 *)(W + woff[ks][1] + a * 16 * WROW);
                    bf16x8 ph, pm, pl;
                    split3(v0, v1, ph, pm, pl);
#pragma unroll
                    for (int tb = 0; tb < TBT; ++tb) {
                        acc[a][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ph, xf[tb], acc[a][tb], 0, 0, 0);
                        acc[a][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pm, xf[tb], acc[a][tb], 0, 0, 0);
                        acc[a][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pl, xf[tb], acc[a][tb], 0, 0, 0);
                    }
                } else {
                    const uint4 v = *(const uint4 *)(W + woff[ks][0] + a * 16 * WROW);
                    const bf16x8 wf = *(const bf16x8 *)&v;
#pragma unroll
                    for (int tb = 0; tb < TBT; ++tb)
                        acc[a][tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xf[tb], acc[a][tb], 0, 0, 0);
                }
            }
        }
    };

    // ---- K loop: steps kt+1 .. kt+depth-1 of a ring are in flight while step kt is multiplied ----
    const int depth = TWO && !xloader ? NSW : NS;              // of the ring this wavefront loads
    const int mine = TWO ? (xloader ? XPW : WPW) : PW;         // copies it issues per K-step
    for (int s = 0; s < depth - 1 && kt0 + s < kt1; ++s) issue(kt0 + s, s);
    int xs = 0, ws = 0, fill = depth - 1;
    for (int kt = kt0; kt < kt1; ++kt) {
        // younger steps that may stay in flight: those issued after step kt, at most depth-2 of them
        const int allowed = min(depth - 2, kt1 - 1 - kt) * mine;
        switch (allowed) {   // the count is an immediate of the wait instruction
#define EMOE_WAIT_CASE(N) case N: wait_loads<N>(); break;
        EMOE_WAIT_CASE(1) EMOE_WAIT_CASE(2) EMOE_WAIT_CASE(3) EMOE_WAIT_CASE(4) EMOE_WAIT_CASE(5) EMOE_WAIT_CASE(6)
        EMOE_WAIT_CASE(8) EMOE_WAIT_CASE(9) EMOE_WAIT_CASE(10) EMOE_WAIT_CASE(12) EMOE_WAIT_CASE(15) EMOE_WAIT_CASE(16)
        EMOE_WAIT_CASE(18) EMOE_WAIT_CASE(20) EMOE_WAIT_CASE(24) EMOE_WAIT_CASE(32)
#undef EMOE_WAIT_CASE
        default: wait_loads<0>(); break;   // a count not listed waits for everything: always safe
        }
        __syncthreads();   // everyone's pieces of step kt have landed; everyone is done reading step kt-1
        if (kt + depth - 1 < kt1) issue(kt + depth - 1, fill);
        multiply(xs, ws);
        xs = xs + 1 == NS ? 0 : xs + 1;
        ws = ws + 1 == (TWO ? NSW : NS) ? 0 : ws + 1;
        fill = fill + 1 == depth ? 0 : fill + 1;
    }

    // ---- epilogue: accumulators -> this wavefront's LDS region [token][expert] -> whole row segments ----
    // A lane holds token n of each token tile and experts 4q .. 4q+3 of each of its expert tiles:
    // stored straight from registers every instruction would touch 16 rows, 64 bytes each.
    __syncthreads();   // all operand reads are done: the ring becomes the staging area
    float *plane = p.logits + (size_t)blockIdx.z * p.T * E;
    const float *bias = blockIdx.z == 0 ? p.logit_bias : nullptr;   // added once
    constexpr int COLS = EBT * 16, STRIDE = COLS + 4;   // floats; +4 keeps the 16 rows of a store apart on the banks
    static_assert(NW * TBT * 16 * STRIDE * 4 <= LDS, "staging fits the ring");
    float *stg = (float *)ring + wave * (TBT * 16 * STRIDE);
#pragma unroll
    for (int a = 0; a < EBT; ++a)
#pragma unroll
        for (int tb = 0; tb < TBT; ++tb)
            *(f32x4 *)(stg + (tb * 16 + n) * STRIDE + a * 16 + 4 * q) = acc[a][tb];
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
    constexpr int LPR = COLS / 4, RPI = 64 / LPR;        // lanes per row, rows per instruction
    const int lr = lane / LPR, lc = (lane % LPR) * 4;
    const int ecol = e0 + we * COLS + lc;
    f32x4 bv = {0.f, 0.f, 0.f, 0.f};
    if (bias) {
#pragma unroll
        for (int r = 0; r < 4; ++r) bv[r] = ecol + r < E ? bias[ecol + r] : 0.f;
    }
    const bool vec = (E & 3) == 0;                        // rows of the plane are 16-byte aligned
#pragma unroll
    for (int r0 = 0; r0 < TBT * 16; r0 += RPI) {
        const int row = r0 + lr;
        const int t = t0 + wt * TBT * 16 + row;
        f32x4 v = *(const f32x4 *)(stg + row * STRIDE + lc);
        v += bv;
        if (t < p.T) {
            float *dst = plane + (size_t)t * E + ecol;
            if (vec && ecol + 3 < E) {
                *(f32x4 *)dst = v;
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (ecol + r < E) dst[r] = v[r];
            }
        }
    }
}

template <typename WT, int TBT, int EBT, int NS, int NW, int WM, int NSW = 0>
hipError_t launch_t(const Pass &p, int planes, hipStream_t st)
{
    constexpr int TB = 16 * TBT * WM, EB = 16 * EBT * (NW / WM);
    dim3 grid((p.T + TB - 1) / TB, (p.E + EB - 1) / EB, planes);
    hipLaunchKernelGGL((k_gate_logits_dma<WT, TBT, EBT, NS, NW, WM, NSW>), grid, dim3(NW * 64), 0, st, p);
    return hipGetLastError();
}

// K splits for a tiling with n_tiles output tiles: enough workgroups for the chip, at least 8
// K-steps each (the ring needs a few steps to reach its depth), at most kGatePlanes
int splits_for(long long n_tiles, int KT)
{
    long long z = (256 + n_tiles - 1) / n_tiles;
    if (z > kGatePlanes) z = kGatePlanes;
    if (z > KT / 8) z = KT / 8;
    return z < 1 ? 1 : (int)z;
}

}  // namespace

// whole K-steps only (the copies cannot zero fill), and 32-bit byte offsets into x and the router
bool gate_dma_supports(const Pass &p)
{
    return p.act_bf16 && p.H % kBK == 0 && p.H >= kBK && (size_t)p.T * p.H * 2 < ((size_t)1 << 32) && (size_t)p.E * p.H * 4 < ((size_t)1 << 32);
}

// Writes *planes partial-sum planes [T,E] to p.logits.
hipError_t launch_gate_logits_dma(const Pass &p, int *planes, hipStream_t st)
{
    // tilings, largest first: tokens x experts per workgroup.  The first one that fills the chip
    // (with its K splits) and whose expert block is not mostly padding is taken.
    const int KT = p.H / kBK;
    auto tiles = [&](int tb, int eb) { return (long long)((p.T + tb - 1) / tb) * ((p.E + eb - 1) / eb); };
    const int ebL = p.router_bf16 ? 256 : 128;
    int cfg = 0;
    if (p.E > ebL / 2 && tiles(128, ebL) * splits_for(tiles(128, ebL), KT) >= 192) cfg = 2;
    else if (p.E > 64 && tiles(64, 128) * splits_for(tiles(64, 128), KT) >= 192) cfg = 1;
    const int z = cfg == 2 ? splits_for(tiles(128, ebL), KT) : cfg == 1 ? splits_for(tiles(64, 128), KT) : splits_for(tiles(32, 64), KT);
    *planes = z;
    // 128 x 256 (bf16 router) or 128 x 128 (fp32 router) on 8 wavefronts (2 x 4) with two rings: 4 stages of
    // token rows (16 KB each), 3 of router rows (32 KB each); 64 x 128 on 8 wavefronts and 32 x 64 on 4, one ring
    if (p.router_bf16) return cfg == 2 ? launch_t<uint16_t, 4, 4, 4, 8, 2, 3>(p, z, st) : cfg == 1 ? launch_t<uint16_t, 2, 2, 6, 8, 2>(p, z, st) : launch_t<uint16_t, 2, 1, 6, 4, 1>(p, z, st);
    return cfg == 2 ? launch_t<float, 4, 2, 4, 8, 2, 3>(p, z, st) : cfg == 1 ? launch_t<float, 4, 1, 4, 8, 1>(p, z, st) : launch_t<float, 2, 1, 6, 4, 1>(p, z, st);
}

}  // namespace emoe
