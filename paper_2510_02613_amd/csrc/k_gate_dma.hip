// Gate logits for prefill-sized batches, staged by direct global -> LDS copies.
//
// logits[t, e] = sum_h x[t, h] * Wr[e, h] (+ logit_bias[e]) in fp32 -- step 1 of the gate of the
// layer of Sec. 2.1 of the paper; scores and the top-k selection follow in k_gate_select.
//
// The contraction is small (2*T*H*E flops) and its operands are read from L2 many times over, so
// what decides its speed is how many bytes a compute unit keeps in flight: a workgroup owns
// 16*TBT tokens x 64*EBT experts and walks K in steps of 64 through an NS-deep LDS ring filled
// by global_load_lds_dwordx4 (NS-1 steps in flight, no register round trip), waiting only for the
// oldest step.  Wavefront w multiplies expert tiles w*EBT .. w*EBT+EBT-1 (16 experts each) with
// all token tiles, v_mfma_f32_16x16x32_bf16.
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

constexpr int kThreads = 256;
constexpr int kWaves = 4;
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

template <typename WT, int TBT, int EBT, int NS>
__global__ __launch_bounds__(kThreads) void k_gate_logits_dma(Pass p)
{
    constexpr bool F32 = sizeof(WT) == 4;
    constexpr int TB = 16 * TBT, EB = 64 * EBT;
    constexpr int XBYTES = TB * 128, WROW = F32 ? 256 : 128, WBYTES = EB * WROW, STAGE = XBYTES + WBYTES;
    constexpr int XP = XBYTES / 1024, WP = WBYTES / 1024;   // 1 KB pieces: 8 rows of 128 B, or 4 rows of 256 B
    constexpr int PW = (XP + WP) / kWaves;                  // pieces per wavefront per K-step
    static_assert((XP + WP) % kWaves == 0, "pieces are dealt evenly to the wavefronts");
    static_assert(NS >= 2 && NS * STAGE <= 160 * 1024 && (NS - 2) * PW < 64, "ring fits LDS and the load counter");
    __shared__ __attribute__((aligned(1024))) char ring[NS * STAGE];

    const int E = p.E, H = p.H;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int t0 = blockIdx.x * TB, e0 = blockIdx.y * EB;
    const char *xbase = (const char *)p.x;
    const char *wbase = (const char *)p.router_w;

    // ---- this lane's share of every K-step: piece (wave + 4 i), its global byte offset at k = 0 ----
    uint32_t src[PW];
    uint32_t dst[PW];   // wave-uniform LDS offset of the piece inside a stage
#pragma unroll
    for (int i = 0; i < PW; ++i) {
        const int pc = wave + kWaves * i;
        if (pc < XP) {
            const int row = pc * 8 + (lane >> 3);
            const int chunk = (lane & 7) ^ ((row >> 1) & 7);
            src[i] = (uint32_t)min(t0 + row, p.T - 1) * (uint32_t)H * 2u + chunk * 16;
            dst[i] = pc * 1024;
        } else if (!F32) {
            const int row = (pc - XP) * 8 + (lane >> 3);
            const int chunk = (lane & 7) ^ ((row >> 1) & 7);
            src[i] = (uint32_t)min(e0 + row, E - 1) * (uint32_t)H * 2u + chunk * 16;
            dst[i] = XBYTES + (pc - XP) * 1024;
        } else {
            const int row = (pc - XP) * 4 + (lane >> 4);
            const int chunk = (lane & 15) ^ (row & 15);
            src[i] = (uint32_t)min(e0 + row, E - 1) * (uint32_t)H * 4u + chunk * 16;
            dst[i] = XBYTES + (pc - XP) * 1024;
        }
    }
    const uint32_t ring_a = lds_addr(ring);
    auto issue = [&](int kt, int slot) {
#pragma unroll
        for (int i = 0; i < PW; ++i) {
            const bool isx = wave + kWaves * i < XP;
            const char *b = isx ? xbase + (size_t)kt * (kBK * 2) : wbase + (size_t)kt * (kBK * (F32 ? 4 : 2));
            dma_piece(b, src[i], ring_a + slot * STAGE + __builtin_amdgcn_readfirstlane(dst[i]));
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

    auto multiply = [&](int slot) {
        const char *X = ring + slot * STAGE;
        const char *W = X + XBYTES + wave * EBT * 16 * WROW;
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

    // ---- K loop: steps kt+1 .. kt+NS-1 are in flight while step kt is multiplied ----
    const int KT = H / kBK;
    for (int s = 0; s < NS - 1 && s < KT; ++s) issue(s, s);
    int slot = 0, fill = NS - 1;
    for (int kt = 0; kt < KT; ++kt) {
        // younger steps that may stay in flight: those issued after step kt, at most NS-2 of them
        const int younger = min(NS - 2, KT - 1 - kt);
        if (younger >= NS - 2)      wait_loads<(NS - 2) * PW>();
        else if (younger == 3)      wait_loads<(NS > 5 ? 3 : 0) * PW>();
        else if (younger == 2)      wait_loads<(NS > 4 ? 2 : 0) * PW>();
        else if (younger == 1)      wait_loads<(NS > 3 ? 1 : 0) * PW>();
        else                        wait_loads<0>();
        __syncthreads();   // everyone's pieces of step kt have landed; everyone is done reading step kt-1
        if (kt + NS - 1 < KT) issue(kt + NS - 1, fill);
        multiply(slot);
        slot = slot + 1 == NS ? 0 : slot + 1;
        fill = fill + 1 == NS ? 0 : fill + 1;
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

template <typename WT, int TBT, int EBT, int NS>
hipError_t launch_t(const Pass &p, hipStream_t st)
{
    dim3 grid((p.T + 16 * TBT - 1) / (16 * TBT), (p.E + 64 * EBT - 1) / (64 * EBT));
    hipLaunchKernelGGL((k_gate_logits_dma<WT, TBT, EBT, NS>), grid, dim3(kThreads), 0, st, p);
    return hipGetLastError();
}

}  // namespace

// whole K-steps only (the copies cannot zero fill), and 32-bit byte offsets into x and the router
bool gate_dma_supports(const Pass &p)
{
    return p.act_bf16 && p.H % kBK == 0 && p.H >= kBK && (size_t)p.T * p.H * 2 < ((size_t)1 << 32) && (size_t)p.E * p.H * 4 < ((size_t)1 << 32);
}

hipError_t launch_gate_logits_dma(const Pass &p, hipStream_t st)
{
    const bool wide = p.E > 64 && p.T >= 8192;   // 64 tokens x 128 experts per workgroup, else 32 x 64
    if (p.router_bf16) return wide ? launch_t<uint16_t, 4, 2, 6>(p, st) : launch_t<uint16_t, 2, 1, 6>(p, st);
    return wide ? launch_t<float, 4, 2, 3>(p, st) : launch_t<float, 2, 1, 6>(p, st);
}

}  // namespace emoe
