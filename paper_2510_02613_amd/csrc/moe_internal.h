// Internal declarations shared by the translation units of libelasticmoe.so.
// Host-side launch wrappers only; every kernel lives in its own .hip file.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elasticmoe.h"

namespace emoe {

// One M-tile of the grouped GEMMs: `rows` consecutive grouped rows starting at
// `row_begin`, all belonging to weight slot `slot`.
struct MTile {
    int32_t slot;
    int32_t row_begin;
    int32_t rows;
    int32_t single;   // 1 when the tile is all of its slot's rows (nobody else reads the slot's weights in this pass)
};

// One work unit of the large-tile GEMMs: an M-tile with a run of its N-slices.  The unit list of a GEMM is
// read as rows of 8: entry 8 i + x is the i-th unit of XCD x (workgroup b serves XCD b mod 8), so which
// column a unit sits in decides where it runs; rows == 0 marks a hole at the end of a column.
struct MUnit {
    int32_t slot;
    int32_t row_begin;
    int32_t rows;
    int32_t info;     // first N-slice of the run << 1 | the tile's single flag
};
struct UnitHdr {
    int32_t n_rows;   // rows of 8 workgroups the launch has to run: unit rows x spp
    int32_t spp;      // N-slices per unit
    int32_t n_units;  // entries of the list, holes included (a multiple of 8)
    int32_t runs;     // runs a tile's N-slices are split into
};

constexpr int kUnitSlack = 2;   // units by which an XCD's column of the unit list may exceed an even deal

// Runs a tile's N-slices are split into so that the units deal out evenly to the 8 XCDs: the smallest
// divisor d of n_slices with at most 5 % of an XCD's share idle if all units were alike, else n_slices.
__host__ __device__ inline int mfma8_runs(int n_chunks, int n_slices)
{
    for (int d = 1; d < n_slices; ++d) {
        const int units = n_chunks * d, dealt = (units + 7) / 8 * 8;
        if (n_slices % d == 0 && (dealt - units) * 20 <= units) return d;
    }
    return n_slices;
}

// Everything the kernels need to know about one forward pass.  Plain device
// pointers into caller-owned memory (x/out/weights) and the caller's workspace.
struct Pass {
    // layer
    int32_t T, H, I, E, k, S, kk;  // kk = k + n_shared : assignment columns per token
    int32_t n_shared;
    int32_t act_bf16, router_bf16;
    int32_t gate, n_group, topk_group, renormalize;
    float routed_scale;
    int32_t shared_begin, shared_end;
    // caller buffers
    const void *x;
    void *out;
    const void *router_w;
    const float *logit_bias, *select_bias;
    const void *w13, *w2;
    // workspace
    const int32_t *map;  // [E + n_shared] active table, shared slots last
    float *logits;       // [logit_planes][T,E] gate logits (bf16-activation path): the planes are partial sums over K ranges
    int32_t logit_planes;
    int32_t *ids;        // [T,k]
    float *w;            // [T,k]
    int32_t *slot_rank;  // [T*kk] (slot << 12 | rank-in-block) or -1
    int32_t *blk_hist;   // [NB,S] per-block histogram, then per-block exclusive base (fused bookkeeping: [S][row stride] token masks)
    uint8_t *blk_cnt;    // fused bookkeeping: [S][row stride] rows per slot and block of 16 tokens
    int32_t *counts;     // [S]
    int32_t *offs;       // [S+1]
    int32_t *perm;       // [A]
    int32_t *inv;        // [T,kk]
    MTile *tiles;        // [max_tiles]
    int32_t *n_tiles;    // [1]
    MUnit *units[2];     // large-tile GEMMs only: the unit lists of GEMM-1 and GEMM-2, unit_cap entries each (else NULL)
    UnitHdr *unit_hdr;   // [2]
    int32_t unit_cap;
    int32_t n_slices[2]; // N-slices of a tile in GEMM-1 and GEMM-2
    void *h;             // [A,I]
    void *y;             // [A,H]
    int32_t max_tiles;
    int32_t gate_tiled;  // the LDS-tiled gate logits kernel is forced (testing aid)
    int32_t self_tiles;  // weight-streaming GEMM-1 only: its workgroups derive their tile from the selection kernel's per-block counts and
                         // masks themselves, and workgroup 0 of the launch writes the tables (offsets, permutation, tile list) beside them
    int32_t fused_hist;  // the selection kernel also ranks the assignments (blocks of kFusedTokens tokens, blk_hist [S][blocks]
                         // of token masks); the scan-and-place kernel finishes the bookkeeping
    float *partials;     // partial sums of the large-tile GEMMs' split tiles, or NULL (no room: never split)
    int32_t n_cus;       // compute units of the device (set by the large-tile launcher)
    int32_t k_split;     // this launch may share the contraction of its last round's tiles out (set by the launcher)
};

constexpr int kGatePlanes = 8;         // partial-sum planes of the gate logits the workspace has room for
constexpr int kAssignPerBlock = 1024;  // assignments ranked by one block of the slot histogram kernel
constexpr int kFusedTokens = 16;       // tokens per workgroup of the fused selection + ranking kernel (one per wavefront)
constexpr int kFusedMaxTokens = 8192;  // largest batch the fused bookkeeping serves: every placing workgroup reads all block masks
// words between the rows of blk_hist [S][blocks] in the fused bookkeeping: whole groups of 64 blocks
__host__ __device__ constexpr int fused_row_stride(int n_blocks) { return (n_blocks + 63) / 64 * 64; }

hipError_t launch_write_map(int32_t *dst, const int32_t *host_vals, int n, hipStream_t st);
hipError_t launch_copy(void *dst, const void *src, size_t bytes, int blocks, hipStream_t st);  // bytes % 16 == 0
hipError_t launch_gate(const Pass &p, hipStream_t st);
hipError_t launch_gate_logits_dma(const Pass &p, int *planes, hipStream_t st);   // logits only, bf16 activations
bool gate_dma_supports(const Pass &p);
hipError_t launch_permute(const Pass &p, int tile_rows, bool sort_tiles, hipStream_t st);
// which: 0 = first GEMM (gather + SwiGLU), 1 = second GEMM
hipError_t launch_experts_generic(const Pass &p, int which, hipStream_t st);
hipError_t launch_experts_mfma(const Pass &p, int which, hipStream_t st);
int mfma_tile_rows();
// 8-wavefront large-tile variant (needs H % 64 == 0 and I % 64 == 0)
hipError_t launch_experts_mfma8(const Pass &p, int which, hipStream_t st);
int mfma8_tile_rows();
bool mfma8_supports(const Pass &p);
int mfma8_n_slices(int H, int I, int which);   // N-slices of a tile in GEMM-1 (which = 0) or GEMM-2
int mfma8_grid_rows(int max_tiles, int n_slices);   // rows of 8 workgroups a launch provides
size_t mfma8_partial_bytes();   // workspace for the partial sums of tiles whose contraction is shared out
hipError_t launch_ceiling_mfma(int blocks, int iters, int random_operands, float *sink, hipStream_t st);
double ceiling_mfma_flops(int blocks, int iters);
hipError_t launch_ceiling_stream(const void *buf, size_t bytes, float *sink, hipStream_t st);
hipError_t launch_ceiling_tile_stream(const void *buf, int n_tiles, size_t row_bytes, int non_temporal, hipStream_t st);
// weight-streaming variant for decode-sized batches (M-tiles of 16 rows)
hipError_t launch_experts_decode(const Pass &p, int which, hipStream_t st);
int decode_tile_rows();
bool decode_self_tiles(const Pass &p);   // GEMM-1 needs no bookkeeping kernel in front of it (Pass::self_tiles)
hipError_t launch_identity_experts(const Pass &p, hipStream_t st);
hipError_t launch_combine(const Pass &p, hipStream_t st);

// A layer that was told which page pools its weights live in (moe_layer_bind_vpools) checks on the host that
// every slot a placement names has a page under it; the pool tells the layer when it goes away.
bool vpool_backed(const moe_vpool *pool, int32_t slot);          // moe_vpool.hip
void vpool_bind(moe_vpool *pool, moe_layer *layer);
void vpool_unbind(moe_vpool *pool, moe_layer *layer);
void layer_drop_vpool(moe_layer *layer, const moe_vpool *pool);  // moe_api.hip

constexpr int kGenericTileRows = 32;  // M-tile of the plain expert kernels

// ---- small device helpers ---------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16, round to nearest even (one v_cvt_pk_bf16_f32 per pair on gfx950)
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    const __bf16 b = (__bf16)f;
    return __builtin_bit_cast(uint16_t, b);
}

// silu(g) * u with the hardware exp2 / reciprocal (about 1 ulp each): g * u / (1 + exp(-g))
__device__ __forceinline__ float silu_mul(float g, float u)
{
    return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u;
}

template <typename T> __device__ __forceinline__ float load_f32(const T *p, size_t i);
template <> __device__ __forceinline__ float load_f32<float>(const float *p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float load_f32<uint16_t>(const uint16_t *p, size_t i) { return bf16_to_f32(p[i]); }

template <typename T> __device__ __forceinline__ void store_f32(T *p, size_t i, float v);
template <> __device__ __forceinline__ void store_f32<float>(float *p, size_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void store_f32<uint16_t>(uint16_t *p, size_t i, float v) { p[i] = f32_to_bf16(v); }

}  // namespace emoe
