// Host side of libelasticmoe.so: argument checking, workspace carving, the
// expert-map switch and the launch sequence of one forward pass.
//
// The library owns no device memory (the paper's execution processes only hold
// references to tensors kept by the memory daemon, Sec. 3.2 "Decoupled Memory and
// Execution Layers"); all intermediates live in the caller's workspace, which is
// carved once at create time, so no later call can allocate.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "moe_internal.h"

using namespace emoe;

// Scratch of moe_forward_static: the whole workspace of its pass lives here, so that the call needs no
// device memory from anybody.  One copy per GPU the library is loaded on, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[MOE_STATIC_SCRATCH_BYTES];

namespace {
thread_local char g_err[512] = "";
}

namespace emoe {
// the message moe_last_error() returns on this thread (shared by every translation unit of the library)
moe_status_t set_error(moe_status_t st, const char *fmt, va_list ap)
{
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    return st;
}
}  // namespace emoe

namespace {

moe_status_t fail(moe_status_t st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    set_error(st, fmt, ap);
    va_end(ap);
    return st;
}

constexpr size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
constexpr int kMinTileRows = 16;  // smallest M-tile any expert kernel uses: sizes the tile list

// Offsets of every intermediate inside the workspace.
struct Layout {
    size_t map, logits, ids, w, slot_rank, blk_hist, blk_cnt, counts, offs, perm, inv, tiles, n_tiles, units[2], unit_hdr, h, y, partials, total;
    size_t unit_cap;
    bool has_partials;
};

size_t esize(int dtype) { return dtype == MOE_BF16 ? 2 : 4; }

moe_status_t check_config(const moe_config_t *c)
{
    if (!c) return fail(MOE_ERR_ARG, "config is NULL");
    if (c->hidden <= 0 || c->inter <= 0 || c->n_experts <= 0 || c->top_k <= 0 || c->n_slots <= 0 || c->max_tokens <= 0)
        return fail(MOE_ERR_SHAPE, "hidden, inter, n_experts, top_k, n_slots, max_tokens must all be positive");
    if (c->act_dtype != MOE_F32 && c->act_dtype != MOE_BF16) return fail(MOE_ERR_ARG, "act_dtype %d is not a moe_dtype_t", c->act_dtype);
    if (c->router_dtype != MOE_F32 && c->router_dtype != MOE_BF16) return fail(MOE_ERR_ARG, "router_dtype %d is not a moe_dtype_t", c->router_dtype);
    if (c->gate != MOE_GATE_SOFTMAX_TOPK && c->gate != MOE_GATE_SIGMOID_GROUP_TOPK) return fail(MOE_ERR_ARG, "gate %d is not a moe_gate_t", c->gate);
    if (c->n_shared < 0 || c->n_group <= 0 || c->topk_group <= 0) return fail(MOE_ERR_SHAPE, "n_shared >= 0, n_group >= 1, topk_group >= 1 required");
    if (c->top_k > c->n_experts) return fail(MOE_ERR_SHAPE, "top_k %d exceeds n_experts %d", c->top_k, c->n_experts);
    if (c->n_experts % c->n_group) return fail(MOE_ERR_SHAPE, "n_group %d does not divide n_experts %d", c->n_group, c->n_experts);
    if (c->topk_group > c->n_group) return fail(MOE_ERR_SHAPE, "topk_group %d exceeds n_group %d", c->topk_group, c->n_group);
    if (c->gate == MOE_GATE_SOFTMAX_TOPK && (c->n_group != 1 || c->topk_group != 1))
        return fail(MOE_ERR_SHAPE, "the softmax gate has no groups: n_group and topk_group must be 1");
    if ((long long)c->top_k > (long long)c->topk_group * (c->n_experts / c->n_group))
        return fail(MOE_ERR_SHAPE, "top_k %d exceeds the %d experts of %d kept groups", c->top_k, c->topk_group * (c->n_experts / c->n_group), c->topk_group);
    if (c->n_shared > c->n_slots) return fail(MOE_ERR_SHAPE, "n_shared %d exceeds n_slots %d", c->n_shared, c->n_slots);
    if (!(c->routed_scale == c->routed_scale)) return fail(MOE_ERR_ARG, "routed_scale is NaN");
    if (c->hidden % 8 || c->inter % 8) return fail(MOE_ERR_UNSUPPORTED, "hidden and inter must be multiples of 8 (16-byte rows)");
    if (c->n_experts > 1024) return fail(MOE_ERR_UNSUPPORTED, "n_experts > 1024");
    if (c->top_k > 32) return fail(MOE_ERR_UNSUPPORTED, "top_k > 32");
    if (c->n_group > 64) return fail(MOE_ERR_UNSUPPORTED, "n_group > 64");
    if (c->n_shared > 4) return fail(MOE_ERR_UNSUPPORTED, "n_shared > 4");
    if (c->n_slots > 2047) return fail(MOE_ERR_UNSUPPORTED, "n_slots > 2047");
    if ((long long)c->max_tokens * (c->top_k + c->n_shared) > (1ll << 26))
        return fail(MOE_ERR_UNSUPPORTED, "max_tokens * (top_k + n_shared) > 2^26");
    return MOE_OK;
}

Layout make_layout(const moe_config_t &c)
{
    Layout L;
    const size_t T = c.max_tokens, k = c.top_k, kk = c.top_k + c.n_shared, S = c.n_slots;
    const size_t A = T * kk;
    const size_t nb = (A + kAssignPerBlock - 1) / kAssignPerBlock;
    const size_t max_tiles = (A + kMinTileRows - 1) / kMinTileRows + S;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    // a table: E + n_shared entries, then the copy lists of replicated experts (count, slots...:
    // at most S slots in lists of at least two, so 3S/2 entries)
    L.map = take(4 * (c.n_experts + c.n_shared + 2 * S));
    L.logits = take(c.act_dtype == MOE_BF16 ? 4 * T * c.n_experts * kGatePlanes : 0);   // partial-sum planes of the K-split logits kernels
    L.ids = take(4 * T * k);
    L.w = take(4 * T * k);
    L.slot_rank = take(4 * A);
    // block words of the bookkeeping: [blocks of 1024 assignments][S], or (fused with the selection) [S][blocks of 16 tokens]
    const size_t nbf = ((T < (size_t)kFusedMaxTokens ? T : (size_t)kFusedMaxTokens) + kFusedTokens - 1) / kFusedTokens;
    const size_t fused_words = (size_t)fused_row_stride((int)nbf) * S;
    L.blk_hist = take(4 * (nb * S > fused_words ? nb * S : fused_words));
    L.blk_cnt = take(fused_words);
    L.counts = take(4 * S);
    L.offs = take(4 * (S + 1));
    L.perm = take(4 * A);
    L.inv = take(4 * A);
    L.tiles = take(sizeof(MTile) * max_tiles);
    L.n_tiles = take(4);
    // unit lists of the large-tile GEMMs (layers they can serve): one entry per (tile, run of N-slices), in rows of 8
    L.unit_cap = 0;
    if (c.act_dtype == MOE_BF16 && c.hidden % 64 == 0 && c.inter % 64 == 0 && A >= 48 * S) {
        const size_t big_tiles = (A + mfma8_tile_rows() - 1) / mfma8_tile_rows() + S;
        const int ns0 = mfma8_n_slices(c.hidden, c.inter, 0), ns1 = mfma8_n_slices(c.hidden, c.inter, 1);
        L.unit_cap = 8 * (size_t)mfma8_grid_rows((int)big_tiles, ns0 > ns1 ? ns0 : ns1);
    }
    L.units[0] = take(sizeof(MUnit) * L.unit_cap);
    L.units[1] = take(sizeof(MUnit) * L.unit_cap);
    L.unit_hdr = take(L.unit_cap ? 2 * sizeof(UnitHdr) : 0);
    L.h = take(esize(c.act_dtype) * A * c.inter);
    L.y = take(esize(c.act_dtype) * A * c.hidden);
    // partial sums of split tiles: only layers whose large-tile GEMMs can have contractions long enough to split
    L.has_partials = c.act_dtype == MOE_BF16 && c.hidden % 64 == 0 && c.inter % 64 == 0 && (c.hidden >= 4096 || c.inter >= 4096) &&
                     A >= 48 * S;
    L.partials = take(L.has_partials ? mfma8_partial_bytes() : 0);
    L.total = o;
    return L;
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

}  // namespace

constexpr int kProfRing = 64;  // forwards whose phase events are kept

struct moe_layer {
    bool prof_on = false;
    long long prof_count = 0;  // forwards recorded since profiling was enabled
    long long prof_seen = 0;   // forwards issued since then
    int prof_every = 1;        // every prof_every-th forward is recorded
    int prof_phase = -1;       // the one phase whose two events are recorded, or -1: all of them
    hipEvent_t ev[kProfRing][MOE_N_PHASES + 1] = {};
    moe_config_t cfg;
    moe_buffers_t buf;
    Layout lay;
    bool has_map;
    std::vector<int32_t> slot_owner;  // per slot: entry (expert, or E + shared expert) of the active table that uses it, or -1
    // slot fills that the next map switch has to wait for (one event per fill, reused after the switch)
    std::vector<hipEvent_t> load_ev;
    int n_pending = 0;
    hipEvent_t serve_ev = nullptr;  // "work enqueued on the serving stream so far", recorded per fill
    moe_vpool *vpool[2] = {nullptr, nullptr};  // the page pools under w13 and w2 when the layer was told (moe_layer_bind_vpools)
};

namespace emoe {
void layer_drop_vpool(moe_layer *l, const moe_vpool *p)
{
    for (int i = 0; i < 2; ++i)
        if (l->vpool[i] == p) l->vpool[i] = nullptr;
}
}  // namespace emoe

// With page pools bound: slot s must have a page under it in both.
static moe_status_t check_backed(const moe_layer *l, int32_t s, const char *what)
{
    static const char *const name[2] = {"w13", "w2"};
    for (int i = 0; i < 2; ++i)
        if (l->vpool[i] && !vpool_backed(l->vpool[i], s))
            return fail(MOE_ERR_MAP, "%s: slot %d has no page under it in the %s pool", what, s, name[i]);
    return MOE_OK;
}
static moe_status_t check_owned_backed(const moe_layer *l, const std::vector<int32_t> &owner, const char *what)
{
    if (!l->vpool[0] && !l->vpool[1]) return MOE_OK;
    for (int32_t s = 0; s < (int32_t)owner.size(); ++s)
        if (owner[s] >= 0) {
            const moe_status_t st = check_backed(l, s, what);
            if (st != MOE_OK) return st;
        }
    return MOE_OK;
}

extern "C" {

const char *moe_last_error(void) { return g_err; }

size_t moe_workspace_bytes(const moe_config_t *cfg)
{
    if (check_config(cfg) != MOE_OK) return 0;
    return make_layout(*cfg).total;
}

moe_status_t moe_layer_create(const moe_config_t *cfg, const moe_buffers_t *buf, moe_layer_t **out)
{
    if (!out) return fail(MOE_ERR_ARG, "out is NULL");
    *out = nullptr;
    moe_status_t st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (!buf) return fail(MOE_ERR_ARG, "buffers is NULL");
    if (!buf->router_w || !buf->w13 || !buf->w2 || !buf->workspace)
        return fail(MOE_ERR_ARG, "router_w, w13, w2 and workspace must be non-NULL");
    if (!aligned(buf->router_w, 16) || !aligned(buf->w13, 16) || !aligned(buf->w2, 16))
        return fail(MOE_ERR_ARG, "router_w, w13 and w2 must be 16-byte aligned");
    if (!aligned(buf->workspace, kAlign)) return fail(MOE_ERR_ARG, "workspace must be 256-byte aligned");
    if ((buf->logit_bias && !aligned(buf->logit_bias, 4)) || (buf->select_bias && !aligned(buf->select_bias, 4)))
        return fail(MOE_ERR_ARG, "bias vectors must be 4-byte aligned");
    Layout L = make_layout(*cfg);
    if (buf->workspace_bytes < L.total)
        return fail(MOE_ERR_CAPACITY, "workspace has %zu bytes, layer needs %zu", buf->workspace_bytes, L.total);
    moe_layer *l = new (std::nothrow) moe_layer;
    if (!l) return fail(MOE_ERR_ARG, "out of host memory");
    l->cfg = *cfg;
    l->buf = *buf;
    l->lay = L;
    l->has_map = false;
    *out = l;
    return MOE_OK;
}

moe_status_t moe_ceiling_mfma(int32_t blocks, int32_t iters, int32_t random_operands, float *sink, void *hip_stream, double *flops)
{
    if (blocks <= 0 || iters <= 0 || !sink || !flops) return fail(MOE_ERR_ARG, "blocks and iters must be positive, sink and flops non-NULL");
    if (blocks > (1 << 20) || iters > (1 << 24)) return fail(MOE_ERR_ARG, "blocks <= 2^20 and iters <= 2^24");
    *flops = ceiling_mfma_flops(blocks, iters);
    const hipError_t e = launch_ceiling_mfma(blocks, iters, random_operands, sink, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "ceiling launch failed: %s", hipGetErrorString(e));
    return MOE_OK;
}

moe_status_t moe_ceiling_stream(const void *buf, size_t bytes, float *sink, void *hip_stream)
{
    if (!buf || !sink || bytes < 16) return fail(MOE_ERR_ARG, "buf and sink must be non-NULL and bytes >= 16");
    if (!aligned(buf, 16)) return fail(MOE_ERR_ARG, "buf must be 16-byte aligned");
    const hipError_t e = launch_ceiling_stream(buf, bytes, sink, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "ceiling launch failed: %s", hipGetErrorString(e));
    return MOE_OK;
}

moe_status_t moe_ceiling_tile_stream(const void *buf, int32_t n_tiles, size_t row_bytes, int32_t non_temporal, void *hip_stream)
{
    if (!buf || !aligned(buf, 16)) return fail(MOE_ERR_ARG, "buf must be non-NULL and 16-byte aligned");
    if (n_tiles <= 0) return fail(MOE_ERR_ARG, "n_tiles %d is not positive", n_tiles);
    if (row_bytes < 128 || row_bytes % 128 != 0 || row_bytes * 256 >= ((size_t)1 << 32))
        return fail(MOE_ERR_ARG, "row_bytes %zu must be a multiple of 128 below 2^24", row_bytes);
    const hipError_t e = launch_ceiling_tile_stream(buf, n_tiles, row_bytes, non_temporal, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "ceiling launch failed: %s", hipGetErrorString(e));
    return MOE_OK;
}

void moe_layer_destroy(moe_layer_t *layer)
{
    if (!layer) return;
    if (layer->prof_on) moe_profile_enable(layer, 0);
    for (hipEvent_t ev : layer->load_ev) (void)hipEventDestroy(ev);
    if (layer->serve_ev) (void)hipEventDestroy(layer->serve_ev);
    for (int i = 0; i < 2; ++i)
        if (layer->vpool[i]) vpool_unbind(layer->vpool[i], layer);
    delete layer;
}

moe_status_t moe_profile_enable(moe_layer_t *l, int32_t enable)
{
    if (!l) return fail(MOE_ERR_ARG, "layer is NULL");
    if (enable < 0) return fail(MOE_ERR_ARG, "enable %d is negative", enable);
    if (enable && l->prof_on) {   // only the sampling changes
        l->prof_every = enable;
        l->prof_seen = 0;          // the next forward is recorded
        return MOE_OK;
    }
    if ((enable != 0) == l->prof_on) return MOE_OK;
    if (enable) {
        for (int i = 0; i < kProfRing; ++i)
            for (int j = 0; j <= MOE_N_PHASES; ++j) {
                hipError_t e = hipEventCreate(&l->ev[i][j]);
                if (e != hipSuccess) {
                    for (int a = 0; a <= i; ++a)
                        for (int b = 0; b <= MOE_N_PHASES; ++b)
                            if (l->ev[a][b]) { (void)hipEventDestroy(l->ev[a][b]); l->ev[a][b] = nullptr; }
                    return fail(MOE_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
                }
            }
        l->prof_count = 0;
        l->prof_seen = 0;
        l->prof_every = enable;
        l->prof_on = true;
    } else {
        for (int i = 0; i < kProfRing; ++i)
            for (int j = 0; j <= MOE_N_PHASES; ++j)
                if (l->ev[i][j]) { (void)hipEventDestroy(l->ev[i][j]); l->ev[i][j] = nullptr; }
        l->prof_on = false;
    }
    return MOE_OK;
}

moe_status_t moe_profile_select(moe_layer_t *l, int32_t phase)
{
    if (!l) return fail(MOE_ERR_ARG, "layer is NULL");
    if (phase < -1 || phase >= MOE_N_PHASES) return fail(MOE_ERR_ARG, "phase %d is outside [-1, %d)", phase, MOE_N_PHASES);
    l->prof_phase = phase;
    l->prof_count = 0;         // recordings made under another selection cannot be read as this one
    l->prof_seen = 0;
    return MOE_OK;
}

moe_status_t moe_profile_read(moe_layer_t *l, int32_t back, float *ms)
{
    if (!l || !ms) return fail(MOE_ERR_ARG, "layer or ms is NULL");
    if (!l->prof_on) return fail(MOE_ERR_ARG, "profiling is not enabled on this layer");
    if (back < 0 || back >= kProfRing || back >= l->prof_count)
        return fail(MOE_ERR_ARG, "no recorded forward %d steps back (recorded %lld, kept %d)", back, l->prof_count, kProfRing);
    hipEvent_t *ev = l->ev[(l->prof_count - 1 - back) % kProfRing];
    const int sel = l->prof_phase;
    hipError_t e = hipEventSynchronize(ev[sel < 0 ? MOE_N_PHASES : sel + 1]);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipEventSynchronize: %s", hipGetErrorString(e));
    for (int j = 0; j < MOE_N_PHASES; ++j) {
        ms[j] = 0.f;
        if (sel >= 0 && j != sel) continue;
        e = hipEventElapsedTime(&ms[j], ev[j], ev[j + 1]);
        if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipEventElapsedTime: %s", hipGetErrorString(e));
    }
    return MOE_OK;
}

namespace {

// Validated placement -> the device table.  There is ONE table at a fixed address, rewritten in place by a
// kernel on hip_stream: passes enqueued on that stream before the switch have read it by then, passes after it
// (a replay of a captured graph included: the table's address is all a captured pass holds) read the new one.
moe_status_t install_table(moe_layer_t *l, std::vector<int32_t> &table, std::vector<int32_t> &owner, void *hip_stream)
{
    int32_t *dst = (int32_t *)((char *)l->buf.workspace + l->lay.map);
    const moe_status_t backed = check_owned_backed(l, owner, "the placement names a slot that cannot be read");
    if (backed != MOE_OK) return backed;
    hipError_t e = hipSuccess;
    // slot fills enqueued by moe_load_expert: everything after this switch on hip_stream sees them complete
    for (int i = 0; i < l->n_pending && e == hipSuccess; ++i) e = hipStreamWaitEvent((hipStream_t)hip_stream, l->load_ev[i], 0);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "waiting for slot fills failed: %s", hipGetErrorString(e));
    l->n_pending = 0;
    e = launch_write_map(dst, table.data(), (int)table.size(), (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "expert map upload failed: %s", hipGetErrorString(e));
    l->has_map = true;
    l->slot_owner.swap(owner);
    return MOE_OK;
}

// entry `who` (expert e, or E + shared expert) claims slot s
moe_status_t claim_slot(const moe_config_t &c, std::vector<int32_t> &owner, int32_t s, int who)
{
    const bool shared = who >= c.n_experts;
    if (s < 0 || s >= c.n_slots)
        return fail(MOE_ERR_MAP, "%s %d -> slot %d is outside [0, %d)", shared ? "shared expert" : "expert",
                    shared ? who - c.n_experts : who, s, c.n_slots);
    if (owner[s] >= 0) return fail(MOE_ERR_MAP, "slot %d is claimed twice (entries %d and %d)", s, owner[s], who);
    owner[s] = who;
    return MOE_OK;
}

}  // namespace

// Checks a plain placement (at most one slot per expert) and writes its device table (E + n_shared
// entries) and the slot -> entry index (S entries) into caller-provided arrays.
static moe_status_t validate_plain_map(const moe_config_t &c, const int32_t *host_map, int32_t n, const int32_t *host_shared_slots,
                                       int32_t *table, int32_t *owner)
{
    if (!host_map) return fail(MOE_ERR_ARG, "host_map is NULL");
    if (n != c.n_experts) return fail(MOE_ERR_MAP, "map has %d entries, layer has %d logical experts", n, c.n_experts);
    if ((c.n_shared > 0) != (host_shared_slots != nullptr))
        return fail(MOE_ERR_MAP, "host_shared_slots must be given exactly when n_shared > 0");
    for (int s = 0; s < c.n_slots; ++s) owner[s] = -1;
    for (int e = 0; e < c.n_experts + c.n_shared; ++e) {
        const bool shared = e >= c.n_experts;
        const int32_t s = shared ? host_shared_slots[e - c.n_experts] : host_map[e];
        if (s < -1 || (shared && s < 0))
            return fail(MOE_ERR_MAP, "%s %d -> slot %d is outside [%s, %d)", shared ? "shared expert" : "expert",
                        shared ? e - c.n_experts : e, s, shared ? "0" : "-1", c.n_slots);
        if (s >= 0) {
            if (s >= c.n_slots)
                return fail(MOE_ERR_MAP, "%s %d -> slot %d is outside [0, %d)", shared ? "shared expert" : "expert",
                            shared ? e - c.n_experts : e, s, c.n_slots);
            if (owner[s] >= 0) return fail(MOE_ERR_MAP, "slot %d is claimed twice (entries %d and %d)", s, owner[s], e);
            owner[s] = e;
        }
        table[e] = s;
    }
    return MOE_OK;
}

moe_status_t moe_set_expert_map(moe_layer_t *l, const int32_t *host_map, int32_t n,
                                const int32_t *host_shared_slots, void *hip_stream)
{
    if (!l) return fail(MOE_ERR_ARG, "layer is NULL");
    const moe_config_t &c = l->cfg;
    std::vector<int32_t> owner(c.n_slots, -1);  // slot -> entry index that claimed it
    std::vector<int32_t> table(c.n_experts + c.n_shared);
    const moe_status_t st = validate_plain_map(c, host_map, n, host_shared_slots, table.data(), owner.data());
    if (st != MOE_OK) return st;
    return install_table(l, table, owner, hip_stream);
}

moe_status_t moe_set_expert_replicas(moe_layer_t *l, const int32_t *host_rep_offsets, const int32_t *host_rep_slots,
                                     int32_t n, const int32_t *host_shared_slots, void *hip_stream)
{
    if (!l) return fail(MOE_ERR_ARG, "layer is NULL");
    if (!host_rep_offsets) return fail(MOE_ERR_ARG, "host_rep_offsets is NULL");
    const moe_config_t &c = l->cfg;
    if (n != c.n_experts) return fail(MOE_ERR_MAP, "placement has %d experts, layer has %d logical experts", n, c.n_experts);
    if ((c.n_shared > 0) != (host_shared_slots != nullptr))
        return fail(MOE_ERR_MAP, "host_shared_slots must be given exactly when n_shared > 0");
    if (host_rep_offsets[0] != 0) return fail(MOE_ERR_MAP, "host_rep_offsets[0] is %d, must be 0", host_rep_offsets[0]);
    for (int e = 0; e < n; ++e)
        if (host_rep_offsets[e + 1] < host_rep_offsets[e] || host_rep_offsets[e + 1] > c.n_slots)
            return fail(MOE_ERR_MAP, "host_rep_offsets must be non-decreasing and end at no more than n_slots = %d (entry %d is %d)",
                        c.n_slots, e + 1, host_rep_offsets[e + 1]);
    if (host_rep_offsets[n] > 0 && !host_rep_slots) return fail(MOE_ERR_ARG, "host_rep_slots is NULL");
    std::vector<int32_t> owner(c.n_slots, -1);
    std::vector<int32_t> table(c.n_experts + c.n_shared);
    for (int e = 0; e < n; ++e) {
        const int b = host_rep_offsets[e], R = host_rep_offsets[e + 1] - b;
        for (int r = 0; r < R; ++r) {
            const moe_status_t st = claim_slot(c, owner, host_rep_slots[b + r], e);
            if (st != MOE_OK) return st;
        }
        if (R == 0) {
            table[e] = -1;
        } else if (R == 1) {
            table[e] = host_rep_slots[b];
        } else {
            // the copy list (count, slots) goes behind the E + n_shared entries; the entry encodes where
            table[e] = -2 - (int32_t)(table.size() - (size_t)(c.n_experts + c.n_shared));
            table.push_back(R);
            for (int r = 0; r < R; ++r) table.push_back(host_rep_slots[b + r]);
        }
    }
    for (int i = 0; i < c.n_shared; ++i) {
        const moe_status_t st = claim_slot(c, owner, host_shared_slots[i], c.n_experts + i);
        if (st != MOE_OK) return st;
        table[c.n_experts + i] = host_shared_slots[i];
    }
    return install_table(l, table, owner, hip_stream);
}

moe_status_t moe_layer_bind_vpools(moe_layer_t *l, moe_vpool_t *w13_pool, moe_vpool_t *w2_pool)
{
    if (!l) return fail(MOE_ERR_ARG, "layer is NULL");
    const moe_config_t &c = l->cfg;
    const size_t es = esize(c.act_dtype);
    const size_t want[2] = {2 * (size_t)c.inter * c.hidden * es, (size_t)c.hidden * c.inter * es};
    moe_vpool_t *pool[2] = {w13_pool, w2_pool};
    const void *base[2] = {l->buf.w13, l->buf.w2};
    static const char *const name[2] = {"w13", "w2"};
    for (int i = 0; i < 2; ++i) {
        if (!pool[i]) continue;
        if (moe_vpool_base(pool[i]) != base[i]) return fail(MOE_ERR_ARG, "the %s pool does not start where the layer's %s does", name[i], name[i]);
        if (moe_vpool_slot_bytes(pool[i]) != want[i])
            return fail(MOE_ERR_ARG, "the %s pool has slots of %zu bytes, the layer's are %zu", name[i], moe_vpool_slot_bytes(pool[i]), want[i]);
        if (moe_vpool_slots(pool[i]) < c.n_slots)
            return fail(MOE_ERR_ARG, "the %s pool has %d slots, the layer has %d", name[i], moe_vpool_slots(pool[i]), c.n_slots);
    }
    moe_vpool *old[2] = {l->vpool[0], l->vpool[1]};
    l->vpool[0] = w13_pool;
    l->vpool[1] = w2_pool;
    if (l->has_map) {   // the placement in force must already be readable
        const moe_status_t st = check_owned_backed(l, l->slot_owner, "the active placement names a slot that cannot be read");
        if (st != MOE_OK) { l->vpool[0] = old[0]; l->vpool[1] = old[1]; return st; }
    }
    for (int i = 0; i < 2; ++i) {
        if (old[i] && old[i] != l->vpool[i]) vpool_unbind(old[i], l);
        if (l->vpool[i]) vpool_bind(l->vpool[i], l);
    }
    return MOE_OK;
}

moe_status_t moe_load_expert(moe_layer_t *l, int32_t slot, const void *src_w13, const void *src_w2,
                             void *copy_stream, void *serve_stream, int32_t copy_blocks)
{
    if (!l) return fail(MOE_ERR_ARG, "layer is NULL");
    const moe_config_t &c = l->cfg;
    if (slot < 0 || slot >= c.n_slots) return fail(MOE_ERR_ARG, "slot %d is outside [0, %d)", slot, c.n_slots);
    if (!src_w13 || !src_w2) return fail(MOE_ERR_ARG, "src_w13 and src_w2 must be non-NULL");
    if (!aligned(src_w13, 16) || !aligned(src_w2, 16)) return fail(MOE_ERR_ARG, "src_w13 and src_w2 must be 16-byte aligned");
    if (copy_blocks < 0 || copy_blocks > 65536) return fail(MOE_ERR_ARG, "copy_blocks %d is outside [0, 65536]", copy_blocks);
    if (copy_stream == serve_stream) return fail(MOE_ERR_ARG, "copy_stream and serve_stream must differ (the fill is meant to run beside the forwards)");
    if (l->has_map && l->slot_owner[slot] >= 0) {
        const int e = l->slot_owner[slot];
        return fail(MOE_ERR_MAP, "slot %d holds %s %d of the active map: it cannot be refilled while forwards may read it", slot,
                    e >= c.n_experts ? "shared expert" : "expert", e >= c.n_experts ? e - c.n_experts : e);
    }
    const moe_status_t backed = check_backed(l, slot, "the fill would write memory that is not there");
    if (backed != MOE_OK) return backed;
    hipError_t e = hipSuccess;
    if (!l->serve_ev) e = hipEventCreateWithFlags(&l->serve_ev, hipEventDisableTiming);
    if (e == hipSuccess && (int)l->load_ev.size() == l->n_pending) {
        hipEvent_t ev = nullptr;
        e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        if (e == hipSuccess) l->load_ev.push_back(ev);
    }
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
    // a forward already enqueued on the serving stream may still read the slot under an older map
    e = hipEventRecord(l->serve_ev, (hipStream_t)serve_stream);
    if (e == hipSuccess) e = hipStreamWaitEvent((hipStream_t)copy_stream, l->serve_ev, 0);
    const size_t es = esize(c.act_dtype);
    const size_t b13 = 2 * (size_t)c.inter * c.hidden * es, b2 = (size_t)c.hidden * c.inter * es;
    const int blocks = copy_blocks ? copy_blocks : 32;
    if (e == hipSuccess) e = launch_copy((char *)const_cast<void *>(l->buf.w13) + (size_t)slot * b13, src_w13, b13, blocks, (hipStream_t)copy_stream);
    if (e == hipSuccess) e = launch_copy((char *)const_cast<void *>(l->buf.w2) + (size_t)slot * b2, src_w2, b2, blocks, (hipStream_t)copy_stream);
    if (e == hipSuccess) e = hipEventRecord(l->load_ev[l->n_pending], (hipStream_t)copy_stream);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "slot fill failed: %s", hipGetErrorString(e));
    l->n_pending++;
    return MOE_OK;
}

moe_status_t moe_workspace_view(const moe_layer_t *l, moe_workspace_view_t *v)
{
    if (!l || !v) return fail(MOE_ERR_ARG, "layer or view is NULL");
    char *ws = (char *)l->buf.workspace;
    v->topk_ids = (const int32_t *)(ws + l->lay.ids);
    v->topk_w = (const float *)(ws + l->lay.w);
    v->counts = (const int32_t *)(ws + l->lay.counts);
    v->offsets = (const int32_t *)(ws + l->lay.offs);
    v->perm = (const int32_t *)(ws + l->lay.perm);
    v->inv = (const int32_t *)(ws + l->lay.inv);
    v->h = ws + l->lay.h;
    v->y = ws + l->lay.y;
    v->active_map = (const int32_t *)(ws + l->lay.map);
    v->tiles = (const int32_t *)(ws + l->lay.tiles);
    v->n_tiles = (const int32_t *)(ws + l->lay.n_tiles);
    v->unit_hdr = l->lay.unit_cap ? (const int32_t *)(ws + l->lay.unit_hdr) : nullptr;
    v->units[0] = l->lay.unit_cap ? (const int32_t *)(ws + l->lay.units[0]) : nullptr;
    v->units[1] = l->lay.unit_cap ? (const int32_t *)(ws + l->lay.units[1]) : nullptr;
    return MOE_OK;
}

// One pass; routed_ids/routed_w non-NULL: the gate is skipped and the caller's routing is read in place.
static moe_status_t forward_pass(moe_layer_t *l, const void *x, int32_t T, const int32_t *routed_ids, const float *routed_w,
                                 int32_t shared_begin, int32_t shared_end, void *out, void *hip_stream, uint32_t flags)
{
    if (!l) return fail(MOE_ERR_ARG, "layer is NULL");
    const moe_config_t &c = l->cfg;
    if (T < 0) return fail(MOE_ERR_ARG, "T is negative");
    if (T > c.max_tokens) return fail(MOE_ERR_CAPACITY, "T %d exceeds max_tokens %d", T, c.max_tokens);
    if (shared_begin < 0 || shared_begin > shared_end || shared_end > T)
        return fail(MOE_ERR_ARG, "shared range [%d,%d) is not inside [0,%d]", shared_begin, shared_end, T);
    if (flags & ~(MOE_FLAG_IDENTITY_EXPERTS | MOE_FLAG_FORCE_GENERIC | MOE_FLAG_GATE_TILED | MOE_FLAG_PERMUTE_UNFUSED)) return fail(MOE_ERR_ARG, "unknown flag bits 0x%x", flags);
    if (!l->has_map) return fail(MOE_ERR_MAP, "no expert map installed: call moe_set_expert_map first");
    {   // page pools bound: a page taken from under a slot of the placement in force would fault the pass
        const moe_status_t backed = check_owned_backed(l, l->slot_owner, "the active placement names a slot whose page is gone");
        if (backed != MOE_OK) return backed;
    }
    if (T == 0) return MOE_OK;
    if (!x || !out) return fail(MOE_ERR_ARG, "x and out must be non-NULL");
    if (!aligned(x, 16) || !aligned(out, 16)) return fail(MOE_ERR_ARG, "x and out must be 16-byte aligned");

    hipStream_t st = (hipStream_t)hip_stream;
    char *ws = (char *)l->buf.workspace;
    Pass p;
    memset(&p, 0, sizeof p);
    p.T = T; p.H = c.hidden; p.I = c.inter; p.E = c.n_experts; p.k = c.top_k; p.S = c.n_slots;
    p.n_shared = c.n_shared; p.kk = c.top_k + c.n_shared;
    p.act_bf16 = c.act_dtype == MOE_BF16; p.router_bf16 = c.router_dtype == MOE_BF16;
    p.gate = c.gate; p.n_group = c.n_group; p.topk_group = c.topk_group; p.renormalize = c.renormalize;
    p.routed_scale = c.routed_scale;
    p.shared_begin = shared_begin; p.shared_end = shared_end;
    p.x = x; p.out = out;
    p.router_w = l->buf.router_w; p.logit_bias = l->buf.logit_bias; p.select_bias = l->buf.select_bias;
    p.w13 = l->buf.w13; p.w2 = l->buf.w2;
    p.map = (const int32_t *)(ws + l->lay.map);
    p.logits = (float *)(ws + l->lay.logits);
    p.logit_planes = 1;
    // the kernels after the gate only read ids and w
    p.ids = routed_ids ? const_cast<int32_t *>(routed_ids) : (int32_t *)(ws + l->lay.ids);
    p.w = routed_w ? const_cast<float *>(routed_w) : (float *)(ws + l->lay.w);
    p.slot_rank = (int32_t *)(ws + l->lay.slot_rank);
    p.blk_hist = (int32_t *)(ws + l->lay.blk_hist);
    p.blk_cnt = (uint8_t *)(ws + l->lay.blk_cnt);
    p.counts = (int32_t *)(ws + l->lay.counts);
    p.offs = (int32_t *)(ws + l->lay.offs);
    p.perm = (int32_t *)(ws + l->lay.perm);
    p.inv = (int32_t *)(ws + l->lay.inv);
    p.tiles = (MTile *)(ws + l->lay.tiles);
    p.n_tiles = (int32_t *)(ws + l->lay.n_tiles);
    p.units[0] = p.units[1] = nullptr;
    p.unit_hdr = nullptr;
    p.h = ws + l->lay.h;
    p.y = ws + l->lay.y;
    p.partials = l->lay.has_partials ? (float *)(ws + l->lay.partials) : nullptr;

    p.gate_tiled = (flags & MOE_FLAG_GATE_TILED) != 0;
    // gated bf16 passes up to kFusedMaxTokens tokens: the selection kernel ranks the assignments, one more kernel places them
    p.fused_hist = p.act_bf16 && !routed_ids && T <= kFusedMaxTokens && !(flags & MOE_FLAG_PERMUTE_UNFUSED);
    const bool identity = flags & MOE_FLAG_IDENTITY_EXPERTS;
    const bool mfma = p.act_bf16 && !(flags & MOE_FLAG_FORCE_GENERIC);
    // large tiles once groups average at least a few MFMA tiles of rows
    const bool big = mfma && mfma8_supports(p) && (long long)T * p.kk >= 48ll * p.S;
    // weight streaming when a slot expects only a handful of rows (routed: T*k/E on average)
    const bool tiny = mfma && !big && (long long)T * p.k <= 4ll * p.E && shared_end - shared_begin <= 2 * decode_tile_rows();
    const int tile_rows = big ? mfma8_tile_rows() : tiny ? decode_tile_rows() : mfma ? mfma_tile_rows() : kGenericTileRows;
    p.max_tiles = (int)(((long long)T * p.kk + tile_rows - 1) / tile_rows) + p.S;
    if (big) {   // the tile-list workgroup also deals the tiles' N-slices to the XCDs, per GEMM
        p.units[0] = (MUnit *)(ws + l->lay.units[0]);
        p.units[1] = (MUnit *)(ws + l->lay.units[1]);
        p.unit_hdr = (UnitHdr *)(ws + l->lay.unit_hdr);
        p.unit_cap = (int32_t)l->lay.unit_cap;
        p.n_slices[0] = mfma8_n_slices(p.H, p.I, 0);
        p.n_slices[1] = mfma8_n_slices(p.H, p.I, 1);
    }

    // optional phase events (benchmarks): event j is recorded before phase j, the last one after the pass
    hipEvent_t *ev = l->prof_on && l->prof_seen++ % l->prof_every == 0 ? l->ev[l->prof_count % kProfRing] : nullptr;
    hipError_t e = hipSuccess;
    const int sel = l->prof_phase;
    auto mark = [&](int j) { if (ev && e == hipSuccess && (sel < 0 || j == sel || j == sel + 1)) e = hipEventRecord(ev[j], st); };
    mark(MOE_PHASE_GATE);
    if (e == hipSuccess && !routed_ids) e = launch_gate(p, st);
    mark(MOE_PHASE_PERMUTE);
    // few tokens, few slots: the weight-streaming GEMM-1 derives its tiles itself and writes the tables beside its stream
    p.self_tiles = tiny && !identity && decode_self_tiles(p);
    if (e == hipSuccess && !p.self_tiles) e = launch_permute(p, tile_rows, big, st);   // the large-tile kernels deal a size-ordered list round-robin to the XCDs
    mark(MOE_PHASE_GEMM1);
    if (e == hipSuccess) {
        if (identity)  e = launch_identity_experts(p, st);
        else if (big)  e = launch_experts_mfma8(p, 0, st);
        else if (tiny) e = launch_experts_decode(p, 0, st);
        else if (mfma) e = launch_experts_mfma(p, 0, st);
        else           e = launch_experts_generic(p, 0, st);
    }
    mark(MOE_PHASE_GEMM2);
    if (e == hipSuccess && !identity)
        e = big ? launch_experts_mfma8(p, 1, st) : tiny ? launch_experts_decode(p, 1, st) : mfma ? launch_experts_mfma(p, 1, st) : launch_experts_generic(p, 1, st);
    mark(MOE_PHASE_COMBINE);
    if (e == hipSuccess) e = launch_combine(p, st);
    mark(MOE_N_PHASES);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "forward launch failed: %s", hipGetErrorString(e));
    if (ev) l->prof_count++;
    return MOE_OK;
}

moe_status_t moe_forward(moe_layer_t *layer, const void *x, int32_t T, int32_t shared_begin, int32_t shared_end,
                         void *out, void *hip_stream, uint32_t flags)
{
    return forward_pass(layer, x, T, nullptr, nullptr, shared_begin, shared_end, out, hip_stream, flags);
}

moe_status_t moe_forward_routed(moe_layer_t *layer, const void *x, int32_t T, const int32_t *topk_ids, const float *topk_w,
                                int32_t shared_begin, int32_t shared_end, void *out, void *hip_stream, uint32_t flags)
{
    if (T > 0 && (!topk_ids || !topk_w)) return fail(MOE_ERR_ARG, "topk_ids and topk_w must be non-NULL");
    if (!aligned(topk_ids, 4) || !aligned(topk_w, 4)) return fail(MOE_ERR_ARG, "topk_ids and topk_w must be 4-byte aligned");
    return forward_pass(layer, x, T, topk_ids, topk_w, shared_begin, shared_end, out, hip_stream, flags);
}

// ---- moe_forward_static: the pass with every intermediate in the library's own device array ----

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU, looked up once per device

// Address of this GPU's copy of `scratch` (the current device's), found once per device.
moe_status_t scratch_of_current_device(void **ptr)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(MOE_ERR_UNSUPPORTED, "device %d: moe_forward_static keeps scratch addresses for devices 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(MOE_ERR_HIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return MOE_OK;
}
}  // namespace

moe_status_t moe_forward_static(const moe_config_t *cfg, const moe_buffers_t *buf,
                                const int32_t *host_map, int32_t n, const int32_t *host_shared_slots,
                                const void *x, int32_t T, int32_t shared_begin, int32_t shared_end,
                                void *out, void *hip_stream, uint32_t flags)
{
    moe_status_t st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (T < 0) return fail(MOE_ERR_ARG, "T is negative");
    if (T > cfg->max_tokens) return fail(MOE_ERR_CAPACITY, "T %d exceeds max_tokens %d", T, cfg->max_tokens);
    // the workspace is laid out for THIS pass's T (max_tokens only bounds T): what must fit is the pass
    moe_config_t c = *cfg;
    c.max_tokens = T > 0 ? T : 1;
    const Layout L = make_layout(c);
    if (L.total > (size_t)MOE_STATIC_SCRATCH_BYTES)
        return fail(MOE_ERR_CAPACITY, "a pass of %d tokens of this layer needs %zu bytes of scratch, moe_forward_static has %zu: "
                    "use moe_forward with a workspace", T, L.total, (size_t)MOE_STATIC_SCRATCH_BYTES);
    if (!buf) return fail(MOE_ERR_ARG, "buffers is NULL");
    if (!buf->router_w || !buf->w13 || !buf->w2) return fail(MOE_ERR_ARG, "router_w, w13 and w2 must be non-NULL");
    if (!aligned(buf->router_w, 16) || !aligned(buf->w13, 16) || !aligned(buf->w2, 16))
        return fail(MOE_ERR_ARG, "router_w, w13 and w2 must be 16-byte aligned");
    if ((buf->logit_bias && !aligned(buf->logit_bias, 4)) || (buf->select_bias && !aligned(buf->select_bias, 4)))
        return fail(MOE_ERR_ARG, "bias vectors must be 4-byte aligned");
    // the placement, checked like moe_set_expert_map does; tables on the host stack (E <= 1024, S <= 2047)
    int32_t table[1024 + 4], owner[2048];
    st = validate_plain_map(c, host_map, n, host_shared_slots, table, owner);
    if (st != MOE_OK) return st;
    if (T == 0) return MOE_OK;

    void *ws = nullptr;
    st = scratch_of_current_device(&ws);
    if (st != MOE_OK) return st;
    moe_layer lay;                       // host object on the stack: no heap, no device memory
    lay.cfg = c;
    lay.buf = *buf;
    lay.buf.workspace = ws;              // kernels get the looked-up device address, never the symbol
    lay.buf.workspace_bytes = MOE_STATIC_SCRATCH_BYTES;
    lay.lay = L;
    lay.has_map = true;
    // every pass writes what it reads (table, histograms, tile list, h, y): nothing has to start at zero
    const hipError_t e = launch_write_map((int32_t *)((char *)ws + L.map), table, c.n_experts + c.n_shared, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(MOE_ERR_HIP, "expert map upload failed: %s", hipGetErrorString(e));
    return forward_pass(&lay, x, T, nullptr, nullptr, shared_begin, shared_end, out, hip_stream, flags);
}

}  // extern "C"
