/*
 * elasticmoe.h -- C ABI of the MI355X (gfx950) MoE expert layer as ONE
 * expert-parallel rank runs it.
 *
 * What the layer is.  The paper (Sec. 2.1, "Distributed Inference for MoE
 * Models") states the computation in one sentence: a layer holds many experts, a
 * gating function selects a few of them per token, and under expert parallelism
 * every device owns a subset of the experts to which tokens are routed.  This
 * library runs that layer for the tokens and the experts of one rank:
 *
 *     gate logits -> scores -> top-k (optionally group limited) -> renormalise
 *     -> logical expert id -> physical weight slot (expert map) -> rows grouped
 *     per slot -> SwiGLU expert FFN per group -> weighted sum back per token.
 *
 * Why there is an expert map.  The paper's "Virtual Expert Management" design
 * choice (Sec. 3.2) and its vpage-remap primitive (Sec. 4.6, App. D) keep the
 * rank's expert weights in place when the expert-parallel degree changes: only a
 * mapping is re-pointed, nothing large is reallocated or copied, and the old
 * mapping stays usable until the switch.  Here the mapping is an int32 table
 * `logical expert -> slot of a preallocated weight pool` that the kernels read;
 * moe_set_expert_map swaps it in O(E) with no allocation and no weight traffic.
 *
 * Memory rules.  Every device buffer (weights, workspace, activations) is owned
 * by the caller and must outlive the layer; the library never calls hipMalloc /
 * hipFree.  This mirrors the paper's split between the memory daemon that owns
 * tensors and the execution side that only holds references (Sec. 3.2,
 * "Decoupled Memory and Execution Layers").  All pointers named "device" are
 * device addresses valid on the GPU that is current when the call is made; all
 * others are host addresses.  All calls are host-thread-safe only when they use
 * different layers.
 *
 * Errors.  Every call returns a moe_status_t; nothing throws or aborts.  On any
 * error the layer (including its active expert map) is unchanged and
 * moe_last_error() describes the problem.
 */
#ifndef ELASTICMOE_H
#define ELASTICMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_layer moe_layer_t; /* opaque host object */
typedef struct moe_vpool moe_vpool_t; /* opaque host object: a weight pool as a contiguous virtual tensor */

typedef enum {
    MOE_OK = 0,
    MOE_ERR_ARG = 1,         /* null pointer, negative size, bad enum, misaligned buffer */
    MOE_ERR_SHAPE = 2,       /* sizes that do not describe a layer (E % n_group != 0, k > E, ...) */
    MOE_ERR_MAP = 3,         /* invalid expert map, or forward before any map was set */
    MOE_ERR_CAPACITY = 4,    /* T > max_tokens, workspace too small */
    MOE_ERR_UNSUPPORTED = 5, /* a shape the kernels do not cover (see moe_layer_create) */
    MOE_ERR_HIP = 6          /* a HIP runtime call failed (message has the HIP error string) */
} moe_status_t;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype_t;

/*
 * Gating rule (Sec. 2.1 names only "a gating function"; these are the rules of
 * the model families the paper serves in Sec. 5).
 *   MOE_GATE_SOFTMAX_TOPK        scores = softmax over all E logits; the k best.
 *   MOE_GATE_SIGMOID_GROUP_TOPK  scores = sigmoid(logit); experts are split into
 *       n_group equal consecutive groups; a group's score is the sum of its two
 *       largest selection scores; only the topk_group best groups stay eligible;
 *       the k best eligible experts are taken.
 * Order is (score descending, lower index first) for experts and for groups.
 * Weights are the un-biased scores of the k selected experts; if `renormalize`
 * they are divided by their sum over all k (local or not); then multiplied by
 * `routed_scale`.
 */
typedef enum { MOE_GATE_SOFTMAX_TOPK = 0, MOE_GATE_SIGMOID_GROUP_TOPK = 1 } moe_gate_t;

typedef struct {
    int32_t hidden;      /* H  : model width; multiple of 8 */
    int32_t inter;       /* I  : SwiGLU intermediate width of one expert; multiple of 8 */
    int32_t n_experts;   /* E  : logical (global) routed experts, 1..1024 */
    int32_t top_k;       /* k  : 1..min(E,32) */
    int32_t n_slots;     /* S  : physical weight slots in the caller's pool, shared included */
    int32_t max_tokens;  /* largest T any moe_forward will pass */
    int32_t act_dtype;   /* moe_dtype_t of x, w13, w2, out */
    int32_t router_dtype;/* moe_dtype_t of router_w */
    int32_t gate;        /* moe_gate_t */
    int32_t n_group;     /* 1 unless MOE_GATE_SIGMOID_GROUP_TOPK; divides E; <= 64 */
    int32_t topk_group;  /* 1..n_group; k <= topk_group * E / n_group */
    int32_t renormalize; /* 0 / 1 */
    float   routed_scale;/* e.g. 1.0 or 2.5 */
    int32_t n_shared;    /* shared (always-on) experts living in the same slot pool, 0..4 */
} moe_config_t;

typedef struct {
    const void  *router_w;    /* device [E,H] row-major, router_dtype */
    const float *logit_bias;  /* device [E] fp32 or NULL; added to the logits before scoring; finite values */
    const float *select_bias; /* device [E] fp32 or NULL; added to scores for SELECTION only; finite values.
                               * (With non-finite biases or activations a token may be left with fewer than k
                               * candidates: its selection is then unspecified -- ids stay inside [0, E), an id
                               * may repeat, and a repeated id carries weight 0 -- and nothing is read or written
                               * out of bounds.) */
    const void  *w13;         /* device [S,2I,H] act_dtype: rows 0..I-1 gate proj, I..2I-1 up proj */
    const void  *w2;          /* device [S,H,I]  act_dtype: down proj */
    void        *workspace;   /* device, 256-byte aligned, >= moe_workspace_bytes(cfg) bytes */
    size_t       workspace_bytes;
} moe_buffers_t;

/* device addresses of the intermediates inside the caller's workspace (for tests) */
typedef struct {
    const int32_t *topk_ids;  /* [T,k]    logical expert ids, best first */
    const float   *topk_w;    /* [T,k]    combine weights of those experts */
    const int32_t *counts;    /* [S]      rows per slot in the last forward */
    const int32_t *offsets;   /* [S+1]    exclusive prefix sum of counts */
    const int32_t *perm;      /* [A]      token index of every grouped row, A = offsets[S] */
    const int32_t *inv;       /* [T,k+n_shared] grouped row of every assignment or -1 */
    const void    *h;         /* [A,I]    act_dtype, silu(gate)*up */
    const void    *y;         /* [A,H]    act_dtype, expert outputs before combine */
    const int32_t *active_map;/* [E + n_shared] the device copy of the active map, shared slots last
                               * (an entry <= -2 stands for an expert with several copies) */
    const int32_t *tiles;     /* [n_tiles][4] the M-tile list of the expert kernels: slot, first grouped row, rows, 1 if the tile is all of its slot's rows else 0 */
    const int32_t *n_tiles;   /* [1] */
    /* Work units of the large-tile expert kernels (NULL when the layer can never run them): per GEMM a header
     * {rows of 8 workgroups, N-slices per unit, entries, runs per tile} and a list read in rows of 8 -- entry
     * 8 i + x is the i-th unit of XCD x: {slot, first grouped row, rows (0: a hole), first N-slice << 1 | single}.
     * Written only by passes that run those kernels. */
    const int32_t *unit_hdr;  /* [2][4] */
    const int32_t *units[2];  /* [entries][4] of GEMM-1 and GEMM-2 */
} moe_workspace_view_t;

/* moe_forward flags */
#define MOE_FLAG_IDENTITY_EXPERTS 1u /* test mode: every expert returns its input row unchanged */
#define MOE_FLAG_FORCE_GENERIC    2u /* run the plain (non-MFMA) expert kernels: debugging aid */
#define MOE_FLAG_GATE_TILED       4u /* bf16 activations: use the LDS-tiled gate logits kernel at any batch size (testing aid) */
#define MOE_FLAG_PERMUTE_UNFUSED  8u /* rank the assignments in the separate histogram kernels (the path of passes whose routing is
                                      * given and of batches over 8192 tokens) instead of inside the selection kernel (testing aid) */

/*
 * Bytes of device workspace a layer of this configuration needs (0 if cfg is
 * invalid; moe_last_error() says why).  Pure host arithmetic.
 */
size_t moe_workspace_bytes(const moe_config_t *cfg);

/*
 * Create a layer object over caller-owned buffers.  Host-only: validates the
 * configuration and the buffer pointers/alignment (router_w, w13, w2 16-byte,
 * workspace 256-byte aligned), carves the workspace, touches no device memory
 * and launches nothing.  The layer has NO expert map yet.
 *   MOE_ERR_UNSUPPORTED: H or I not a multiple of 8, E > 1024, k > 32,
 *   n_group > 64, n_shared > 4.
 */
moe_status_t moe_layer_create(const moe_config_t *cfg, const moe_buffers_t *buf, moe_layer_t **out);

/*
 * Install a new expert placement (paper: vpage-remap, Sec. 4.6 / App. D; scale-up
 * step "HMM Reconfigures Memory Layout", Sec. 4.7).
 *   host_map [n]           n must equal E; entry e is the slot holding logical expert e,
 *                          or -1 when the expert lives on another rank.
 *   host_shared_slots [n_shared]  slots of the shared experts (NULL iff n_shared == 0).
 * Rejected with MOE_ERR_MAP, leaving the old map active: n != E, an entry < -1 or
 * >= S, two experts (or an expert and a shared expert) on one slot.
 * The table is copied out of the host arrays before the call returns.  The layer has
 * ONE device table at a fixed address in the workspace, rewritten in place by a tiny
 * kernel enqueued on `hip_stream`: passes enqueued on that stream before this call have
 * read the old table by then (the old placement stays in force for them), passes
 * enqueued after it read the new one -- a replay of a HIP graph captured earlier
 * included, since a captured pass holds nothing of the placement but the table's
 * address.  Passes that run on OTHER streams are the caller's to order against the
 * switch (a pass that overlaps the rewrite could read a mixture of the two
 * placements).  No allocation, no synchronisation, no weight traffic.  The caller
 * must have filled the newly
 * referenced weight slots (stream-ordered before the next forward).
 */
moe_status_t moe_set_expert_map(moe_layer_t *layer, const int32_t *host_map, int32_t n,
                                const int32_t *host_shared_slots, void *hip_stream);

/*
 * Install a placement in which an expert may be held in SEVERAL slots of this rank
 * (placements that copy heavily used experts to balance load: the paper lists them among
 * the expert distribution strategies in Sec. 2.1 and leaves the choice of copy open).
 *   host_rep_offsets [n+1]  n must equal E; expert e's copies are the slots
 *                           host_rep_slots[host_rep_offsets[e] .. host_rep_offsets[e+1]);
 *                           no copy = the expert lives on another rank.
 *   host_rep_slots          all copies, expert by expert (may be NULL when there are none).
 *   host_shared_slots [n_shared]  as in moe_set_expert_map.
 * Token t's assignment to expert e goes to copy t mod R of its R copies: a choice that
 * needs no state, is the same on every pass, and spreads an expert's rows evenly over its
 * copies whenever its tokens are spread over the batch.  All copies of an expert must hold
 * the same weights for the layer to compute the same function (not checked).
 * Rejected with MOE_ERR_MAP, leaving the old placement active: n != E, offsets that do not
 * start at 0, decrease or exceed S, a slot outside [0, S), a slot used twice.
 * Everything else -- the one device table, ordering on `hip_stream`, no allocation, no
 * weight traffic, the wait for pending slot fills -- as in moe_set_expert_map, which is
 * the case of at most one copy per expert.
 */
moe_status_t moe_set_expert_replicas(moe_layer_t *layer, const int32_t *host_rep_offsets,
                                     const int32_t *host_rep_slots, int32_t n,
                                     const int32_t *host_shared_slots, void *hip_stream);

/*
 * Fill one slot of the weight pools in the background while forwards keep running
 * (paper: new or migrated experts are copied into freshly mapped pages while the old
 * instance serves, and only then the mapping is switched -- Sec. 3.2 "zero-downtime",
 * Sec. 4.7 scale-up steps, p2p-copy in Sec. 4.6).  On one GPU the source is a device
 * buffer the caller has staged (the landing buffer of a peer transfer).
 *   slot        pool slot to fill; it must NOT be referenced by the active map
 *               (MOE_ERR_MAP otherwise: forwards may be reading it)
 *   src_w13     device [2I,H] act_dtype, 16-byte aligned     src_w2  device [H,I]
 *   copy_stream stream the copy kernels run on               serve_stream  the stream
 *               the forwards run on (must differ from copy_stream)
 *   copy_blocks workgroups of the copy kernels (0 = 32): the throttle on how much HBM
 *               bandwidth the fill may take from the forwards
 * Ordering, all by events, no host synchronisation and no allocation: the copy starts
 * after the work ALREADY enqueued on serve_stream (a forward that still reads the slot
 * under an older map); the next moe_set_expert_map makes its stream wait for every
 * fill issued since the previous switch, so forwards after that switch see the
 * weights.  The weight pools given at moe_layer_create must be writable.  Forwards
 * that run on other streams than serve_stream are the caller's to order.
 */
moe_status_t moe_load_expert(moe_layer_t *layer, int32_t slot, const void *src_w13, const void *src_w2,
                             void *copy_stream, void *serve_stream, int32_t copy_blocks);

/*
 * One forward pass of the layer, enqueued on `hip_stream` (a hipStream_t; NULL =
 * the default stream).  Asynchronous, never synchronises, never allocates.
 *   x    device [T,H] act_dtype, 16-byte aligned
 *   out  device [T,H] act_dtype, 16-byte aligned; row t = sum over the token's
 *        LOCAL selected experts of weight * FFN_slot(x_t), plus 1.0 * FFN(x_t)
 *        of every shared expert when shared_begin <= t < shared_end; a token with
 *        no local work gets an all-zero row (a partial sum for the cross-rank
 *        reduction).  The sum runs in selection order, shared experts last, in
 *        fp32 with one final rounding.
 *   T == 0 is a no-op.  T > max_tokens -> MOE_ERR_CAPACITY.
 *   shared range must satisfy 0 <= shared_begin <= shared_end <= T.
 * After the pass the workspace holds the intermediates moe_workspace_view names.
 */
moe_status_t moe_forward(moe_layer_t *layer, const void *x, int32_t T,
                         int32_t shared_begin, int32_t shared_end,
                         void *out, void *hip_stream, uint32_t flags);

/*
 * The same pass for a rank that receives its tokens ALREADY ROUTED -- the input of an
 * expert-parallel rank after the dispatch exchange (paper Sec. 2.1: tokens are routed
 * to the devices that hold their experts): the gate is skipped.
 *   topk_ids device [T,k] int32: logical expert ids per token; an id outside [0,E)
 *            (e.g. -1) is an assignment that does not exist and contributes nothing;
 *            ids whose map entry is -1 are skipped as in moe_forward; an id may repeat
 *            within a token (it then counts once per occurrence).
 *   topk_w   device [T,k] float: combine weights, used as given.
 * Both are read in place during the pass (keep them unchanged until it has run on the
 * stream) and never written.  Everything else (x, out, shared range, flags, errors,
 * asynchrony, no allocation) as in moe_forward.  Afterwards moe_workspace_view's
 * topk_ids/topk_w still name the workspace copies of the last GATED pass; all other
 * intermediates are this pass's.
 */
moe_status_t moe_forward_routed(moe_layer_t *layer, const void *x, int32_t T,
                                const int32_t *topk_ids, const float *topk_w,
                                int32_t shared_begin, int32_t shared_end,
                                void *out, void *hip_stream, uint32_t flags);

/*
 * moe_forward for callers that can neither allocate device memory nor hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  No layer
 * object: the configuration, the weight buffers and the placement travel with the call, and every
 * intermediate of the pass (expert table, routing, histograms, tile list, h, y) lives in a device
 * array of MOE_STATIC_SCRATCH_BYTES that is part of the library image -- every GPU the library runs
 * on holds one copy until the process ends.  The call allocates nothing (no hipMalloc / hipFree, no
 * allocating library routine) and never synchronises.
 *   cfg, buf   as for moe_layer_create; buf->workspace and workspace_bytes are ignored (may be 0);
 *              cfg->max_tokens only bounds T.
 *   host_map [n], host_shared_slots   the placement, as for moe_set_expert_map (plain placements
 *              only: one slot per expert); checked on every call, MOE_ERR_MAP as there.
 *   x, T, shared range, out, hip_stream, flags   as for moe_forward.
 * MOE_ERR_CAPACITY when a pass of T tokens of this layer needs more scratch than the array holds
 * (moe_workspace_bytes of the configuration with max_tokens = T); nothing is launched then.
 * All calls on one GPU share that GPU's array, which keeps the previous call's contents (a pass
 * writes everything it reads, so nothing needs clearing): calls that overlap on one GPU -- on
 * different streams, or from different host threads -- race; calls on one stream are ordered.
 * The result is bit-identical to moe_forward on a layer of the same configuration and placement.
 */
#define MOE_STATIC_SCRATCH_BYTES (32u << 20)
moe_status_t moe_forward_static(const moe_config_t *cfg, const moe_buffers_t *buf,
                                const int32_t *host_map, int32_t n, const int32_t *host_shared_slots,
                                const void *x, int32_t T, int32_t shared_begin, int32_t shared_end,
                                void *out, void *hip_stream, uint32_t flags);

/* Addresses of the intermediates (valid for the layer's lifetime). */
moe_status_t moe_workspace_view(const moe_layer_t *layer, moe_workspace_view_t *view);

/*
 * Phase timing for benchmarks (not part of the method; it exists so that a
 * benchmark can time each kernel of a pass on the very stream the pass runs on).
 * While enabled, every enable-th moe_forward (enable = 1: every one; a larger value
 * samples, so that the events' own cost -- a microsecond or two each -- stays out of
 * most passes) records HIP events around its phases; the last 64 recorded forwards are
 * kept.  moe_profile_read waits for the recorded forward `back` recordings ago
 * (0 = most recent) and writes the milliseconds of each phase to ms[MOE_N_PHASES].
 * Enabling creates the events (host objects), disabling or destroying the layer
 * destroys them.  moe_profile_select(phase) restricts the recording to the two events
 * around ONE phase (moe_profile_read then writes 0 for the others), -1 (the default)
 * records all six; it forgets what was recorded before.
 */
enum { MOE_PHASE_GATE = 0, MOE_PHASE_PERMUTE = 1, MOE_PHASE_GEMM1 = 2, MOE_PHASE_GEMM2 = 3,
       MOE_PHASE_COMBINE = 4, MOE_N_PHASES = 5 };
moe_status_t moe_profile_enable(moe_layer_t *layer, int32_t enable);
moe_status_t moe_profile_select(moe_layer_t *layer, int32_t phase);
moe_status_t moe_profile_read(moe_layer_t *layer, int32_t back, float *ms);

/*
 * Measuring sticks for benchmarks (not part of the method): what this chip sustains
 * with nothing else in the way, so that a fraction of the data-sheet peak can be read
 * beside the fraction of what is reachable.  Both only enqueue one kernel on
 * `hip_stream`; the caller times it.  `sink` is a device float the kernels may
 * write (they practically never do); nothing is allocated.
 *   moe_ceiling_mfma:   `blocks` workgroups of 8 wavefronts each run `iters` rounds of
 *                       8 independent register-only v_mfma_f32_32x32x16_bf16;
 *                       *flops receives the flops of the launch.  random_operands != 0
 *                       multiplies pseudo-random values in (-1, 1) that change from one
 *                       MFMA to the next (the sustained rate under realistic switching
 *                       power), 0 small constants (the issue-rate ceiling).
 *   moe_ceiling_stream: reads `bytes` (rounded down to 16) of device memory at `buf`
 *                       (16-byte aligned) once, 16 bytes per lane.
 *   moe_ceiling_tile_stream: the weight stream of the large-tile expert kernels with nothing
 *                       else running: reads n_tiles x 256 x row_bytes bytes at `buf` (device,
 *                       16-byte aligned; the caller owns at least that much) as n_tiles tiles of
 *                       256 consecutive rows, one workgroup per tile, 128 bytes of every row per
 *                       step, global -> LDS, 2 steps in flight.  row_bytes: a multiple of 128
 *                       below 2^24 (the row stride of a weight matrix: hidden or inter elements).
 *                       non_temporal != 0 marks the copies read-once, as the kernels do for a
 *                       slot whose rows are one tile.  MOE_ERR_ARG on anything else; nothing
 *                       is written.
 */
moe_status_t moe_ceiling_mfma(int32_t blocks, int32_t iters, int32_t random_operands, float *sink,
                              void *hip_stream, double *flops);
moe_status_t moe_ceiling_stream(const void *buf, size_t bytes, float *sink, void *hip_stream);
moe_status_t moe_ceiling_tile_stream(const void *buf, int32_t n_tiles, size_t row_bytes, int32_t non_temporal, void *hip_stream);

/*
 * A weight pool as ONE contiguous virtual tensor over separately allocated physical pages
 * (paper: Virtual Expert Management, Sec. 3.2; the vpage-remap primitive, Sec. 4.6 / App. D):
 * kernels see slots 0..n-1 back to back at moe_vpool_base(), slot_bytes apart, and which
 * physical page lies under a slot is changed in O(1) without moving a byte -- map a fresh
 * page behind the resident ones to grow, exchange the pages under two slots to re-place
 * experts, unmap and free pages to shrink.  A layer uses such a pool by being given its base
 * as moe_buffers_t.w13 / .w2 (one pool each); the expert map then names VIRTUAL slots and an
 * identity map is all that kernels written for contiguous experts need.
 *   moe_vpool_create      reserves the address range only (slot_bytes must be a multiple of
 *                         the device's mapping granularity, MOE_ERR_UNSUPPORTED otherwise).
 *   moe_vpool_page_alloc  allocates one slot-sized physical page; *page = its id.
 *   moe_vpool_map         puts a page under a slot (both must be free: MOE_ERR_MAP), read/write.
 *   moe_vpool_unmap       takes the page from under a slot; the page keeps its contents.
 *   moe_vpool_page_free   releases an unmapped page.       moe_vpool_page_of  page under a slot, or -1.
 *   moe_vpool_destroy     unmaps and releases everything and frees the address range.
 *   moe_vpool_slot_bytes / moe_vpool_slots   what the pool was created with (0 for NULL).
 * These are the only calls of the library that own device memory.  Mapping calls are host
 * operations, not stream ordered: unmap a slot only when no kernel that can read it is in
 * flight, and never let an expert map name a slot that has no page (reading it faults).
 *
 * moe_layer_bind_vpools tells a layer which pools lie under its w13 and w2 (either may be NULL:
 * that buffer is plain memory); each pool must start at the layer's buffer, have the layer's slot
 * size and at least its slots (MOE_ERR_ARG otherwise).  From then on the host refuses, with
 * MOE_ERR_MAP and before anything is enqueued, what would make a kernel touch a slot without a
 * page: a placement (moe_set_expert_map / moe_set_expert_replicas) that names one, a forward while
 * the placement in force names one (a page unmapped after the switch), a moe_load_expert into
 * one; binding itself fails that way when the placement in force is not readable.  Pages under
 * slots the placement does not name may come and go freely.  A replay of a captured graph runs
 * no host check.  Destroying a pool unbinds it from its layers; destroying a layer unbinds it.
 */
moe_status_t moe_vpool_create(size_t slot_bytes, int32_t n_vslots, moe_vpool_t **out);
void *moe_vpool_base(const moe_vpool_t *pool);
moe_status_t moe_vpool_page_alloc(moe_vpool_t *pool, int32_t *page);
moe_status_t moe_vpool_page_free(moe_vpool_t *pool, int32_t page);
moe_status_t moe_vpool_map(moe_vpool_t *pool, int32_t vslot, int32_t page);
moe_status_t moe_vpool_unmap(moe_vpool_t *pool, int32_t vslot);
int32_t moe_vpool_page_of(const moe_vpool_t *pool, int32_t vslot);
size_t moe_vpool_slot_bytes(const moe_vpool_t *pool);
int32_t moe_vpool_slots(const moe_vpool_t *pool);
moe_status_t moe_vpool_destroy(moe_vpool_t *pool);
moe_status_t moe_layer_bind_vpools(moe_layer_t *layer, moe_vpool_t *w13_pool, moe_vpool_t *w2_pool);

/*
 * Zero-copy attach of a weight pool from another process (paper: the zero-copy primitive, Sec. 4.6; its
 * export_handle / open_tensor pair, App. D; the serving instances of Sec. 3.2 that hold references to
 * tensors kept by the memory daemon).  The process that owns a pool exports a handle; a serving process
 * on the same GPU opens it and passes the address as moe_buffers_t.w13 / .w2: no weight byte is copied,
 * and serving processes come and go while the owner keeps the experts resident.
 *   moe_pool_export  dev_ptr: an address inside a device allocation of THIS process (e.g. the base of a
 *                    pool).  handle receives MOE_IPC_HANDLE_BYTES opaque bytes that name the whole
 *                    allocation, *offset the distance of dev_ptr from its start; both travel to the other
 *                    process by any means (pipe, socket, file).  MOE_ERR_UNSUPPORTED for allocations of
 *                    2 GiB and more (split such a pool over several allocations).
 *   moe_pool_open    in the OTHER process: maps the allocation and returns the address that corresponds
 *                    to dev_ptr.  The memory stays owned by the exporter, which must keep it allocated
 *                    while it is open elsewhere; writes by either side are seen by the other (stream and
 *                    process synchronisation are the callers').
 *   moe_pool_close   unmaps it again (same address and offset as returned / given to moe_pool_open).
 * A handle cannot be opened in the process that exported it.  Pools of moe_vpool_* are not exportable
 * through these calls.
 */
#define MOE_IPC_HANDLE_BYTES 64
moe_status_t moe_pool_export(const void *dev_ptr, void *handle, size_t *offset);
moe_status_t moe_pool_open(const void *handle, size_t offset, void **dev_ptr);
moe_status_t moe_pool_close(void *dev_ptr, size_t offset);

/* Frees the host object only (the library owns no device memory). NULL is allowed. */
void moe_layer_destroy(moe_layer_t *layer);

/* Message of the last failing call on this host thread ("" if none). */
const char *moe_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ELASTICMOE_H */
