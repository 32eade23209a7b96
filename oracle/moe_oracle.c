/*
 * CPU oracle for the MoE expert layer as one expert-parallel rank runs it.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the parity reference for the HIP path
 * and the reported CPU baseline; nothing in the product path may call it.  It
 * shares no code, header, table or helper with the HIP library.
 *
 * What it computes.  The paper (Sec. 2.1, "Distributed Inference for MoE
 * Models") defines the layer only as: many experts, a gating function selects a
 * few per token, and under expert parallelism each device holds a subset of the
 * experts to which tokens are routed.  Its "Virtual Expert Management" design
 * choice and the vpage-remap primitive (Sec. 4.6, App. D) say kernels see the
 * rank's experts through a mapping that may be re-pointed without moving
 * weights.  The arithmetic below is the plain definition of such a layer for
 * the gating families of the models the paper serves (Sec. 5: softmax top-k
 * with renormalisation; sigmoid scores with group-limited top-k, renormalised
 * and scaled), written as one straight loop per token in fp64:
 *
 *   1. logits   l[e] = sum_h x[t,h] * Wr[e,h]  (+ logit_bias[e])
 *   2. scores   softmax over all E, or sigmoid; s32 = (float) s;
 *               selection score c[e] = s32[e] (+ select_bias[e])
 *   3. select   order by (c descending, index ascending); take the first k.
 *               Grouped gate: experts are split into n_group equal consecutive
 *               groups, a group's score is the sum of its two largest c, the
 *               topk_group best groups (score descending, index ascending) stay
 *               eligible, then the first k eligible experts are taken.
 *   4. weights  w_j = s[e_j] (fp64, never the biased score); if renormalize,
 *               divided by their sum over all k selected; times routed_scale.
 *   5. locality slot_j = expert_map[e_j]; assignments with slot -1 belong to
 *               another rank and are skipped.
 *   6. expert   g = W13[slot][0:I] x,  u = W13[slot][I:2I] x,
 *               a = g / (1 + exp(-g)) * u,  y = W2[slot] a.
 *               (identity_experts != 0 replaces this by y = x: a test mode.)
 *   7. combine  out[t] = sum_j w_j y_j  + for every shared slot, if
 *               shared_begin <= t < shared_end, 1.0 * FFN_shared(x_t).
 *               A token with no contribution gets an all-zero row.
 *      (oracle_forward_replicated: a placement may hold several copies of an
 *               expert; token t then uses copy t mod R -- see that function.)
 *   8. tie flags (fp32 selection scores): bit 0 set when the k-th and the best
 *               unselected eligible score differ by < 1e-5; bit 1 set when the
 *               topk_group-th and next group score differ by < 1e-5.
 *
 * There is no permutation, blocking, fusion or reordering: a reader can check
 * each step against the list above.  Inputs are fp32 arrays or bf16 bit
 * patterns (widened exactly); every product and sum is fp64.
 *
 * Parity pins: see tests/test_oracle_pins.py (closed forms, library routines,
 * brute force, a hand-worked grouped-selection example).  The numerical
 * conventions of the real checkpoints (DeepSeek-V3 / Qwen3 gating constants
 * beyond what is listed above) are "parity unpinned": no trained weights or
 * reference outputs exist in this build.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_GATE_SOFTMAX = 0, ORACLE_GATE_SIGMOID_GROUP = 1 };

typedef struct {
    int32_t T, H, I, E, k, S;
    int32_t gate;        /* ORACLE_GATE_* */
    int32_t n_group;     /* 1 for the softmax gate */
    int32_t topk_group;  /* 1 for the softmax gate */
    int32_t renormalize;
    double routed_scale;
    int32_t n_shared;
    int32_t act_dtype;    /* storage of x, w13, w2 : ORACLE_F32 / ORACLE_BF16 */
    int32_t router_dtype; /* storage of router_w */
} oracle_cfg;

/* value of element i of an array stored as fp32 or as bf16 bit patterns */
static double ld(const void *p, int dtype, size_t i)
{
    if (dtype == ORACLE_BF16) {
        uint32_t bits = ((uint32_t)((const uint16_t *)p)[i]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    return (double)((const float *)p)[i];
}

/* does candidate a come before candidate b in (score descending, index ascending)? */
static int before(float ca, int ia, float cb, int ib)
{
    if (ca != cb) return ca > cb;
    return ia < ib;
}

/*
 * Steps 1-4 and 8 for one token.
 *   forced_ids != NULL: step 3 is skipped and those k experts are used instead
 *   (weights still come from this token's own scores).
 * scratch: s[E] doubles, c[E] floats, eligible[E] bytes, gscore[n_group] floats.
 */
static void route_token(const oracle_cfg *cfg, const void *x, const void *router_w,
                        const float *logit_bias, const float *select_bias, int t,
                        const int32_t *forced_ids, int32_t *ids, double *w, uint8_t *flags,
                        float *c_out, double *s, float *c, uint8_t *eligible, float *gscore)
{
    const int H = cfg->H, E = cfg->E, k = cfg->k;
    /* 1. logits */
    for (int e = 0; e < E; ++e) {
        double acc = 0.0;
        for (int h = 0; h < H; ++h)
            acc += ld(x, cfg->act_dtype, (size_t)t * H + h) * ld(router_w, cfg->router_dtype, (size_t)e * H + h);
        if (logit_bias) acc += (double)logit_bias[e];
        s[e] = acc;
    }
    /* 2. scores */
    if (cfg->gate == ORACLE_GATE_SOFTMAX) {
        double m = s[0], z = 0.0;
        for (int e = 1; e < E; ++e) if (s[e] > m) m = s[e];
        for (int e = 0; e < E; ++e) { s[e] = exp(s[e] - m); z += s[e]; }
        for (int e = 0; e < E; ++e) s[e] /= z;
    } else {
        for (int e = 0; e < E; ++e) s[e] = 1.0 / (1.0 + exp(-s[e]));
    }
    for (int e = 0; e < E; ++e) {
        c[e] = (float)s[e];
        if (select_bias) c[e] = c[e] + select_bias[e];
        if (c_out) c_out[e] = c[e];
    }
    /* 3. selection */
    uint8_t fl = 0;
    for (int e = 0; e < E; ++e) eligible[e] = 1;
    if (cfg->gate == ORACLE_GATE_SIGMOID_GROUP && cfg->n_group > 1) {
        const int G = cfg->n_group, per = E / G;
        for (int g = 0; g < G; ++g) {
            /* two largest c of the group */
            int b1 = -1, b2 = -1;
            for (int e = g * per; e < (g + 1) * per; ++e)
                if (b1 < 0 || before(c[e], e, c[b1], b1)) b1 = e;
            for (int e = g * per; e < (g + 1) * per; ++e)
                if (e != b1 && (b2 < 0 || before(c[e], e, c[b2], b2))) b2 = e;
            gscore[g] = (b2 >= 0) ? (c[b1] + c[b2]) : c[b1];
        }
        /* keep the topk_group best groups */
        uint8_t kept[256];
        for (int g = 0; g < G; ++g) kept[g] = 0;
        float last_kept = 0.f;
        for (int r = 0; r < cfg->topk_group; ++r) {
            int best = -1;
            for (int g = 0; g < G; ++g)
                if (!kept[g] && (best < 0 || before(gscore[g], g, gscore[best], best))) best = g;
            kept[best] = 1;
            last_kept = gscore[best];
        }
        if (cfg->topk_group < G) {
            int best = -1;
            for (int g = 0; g < G; ++g)
                if (!kept[g] && (best < 0 || before(gscore[g], g, gscore[best], best))) best = g;
            if (fabsf(last_kept - gscore[best]) < 1e-5f) fl |= 2;
        }
        for (int e = 0; e < E; ++e) eligible[e] = kept[e / per];
    }
    if (forced_ids) {
        for (int j = 0; j < k; ++j) ids[j] = forced_ids[j];
    } else {
        float kth = 0.f;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e)
                if (eligible[e] && (best < 0 || before(c[e], e, c[best], best))) best = e;
            ids[j] = best;
            eligible[best] = 0;
            kth = c[best];
        }
        /* 8. expert tie flag: k-th selected vs best of what is left */
        int best = -1;
        for (int e = 0; e < E; ++e)
            if (eligible[e] && (best < 0 || before(c[e], e, c[best], best))) best = e;
        if (best >= 0 && fabsf(kth - c[best]) < 1e-5f) fl |= 1;
    }
    /* 4. weights */
    double sum = 0.0;
    for (int j = 0; j < k; ++j) { w[j] = s[ids[j]]; sum += w[j]; }
    for (int j = 0; j < k; ++j) {
        if (cfg->renormalize) w[j] /= sum;
        w[j] *= cfg->routed_scale;
    }
    if (flags) *flags = fl;
}

/* step 6 for one token and one slot: acc[h] += weight * FFN_slot(x_t)[h] */
static void expert_token(const oracle_cfg *cfg, const void *x, const void *w13, const void *w2,
                         int t, int slot, double weight, int identity, double *acc, double *a)
{
    const int H = cfg->H, I = cfg->I;
    if (identity) {
        for (int h = 0; h < H; ++h) acc[h] += weight * ld(x, cfg->act_dtype, (size_t)t * H + h);
        return;
    }
    const size_t w13_base = (size_t)slot * 2 * I * H;
    const size_t w2_base = (size_t)slot * H * I;
    for (int i = 0; i < I; ++i) {
        double g = 0.0, u = 0.0;
        for (int h = 0; h < H; ++h) {
            double xv = ld(x, cfg->act_dtype, (size_t)t * H + h);
            g += ld(w13, cfg->act_dtype, w13_base + (size_t)i * H + h) * xv;
            u += ld(w13, cfg->act_dtype, w13_base + (size_t)(I + i) * H + h) * xv;
        }
        a[i] = g / (1.0 + exp(-g)) * u;
    }
    for (int h = 0; h < H; ++h) {
        double y = 0.0;
        for (int i = 0; i < I; ++i) y += ld(w2, cfg->act_dtype, w2_base + (size_t)h * I + i) * a[i];
        acc[h] += weight * y;
    }
}

/*
 * Routing of every token (steps 1-4, 8).
 *   ids [T,k] int32, w [T,k] fp64, flags [T] bytes (may be NULL),
 *   c_out [T,E] fp32 selection scores (may be NULL).
 */
void oracle_route(const oracle_cfg *cfg, const void *x, const void *router_w,
                  const float *logit_bias, const float *select_bias,
                  int32_t *ids, double *w, uint8_t *flags, float *c_out)
{
#pragma omp parallel
    {
        double *s = malloc(sizeof(double) * cfg->E);
        float *c = malloc(sizeof(float) * cfg->E);
        uint8_t *el = malloc(cfg->E);
        float *gs = malloc(sizeof(float) * (cfg->n_group > 0 ? cfg->n_group : 1));
#pragma omp for schedule(dynamic, 4)
        for (int t = 0; t < cfg->T; ++t)
            route_token(cfg, x, router_w, logit_bias, select_bias, t, NULL,
                        ids + (size_t)t * cfg->k, w + (size_t)t * cfg->k,
                        flags ? flags + t : NULL, c_out ? c_out + (size_t)t * cfg->E : NULL,
                        s, c, el, gs);
        free(s); free(c); free(el); free(gs);
    }
}

/*
 * The whole layer (steps 1-7) for the tokens tok[0..n_tok).
 *   w13 [S,2I,H], w2 [S,H,I] : physical slot pools
 *   expert_map [E]  : logical expert -> slot, -1 = not on this rank
 *   shared_slots [n_shared]
 *   forced_ids : NULL, or [T,k] expert ids to use instead of step 3
 *   out [n_tok,H] fp64
 */
void oracle_forward(const oracle_cfg *cfg, const void *x, const void *router_w,
                    const float *logit_bias, const float *select_bias,
                    const void *w13, const void *w2, const int32_t *expert_map,
                    const int32_t *shared_slots, int32_t shared_begin, int32_t shared_end,
                    const int32_t *tok, int32_t n_tok, const int32_t *forced_ids,
                    int32_t identity_experts, double *out)
{
#pragma omp parallel
    {
        double *s = malloc(sizeof(double) * cfg->E);
        float *c = malloc(sizeof(float) * cfg->E);
        uint8_t *el = malloc(cfg->E);
        float *gs = malloc(sizeof(float) * (cfg->n_group > 0 ? cfg->n_group : 1));
        int32_t *ids = malloc(sizeof(int32_t) * cfg->k);
        double *w = malloc(sizeof(double) * cfg->k);
        double *a = malloc(sizeof(double) * cfg->I);
#pragma omp for schedule(dynamic, 1)
        for (int n = 0; n < n_tok; ++n) {
            const int t = tok[n];
            double *acc = out + (size_t)n * cfg->H;
            for (int h = 0; h < cfg->H; ++h) acc[h] = 0.0;
            route_token(cfg, x, router_w, logit_bias, select_bias, t,
                        forced_ids ? forced_ids + (size_t)t * cfg->k : NULL,
                        ids, w, NULL, NULL, s, c, el, gs);
            for (int j = 0; j < cfg->k; ++j) {
                const int slot = expert_map[ids[j]];          /* 5. locality */
                if (slot < 0) continue;
                expert_token(cfg, x, w13, w2, t, slot, w[j], identity_experts, acc, a);
            }
            for (int i = 0; i < cfg->n_shared; ++i)           /* 7. shared experts */
                if (t >= shared_begin && t < shared_end)
                    expert_token(cfg, x, w13, w2, t, shared_slots[i], 1.0, identity_experts, acc, a);
        }
        free(s); free(c); free(el); free(gs); free(ids); free(w); free(a);
    }
}

/*
 * Steps 5-7 alone, for a rank that receives tokens already routed (the input of an
 * expert-parallel rank after the dispatch exchange, paper Sec. 2.1): the k expert
 * ids and combine weights of every token are given instead of computed.
 *   ids [T,k] int32 : logical expert ids; an id outside [0,E) is an assignment that
 *                     does not exist (padding) and contributes nothing
 *   wts [T,k] fp32  : combine weights, used as given (no renormalisation, no scale)
 * Everything else as in oracle_forward.
 */
void oracle_forward_routed(const oracle_cfg *cfg, const void *x, const void *w13, const void *w2,
                           const int32_t *expert_map, const int32_t *shared_slots,
                           int32_t shared_begin, int32_t shared_end,
                           const int32_t *tok, int32_t n_tok, const int32_t *ids, const float *wts,
                           int32_t identity_experts, double *out)
{
#pragma omp parallel
    {
        double *a = malloc(sizeof(double) * cfg->I);
#pragma omp for schedule(dynamic, 1)
        for (int n = 0; n < n_tok; ++n) {
            const int t = tok[n];
            double *acc = out + (size_t)n * cfg->H;
            for (int h = 0; h < cfg->H; ++h) acc[h] = 0.0;
            for (int j = 0; j < cfg->k; ++j) {
                const int e = ids[(size_t)t * cfg->k + j];
                if (e < 0 || e >= cfg->E) continue;
                const int slot = expert_map[e];               /* 5. locality */
                if (slot < 0) continue;
                expert_token(cfg, x, w13, w2, t, slot, (double)wts[(size_t)t * cfg->k + j], identity_experts, acc, a);
            }
            for (int i = 0; i < cfg->n_shared; ++i)           /* 7. shared experts */
                if (t >= shared_begin && t < shared_end)
                    expert_token(cfg, x, w13, w2, t, shared_slots[i], 1.0, identity_experts, acc, a);
        }
        free(a);
    }
}

/*
 * The whole layer with a REPLICATED placement: a logical expert may be held in several
 * slots of this rank (placements that copy heavily used experts to balance load; the paper
 * names them among the distribution strategies in Sec. 2.1 and does not fix how a copy is
 * chosen).  Step 5 becomes: expert e has R = rep_off[e+1] - rep_off[e] copies in slots
 * rep_slots[rep_off[e] ..]; R = 0 means the expert is on another rank; token t uses copy
 * t mod R.  Everything else as in oracle_forward (which is the case R <= 1 everywhere).
 */
void oracle_forward_replicated(const oracle_cfg *cfg, const void *x, const void *router_w,
                               const float *logit_bias, const float *select_bias,
                               const void *w13, const void *w2,
                               const int32_t *rep_off, const int32_t *rep_slots,
                               const int32_t *shared_slots, int32_t shared_begin, int32_t shared_end,
                               const int32_t *tok, int32_t n_tok, const int32_t *forced_ids,
                               int32_t identity_experts, double *out)
{
#pragma omp parallel
    {
        double *s = malloc(sizeof(double) * cfg->E);
        float *c = malloc(sizeof(float) * cfg->E);
        uint8_t *el = malloc(cfg->E);
        float *gs = malloc(sizeof(float) * (cfg->n_group > 0 ? cfg->n_group : 1));
        int32_t *ids = malloc(sizeof(int32_t) * cfg->k);
        double *w = malloc(sizeof(double) * cfg->k);
        double *a = malloc(sizeof(double) * cfg->I);
#pragma omp for schedule(dynamic, 1)
        for (int n = 0; n < n_tok; ++n) {
            const int t = tok[n];
            double *acc = out + (size_t)n * cfg->H;
            for (int h = 0; h < cfg->H; ++h) acc[h] = 0.0;
            route_token(cfg, x, router_w, logit_bias, select_bias, t,
                        forced_ids ? forced_ids + (size_t)t * cfg->k : NULL,
                        ids, w, NULL, NULL, s, c, el, gs);
            for (int j = 0; j < cfg->k; ++j) {
                const int e = ids[j];
                const int R = rep_off[e + 1] - rep_off[e];    /* 5. locality, with copies */
                if (R == 0) continue;
                const int slot = rep_slots[rep_off[e] + t % R];
                expert_token(cfg, x, w13, w2, t, slot, w[j], identity_experts, acc, a);
            }
            for (int i = 0; i < cfg->n_shared; ++i)           /* 7. shared experts */
                if (t >= shared_begin && t < shared_end)
                    expert_token(cfg, x, w13, w2, t, shared_slots[i], 1.0, identity_experts, acc, a);
        }
        free(s); free(c); free(el); free(gs); free(ids); free(w); free(a);
    }
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
