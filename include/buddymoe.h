/* buddymoe.h - C ABI of the MI355X (gfx950) library for one Mixture-of-Experts
 * layer's forward pass with buddy-expert substitution (BuddyMoE).
 *
 * The pass: router logits -> softmax / top-k gates -> substitution of every
 * selected expert that is not resident in device memory by its highest-ranked
 * resident buddy (Section 4, Algorithm 1) -> grouping of the surviving
 * (token, slot) assignments by expert -> SwiGLU expert FFN over resident
 * experts only -> gate-weighted aggregation (+ always-on shared experts).
 *
 * Conventions
 *  - Plain C.  No hidden allocation, no global state, no host synchronisation:
 *    every call enqueues its kernels on `stream` (a hipStream_t passed as
 *    void*; NULL = the default stream) and returns.
 *  - "device" pointers are HIP device memory owned by the caller, row-major,
 *    contiguous, 16-byte aligned.  The library never frees or retains them.
 *    "host" pointers are ordinary memory read during the call.
 *  - T tokens, d hidden size, E routed experts, F expert FFN width, K experts
 *    per token, R buddy-table width, H search limit (0 <= H <= R),
 *    A = T*K assignments.
 *  - Return value: BM_OK (0) or a negative bm_status.  Shape and pointer
 *    errors are detected on the host before anything is launched; no kernel
 *    faults on arbitrary table or id contents (ids outside [0,E) are treated
 *    as "not resident").
 */
#ifndef BUDDYMOE_H
#define BUDDYMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BM_OK = 0,
    BM_ERR_NULL = -1,       /* a required pointer is NULL                           */
    BM_ERR_SHAPE = -2,      /* K>E, H>R, E or K above the supported maximum, d or F
                               not a multiple of 32 for bf16, non-positive sizes    */
    BM_ERR_DTYPE = -3,      /* dtype is neither BM_F32 nor BM_BF16                  */
    BM_ERR_WORKSPACE = -4,  /* workspace NULL, misaligned or smaller than required  */
    BM_ERR_BAD_TABLE = -5,  /* bm_validate_tables: entry outside [-1,E) or == row   */
    BM_ERR_HIP = -6         /* a kernel launch failed (hipGetLastError != success)  */
} bm_status;

typedef enum { BM_F32 = 0, BM_BF16 = 1 } bm_dtype;

enum {
    BM_RENORM_TOPK  = 1u << 0, /* gate weights are the softmax renormalised over the K
                                  selected experts (p-tilde of Section 3, "Notation");
                                  off: the plain softmax probabilities               */
    BM_REMAP_UNIQUE = 1u << 1, /* Algorithm 1's "b not in U_t" test: a buddy already
                                  held by the token is skipped.  Off: the substitute
                                  is the first resident entry of the buddy row        */
    BM_Y_F32        = 1u << 2, /* bm_moe_forward writes y as fp32 whatever dtype is   */
    /* Gates in front of the substitution, decided per token from its K gate weights
     * renormalised to sum 1 (p-tilde), before any drop.  A miss of a token that may
     * not be given a substitute is dropped like a miss without an acceptable buddy
     * (the paper fetches such an expert from host memory instead; a single layer's
     * forward pass has no such channel). */
    BM_GATE_TAE       = 1u << 3, /* Section 3.1, Eq. 1: no substitution for a token whose
                                    TAE = -(sum p~ log p~)/log K is <= desc.tae_tau       */
    BM_GATE_MARGIN    = 1u << 4, /* Section 3.1: nor when p~_max - p~_2nd >= desc.margin_gamma
                                    (second value 0 when K == 1)                          */
    BM_REPLACE_BUDGET = 1u << 5, /* Section 5.1: at most desc.rho substitutions per token,
                                    counted in slot order; later misses are dropped      */
    BM_GATE_DIST      = 1u << 6, /* Section 3.1, Eq. 2: over the batch of the call (its T
                                    tokens), delta = share of the distinct routed experts
                                    that are not resident; no substitution for any token
                                    when delta >= desc.dist_beta.  Decided exactly
                                    (offloaded >= beta * requested, in fp64)              */
    BM_PSI_TOKEN      = 1u << 7  /* Section 3.1, Eq. 3 with kappa = 0 (bm_moe_forward only): the
                                    substitute is the acceptable entry - same test, same first H
                                    entries - of largest q[j|i] * (1 + desc.psi_eta * p_j(x)),
                                    p_j(x) the softmax probability of expert j for the token
                                    (fp32); equal scores keep the earlier entry.  Needs
                                    weights.buddy_q                                          */
};
#define BM_GATE_ANY (BM_GATE_TAE | BM_GATE_MARGIN | BM_REPLACE_BUDGET)   /* the per-token ones */

/* Limits of this build. */
#define BM_MAX_E 256
#define BM_MAX_K 32
#define BM_MAX_R 32

typedef struct {
    int32_t T, d, E, F, K;
    int32_t n_shared;   /* always-on experts added with weight 1 (0 for none)        */
    int32_t R, H;       /* buddy-table width and search limit                         */
    int32_t dtype;      /* bm_dtype of x, all weights and (unless BM_Y_F32) y         */
    uint32_t flags;     /* BM_* flag bits                                             */
    float tae_tau;      /* read only with BM_GATE_TAE                                 */
    float margin_gamma; /* read only with BM_GATE_MARGIN                              */
    int32_t rho;        /* read only with BM_REPLACE_BUDGET; >= 0                     */
    float dist_beta;    /* read only with BM_GATE_DIST                                */
    float psi_eta;      /* read only with BM_PSI_TOKEN; >= 0                          */
} bm_layer_desc;

/* Weights, all device pointers in `dtype`.  The reduction dimension is
 * contiguous.  Pointers cover all E experts, but rows of an expert that is not
 * resident are never read. */
typedef struct {
    const void *w_router;      /* [E][d]                                  */
    const float *router_bias;  /* [E] fp32, or NULL                       */
    const void *w_gate;        /* [E][F][d]                               */
    const void *w_up;          /* [E][F][d]                               */
    const void *w_down;        /* [E][d][F]                               */
    const void *ws_gate;       /* [n_shared][F][d], NULL when n_shared==0 */
    const void *ws_up;         /* [n_shared][F][d]                        */
    const void *ws_down;       /* [n_shared][d][F]                        */
    /* Optional fragment-major copies written by bm_pack_weights (bf16 only; NULL =
     * not available).  When all copies a layer needs are given, the decode-sized
     * path streams them instead of the arrays above; results are identical. */
    const void *wp_gateup;     /* routed gate+up, bm_packed_bytes(desc, 0) bytes */
    const void *wp_down;       /* routed down,    bm_packed_bytes(desc, 1) bytes */
    const void *wsp_gateup;    /* shared gate+up, bm_packed_bytes(desc, 2) bytes */
    const void *wsp_down;      /* shared down,    bm_packed_bytes(desc, 3) bytes */
    /* q[j|i] of every buddy-table entry, [E][R] fp32 as bm_build_buddy_table writes it;
     * read only with BM_PSI_TOKEN (NULL otherwise) */
    const float *buddy_q;
} bm_weights;

typedef struct {
    int32_t n_miss;         /* selected experts that were not resident  */
    int32_t n_substituted;  /* of those, replaced by a resident buddy   */
    int32_t n_dropped;      /* of those, dropped (no acceptable buddy)  */
    /* Distribution gate (Eq. 2); all three are 0 without BM_GATE_DIST */
    int32_t n_requested;            /* distinct experts routed to by the batch       */
    int32_t n_requested_offloaded;  /* of those, not resident                        */
    int32_t bypassed;               /* 1 if delta >= beta switched substitution off  */
} bm_remap_stats;

/* Optional outputs of bm_moe_forward; any member may be NULL.  Pointers are
 * device memory. */
typedef struct {
    int32_t *ids;            /* [T][K] router's choice                      */
    int32_t *ids_remapped;   /* [T][K] after substitution, -1 = dropped     */
    float *w;                /* [T][K] gate weights after drops             */
    int32_t *offsets;        /* [E+1]                                       */
    int32_t *perm;           /* [T*K]                                       */
    int32_t *inv_perm;       /* [T*K]                                       */
    bm_remap_stats *stats;   /* one struct                                  */
    void *stage_events[5];   /* hipEvent_t handles, all NULL or all set; recorded on
                                `stream` before the front end, after the grouping,
                                after the gate/up projection, after the down
                                projection and after the aggregation (timing only) */
} bm_debug_out;

/* Router and gates (Section 3, "Notation and Preliminaries"; Section 2.2):
 *   z[t][e] = bias[e] + sum_j x[t][j] * w_router[e][j]      (fp32 accumulation)
 *   p = softmax(z);  ids[t][0..K) = the K experts of largest z, slot 0 the
 *   largest, equal logits to the lower index;  w[t][k] = p of slot k,
 *   renormalised over the K slots when BM_RENORM_TOPK is set.
 * x [T][d] dtype (device), w_router [E][d] dtype (device), bias [E] fp32 or
 * NULL (device), ids [T][K] int32 and w [T][K] fp32 (device, written).
 * Uses T, d, E, K, dtype, flags of desc.  T == 0 is a no-op. */
int bm_route_topk(const bm_layer_desc *desc, const void *x, const void *w_router,
                  const float *bias, int32_t *ids, float *w, void *stream);

/* Buddy substitution (Section 4, Algorithm 1; fallback of Section 3.1):
 * per token, slots in order k = 0..K-1; a slot whose expert e is resident is
 * kept; otherwise it takes the first b = buddy_table[e][r], r < H, that is in
 * [0,E), resident and - with BM_REMAP_UNIQUE - not in the token's set U_t
 * (the token's K input ids plus the buddies accepted at earlier slots).  If
 * none qualifies the slot is dropped: id -1 and, when w is given, w = 0 (the
 * other slots' weights are not renormalised).  A substitute keeps the slot's
 * gate weight.  Input ids outside [0,E) come out as -1 / w = 0.
 * residency_bitmap: ceil(E/64) uint64 words (device), expert e resident iff
 *   bit (e % 64) of word (e / 64) is set.
 * buddy_table [E][R] int32 (device), best buddy first, short rows padded -1.
 * ids_in [T][K] (device); ids_out [T][K] (device, may alias ids_in);
 * w [T][K] fp32 in/out (device, nullable); stats (device, nullable, written).
 * With BM_GATE_TAE / BM_GATE_MARGIN (Section 3.1) the gates are evaluated per
 * token in fp32 from w as passed in (w is then required: BM_ERR_NULL without it;
 * BM_REPLACE_BUDGET, Section 5.1, counts substitutions and does not read w); a miss
 * of a gated token, or one beyond the token's budget, counts as a miss and as
 * dropped.  TAE and the margin are fp32 values compared with fp32 thresholds: a
 * token whose exact TAE (or margin) lies within about 2e-5 of the threshold may
 * fall on either side of it.  BM_GATE_DIST takes the
 * T tokens of the call as the batch; with it and ids_out == ids_in the call
 * runs in a single workgroup (the request set has to be read before any id is
 * overwritten).  BM_PSI_TOKEN needs the router's probabilities and is refused
 * here (BM_ERR_SHAPE): it is served by bm_moe_forward.
 * Uses T, E, K, R, H, flags, tae_tau, margin_gamma, rho, dist_beta of desc. */
int bm_buddy_remap(const bm_layer_desc *desc, const uint64_t *residency_bitmap,
                   const int32_t *buddy_table, const int32_t *ids_in, int32_t *ids_out,
                   float *w, bm_remap_stats *stats, void *stream);

/* Profiling statistics (Section 3.2, "Empirical Evidence from Profiling"): for
 * the batch of routed ids [T][K] (device int32),
 *   activations[i]      += number of tokens with i in S(x)
 *   coactivations[i][j] += number of tokens with i and j both in S(x), i != j
 * activations [E] and coactivations [E][E] are device int64 running totals that
 * the caller zeroes before the first batch; the diagonal is never written.  Ids
 * outside [0,E) are ignored and an expert listed twice by a token counts once.
 * Exact (integer atomics); batches may be fed in any order.  Uses T, E, K. */
int bm_coactivation_accumulate(const bm_layer_desc *desc, const int32_t *ids, int64_t *activations,
                               int64_t *coactivations, void *stream);

/* Buddy lists from the co-activation counts (Section 3.2 Eq. 4, Section 3.3
 * Eq. 5-6).  Per pivot i: q[j|i] = coactivations[i][j] / (sum of row i without
 * the diagonal); peers sorted by descending q, equal q to the lower index; the
 * list is the shortest prefix whose q sums to at least alpha, at most R entries,
 * at least one when the row sum is positive, none when it is zero; peers with
 * q = 0 are never listed.  The threshold test is made on the counts,
 * prefix count >= (double)alpha * (double)row sum, in fp64.
 * buddy_table [E][R] int32 (device, written; best first, padded with -1) has the
 * layout bm_buddy_remap and bm_moe_forward read.  list_len [E] int32 and
 * q [E][R] fp32 (the q of each listed entry, 0 in the padding) are optional
 * device outputs.  0 < alpha <= 1.  Uses E, R of desc.  Not modelled: the
 * optional stabilisers of Section 3.3 (probability-weighted counts, Laplace
 * smoothing, warm-up down-weighting). */
int bm_build_buddy_table(const bm_layer_desc *desc, const int64_t *coactivations, float alpha,
                         int32_t *buddy_table, int32_t *list_len, float *q, void *stream);

/* Grouping of the surviving assignments by expert, the execution order of the
 * expert FFNs (Section 2.2: the selected experts run, their outputs are
 * aggregated): a stable counting sort of the flat indices a = t*K + k with
 * ids[a] >= 0, keyed by ids[a].
 *   offsets [E+1]: first position of each expert, offsets[E] = live count
 *   perm [T*K]: perm[pos] = a for pos < live count, -1 after
 *   inv_perm [T*K]: position of assignment a, -1 if dropped
 * All device int32.  Uses T, E, K of desc only.  workspace: device scratch,
 * 256-byte aligned, of at least bm_workspace_bytes of a desc with the same T, E, K
 * and d = F = 0 (a few hundred bytes to a few hundred KB: per-tile histograms);
 * the size of a whole layer's desc is always enough as well.
 * T = 0 writes offsets (all zero) only; the other arrays may then be NULL. */
int bm_permute_by_expert(const bm_layer_desc *desc, const int32_t *ids_remapped,
                         int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                         void *workspace, size_t workspace_bytes, void *stream);

/* The whole layer (Sections 2.2, 3 and 4 as above) plus expert execution:
 *   for every surviving slot: h = silu(W_g[e] x) * (W_u[e] x), o = W_d[e] h
 *   y[t] = sum_k w[t][k] * o[t][k] + sum_{s<n_shared} FFN^shared_s(x[t])
 * x [T][d] dtype (device), y [T][d] dtype or fp32 with BM_Y_F32 (device,
 * written; must not alias x).  workspace as above.  dbg may be NULL.
 * bf16: MFMA with fp32 accumulation, h and o held in bf16 between the two
 * projections; fp32: fp32 FMA throughout. */
int bm_moe_forward(const bm_layer_desc *desc, const void *x, const bm_weights *weights,
                   const uint64_t *residency_bitmap, const int32_t *buddy_table, void *y,
                   void *workspace, size_t workspace_bytes, const bm_debug_out *dbg,
                   void *stream);

/* bm_moe_forward for callers that cannot allocate device memory or carry a
 * workspace: code running under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, kernels and results as bm_moe_forward,
 * but the scratch is a BM_STATIC_WORKSPACE_BYTES array built into the library's
 * device code (each GPU the library is loaded on holds one copy until the process
 * ends); the call allocates and frees nothing.  A desc whose
 * bm_workspace_bytes exceeds BM_STATIC_WORKSPACE_BYTES is refused with
 * BM_ERR_WORKSPACE before anything is launched (decode-sized batches of the large
 * layers and small prefill batches fit; use bm_moe_forward beyond that).  Every
 * call on a GPU shares that GPU's array: calls that overlap on one GPU (different
 * streams or threads) race - serialise them.  Nothing in the array has to survive
 * between calls and every kernel writes what it later reads, so no clearing is
 * needed and none is done.  The array's address is looked up once per device, on
 * the first call with that device current (BM_ERR_HIP if the lookup fails). */
#define BM_STATIC_WORKSPACE_BYTES (32u << 20)
int bm_moe_forward_static(const bm_layer_desc *desc, const void *x, const bm_weights *weights,
                          const uint64_t *residency_bitmap, const int32_t *buddy_table, void *y,
                          const bm_debug_out *dbg, void *stream);

/* One-time repacking of the expert weights for decode-sized batches (model
 * load time, not part of the forward pass).  The public layout above stays the
 * reference; the packed copy holds, for every block of 16 weight rows and every
 * 32 values of the reduction dimension, the 1 KB MFMA operand fragment
 * contiguously (gate and up fragments interleaved), so a wave streams its rows
 * as one contiguous run.  Optional: without it the decode kernels fetch the
 * public layout as whole cache lines and re-order them on chip, a few per cent
 * slower; the copy costs the memory of the resident experts once more.
 * bf16 only; needs F % 32 == 0 and d % 32 == 0.
 * which: 0 routed gate+up, 1 routed down, 2 shared gate+up, 3 shared down. */
size_t bm_packed_bytes(const bm_layer_desc *desc, int which);

/* Fills the packed buffers named in weights->wp_* / wsp_* (device, caller-owned,
 * at least bm_packed_bytes each; a NULL member is skipped) from the public
 * arrays of the same struct.  residency_bitmap (device, nullable): only routed
 * experts whose bit is set are read and packed - weights of absent experts are
 * not touched; NULL packs all.  Shared experts are always packed. */
int bm_pack_weights(const bm_layer_desc *desc, const bm_weights *weights,
                    const uint64_t *residency_bitmap, void *stream);

/* Bytes of device scratch bm_moe_forward needs for this desc (host, pure function
 * of desc: T, d, E, F, K, n_shared, dtype and flags enter; 0 if desc is invalid).
 * With d = 0 and F = 0 it is the scratch of bm_permute_by_expert alone, a function
 * of T, E and K. */
size_t bm_workspace_bytes(const bm_layer_desc *desc);

/* Host-side check of a residency bitmap and buddy table (host pointers):
 * every table entry is -1 or in [0,E) and differs from its row index
 * (Eq. 4: an expert is not its own buddy).  BM_OK or BM_ERR_BAD_TABLE. */
int bm_validate_tables(const bm_layer_desc *desc, const uint64_t *bitmap_host,
                       const int32_t *table_host);

/* Static string for a bm_status. */
const char *bm_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* BUDDYMOE_H */
