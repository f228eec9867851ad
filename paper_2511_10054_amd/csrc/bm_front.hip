// Front end of the layer: router logits, softmax / top-k gates, buddy
// substitution (Section 4, Algorithm 1) and the stable grouping of the
// surviving assignments by expert.
//
// Tokens are processed in tiles of TILE_T = 32 (16 for small bf16 batches, see
// front_tile_tokens).  One workgroup owns one tile:
// its waves split the hidden dimension for the router product (MFMA for bf16,
// fp32 FMA for fp32), the partial logits meet in LDS, then each wave ranks
// whole tokens (one expert per lane), 32 lanes walk Algorithm 1 for the 32
// tokens, and the tile's per-expert histogram goes to global memory.  A
// one-workgroup scan turns the histograms into group offsets, per-tile bases
// and the row-tile table of the grouped GEMMs; a scatter kernel then places
// every assignment (rank inside the tile by counting earlier equal keys, so
// the order is the stable one and no atomics decide a position).  Small batches
// get offsets and placement from one workgroup instead (group_small_kernel), or
// from the front kernel itself (FUSED).
#include "bm_kernels.h"

namespace bm {

// ---------------------------------------------------------------------------
// Algorithm 1 for one token.  Slots are visited in order; the scan over a
// buddy row has a fixed trip count H and selects the first acceptable entry
// without an early exit.  `bitmap` is the residency mask (LDS), `table` the
// buddy table (LDS or global), `ids` the token's K slots (read, then
// overwritten in place), `w` its gate weights (nullable).
// ---------------------------------------------------------------------------
__device__ __forceinline__ bool test_bit4(const uint64_t (&m)[4], int b) {
    const int wi = b >> 6;
    uint64_t wv = wi == 0 ? m[0] : wi == 1 ? m[1] : wi == 2 ? m[2] : m[3];
    return (wv >> (b & 63)) & 1ull;
}
__device__ __forceinline__ void set_bit4(uint64_t (&m)[4], int b) {
    const int wi = b >> 6;
    const uint64_t bit = 1ull << (b & 63);
    m[0] |= wi == 0 ? bit : 0ull;
    m[1] |= wi == 1 ? bit : 0ull;
    m[2] |= wi == 2 ? bit : 0ull;
    m[3] |= wi == 3 ? bit : 0ull;
}

// Gates in front of the substitution (Section 3.1: TAE, Eq. 1, and probability margin;
// Section 5.1: replacement budget).  From the token's K gate weights renormalised to sum 1:
// the token may be given substitutes unless (BM_GATE_TAE and TAE <= tau) or (BM_GATE_MARGIN and
// largest - second largest >= gamma); returns how many slots may be replaced (0 = none).
__device__ __forceinline__ int replacement_budget(int K, uint32_t flags, float tau, float gamma, int rho,
                                                  const float *w) {
    int budget = (flags & BM_REPLACE_BUDGET) ? rho : 0x7fffffff;
    if (flags & (BM_GATE_TAE | BM_GATE_MARGIN)) {
        float sum = 0.0f;
        for (int k = 0; k < K; ++k) sum += w[k];
        float h = 0.0f, p1 = 0.0f, p2 = 0.0f;
        for (int k = 0; k < K; ++k) {
            const float pk = w[k] / sum;
            h -= pk > 0.0f ? pk * logf(pk) : 0.0f;
            const float lo = fminf(p1, pk);
            p1 = fmaxf(p1, pk);
            p2 = fmaxf(p2, lo);
        }
        const float tae = K > 1 ? h / logf((float)K) : 0.0f;
        if ((flags & BM_GATE_TAE) && tae <= tau) budget = 0;
        if ((flags & BM_GATE_MARGIN) && (p1 - p2) >= gamma) budget = 0;
    }
    return budget;
}

// Distribution gate (Section 3.1, Eq. 2): delta = n_cpu / n_req >= beta, decided without rounding
// (both products are exact in fp64 for counts up to BM_MAX_E and an fp32 threshold).
__device__ __forceinline__ bool dist_bypass(int n_req, int n_cpu, float beta) {
    return n_req > 0 && (double)n_cpu >= (double)beta * (double)n_req;
}

// Token-aware buddy priority (Section 3.1, Eq. 3 with kappa = 0): how the normalised router logit of
// expert b (its softmax probability over all experts) is obtained for the token at hand.
struct PsiSource {
    const float *q;        // [E][R] q[j|i] of every table entry; null: priority = table order
    float eta;
    const float *logits;   // the token's logit row (bias included), with zmax and inv_den; or null
    float zmax, inv_den;
    const float *probs;    // the token's probability row; used when logits is null
    __device__ __forceinline__ float zhat(int b) const {
        return logits != nullptr ? __expf(logits[b] - zmax) * inv_den : probs[b];
    }
};

__device__ __forceinline__ void remap_token(int K, int E, int R, int H, uint32_t flags, float tau, float gamma,
                                            int rho, const uint64_t *bitmap, const int32_t *table,
                                            const int32_t *ids_in, int32_t *ids_out, float *w,
                                            int &n_miss, int &n_sub, int &n_drop, const PsiSource &psi) {
    const bool unique = (flags & BM_REMAP_UNIQUE) != 0;
    int budget = 0x7fffffff;
    if (flags & BM_GATE_ANY) budget = replacement_budget(K, flags, tau, gamma, rho, w);   // before any drop
    uint64_t used[4] = {0ull, 0ull, 0ull, 0ull};   // U_t
    for (int k = 0; k < K; ++k) {
        int e = ids_in[k];
        if ((unsigned)e < (unsigned)E) set_bit4(used, e);
    }
    for (int k = 0; k < K; ++k) {
        const int e = ids_in[k];
        const bool valid = (unsigned)e < (unsigned)E;
        const bool res = valid && ((bitmap[e >> 6 & 3] >> (e & 63)) & 1ull);
        int out = res ? e : -1;
        if (valid && !res) {
            ++n_miss;
            bool found = false;
            const int32_t *row = table + (size_t)e * R;
            const int depth = budget > 0 ? H : 0;          // budget used up or token gated: no search
            if (psi.q == nullptr) {
                for (int r = 0; r < depth; ++r) {
                    const int b = row[r];
                    const bool bvalid = (unsigned)b < (unsigned)E;
                    const int bc = bvalid ? b : 0;
                    bool ok = bvalid && ((bitmap[bc >> 6] >> (bc & 63)) & 1ull);
                    ok = ok && !(unique && test_bit4(used, bc));
                    out = (ok && !found) ? b : out;
                    found = found || ok;
                }
            } else {
                // the acceptable entry of largest q * (1 + eta * zhat); equal scores keep the earlier entry
                const float *qrow = psi.q + (size_t)e * R;
                float best = 0.0f;
                for (int r = 0; r < depth; ++r) {
                    const int b = row[r];
                    const bool bvalid = (unsigned)b < (unsigned)E;
                    const int bc = bvalid ? b : 0;
                    bool ok = bvalid && ((bitmap[bc >> 6] >> (bc & 63)) & 1ull);
                    ok = ok && !(unique && test_bit4(used, bc));
                    const float score = qrow[r] * (1.0f + psi.eta * psi.zhat(bc));
                    const bool take = ok && (!found || score > best);
                    out = take ? b : out;
                    best = take ? score : best;
                    found = found || ok;
                }
            }
            if (found) { ++n_sub; --budget; set_bit4(used, out); } else { ++n_drop; }
        }
        ids_out[k] = out;
        if (w != nullptr && out < 0) w[k] = 0.0f;
    }
}

// ---------------------------------------------------------------------------
// Shared LDS block of the front kernels.
// ---------------------------------------------------------------------------
struct FrontLds {
    int32_t ids[TILE_T * BM_MAX_K];
    float w[TILE_T * BM_MAX_K];
    int32_t counts[BM_MAX_E];
    int32_t lut[BM_MAX_E];
    int32_t stats[4];
    int32_t dist[4];         // distribution gate: requested, requested and offloaded, bypassed
    uint64_t bitmap[4];
    unsigned long long req[4];
    float zmax[TILE_T], inv_den[TILE_T];   // per token: largest logit, 1 / sum of exp over all experts
};

// Ranks the tile's tokens from the logits in LDS and finishes the tile.
// logits: [TILE_T][stride] fp32, bias already added.  The logits region is
// reused for the buddy table once ranking is done (cap = its size in ints).
template <int EC>   // EC = ceil(E / 64) experts per lane (compile-time bound)
__device__ void tile_epilogue(const FrontParams &p, float *logits, int stride, int cap_ints,
                              FrontLds &s, int tile) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    const int t0 = tile * p.tile_tokens;
    const int ntok = min(p.tile_tokens, p.T - t0);
    const int E = p.E, K = p.K;
    const int ec = (E + 63) >> 6;

    // Lane l owns experts l, l+64, ...  Few experts - ranking by counting: the rank of an expert is the
    // number of experts that beat it (larger logit, or equal logit and lower index), found with E
    // broadcast reads of the logit row, no cross-lane traffic; experts of rank < K are the selection,
    // slot = rank.  Many experts - K rounds of a wave-wide maximum (see below).  Same order either way.
    for (int i = wave; i < ntok; i += nw) {
        const float *zr = logits + i * stride;
        float myv[EC];
        int rank[EC];
#pragma unroll
        for (int c = 0; c < EC; ++c) {
            const int e = lane + 64 * c;
            myv[c] = (e < E) ? zr[e] : -INFINITY;
            rank[c] = 0;
        }
        if (E <= 16) {
#pragma unroll 16
            for (int j = 0; j < E; ++j) {              // branch-free body, unrolled: the LDS reads go out in batches
                const float zj = zr[j];
#pragma unroll
                for (int c = 0; c < EC; ++c)
                    rank[c] += (int)(zj > myv[c]) | ((int)(zj == myv[c]) & (int)(j < lane + 64 * c));
            }
#pragma unroll
            for (int c = 0; c < EC; ++c) {
                const int e = lane + 64 * c;
                if (e < E && rank[c] < K) {
                    s.ids[i * K + rank[c]] = e;
                    s.w[i * K + rank[c]] = myv[c];        // the logit for now; replaced by the gate weight below
                }
            }
        } else {
            // Many experts: K rounds of "largest remaining" instead (counting costs E reads per lane).
            // A round takes the wave-wide maximum of the order-preserving integer image of the logits,
            // then the lowest expert index that holds it (ballots, lowest set lane of the lowest c);
            // that expert's owner takes it out of the race (0 is below the image of every float).
            uint32_t key[EC];
#pragma unroll
            for (int c = 0; c < EC; ++c) key[c] = (lane + 64 * c < E) ? float_to_ordered(myv[c]) : 0u;
            for (int r = 0; r < K; ++r) {
                uint32_t mine = key[0];
#pragma unroll
                for (int c = 1; c < EC; ++c) mine = key[c] > mine ? key[c] : mine;
                const uint32_t best = wave_max_u32(mine);
                int e_win = -1;
#pragma unroll
                for (int c = EC - 1; c >= 0; --c) {
                    const unsigned long long m = __ballot(key[c] == best);
                    if (m != 0ull) e_win = 64 * c + (int)__builtin_ctzll(m);
                }
#pragma unroll
                for (int c = 0; c < EC; ++c)
                    if (lane + 64 * c == e_win) key[c] = 0u;
                if (lane == 0) {
                    s.ids[i * K + r] = e_win;
                    s.w[i * K + r] = ordered_to_float(best);
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        const float zmax = s.w[i * K];
        float denom = 0.0f;
        if (p.flags & BM_RENORM_TOPK) {
            for (int k = 0; k < K; ++k) denom += expf(s.w[i * K + k] - zmax);     // same order in every lane
        } else {
            float part = 0.0f;
#pragma unroll
            for (int c = 0; c < EC; ++c) part += (myv[c] == -INFINITY) ? 0.0f : expf(myv[c] - zmax);
            denom = wave_sum(part);
        }
        const float pk = (lane < K) ? expf(s.w[i * K + lane] - zmax) : 0.0f;
        if (p.flags & BM_PSI_TOKEN) {
            // token-aware buddy priority needs every expert's softmax probability for this token: keep
            // (zmax, 1 / sum over all experts) for the substitution below, or write the probabilities out
            // when the substitution runs in a later kernel
            float part = 0.0f;
#pragma unroll
            for (int c = 0; c < EC; ++c) part += (myv[c] == -INFINITY) ? 0.0f : __expf(myv[c] - zmax);
            const float inv_all = 1.0f / wave_sum(part);
            if (lane == 0) { s.zmax[i] = zmax; s.inv_den[i] = inv_all; }
            if (p.probs_out != nullptr) {
#pragma unroll
                for (int c = 0; c < EC; ++c) {
                    const int e = lane + 64 * c;
                    if (e < E) p.probs_out[(size_t)(t0 + i) * E + e] = __expf(myv[c] - zmax) * inv_all;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        if (lane < K) {
            p.ids[(size_t)(t0 + i) * K + lane] = s.ids[i * K + lane];
            s.w[i * K + lane] = pk / denom;
        }
    }
    __syncthreads();

    const int n = ntok * K;
    if (p.bitmap == nullptr) {                   // routing only
        for (int idx = tid; idx < n; idx += blockDim.x) p.w[(size_t)t0 * K + idx] = s.w[idx];
        return;
    }

    // stage residency bitmap and buddy table in LDS
    const bool psi_mode = (p.flags & BM_PSI_TOKEN) != 0;         // the logits stay where they are
    const bool tab_in_lds = !psi_mode && E * p.R <= cap_ints;
    int32_t *s_table = reinterpret_cast<int32_t *>(logits);
    if (tab_in_lds)
        for (int idx = tid; idx < E * p.R; idx += blockDim.x) s_table[idx] = p.table[idx];
    for (int idx = tid; idx < BM_MAX_E; idx += blockDim.x) s.counts[idx] = 0;
    if (tid < 4) { s.bitmap[tid] = (tid < ec) ? p.bitmap[tid] : 0ull; s.stats[tid] = 0; s.req[tid] = 0ull; s.dist[tid] = 0; }
    __syncthreads();

    int H = p.H;
    if (p.flags & BM_GATE_DIST) {
        // this tile holds the whole batch (the host guarantees it): set of requested experts, Eq. 2
        for (int idx = tid; idx < n; idx += blockDim.x) {
            const int e = s.ids[idx];
            atomicOr(&s.req[e >> 6], 1ull << (e & 63));
        }
        __syncthreads();
        int n_req = 0, n_cpu = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            n_req += __popcll(s.req[i]);
            n_cpu += __popcll(s.req[i] & ~s.bitmap[i]);
        }
        const bool bypass = dist_bypass(n_req, n_cpu, p.beta);
        if (bypass) H = 0;                       // every miss is dropped
        if (tid == 0) { s.dist[0] = n_req; s.dist[1] = n_cpu; s.dist[2] = bypass ? 1 : 0; }
    }

    if (p.flags & (BM_REMAP_UNIQUE | BM_GATE_ANY | BM_PSI_TOKEN)) {
        // Algorithm 1 proper (and its per-token gates and priorities): a lane walks its token's slots in order
        if (tid < ntok) {
            int n_miss = 0, n_sub = 0, n_drop = 0;
            int32_t *tok_ids = &s.ids[tid * K];
            float *tok_w = &s.w[tid * K];
            PsiSource psi{};
            if (psi_mode) {
                psi.q = p.q; psi.eta = p.eta;
                psi.logits = logits + tid * stride; psi.zmax = s.zmax[tid]; psi.inv_den = s.inv_den[tid];
            }
            remap_token(K, E, p.R, H, p.flags, p.tau, p.gamma, p.rho, s.bitmap,
                        tab_in_lds ? s_table : p.table, tok_ids, tok_ids, tok_w, n_miss, n_sub, n_drop, psi);
            if (n_miss) atomicAdd(&s.stats[0], n_miss);
            if (n_sub) atomicAdd(&s.stats[1], n_sub);
            if (n_drop) atomicAdd(&s.stats[2], n_drop);
            for (int k = 0; k < K; ++k) {
                const int e = tok_ids[k];
                if (e >= 0) atomicAdd(&s.counts[e], 1);
            }
        }
    } else {
        // without the U_t test the substitute depends on the expert alone: one lane per expert scans
        // its buddy row once (same fixed-trip select scan), then every assignment is a table lookup
        const int32_t *tab = tab_in_lds ? s_table : p.table;
        for (int e = tid; e < E; e += blockDim.x) {
            const bool res = (s.bitmap[e >> 6] >> (e & 63)) & 1ull;
            int out = res ? e : -1;
            bool found = res;
            for (int r = 0; r < H; ++r) {
                const int b = tab[e * p.R + r];
                const bool bvalid = (unsigned)b < (unsigned)E;
                const int bc = bvalid ? b : 0;
                const bool ok = bvalid && ((s.bitmap[bc >> 6] >> (bc & 63)) & 1ull);
                out = (ok && !found) ? b : out;
                found = found || ok;
            }
            s.lut[e] = out | (res ? 0 : 0x40000000);       // bit 30 marks "was not resident"
        }
        __syncthreads();
        for (int idx = tid; idx < n; idx += blockDim.x) {
            const int v = s.lut[s.ids[idx]];
            const bool miss = (v & 0x40000000) != 0 || v < 0;
            const int out = v < 0 ? -1 : (v & 0x3fffffff);
            s.ids[idx] = out;
            if (out < 0) s.w[idx] = 0.0f;
            if (miss) atomicAdd(&s.stats[0], 1);
            if (miss && out >= 0) atomicAdd(&s.stats[1], 1);
            if (out < 0) atomicAdd(&s.stats[2], 1);
            if (out >= 0) atomicAdd(&s.counts[out], 1);
        }
    }
    __syncthreads();

    for (int idx = tid; idx < n; idx += blockDim.x) {
        p.ids2[(size_t)t0 * K + idx] = s.ids[idx];
        p.w[(size_t)t0 * K + idx] = s.w[idx];
    }
    // histograms are stored expert-major ([E][tiles]): the single workgroup that scans them reads and writes
    // whole lines, the strided side is spread over the many workgroups here
    const int n_tiles_all = (p.T + p.tile_tokens - 1) / p.tile_tokens;
    for (int e = tid; e < E; e += blockDim.x) p.tile_counts[(size_t)e * n_tiles_all + tile] = s.counts[e];
    if (tid < 3) p.tile_stats[tile * 4 + tid] = s.stats[tid];
}

// ---------------------------------------------------------------------------
// Tail of the front end when one workgroup owns every tile (at most
// FUSED_TILES tiles, i.e. decode-sized batches): group offsets, row-tile table,
// statistics and the stable placement, from the per-tile histograms and
// substituted ids kept in LDS.  Saves the scan and scatter launches.
// ---------------------------------------------------------------------------
constexpr int FUSED_TILES = 1;

struct FusedLds {
    int32_t ids[FUSED_TILES][TILE_T * BM_MAX_K];   // substituted ids of every tile
    int32_t counts[FUSED_TILES][BM_MAX_E];         // per-tile histograms
    int32_t stats[FUSED_TILES][4];
    int32_t dist[4];                               // distribution gate counters (single-tile batches)
    int32_t start[BM_MAX_E + 16];                  // group offsets
    int32_t tstart[BM_MAX_E + 16];                 // first row tile of each group
};

// exclusive prefix sum over the wave; `total` = sum over all lanes
__device__ __forceinline__ int wave_excl_scan(int v, int &total) {
    const int lane = threadIdx.x & 63;
    int incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(incl, d, WAVE);
        if (lane >= d) incl += o;
    }
    total = __shfl(incl, 63, WAVE);
    return incl - v;
}

// Stable placement of A assignments whose substituted ids sit in LDS (-1 = dropped): the position of
// assignment a is start[e] plus the number of earlier assignments with the same expert e.  One wave
// per expert walks the assignments 64 at a time; the rank inside a step is a ballot and a popcount.
__device__ void place_assignments(const int32_t *ids, int A, int E, int K, const int32_t *start,
                                  const ScatterParams &c) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    for (int e = wave; e < E; e += nw) {
        int run = start[e];
        if (start[e + 1] == run) continue;             // nothing routed to this expert
        for (int base = 0; base < A; base += WAVE) {
            const int a = base + lane;
            const bool mine = a < A && ids[a] == e;
            const unsigned long long m = __ballot(mine);
            if (mine) {
                const int pos = run + __popcll(m & ((1ull << lane) - 1ull));
                c.perm[pos] = a;
                if (c.row_token) c.row_token[pos] = a / K;
                c.inv_perm[a] = pos;
            }
            run += __popcll(m);
        }
    }
    for (int a = tid; a < A; a += blockDim.x)
        if (ids[a] < 0) c.inv_perm[a] = -1;
}

// The two row-tile lists of a projection that runs both tile heights in one launch (p.mixed): a group of n rows
// gives n / 256 tiles of 256 rows, and its rest one more of them when it exceeds 128 rows, else (when there is
// a rest) one 128-row tile.  Called by every thread of the workgroup once `start` (G + 1 group starts in LDS)
// is valid; the last wave does the work - scans over the groups in registers, a few consecutive groups per
// lane - while the others go on.
__device__ void write_mixed_tile_tables(const ScanParams &p, const int32_t *start) {
    if (!p.mixed) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if (wave != nw - 1) return;
    const int G = p.E + p.n_shared;
    constexpr int PER = (BM_MAX_E + 8 + 63) / 64;
    int nb[PER], ns[PER], sum_b = 0, sum_s = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int g = lane * PER + i;
        const int n = g < G ? start[g + 1] - start[g] : 0;
        const int rest = n & 255;
        nb[i] = (n >> 8) + (rest > 128 ? 1 : 0);
        ns[i] = (rest >= 1 && rest <= 128) ? 1 : 0;
        sum_b += nb[i];
        sum_s += ns[i];
    }
    int tot_b, tot_s;
    int run_b = wave_excl_scan(sum_b, tot_b), run_s = wave_excl_scan(sum_s, tot_s);
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int g = lane * PER + i;
        for (int j = 0; j < nb[i]; ++j) {
            p.mt_group_b[run_b + j] = g;
            p.mt_row0_b[run_b + j] = start[g] + j * 256;
        }
        if (ns[i]) {
            p.mt_group_s[run_s] = g;
            p.mt_row0_s[run_s] = start[g] + nb[i] * 256;
        }
        run_b += nb[i];
        run_s += ns[i];
    }
    if (lane == 0) {
        p.n_mtiles_b[0] = tot_b; p.n_mtiles_b[1] = start[G];
        p.n_mtiles_s[0] = tot_s; p.n_mtiles_s[1] = start[G];
    }
}

// Offsets and the list of row tiles from the group starts in LDS (start: G + 1 rows, tstart: G + 1 tiles);
// every thread of one workgroup calls it.  For the decode projections (largest_first) the list holds the
// live groups by falling row count: a group is one work-item column of their grid, groups with more rows take
// longer per item, and handing the big ones out first leaves the short items for the end of the launch.
__device__ void write_group_tables(const ScanParams &p, const int32_t *start, const int32_t *tstart) {
    const int tid = threadIdx.x, G = p.E + p.n_shared;
    for (int g = tid; g <= G; g += blockDim.x) p.offsets[g] = start[g];
    if (p.largest_first) {
        for (int g = tid; g < G; g += blockDim.x) {
            const int n = start[g + 1] - start[g];
            if (n == 0) continue;
            int rank = 0;
            for (int h = 0; h < G; ++h) {
                const int m = start[h + 1] - start[h];
                rank += (m > n || (m == n && h < g)) ? 1 : 0;
            }
            p.mt_group[rank] = g;
            p.mt_row0[rank] = start[g];
        }
    } else {
        for (int g = tid; g < G; g += blockDim.x) {
            const int nt = tstart[g + 1] - tstart[g];
            for (int i = 0; i < nt; ++i) {
                p.mt_group[tstart[g] + i] = g;
                p.mt_row0[tstart[g] + i] = start[g] + i * p.BM;
            }
        }
    }
}

// Everything after the per-expert counts of a batch whose substituted ids sit in LDS (one workgroup):
// group offsets, the list of row tiles (or of live groups, largest first, for the decode projections),
// statistics, stable placement.  counts: E entries in LDS; start / tstart: LDS scratch of G + 1 entries;
// local_stats: the three substitution counters in LDS, or null to add up the per-tile ones.  Every thread of
// the workgroup calls it, after a barrier behind the writes of ids and counts.
__device__ void finish_groups(const ScanParams &p, const ScatterParams &c, const int32_t *ids, int A,
                              const int32_t *counts, int32_t *start, int32_t *tstart, const int32_t *local_stats) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int E = p.E, G = p.E + p.n_shared, K = c.K;
    if (wave == 0) {                               // exclusive scans over the groups, a few consecutive groups per lane
        constexpr int PER = (BM_MAX_E + 8 + 63) / 64;
        int cnt[PER], nt[PER], sum_c = 0, sum_t = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int g = lane * PER + i;
            const int n = g < E ? counts[g] : (g < G ? p.T : 0);
            cnt[i] = n;
            nt[i] = (n + p.BM - 1) / p.BM;
            sum_c += n;
            sum_t += nt[i];
        }
        int tot_c, tot_t;
        int run_c = wave_excl_scan(sum_c, tot_c), run_t = wave_excl_scan(sum_t, tot_t);
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int g = lane * PER + i;
            if (g <= G) { start[g] = run_c; tstart[g] = run_t; }
            run_c += cnt[i];
            run_t += nt[i];
        }
        if (lane == 0) { p.n_mtiles[0] = tot_t; p.n_mtiles[1] = tot_c; }
    }
    __syncthreads();
    write_group_tables(p, start, tstart);
    write_mixed_tile_tables(p, start);
    if (p.stats != nullptr && wave < 3) {          // one wave per counter
        int sum = 0;
        if (local_stats != nullptr) sum = local_stats[wave];
        else {
            if (p.tile_stats != nullptr)
                for (int t = lane; t < p.n_tiles; t += WAVE) sum += p.tile_stats[t * 4 + wave];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, WAVE);
        }
        if (lane == 0) { p.stats[wave] = sum; p.stats[3 + wave] = 0; }
    }
    place_assignments(ids, A, E, K, start, c);
    const int live = start[E];
    for (int pos = live + tid; pos < A; pos += blockDim.x) c.perm[pos] = -1;
    if (c.row_token)
        for (int sidx = 0; sidx < p.n_shared; ++sidx)
            for (int t = tid; t < p.T; t += blockDim.x) c.row_token[start[E + sidx] + t] = t;
}

__device__ void fused_tail(const FrontParams &p, FusedLds &fs, int n_tiles) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int E = p.E, K = p.K, n_shared = p.scan.n_shared, G = E + n_shared, BM = p.scan.BM;
    // group offsets and row-tile starts: one wave, up to 5 consecutive groups per lane
    if (wave == 0) {
        constexpr int PER = (BM_MAX_E + 8 + 63) / 64;
        int cnt[PER], nt[PER], sum_c = 0, sum_t = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int g = lane * PER + i;
            int c = 0;
            if (g < E) { for (int t = 0; t < n_tiles; ++t) c += fs.counts[t][g]; }
            else if (g < G) c = p.T;
            cnt[i] = c;
            nt[i] = (c + BM - 1) / BM;
            sum_c += c;
            sum_t += nt[i];
        }
        int tot_c, tot_t;
        int run_c = wave_excl_scan(sum_c, tot_c), run_t = wave_excl_scan(sum_t, tot_t);
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int g = lane * PER + i;
            if (g <= G) { fs.start[g] = run_c; fs.tstart[g] = run_t; }
            run_c += cnt[i];
            run_t += nt[i];
        }
        if (lane == 0) { p.scan.n_mtiles[0] = tot_t; p.scan.n_mtiles[1] = tot_c; }
    }
    __syncthreads();
    for (int g = tid; g <= G; g += blockDim.x) p.scan.offsets[g] = fs.start[g];
    for (int g = tid; g < G; g += blockDim.x) {
        const int ntile = fs.tstart[g + 1] - fs.tstart[g];
        for (int i = 0; i < ntile; ++i) {
            p.scan.mt_group[fs.tstart[g] + i] = g;
            p.scan.mt_row0[fs.tstart[g] + i] = fs.start[g] + i * BM;
        }
    }
    write_mixed_tile_tables(p.scan, fs.start);
    if (p.scan.stats != nullptr && tid < 3) {
        int sum = 0;
        for (int t = 0; t < n_tiles; ++t) sum += fs.stats[t][tid];
        p.scan.stats[tid] = sum;
        p.scan.stats[3 + tid] = (p.flags & BM_GATE_DIST) ? fs.dist[tid] : 0;
    }
    // stable placement (the batch is one tile)
    const int live = fs.start[E];
    place_assignments(fs.ids[0], p.T * K, E, K, fs.start, p.scat);
    for (int pos = live + tid; pos < p.T * K; pos += blockDim.x) p.scat.perm[pos] = -1;
    if (p.scat.row_token)
        for (int sidx = 0; sidx < n_shared; ++sidx)
            for (int t = tid; t < p.T; t += blockDim.x) p.scat.row_token[fs.start[E + sidx] + t] = t;
}

// ---------------------------------------------------------------------------
// bf16 front kernel: router product on MFMA 16x16x32 (tokens x experts),
// operands read from global memory directly in the instruction's layout:
// lane l supplies row/column (l % 16) and the 8 consecutive k values starting
// at 8 * (l / 16), i.e. one 16-byte load per operand per k-step, 64 contiguous
// bytes per row.  (The vector memory path moves one 128-byte line per two
// cycles whatever part of it is used, and with many experts these loads bound
// the kernel; the 32x32x16 form reads 32 bytes per row and instruction.)  The
// waves split the hidden dimension in batches of U k-steps; the loads of a
// batch are all issued before its MFMAs.  The partial logit tiles of the waves
// are written to LDS side by side and added in wave order (reproducible sum),
// or, when NW tiles do not fit, added into one tile wave after wave.
// NB = number of 16-expert column blocks, NW = waves per workgroup.
// FUSED: one workgroup walks all (<= FUSED_TILES) tiles and finishes the
// grouping itself.
// ---------------------------------------------------------------------------
template <int NB, int NW, int U, bool FUSED>
__global__ void __launch_bounds__(NW * 64) front_bf16_kernel(FrontParams p) {
    static_assert(TILE_T == 32, "two 16-token row blocks per tile");
    constexpr int STRIDE = NB * 16 + 1;
    constexpr int TILE = TILE_T * STRIDE;
    constexpr int NS_FIT = (68 * 1024) / (TILE * 4);
    constexpr int NS = NS_FIT >= NW ? NW : (NS_FIT < 1 ? 1 : NS_FIT);   // partial tiles kept side by side
    __shared__ float part[NS * TILE];
    constexpr bool CAN_STAGE = !FUSED && U >= 2 && U % 2 == 0;
    __shared__ u32x4 stage[CAN_STAGE ? NW * 256 : 1];            // 4 KB per wave (see the staged product below)
    __shared__ FrontLds s;
    __shared__ FusedLds fs_store[FUSED ? 1 : 0 + 1];
    FusedLds &fs = fs_store[0];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, kq = lane >> 4;
    const uint16_t *x = static_cast<const uint16_t *>(p.x);
    const uint16_t *wr = static_cast<const uint16_t *>(p.wr);
    const int n_tiles = (p.T + p.tile_tokens - 1) / p.tile_tokens;
    const int tile_begin = FUSED ? 0 : blockIdx.x, tile_end = FUSED ? n_tiles : blockIdx.x + 1;

    const uint16_t *wb[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) wb[nb] = wr + (size_t)min(nb * 16 + r16, p.E - 1) * p.d + kq * 8;
    const int ksteps = p.d >> 5;
    const int nbatch = ksteps / U;

    for (int tile = tile_begin; tile < tile_end; ++tile) {
        const int t0 = tile * p.tile_tokens;
        const bool two = min(p.tile_tokens, p.T - t0) > 16;   // the tile's second 16-token block holds tokens (uniform)
        const uint16_t *xa[2];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) xa[tb] = x + (size_t)min(t0 + tb * 16 + r16, p.T - 1) * p.d + kq * 8;
        f32x4 acc[2][NB];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) acc[tb][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

        // Staged product: the operands are fetched as whole 128-byte lines (8 rows per instruction, half as
        // many lines touched as with 64 bytes per row - and with many experts the lines touched bound the
        // kernel) and turned into the MFMA operand order through a wave-private LDS area of two 2 KB
        // blocks: stored 8 rows x 128 bytes per register, read back 16 rows x 16 bytes per fragment, the
        // 16-byte pieces of a row rotated by the row index against bank conflicts.  The blocks are reused
        // operand block after operand block; no barrier: only the writing wave touches its area, and a
        // wave's LDS operations stay in order.  A batch is LPB lines (two k-steps each) of every operand.
        // (not in the fused kernel, which has no registers to spare: it serves batches of a few tokens,
        // whose direct loads touch few lines anyway; not with 256 experts, whose batch would not fit)
        const bool staged = CAN_STAGE;
        int ks_done = nbatch * U;                                      // k-steps covered by the batched loops
        if (CAN_STAGE) {
            constexpr int LPB = U / 2 > 0 ? U / 2 : 1;
            u32x4 *area = stage + (CAN_STAGE ? wave : 0) * 256;       // [block 0..1][row 0..15][piece 0..7]
            const int lrow = lane >> 3, lpiece = lane & 7;
            const uint16_t *xs_[2][2];
            int woff[NB][2], wslot[2], rslot[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int r = 8 * j + lrow;
#pragma unroll
                for (int tb = 0; tb < 2; ++tb) xs_[tb][j] = x + (size_t)min(t0 + tb * 16 + r, p.T - 1) * p.d + lpiece * 8;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) woff[nb][j] = min(nb * 16 + r, p.E - 1) * p.d + lpiece * 8;
                wslot[j] = r * 8 + (lpiece ^ (r & 7));
                rslot[j] = r16 * 8 + ((j * 4 + kq) ^ (r16 & 7));     // fragment of the line's k-step j
            }
            const int nlb = p.d / (64 * LPB);
            ks_done = nlb * 2 * LPB;
            for (int bt = wave; bt < nlb; bt += NW) {
                const int k0 = bt * 64 * LPB;
                u32x4 rx[LPB][2][2], rw[LPB][NB][2];                   // [line][operand block][row group]
#pragma unroll
                for (int h = 0; h < LPB; ++h)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        rx[h][0][j] = ldg128(xs_[0][j] + k0 + h * 64);
                        if (two) rx[h][1][j] = ldg128(xs_[1][j] + k0 + h * 64);
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) rw[h][nb][j] = ldg128(wr + woff[nb][j] + k0 + h * 64);
                    }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int h = 0; h < LPB; ++h) {
                    bf16x8 fa[2][2];
#pragma unroll
                    for (int tb = 0; tb < 2; ++tb) {
                        if (tb == 1 && !two) break;
#pragma unroll
                        for (int j = 0; j < 2; ++j) area[tb * 128 + wslot[j]] = rx[h][tb][j];
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) fa[tb][ks] = as_bf16x8(area[tb * 128 + rslot[ks]]);
                    }
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        u32x4 *ar = area + (nb & 1) * 128;
#pragma unroll
                        for (int j = 0; j < 2; ++j) ar[wslot[j]] = rw[h][nb][j];
#pragma unroll
                        for (int ks = 0; ks < 2; ++ks) {
                            const bf16x8 b = as_bf16x8(ar[rslot[ks]]);
                            acc[0][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[0][ks], b, acc[0][nb], 0, 0, 0);
                            if (two)
                                acc[1][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[1][ks], b, acc[1][nb], 0, 0, 0);
                        }
                    }
                }
            }
        }
        for (int bt = wave; !staged && bt < nbatch; bt += NW) {
            const int k0 = bt * U * 32;
            u32x4 ra[2][U], rb[NB][U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                ra[0][u] = ldg128(xa[0] + k0 + u * 32);
                if (two) ra[1][u] = ldg128(xa[1] + k0 + u * 32);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) rb[nb][u] = ldg128(wb[nb] + k0 + u * 32);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    acc[0][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ra[0][u]), as_bf16x8(rb[nb][u]), acc[0][nb], 0, 0, 0);
                    if (two)
                        acc[1][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ra[1][u]), as_bf16x8(rb[nb][u]), acc[1][nb], 0, 0, 0);
                }
        }
        for (int ks = ks_done + wave; ks < ksteps; ks += NW) {          // k-steps past the last full batch
            const bf16x8 a0 = as_bf16x8(ldg128(xa[0] + ks * 32)), a1 = as_bf16x8(ldg128(xa[1] + ks * 32));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const bf16x8 b = as_bf16x8(ldg128(wb[nb] + ks * 32));
                acc[0][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b, acc[0][nb], 0, 0, 0);
                acc[1][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b, acc[1][nb], 0, 0, 0);
            }
        }

        // D[i][j] of a 16x16 block: lane holds column j = l % 16 and rows i = 4 * (l / 16) + v.
        // NS partial tiles sit side by side in LDS; wave w adds into slot w % NS in round w / NS,
        // then the slots are added in slot order: one fixed association, reproducible.
        for (int r = 0; r < (NW + NS - 1) / NS; ++r) {
            if (wave / NS == r) {
                float *mine = part + (wave % NS) * TILE;
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            float *q = &mine[(tb * 16 + 4 * kq + v) * STRIDE + nb * 16 + r16];
                            *q = (r == 0 ? 0.0f : *q) + acc[tb][nb][v];
                        }
            }
            __syncthreads();
        }
        for (int idx = tid; idx < TILE_T * NB * 16; idx += NW * 64) {
            const int i = idx / (NB * 16), e = idx - i * (NB * 16);
            float sum = (p.bias != nullptr && e < p.E) ? p.bias[e] : 0.0f;
#pragma unroll
            for (int w = 0; w < NS; ++w) sum += part[w * TILE + i * STRIDE + e];
            part[i * STRIDE + e] = sum;                // slot 0 becomes the logit tile (own element only)
        }
        __syncthreads();
        tile_epilogue<(NB + 3) / 4>(p, part, STRIDE, TILE, s, tile);
        if (FUSED) {
            __syncthreads();
            const int n = min(p.tile_tokens, p.T - t0) * p.K;
            for (int idx = tid; idx < n; idx += NW * 64) fs.ids[tile][idx] = s.ids[idx];
            for (int e = tid; e < p.E; e += NW * 64) fs.counts[tile][e] = s.counts[e];
            if (tid < 3) { fs.stats[tile][tid] = s.stats[tid]; fs.dist[tid] = s.dist[tid]; }
            __syncthreads();
        }
    }
    if (FUSED) fused_tail(p, fs, n_tiles);
    // a batch of one tile: this workgroup holds every substituted id and the histogram, and finishes the
    // grouping itself instead of leaving it to a launch of its own
    if (!FUSED && p.tail) {
        __syncthreads();
        finish_groups(p.scan, p.scat, s.ids, p.T * p.K, s.counts, fs.start, fs.tstart, s.stats);
    }
}

// ---------------------------------------------------------------------------
// fp32 front kernel: every (token, expert) logit is a lane-strided fp32 FMA
// dot product reduced over the wave.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) front_f32_kernel(FrontParams p) {
    constexpr int STRIDE = BM_MAX_E + 1;
    __shared__ float logits[TILE_T * STRIDE];
    __shared__ FrontLds s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    const int tile = blockIdx.x, t0 = tile * TILE_T;
    const int ntok = min(TILE_T, p.T - t0);
    const float *x = static_cast<const float *>(p.x);
    const float *wr = static_cast<const float *>(p.wr);
    for (int pair = wave; pair < ntok * p.E; pair += nw) {
        const int i = pair / p.E, e = pair - i * p.E;
        const float *xr = x + (size_t)(t0 + i) * p.d, *wrow = wr + (size_t)e * p.d;
        float acc = 0.0f;
        for (int j = lane; j < p.d; j += WAVE) acc = fmaf(xr[j], wrow[j], acc);
        acc = wave_sum(acc);
        if (lane == 0) logits[i * STRIDE + e] = acc + (p.bias ? p.bias[e] : 0.0f);
    }
    __syncthreads();
    tile_epilogue<4>(p, logits, STRIDE, TILE_T * STRIDE, s, tile);
}

// ---------------------------------------------------------------------------
// Stand-alone substitution kernel: one lane per token, bitmap and table in LDS.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) remap_kernel(RemapParams p) {
    extern __shared__ int32_t s_table[];
    __shared__ uint64_t s_bitmap[4];
    __shared__ unsigned long long s_req[4];
    __shared__ int32_t s_stats[3];
    const int tid = threadIdx.x;
    const int ec = (p.E + 63) >> 6;
    for (int idx = tid; idx < p.E * p.R; idx += blockDim.x) s_table[idx] = p.table[idx];
    if (tid < 4) { s_bitmap[tid] = (tid < ec) ? p.bitmap[tid] : 0ull; s_req[tid] = 0ull; }
    if (tid < 3) s_stats[tid] = 0;
    __syncthreads();
    int H = p.H;
    if (p.flags & BM_GATE_DIST) {
        // Eq. 2 over the whole batch, recomputed by every workgroup (no scratch memory, no grid-wide wait)
        const size_t n = (size_t)p.T * p.K;
        unsigned long long mine[4] = {0ull, 0ull, 0ull, 0ull};
        for (size_t a = tid; a < n; a += blockDim.x) {
            const int e = p.ids_in[a];
            if ((unsigned)e < (unsigned)p.E) {
                const unsigned long long bit = 1ull << (e & 63);
                const int wi = e >> 6;
                mine[0] |= wi == 0 ? bit : 0ull; mine[1] |= wi == 1 ? bit : 0ull;
                mine[2] |= wi == 2 ? bit : 0ull; mine[3] |= wi == 3 ? bit : 0ull;
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) if (mine[i]) atomicOr(&s_req[i], mine[i]);
        __syncthreads();
        int n_req = 0, n_cpu = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            n_req += __popcll(s_req[i]);
            n_cpu += __popcll(s_req[i] & ~s_bitmap[i]);
        }
        const bool bypass = dist_bypass(n_req, n_cpu, p.beta);
        if (bypass) H = 0;
        if (p.stats != nullptr && blockIdx.x == 0 && tid == 0) {
            p.stats[3] = n_req; p.stats[4] = n_cpu; p.stats[5] = bypass ? 1 : 0;
        }
    }
    int n_miss = 0, n_sub = 0, n_drop = 0;
    for (int t = blockIdx.x * blockDim.x + tid; t < p.T; t += gridDim.x * blockDim.x) {
        const int32_t *in = p.ids_in + (size_t)t * p.K;
        int32_t *out = p.ids_out + (size_t)t * p.K;
        float *w = p.w ? p.w + (size_t)t * p.K : nullptr;
        PsiSource psi{};
        if (p.flags & BM_PSI_TOKEN) { psi.q = p.q; psi.eta = p.eta; psi.probs = p.probs + (size_t)t * p.E; }
        remap_token(p.K, p.E, p.R, H, p.flags, p.tau, p.gamma, p.rho, s_bitmap, s_table, in, out, w, n_miss,
                    n_sub, n_drop, psi);
    }
    if (n_miss) atomicAdd(&s_stats[0], n_miss);
    if (n_sub) atomicAdd(&s_stats[1], n_sub);
    if (n_drop) atomicAdd(&s_stats[2], n_drop);
    __syncthreads();
    if (p.stats != nullptr && tid < 3 && s_stats[tid]) atomicAdd(&p.stats[tid], s_stats[tid]);
}

__global__ void zero_ints_kernel(int32_t *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// Per-tile histogram of given ids (stand-alone grouping entry point).
__global__ void __launch_bounds__(256) count_kernel(const int32_t *ids, int T, int K, int E, int tile_tokens,
                                                    int32_t *tile_counts) {
    __shared__ int32_t counts[BM_MAX_E];
    const int tid = threadIdx.x, tile = blockIdx.x, t0 = tile * tile_tokens;
    const int n = min(tile_tokens, T - t0) * K;
    for (int e = tid; e < E; e += blockDim.x) counts[e] = 0;
    __syncthreads();
    for (int idx = tid; idx < n; idx += blockDim.x) {
        const int e = ids[(size_t)t0 * K + idx];
        if ((unsigned)e < (unsigned)E) atomicAdd(&counts[e], 1);
    }
    __syncthreads();
    const int n_tiles_all = (T + tile_tokens - 1) / tile_tokens;
    for (int e = tid; e < E; e += blockDim.x) tile_counts[(size_t)e * n_tiles_all + tile] = counts[e];
}

// ---------------------------------------------------------------------------
// One-workgroup scan: tile histograms -> per-tile bases (relative to the
// group start), group offsets (routed experts, then shared experts with T
// rows each), the row-tile table of the grouped GEMMs, and the summed
// substitution statistics.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(1024) scan_kernel(ScanParams p) {
    __shared__ int32_t total[BM_MAX_E + 8];
    __shared__ int32_t start[BM_MAX_E + 9];
    __shared__ int32_t tstart[BM_MAX_E + 9];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    const int G = p.E + p.n_shared;
    // per expert: exclusive scan of its counts over the tiles, 64 tiles per wave step.  A wave takes EB
    // experts at a time and issues the loads of SB steps of each together: every load is a round trip
    // to memory, the scans between them are short.
    constexpr int SB = 4, EB = 4;
    for (int e0 = wave; e0 < p.E; e0 += nw * EB) {          // experts e0, e0 + nw, ..: few experts spread over the waves
        int run[EB];
#pragma unroll
        for (int j = 0; j < EB; ++j) run[j] = 0;
        for (int tb = 0; tb < p.n_tiles; tb += SB * WAVE) {
            int c[EB][SB];
#pragma unroll
            for (int j = 0; j < EB; ++j)
#pragma unroll
                for (int i = 0; i < SB; ++i) {
                    const int t = tb + i * WAVE + lane;
                    c[j][i] = (e0 + j * nw < p.E && t < p.n_tiles) ? p.tile_counts[(size_t)(e0 + j * nw) * p.n_tiles + t] : 0;
                }
#pragma unroll
            for (int j = 0; j < EB; ++j)
#pragma unroll
                for (int i = 0; i < SB; ++i) {
                    if (tb + i * WAVE >= p.n_tiles || e0 + j * nw >= p.E) continue;   // uniform over the wave
                    const int t = tb + i * WAVE + lane;
                    int tot;
                    const int ex = wave_excl_scan(c[j][i], tot);
                    if (e0 + j * nw < p.E && t < p.n_tiles) p.tile_base[(size_t)(e0 + j * nw) * p.n_tiles + t] = run[j] + ex;
                    run[j] += tot;
                }
        }
#pragma unroll
        for (int j = 0; j < EB; ++j)
            if (lane == 0 && e0 + j * nw < p.E) total[e0 + j * nw] = run[j];
    }
    for (int g = p.E + tid; g < G; g += blockDim.x) total[g] = p.T;
    __syncthreads();
    if (wave == 0) {                               // exclusive scans over the groups, a few consecutive groups per lane
        constexpr int PER = (BM_MAX_E + 8 + 63) / 64;
        int cnt[PER], nt[PER], sum_c = 0, sum_t = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int g = lane * PER + i;
            const int c = g < G ? total[g] : 0;
            cnt[i] = c;
            nt[i] = (c + p.BM - 1) / p.BM;
            sum_c += c;
            sum_t += nt[i];
        }
        int tot_c, tot_t;
        int run_c = wave_excl_scan(sum_c, tot_c), run_t = wave_excl_scan(sum_t, tot_t);
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int g = lane * PER + i;
            if (g <= G) { start[g] = run_c; tstart[g] = run_t; }
            run_c += cnt[i];
            run_t += nt[i];
        }
        if (lane == 0) { p.n_mtiles[0] = tot_t; p.n_mtiles[1] = tot_c; }
    }
    __syncthreads();
    for (int g = tid; g <= G; g += blockDim.x) p.offsets[g] = start[g];
    for (int g = tid; g < G; g += blockDim.x) {
        const int nt = tstart[g + 1] - tstart[g];
        for (int i = 0; i < nt; ++i) {
            p.mt_group[tstart[g] + i] = g;
            p.mt_row0[tstart[g] + i] = start[g] + i * p.BM;
        }
    }
    write_mixed_tile_tables(p, start);
    if (p.stats != nullptr && wave < 3) {          // one wave per counter, lanes over the tiles
        int sum = 0;
        if (p.tile_stats != nullptr)
            for (int t = lane; t < p.n_tiles; t += WAVE) sum += p.tile_stats[t * 4 + wave];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, WAVE);
        if (lane == 0) { p.stats[wave] = sum; p.stats[3 + wave] = 0; }
    }
}

// ---------------------------------------------------------------------------
// Scatter: position of assignment a = offsets[e] + base of its tile + number
// of earlier assignments of the tile with the same expert.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) scatter_kernel(ScatterParams p) {
    __shared__ int32_t s_ids[TILE_T * BM_MAX_K];
    const int tid = threadIdx.x, tile = blockIdx.x, t0 = tile * p.tile_tokens;
    const int n_tiles_all = (p.T + p.tile_tokens - 1) / p.tile_tokens;
    const int K = p.K, E = p.E;
    const int ntok = min(p.tile_tokens, p.T - t0);
    const int n = ntok * K;
    for (int idx = tid; idx < n; idx += blockDim.x) {
        const int e = p.ids[(size_t)t0 * K + idx];
        s_ids[idx] = ((unsigned)e < (unsigned)E) ? e : -1;
    }
    __syncthreads();
    const int live = p.offsets[E];
    for (int idx = tid; idx < n; idx += blockDim.x) {
        const int e = s_ids[idx];
        const int a = t0 * K + idx;
        int pos = -1;
        if (e >= 0) {
            int rank = 0;
            for (int j = 0; j < idx; ++j) rank += (s_ids[j] == e) ? 1 : 0;
            pos = p.offsets[e] + p.tile_base[(size_t)e * n_tiles_all + tile] + rank;
            p.perm[pos] = a;
            if (p.row_token) p.row_token[pos] = a / K;
        }
        p.inv_perm[a] = pos;
    }
    // positions past the live count hold -1
    for (int idx = tid; idx < p.tile_tokens * K; idx += blockDim.x) {
        const int pos = t0 * K + idx;
        if (pos >= live && pos < p.T * K) p.perm[pos] = -1;
    }
    // rows of the shared experts map to their own token
    if (p.row_token)
        for (int sidx = 0; sidx < p.n_shared; ++sidx) {
            const int base = p.offsets[E + sidx];
            for (int i = tid; i < ntok; i += blockDim.x) p.row_token[base + t0 + i] = t0 + i;
        }
}

// ---------------------------------------------------------------------------
// Scan and scatter in one launch for batches whose histogram (experts x tiles)
// is small enough for every workgroup to sum it by itself: the workgroup of a
// tile adds up, per expert, all tiles (group size) and the tiles before its
// own (its base inside the group) - a wave per expert, lanes over the tiles,
// the loads of EB experts going out together - scans the group sizes, and
// places its assignments.  The workgroup of tile 0 also writes the offsets,
// the row-tile table and the statistics.  Saves the one-workgroup scan launch,
// a chain of dependent round trips to memory (11 us for 64-128 experts).
// ---------------------------------------------------------------------------
constexpr long long TILE_SUM_MAX = 32768;          // histogram entries every workgroup re-reads (128 KB)

__global__ void __launch_bounds__(1024) group_tiles_kernel(ScanParams p, ScatterParams c) {
    __shared__ int32_t total[BM_MAX_E + 8];
    __shared__ int32_t before[BM_MAX_E];
    __shared__ int32_t start[BM_MAX_E + 9];
    __shared__ int32_t tstart[BM_MAX_E + 9];
    __shared__ int32_t s_ids[TILE_T * BM_MAX_K];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    const int tile = blockIdx.x, t0 = tile * c.tile_tokens;
    const int K = c.K, E = p.E, G = p.E + p.n_shared;
    const int ntok = min(c.tile_tokens, c.T - t0);
    const int n = ntok * K;
    for (int idx = tid; idx < n; idx += blockDim.x) {
        const int e = c.ids[(size_t)t0 * K + idx];
        s_ids[idx] = ((unsigned)e < (unsigned)E) ? e : -1;
    }
    constexpr int EB = 8, SB = 4;                         // every load is a round trip to memory: EB * SB go out together
    for (int e0 = wave; e0 < E; e0 += nw * EB) {          // experts e0, e0 + nw, ..
        int tot[EB], bef[EB];
#pragma unroll
        for (int j = 0; j < EB; ++j) tot[j] = bef[j] = 0;
        for (int tb = 0; tb < p.n_tiles; tb += SB * WAVE) {
            int cnt[EB][SB];
#pragma unroll
            for (int j = 0; j < EB; ++j)
#pragma unroll
                for (int i = 0; i < SB; ++i) {
                    const int t = tb + i * WAVE + lane;
                    cnt[j][i] = (e0 + j * nw < E && t < p.n_tiles) ? p.tile_counts[(size_t)(e0 + j * nw) * p.n_tiles + t] : 0;
                }
#pragma unroll
            for (int j = 0; j < EB; ++j)
#pragma unroll
                for (int i = 0; i < SB; ++i) {
                    tot[j] += cnt[j][i];
                    bef[j] += tb + i * WAVE + lane < tile ? cnt[j][i] : 0;
                }
        }
#pragma unroll
        for (int j = 0; j < EB; ++j) {
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) {
                tot[j] += __shfl_xor(tot[j], m, WAVE);
                bef[j] += __shfl_xor(bef[j], m, WAVE);
            }
            if (lane == 0 && e0 + j * nw < E) { total[e0 + j * nw] = tot[j]; before[e0 + j * nw] = bef[j]; }
        }
    }
    for (int g = E + tid; g < G; g += blockDim.x) total[g] = p.T;
    __syncthreads();
    if (wave == 0) {                               // exclusive scans over the groups, a few consecutive groups per lane
        constexpr int PER = (BM_MAX_E + 8 + 63) / 64;
        int cnt[PER], nt[PER], sum_c = 0, sum_t = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int g = lane * PER + i;
            const int cg = g < G ? total[g] : 0;
            cnt[i] = cg;
            nt[i] = (cg + p.BM - 1) / p.BM;
            sum_c += cg;
            sum_t += nt[i];
        }
        int tot_c, tot_t;
        int run_c = wave_excl_scan(sum_c, tot_c), run_t = wave_excl_scan(sum_t, tot_t);
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int g = lane * PER + i;
            if (g <= G) { start[g] = run_c; tstart[g] = run_t; }
            run_c += cnt[i];
            run_t += nt[i];
        }
        if (tile == 0 && lane == 0) { p.n_mtiles[0] = tot_t; p.n_mtiles[1] = tot_c; }
    }
    __syncthreads();
    if (tile == 0) {
        write_group_tables(p, start, tstart);
        write_mixed_tile_tables(p, start);
        if (p.stats != nullptr && wave >= nw - 3) {    // one wave per counter, lanes over the tiles
            const int k = wave - (nw - 3);
            int sum = 0;
            if (p.tile_stats != nullptr)
                for (int t = lane; t < p.n_tiles; t += WAVE) sum += p.tile_stats[t * 4 + k];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, WAVE);
            if (lane == 0) { p.stats[k] = sum; p.stats[3 + k] = 0; }
        }
    }
    // placement: group start + the tile's base inside the group + earlier assignments of the tile with the same expert
    const int live = start[E];
    for (int idx = tid; idx < n; idx += blockDim.x) {
        const int e = s_ids[idx];
        const int a = t0 * K + idx;
        int pos = -1;
        if (e >= 0) {
            int rank = 0;
            for (int j = 0; j < idx; ++j) rank += (s_ids[j] == e) ? 1 : 0;
            pos = start[e] + before[e] + rank;
            c.perm[pos] = a;
            if (c.row_token) c.row_token[pos] = a / K;
        }
        c.inv_perm[a] = pos;
    }
    for (int idx = tid; idx < c.tile_tokens * K; idx += blockDim.x) {      // positions past the live count hold -1
        const int pos = t0 * K + idx;
        if (pos >= live && pos < c.T * K) c.perm[pos] = -1;
    }
    if (c.row_token)                                                         // rows of the shared experts map to their own token
        for (int sidx = 0; sidx < c.n_shared; ++sidx)
            for (int i = tid; i < ntok; i += blockDim.x) c.row_token[start[E + sidx] + t0 + i] = t0 + i;
}

// ---------------------------------------------------------------------------
// Scan and scatter in one workgroup for small batches (at most SMALL_A
// assignments): the substituted ids are staged in LDS, every expert's count
// and the stable positions come from ballots over them (place_assignments).
// Writes what scan_kernel and scatter_kernel write, except the per-tile bases.
// ---------------------------------------------------------------------------
constexpr int SMALL_A = 1024;

__global__ void __launch_bounds__(1024) group_small_kernel(ScanParams p, ScatterParams c) {
    __shared__ int32_t ids[SMALL_A];
    __shared__ int32_t total[BM_MAX_E + 8];
    __shared__ int32_t start[BM_MAX_E + 9];
    __shared__ int32_t tstart[BM_MAX_E + 9];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    const int E = p.E, A = c.T * c.K;
    for (int a = tid; a < A; a += blockDim.x) {
        const int e = c.ids[a];
        ids[a] = ((unsigned)e < (unsigned)E) ? e : -1;
    }
    __syncthreads();
    for (int e = wave; e < E; e += nw) {
        int cnt = 0;
        for (int base = 0; base < A; base += WAVE) {
            const int a = base + lane;
            cnt += __popcll(__ballot(a < A && ids[a] == e));
        }
        if (lane == 0) total[e] = cnt;
    }
    __syncthreads();
    finish_groups(p, c, ids, A, total, start, tstart, nullptr);
}

// ---------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------
template <int NB, int NW, int U>
static void launch_front_bf16(const FrontParams &p, int n_tiles, hipStream_t st) {
    if (p.fused) hipLaunchKernelGGL((front_bf16_kernel<NB, NW, U, true>), dim3(1), dim3(NW * 64), 0, st, p);
    else hipLaunchKernelGGL((front_bf16_kernel<NB, NW, U, false>), dim3(n_tiles), dim3(NW * 64), 0, st, p);
}

// One workgroup for the whole front end (router to placement): only with the distribution gate and a
// batch of at most one tile - the gate's in-tile form needs the whole batch in one workgroup and saves two
// launches.  Otherwise workgroups of 16 tokens plus the grouping kernel are faster at every batch size
// (front end at 1 / 8 / 16 tokens: 13.8 / 13.6 / 14.2 us against 15.0 / 16.0 / 17.7 us); a batch of one such
// workgroup finishes the grouping itself (FrontParams::tail).
bool front_can_fuse(int T, int dtype, uint32_t flags) {
    return dtype == BM_BF16 && (flags & BM_GATE_DIST) && T > 0 && T <= TILE_T;
}

// Tokens per workgroup of the bf16 front kernel (and per tile of the histograms that the scan and scatter
// kernels work on).  A tile's router product is bound by the number of cache lines its loads touch, so
// as long as 32-token tiles would not give every compute unit a workgroup, the batch is cut into 16-token
// tiles on twice the units (measured at 64 tokens: front kernel 12 us instead of 18).
int front_tile_tokens(int T, int dtype, bool fused) {
    return (dtype == BM_BF16 && !fused && (T + TILE_T - 1) / TILE_T < 256) ? 16 : TILE_T;
}

int launch_front(const FrontParams &p, int dtype, hipStream_t st) {
    const int n_tiles = (p.T + p.tile_tokens - 1) / p.tile_tokens;
    if (n_tiles == 0) return 0;
    if (dtype == BM_F32) {
        hipLaunchKernelGGL(front_f32_kernel, dim3(n_tiles), dim3(256), 0, st, p);
    } else {
        const int nb = (p.E + 15) / 16;
        // a tile is latency-bound: 16 waves split the product and rank two tokens each; U keeps a batch
        // of loads ((2 + NB) * U registers quadruples) inside the 128 registers a wave of 16 has
        if (nb <= 1) launch_front_bf16<1, 16, 4>(p, n_tiles, st);
        else if (nb <= 2) launch_front_bf16<2, 16, 4>(p, n_tiles, st);
        else if (nb <= 4) launch_front_bf16<4, 16, 2>(p, n_tiles, st);
        else if (nb <= 8) launch_front_bf16<8, 8, 2>(p, n_tiles, st);
        else launch_front_bf16<16, 8, 1>(p, n_tiles, st);
    }
    return launch_status(__func__);
}

int launch_remap(const RemapParams &p, hipStream_t st) {
    if (p.stats) hipLaunchKernelGGL(zero_ints_kernel, dim3(1), dim3(64), 0, st, p.stats, 6);
    if (p.T > 0) {
        const size_t lds = (size_t)p.E * p.R * sizeof(int32_t);
        int blocks = (p.T + 255) / 256;
        if (p.flags & BM_GATE_DIST) {
            // every workgroup reads all ids for the request set: bound their number; in place, a single
            // workgroup reads the set before it overwrites anything
            blocks = p.ids_out == p.ids_in ? 1 : (blocks > 256 ? 256 : blocks);
        }
        hipLaunchKernelGGL(remap_kernel, dim3(blocks), dim3(256), lds, st, p);
    }
    return launch_status(__func__);
}

int launch_count(const int32_t *ids, int T, int K, int E, int tile_tokens, int32_t *tile_counts, hipStream_t st) {
    const int n_tiles = (T + tile_tokens - 1) / tile_tokens;
    if (n_tiles) hipLaunchKernelGGL(count_kernel, dim3(n_tiles), dim3(256), 0, st, ids, T, K, E, tile_tokens, tile_counts);
    return launch_status(__func__);
}

int launch_scan(const ScanParams &p, hipStream_t st) {
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, st, p);
    return launch_status(__func__);
}

// The one-workgroup kernel walks every assignment once per expert (a wave per expert, 64 assignments a
// step): fine for a few experts, slow for many (128 experts x 1024 assignments: 25 us against 12 us for the
// per-tile kernel).
bool grouping_small(long long assignments, int E) { return assignments <= SMALL_A && assignments * E <= 32768; }

// scan + scatter: one kernel for small batches and for small histograms
int launch_grouping(const ScanParams &sp, const ScatterParams &cp, hipStream_t st) {
    if (grouping_small((long long)cp.T * cp.K, cp.E)) {
        hipLaunchKernelGGL(group_small_kernel, dim3(1), dim3(1024), 0, st, sp, cp);   // also for an empty batch: offsets
        return launch_status(__func__);
    }
    const int n_tiles = (cp.T + cp.tile_tokens - 1) / cp.tile_tokens;
    if ((long long)sp.E * n_tiles <= TILE_SUM_MAX) {
        hipLaunchKernelGGL(group_tiles_kernel, dim3(n_tiles), dim3(1024), 0, st, sp, cp);
        return launch_status(__func__);
    }
    const int rc = launch_scan(sp, st);
    return rc | launch_scatter(cp, st);
}

int launch_scatter(const ScatterParams &p, hipStream_t st) {
    const int n_tiles = (p.T + p.tile_tokens - 1) / p.tile_tokens;
    if (n_tiles) hipLaunchKernelGGL(scatter_kernel, dim3(n_tiles), dim3(256), 0, st, p);
    return launch_status(__func__);
}

}  // namespace bm
