// CPU oracle for one MoE layer's forward pass with buddy-expert substitution.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
// tests, the smoke check and the benchmark's cpu_baseline leg compare the HIP
// library against.  It shares no code with the HIP library and the product
// path never calls it.
//
// Precision: inputs are fp32 arrays (bf16 workloads are widened exactly
// before they get here); every sum, exponential and product is evaluated in
// fp64; outputs are fp64.  The one place floating point decides an integer is
// the top-k selection: logits are rounded to fp32 first, because fp32 is the
// precision the device kernel holds its logits in.
//
// Parity pins (tests/test_oracle_*.py): routing against a library argsort and
// softmax; the substitution against hand-worked cases of Algorithm 1, an
// independent per-slot checker and the per-expert lookup-table form; the
// permutation against a library stable sort; the layer output against a
// brute-force dense evaluation of every expert masked by the gate matrix;
// TAE against closed forms.  Unpinned by the paper: the error of the
// substituted layer against the unsubstituted one (no bound is given).
//
// Plain loops, one per definition, with no blocking, fusion or reordering.
// OpenMP splits the token loop only (tokens are independent).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

extern "C" {

// Section 3 "Notation and Preliminaries": router logits z(x) in R^E.
//   z[t][e] = bias[e] + sum_j x[t][j] * w_router[e][j]
// x [T][d], w_router [E][d], bias [E] or NULL, z [T][E].
int bm_oracle_router_logits(int T, int d, int E, const float* x, const float* w_router,
                            const float* bias, double* z) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int e = 0; e < E; ++e) {
            double acc = bias ? (double)bias[e] : 0.0;
            for (int j = 0; j < d; ++j) acc += (double)x[(size_t)t * d + j] * (double)w_router[(size_t)e * d + j];
            z[(size_t)t * E + e] = acc;
        }
    }
    return 0;
}

// Section 3 "Notation and Preliminaries": p = softmax(z); S(x) = the k experts
// of largest probability; p-tilde = p renormalised over S(x).
// Slot 0 holds the largest logit; equal logits go to the lower expert index.
// renorm != 0: w = p-tilde (sums to 1 over the K slots); renorm == 0: w = p.
// ids [T][K], w [T][K].
int bm_oracle_topk_gates(int T, int E, int K, int renorm, const double* z, int32_t* ids, double* w) {
    if (K > E) return -1;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        const double* zt = z + (size_t)t * E;
        std::vector<float> z32(E);
        std::vector<char> taken(E, 0);
        for (int e = 0; e < E; ++e) z32[e] = (float)zt[e];
        double zmax = zt[0];
        for (int e = 1; e < E; ++e) if (zt[e] > zmax) zmax = zt[e];
        double sum_all = 0.0;
        for (int e = 0; e < E; ++e) sum_all += std::exp(zt[e] - zmax);
        double sum_sel = 0.0;
        for (int k = 0; k < K; ++k) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || z32[e] > z32[best]) best = e;   // strict '>' keeps the lowest index on ties
            }
            taken[best] = 1;
            ids[(size_t)t * K + k] = best;
            double p = std::exp(zt[best] - zmax);
            w[(size_t)t * K + k] = p;
            sum_sel += p;
        }
        double denom = renorm ? sum_sel : sum_all;
        for (int k = 0; k < K; ++k) w[(size_t)t * K + k] /= denom;
    }
    return 0;
}

// Section 3.1 Eq. 1: Token Activating Entropy of the renormalised top-k gates,
//   TAE = -( sum_{i in S} p~_i log p~_i ) / log k,  in [0,1].
// w [T][K] must be p-tilde (sum to 1 per token).  For K == 1 the entropy and
// its normaliser are both 0; the value is defined as 0 here.
int bm_oracle_tae(int T, int K, const double* w, double* tae) {
    for (int t = 0; t < T; ++t) {
        double h = 0.0;
        for (int k = 0; k < K; ++k) {
            double p = w[(size_t)t * K + k];
            if (p > 0.0) h -= p * std::log(p);
        }
        tae[t] = (K > 1) ? h / std::log((double)K) : 0.0;
    }
    return 0;
}

// Section 4, Algorithm 1 (BuddySubstitute): per token, walk the K slots in
// order; a selected expert that is not resident is replaced by the first
// entry b of its buddy row, among ranks 1..H, that is resident and (unique
// mode) not yet in the token's set U_t; U_t starts as the token's K selected
// experts and grows by every accepted buddy.
//
// Readings where the algorithm is silent:
//  * unique == 0 drops the "b not in U_t" test: the substitute is the first
//    resident entry of the row, whatever the token already holds.
//  * a table entry outside [0,E) (the -1 padding of short rows) is never
//    resident; the scan continues past it.
//  * no acceptable buddy among the first H entries: the slot is dropped
//    (Section 3.1, the fallback that skips the expert): id -1, gate weight 0,
//    the other slots' weights are left as they are.
//  * a substitute inherits the gate weight of the slot it fills.
// resident [E] (0/1 bytes), table [E][R], ids_in/ids_out [T][K] (may alias),
// w [T][K] in/out (nullable), stats[3] = {misses, substituted, dropped}.
int bm_oracle_buddy_remap(int T, int K, int E, int R, int H, int unique, const uint8_t* resident,
                          const int32_t* table, const int32_t* ids_in, int32_t* ids_out, double* w,
                          int64_t* stats);   // defined after the general form below, which it reduces to

// Section 3.1 Eq. 2, Expert Distribution Gate: over the micro-batch (here: the
// T tokens of the call) R(B) = the set of distinct experts some token selected;
//   delta = |{i in R(B) : i not resident}| / |R(B)|.
// counts[0] = |R(B)|, counts[1] = the numerator.  Returns delta (0 for an empty
// batch).  Ids outside [0,E) request nothing.
double bm_oracle_distribution_delta(int T, int K, int E, const uint8_t* resident, const int32_t* ids,
                                    int64_t* counts) {
    std::vector<char> requested(E, 0);
    for (size_t a = 0; a < (size_t)T * K; ++a)
        if (ids[a] >= 0 && ids[a] < E) requested[ids[a]] = 1;
    int64_t n_req = 0, n_cpu = 0;
    for (int e = 0; e < E; ++e) {
        if (!requested[e]) continue;
        ++n_req;
        if (!resident[e]) ++n_cpu;
    }
    if (counts) { counts[0] = n_req; counts[1] = n_cpu; }
    return n_req ? (double)n_cpu / (double)n_req : 0.0;
}

// Section 3.1 (the three-stage decision: TAE gate with optional margin gate,
// distribution gate, buddy selection) and Section 5.1 (replacement budget rho)
// around Algorithm 1.
// Per token, from its gate weights renormalised over the K slots (p~):
//   TAE = -(sum p~ log p~) / log K  (Eq. 1);  m = p~_max - p~_2nd  (0 for the
//   missing second value when K == 1).
//   Replacement is forbidden for the token when (use_tae and TAE <= tau) or
//   (use_margin and m >= gamma).
// Per batch: with use_dist, replacement is bypassed for every token when
//   delta >= beta (Eq. 2).
// With use_budget, at most rho slots of a token are replaced, counted in slot
// order.
// Reading (the paper lets such a miss be fetched from host memory, which this
// layer cannot do): a miss that may not be replaced - forbidden token, bypassed
// batch, or budget used up - is dropped exactly like a miss without an
// acceptable buddy.  Everything else is bm_oracle_buddy_remap.  w [T][K] is
// required with use_tae / use_margin (read for the gates before any drop, then
// updated).  stats[6] = {misses, substituted, dropped, |R(B)|, offloaded among
// R(B), bypassed 0/1}; the last three are 0 without use_dist.
//
// Token-aware buddy priority (Section 3.1, Eq. 3, with kappa = 0): with use_psi the
// substitute is not the first acceptable entry of the row but the acceptable entry
// (same acceptance test, same first H entries) of largest
//   Psi(j|i,x) = q[j|i] * (1 + eta * zhat_j(x)),
// equal Psi going to the earlier entry.  q [E][R] holds q[j|i] of every table entry;
// zhat [T][E] is the normalised router logit of every expert for every token
// (reading: the softmax probability p_j(x) over all experts).  eta = 0 reproduces
// the table order whenever the rows are sorted by q.  margin_out [T] (nullable):
// per token the smallest relative gap (best - second) / best over its decisions
// that had at least two acceptable entries (1e300 if none) - how close the token
// came to a different choice.
// The ranks r < H of expert e's buddy row whose entry may stand in for e for this
// token (Algorithm 1's acceptance test): a valid expert id, resident, and - unique
// mode - not among the experts the token holds already.
static std::vector<int> acceptable_ranks(int e, int E, int R, int H, bool unique, const uint8_t* resident,
                                         const int32_t* table, const std::vector<char>& held) {
    std::vector<int> ranks;
    for (int r = 0; r < H; ++r) {
        const int32_t b = table[(size_t)e * R + r];
        const bool valid = b >= 0 && b < E;
        if (valid && resident[b] && !(unique && held[b])) ranks.push_back(r);
    }
    return ranks;
}

// Whether a token may be given substitutes at all (Section 3.1): Eq. 1 on its gate
// weights renormalised to sum 1, and the top-two margin.
static bool token_may_substitute(int K, const double* wt, bool use_tae, double tau, bool use_margin, double gamma) {
    if (!use_tae && !use_margin) return true;
    double sum = 0.0;
    for (int k = 0; k < K; ++k) sum += wt[k];
    double entropy = 0.0, largest = 0.0, second = 0.0;
    for (int k = 0; k < K; ++k) {
        const double pk = wt[k] / sum;
        if (pk > 0.0) entropy -= pk * std::log(pk);
        if (pk > largest) { second = largest; largest = pk; } else if (pk > second) { second = pk; }
    }
    const double tae = (K > 1) ? entropy / std::log((double)K) : 0.0;
    if (use_tae && tae <= tau) return false;
    if (use_margin && (largest - second) >= gamma) return false;
    return true;
}

int bm_oracle_buddy_remap_psi(int T, int K, int E, int R, int H, int unique, int use_tae, double tau,
                              int use_margin, double gamma, int use_budget, int rho, int use_dist,
                              double beta, int use_psi, double eta, const double* q, const double* zhat,
                              const uint8_t* resident, const int32_t* table, const int32_t* ids_in,
                              int32_t* ids_out, double* w, int64_t* stats, double* margin_out) {
    if (H > R || H < 0 || ((use_tae || use_margin) && !w) || (use_psi && (!q || !zhat))) return -1;
    int64_t n_miss = 0, n_sub = 0, n_drop = 0, dist[2] = {0, 0};
    bool bypass = false;
    if (use_dist) bypass = bm_oracle_distribution_delta(T, K, E, resident, ids_in, dist) >= beta && dist[0] > 0;
    for (int t = 0; t < T; ++t) {
        const int32_t* s_in = ids_in + (size_t)t * K;
        int32_t* s_out = ids_out + (size_t)t * K;
        double* wt = w ? w + (size_t)t * K : nullptr;
        const bool open = !bypass && (!wt || token_may_substitute(K, wt, use_tae, tau, use_margin, gamma));

        std::vector<int32_t> selected(s_in, s_in + K);       // the token's routed experts (ids_out may alias ids_in)
        std::vector<char> held(E, 0);                        // U_t: the routed experts, then every accepted buddy
        for (int32_t e : selected) if (e >= 0 && e < E) held[e] = 1;

        int replaced = 0;
        double closest = 1e300;
        for (int k = 0; k < K; ++k) {
            const int32_t e = selected[k];
            int32_t runs = e;                                // the expert that will run in this slot
            if (e < 0 || e >= E) {
                runs = -1;                                   // not a routed expert: nothing to run
            } else if (!resident[e]) {
                ++n_miss;
                runs = -1;
                std::vector<int> ranks;
                if (open && !(use_budget && replaced >= rho))
                    ranks = acceptable_ranks(e, E, R, H, unique != 0, resident, table, held);
                if (!ranks.empty()) {
                    int pick = ranks.front();                // Algorithm 1: the highest-ranked acceptable entry
                    if (use_psi) {                           // Eq. 3: the acceptable entry of largest priority
                        double best = -1.0, second = -1.0;
                        for (int r : ranks) {
                            const int32_t b = table[(size_t)e * R + r];
                            const double psi = q[(size_t)e * R + r] * (1.0 + eta * zhat[(size_t)t * E + b]);
                            if (psi > best) { second = best; best = psi; pick = r; }
                            else if (psi > second) second = psi;
                        }
                        if (ranks.size() > 1 && best > 0.0) closest = std::min(closest, (best - second) / best);
                    }
                    runs = table[(size_t)e * R + pick];
                    held[runs] = 1;
                    ++replaced;
                    ++n_sub;
                } else {
                    ++n_drop;
                }
            }
            s_out[k] = runs;
            if (runs < 0 && wt) wt[k] = 0.0;
        }
        if (margin_out) margin_out[t] = closest;
    }
    if (stats) {
        stats[0] = n_miss; stats[1] = n_sub; stats[2] = n_drop;
        stats[3] = dist[0]; stats[4] = dist[1]; stats[5] = bypass ? 1 : 0;
    }
    return 0;
}

int bm_oracle_buddy_remap(int T, int K, int E, int R, int H, int unique, const uint8_t* resident,
                          const int32_t* table, const int32_t* ids_in, int32_t* ids_out, double* w,
                          int64_t* stats) {
    int64_t all[6];
    const int rc = bm_oracle_buddy_remap_psi(T, K, E, R, H, unique, 0, 0.0, 0, 0.0, 0, 0, 0, 0.0, 0, 0.0, nullptr,
                                             nullptr, resident, table, ids_in, ids_out, w, all, nullptr);
    if (rc == 0 && stats) { stats[0] = all[0]; stats[1] = all[1]; stats[2] = all[2]; }
    return rc;
}

int bm_oracle_buddy_remap_gated(int T, int K, int E, int R, int H, int unique, int use_tae, double tau,
                                int use_margin, double gamma, int use_budget, int rho, int use_dist,
                                double beta, const uint8_t* resident, const int32_t* table,
                                const int32_t* ids_in, int32_t* ids_out, double* w, int64_t* stats) {
    return bm_oracle_buddy_remap_psi(T, K, E, R, H, unique, use_tae, tau, use_margin, gamma, use_budget, rho,
                                     use_dist, beta, 0, 0.0, nullptr, nullptr, resident, table, ids_in, ids_out,
                                     w, stats, nullptr);
}

// Section 3.2, "Empirical Evidence from Profiling": over the routed tokens,
//   A[i]    = number of tokens with i in S(x)
//   M[i][j] = number of tokens with i and j both in S(x), i != j (M[i][i] = 0)
// The counts of this batch are ADDED to A [E] and M [E][E] (int64), so a corpus
// can be fed batch by batch.  Ids outside [0,E) are ignored; an expert that a
// token lists twice counts once for that token.
int bm_oracle_coactivation(int T, int K, int E, const int32_t* ids, int64_t* A, int64_t* M) {
    for (int t = 0; t < T; ++t) {
        std::vector<char> in_s(E, 0);
        for (int k = 0; k < K; ++k) {
            int32_t e = ids[(size_t)t * K + k];
            if (e >= 0 && e < E) in_s[e] = 1;
        }
        for (int i = 0; i < E; ++i) {
            if (!in_s[i]) continue;
            A[i] += 1;
            for (int j = 0; j < E; ++j)
                if (j != i && in_s[j]) M[(size_t)i * E + j] += 1;
        }
    }
    return 0;
}

// Section 3.2 Eq. 4 and Section 3.3 Eq. 5-6: buddy lists from the co-activation
// counts.  Per pivot i:
//   q[j|i] = M[i][j] / sum_{j' != i} M[i][j'],  q[i|i] = 0           (Eq. 4)
//   pi_i   = peers by descending q (equal q: lower expert index first)
//   t_i    = min { t : sum_{r<=t} q[pi_i(r)|i] >= alpha }            (Eq. 5)
//   B(i)   = { pi_i(1..t_i) }, cut to at most k_max entries          (Eq. 6)
// A pivot with no co-activation at all (row sum 0) gets an empty list; any
// other pivot gets at least one entry.  Peers with q = 0 are never listed.
// table [E][k_max] is filled best first and padded with -1; len [E] (nullable)
// receives the list lengths; q_out [E][k_max] (nullable) the q of each entry.
// Not modelled (the paper calls them optional stabilisers): probability-
// weighted counts, Laplace smoothing, warm-up down-weighting.
int bm_oracle_build_buddy_lists(int E, int k_max, const int64_t* M, double alpha, int32_t* table,
                                int32_t* len, double* q_out) {
    for (int i = 0; i < E; ++i) {
        double total = 0.0;
        for (int j = 0; j < E; ++j) if (j != i) total += (double)M[(size_t)i * E + j];
        std::vector<double> q(E, 0.0);
        if (total > 0.0)
            for (int j = 0; j < E; ++j) if (j != i) q[j] = (double)M[(size_t)i * E + j] / total;
        std::vector<int> order;
        for (int j = 0; j < E; ++j) if (j != i && q[j] > 0.0) order.push_back(j);
        // insertion sort: descending q, equal q keep ascending index (stable)
        for (size_t a = 1; a < order.size(); ++a) {
            int x = order[a];
            size_t b = a;
            while (b > 0 && q[order[b - 1]] < q[x]) { order[b] = order[b - 1]; --b; }
            order[b] = x;
        }
        // Eq. 5 with both sides multiplied by the row sum: the prefix sum of q is a ratio of counts, and
        // "count >= alpha * total" has a single rounding (the device evaluates the same fp64 expression)
        int t_i = 0;
        int64_t cum = 0;
        for (size_t r = 0; r < order.size(); ++r) {
            cum += M[(size_t)i * E + order[r]];
            t_i = (int)r + 1;
            if ((double)cum >= alpha * total) break;
        }
        if (t_i > k_max) t_i = k_max;
        for (int r = 0; r < k_max; ++r) {
            table[(size_t)i * k_max + r] = r < t_i ? order[r] : -1;
            if (q_out) q_out[(size_t)i * k_max + r] = r < t_i ? q[order[r]] : 0.0;
        }
        if (len) len[i] = t_i;
    }
    return 0;
}

// Grouping of the surviving assignments by expert (Section 2.2: each token's
// selected experts run and their outputs are aggregated; the grouping itself
// is the execution order of this build): a stable counting sort of the flat
// assignment indices a = t*K + k with ids[a] >= 0, keyed by ids[a].
//   offsets [E+1]: offsets[e] = first position of expert e, offsets[E] = live count
//   perm [T*K]: perm[pos] = a (entries past the live count are -1)
//   inv_perm [T*K]: inv_perm[a] = pos, or -1 for a dropped assignment
int bm_oracle_permute(int T, int K, int E, const int32_t* ids, int32_t* offsets, int32_t* perm,
                      int32_t* inv_perm) {
    const int A = T * K;
    std::vector<int32_t> count(E, 0);
    for (int a = 0; a < A; ++a) if (ids[a] >= 0) ++count[ids[a]];
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + count[e];
    std::vector<int32_t> cursor(offsets, offsets + E);
    for (int a = 0; a < A; ++a) { perm[a] = -1; inv_perm[a] = -1; }
    for (int a = 0; a < A; ++a) {
        if (ids[a] < 0) continue;
        int32_t pos = cursor[ids[a]]++;
        perm[pos] = a;
        inv_perm[a] = pos;
    }
    return 0;
}

static inline double silu(double a) { return a / (1.0 + std::exp(-a)); }

// One SwiGLU expert on one token (the expert FFN of Section 2.1, in the gated
// form the workload configs name):
//   g = W_g x, u = W_u x, h = silu(g) * u, out = W_d h
// w_gate, w_up [F][d]; w_down [d][F]; x [d]; out [d].
int bm_oracle_expert_ffn(int d, int F, const float* w_gate, const float* w_up, const float* w_down,
                         const float* x, double* out) {
    std::vector<double> h(F);
    for (int f = 0; f < F; ++f) {
        double g = 0.0, u = 0.0;
        for (int j = 0; j < d; ++j) {
            g += (double)w_gate[(size_t)f * d + j] * (double)x[j];
            u += (double)w_up[(size_t)f * d + j] * (double)x[j];
        }
        h[f] = silu(g) * u;
    }
    for (int i = 0; i < d; ++i) {
        double acc = 0.0;
        for (int f = 0; f < F; ++f) acc += (double)w_down[(size_t)i * F + f] * h[f];
        out[i] = acc;
    }
    return 0;
}

// Expert execution and aggregation (Section 2.2) over rewritten ids:
//   y[t] = sum_k w[t][k] * FFN_{ids[t][k]}(x[t])   (slots with id -1 skipped)
//        + sum_{s < n_shared} FFN^shared_s(x[t])   (always on, weight 1)
// w_gate/w_up [E][F][d], w_down [E][d][F]; shared stacks likewise; y [T][d].
int bm_oracle_experts_combine(int T, int d, int E, int F, int K, int n_shared, const float* x,
                              const int32_t* ids, const double* w, const float* w_gate,
                              const float* w_up, const float* w_down, const float* ws_gate,
                              const float* ws_up, const float* ws_down, double* y) {
    const size_t fd = (size_t)F * d;
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
        std::vector<double> o(d);
        double* yt = y + (size_t)t * d;
        for (int i = 0; i < d; ++i) yt[i] = 0.0;
        for (int k = 0; k < K; ++k) {
            int32_t e = ids[(size_t)t * K + k];
            if (e < 0) continue;
            bm_oracle_expert_ffn(d, F, w_gate + e * fd, w_up + e * fd, w_down + e * fd, x + (size_t)t * d, o.data());
            double wk = w[(size_t)t * K + k];
            for (int i = 0; i < d; ++i) yt[i] += wk * o[i];
        }
        for (int s = 0; s < n_shared; ++s) {
            bm_oracle_expert_ffn(d, F, ws_gate + s * fd, ws_up + s * fd, ws_down + s * fd, x + (size_t)t * d, o.data());
            for (int i = 0; i < d; ++i) yt[i] += o[i];
        }
    }
    return 0;
}

// The whole layer: logits -> gates -> Algorithm 1 -> experts + aggregation.
// Optional outputs (any may be NULL): ids, ids_remapped [T][K], w_out [T][K]
// (after drops), stats[3].
int bm_oracle_moe_forward(int T, int d, int E, int F, int K, int n_shared, int R, int H, int renorm,
                          int unique, const float* x, const float* w_router, const float* bias,
                          const float* w_gate, const float* w_up, const float* w_down,
                          const float* ws_gate, const float* ws_up, const float* ws_down,
                          const uint8_t* resident, const int32_t* table, double* y, int32_t* ids_out,
                          int32_t* ids_remapped_out, double* w_out, int64_t* stats) {
    std::vector<double> z((size_t)T * E), w((size_t)T * K);
    std::vector<int32_t> ids((size_t)T * K), ids2((size_t)T * K);
    int rc = bm_oracle_router_logits(T, d, E, x, w_router, bias, z.data());
    if (rc) return rc;
    rc = bm_oracle_topk_gates(T, E, K, renorm, z.data(), ids.data(), w.data());
    if (rc) return rc;
    rc = bm_oracle_buddy_remap(T, K, E, R, H, unique, resident, table, ids.data(), ids2.data(), w.data(), stats);
    if (rc) return rc;
    rc = bm_oracle_experts_combine(T, d, E, F, K, n_shared, x, ids2.data(), w.data(), w_gate, w_up, w_down,
                                   ws_gate, ws_up, ws_down, y);
    if (rc) return rc;
    if (ids_out) std::memcpy(ids_out, ids.data(), sizeof(int32_t) * ids.size());
    if (ids_remapped_out) std::memcpy(ids_remapped_out, ids2.data(), sizeof(int32_t) * ids2.size());
    if (w_out) std::memcpy(w_out, w.data(), sizeof(double) * w.size());
    return 0;
}

// The whole layer with the gates of Section 3.1 / budget of Section 5.1 in front of Algorithm 1
// (stats[6] as in bm_oracle_buddy_remap_gated).
int bm_oracle_moe_forward_gated(int T, int d, int E, int F, int K, int n_shared, int R, int H, int renorm,
                                int unique, int use_tae, double tau, int use_margin, double gamma,
                                int use_budget, int rho, int use_dist, double beta, const float* x,
                                const float* w_router,
                                const float* bias, const float* w_gate, const float* w_up,
                                const float* w_down, const float* ws_gate, const float* ws_up,
                                const float* ws_down, const uint8_t* resident, const int32_t* table,
                                double* y, int32_t* ids_out, int32_t* ids_remapped_out, double* w_out,
                                int64_t* stats) {
    std::vector<double> z((size_t)T * E), w((size_t)T * K);
    std::vector<int32_t> ids((size_t)T * K), ids2((size_t)T * K);
    int rc = bm_oracle_router_logits(T, d, E, x, w_router, bias, z.data());
    if (rc) return rc;
    rc = bm_oracle_topk_gates(T, E, K, renorm, z.data(), ids.data(), w.data());
    if (rc) return rc;
    rc = bm_oracle_buddy_remap_gated(T, K, E, R, H, unique, use_tae, tau, use_margin, gamma, use_budget, rho,
                                     use_dist, beta, resident, table, ids.data(), ids2.data(), w.data(), stats);
    if (rc) return rc;
    rc = bm_oracle_experts_combine(T, d, E, F, K, n_shared, x, ids2.data(), w.data(), w_gate, w_up, w_down,
                                   ws_gate, ws_up, ws_down, y);
    if (rc) return rc;
    if (ids_out) std::memcpy(ids_out, ids.data(), sizeof(int32_t) * ids.size());
    if (ids_remapped_out) std::memcpy(ids_remapped_out, ids2.data(), sizeof(int32_t) * ids2.size());
    if (w_out) std::memcpy(w_out, w.data(), sizeof(double) * w.size());
    return 0;
}

// Softmax probabilities of all experts, p [T][E], from logits z [T][E] (Section 3, "Notation").
int bm_oracle_softmax(int T, int E, const double* z, double* p) {
    for (int t = 0; t < T; ++t) {
        const double* zt = z + (size_t)t * E;
        double zmax = zt[0], sum = 0.0;
        for (int e = 1; e < E; ++e) if (zt[e] > zmax) zmax = zt[e];
        for (int e = 0; e < E; ++e) sum += std::exp(zt[e] - zmax);
        for (int e = 0; e < E; ++e) p[(size_t)t * E + e] = std::exp(zt[e] - zmax) / sum;
    }
    return 0;
}

// The whole layer with token-aware buddy priority (and optionally the gates); zhat = softmax(z).
int bm_oracle_moe_forward_psi(int T, int d, int E, int F, int K, int n_shared, int R, int H, int renorm,
                              int unique, int use_tae, double tau, int use_margin, double gamma,
                              int use_budget, int rho, int use_dist, double beta, double eta, const double* q,
                              const float* x, const float* w_router, const float* bias, const float* w_gate,
                              const float* w_up, const float* w_down, const float* ws_gate, const float* ws_up,
                              const float* ws_down, const uint8_t* resident, const int32_t* table, double* y,
                              int32_t* ids_out, int32_t* ids_remapped_out, double* w_out, int64_t* stats,
                              double* margin_out) {
    std::vector<double> z((size_t)T * E), w((size_t)T * K), p((size_t)T * E);
    std::vector<int32_t> ids((size_t)T * K), ids2((size_t)T * K);
    int rc = bm_oracle_router_logits(T, d, E, x, w_router, bias, z.data());
    if (rc) return rc;
    rc = bm_oracle_topk_gates(T, E, K, renorm, z.data(), ids.data(), w.data());
    if (rc) return rc;
    bm_oracle_softmax(T, E, z.data(), p.data());
    rc = bm_oracle_buddy_remap_psi(T, K, E, R, H, unique, use_tae, tau, use_margin, gamma, use_budget, rho,
                                   use_dist, beta, 1, eta, q, p.data(), resident, table, ids.data(), ids2.data(),
                                   w.data(), stats, margin_out);
    if (rc) return rc;
    rc = bm_oracle_experts_combine(T, d, E, F, K, n_shared, x, ids2.data(), w.data(), w_gate, w_up, w_down,
                                   ws_gate, ws_up, ws_down, y);
    if (rc) return rc;
    if (ids_out) std::memcpy(ids_out, ids.data(), sizeof(int32_t) * ids.size());
    if (ids_remapped_out) std::memcpy(ids_remapped_out, ids2.data(), sizeof(int32_t) * ids2.size());
    if (w_out) std::memcpy(w_out, w.data(), sizeof(double) * w.size());
    return 0;
}

int bm_oracle_num_threads(void);

}  // extern "C"

#ifdef _OPENMP
#include <omp.h>
extern "C" int bm_oracle_num_threads(void) { return omp_get_max_threads(); }
#else
extern "C" int bm_oracle_num_threads(void) { return 1; }
#endif
