// Front end of the layer: router logits, softmax / top-k gates, buddy
// substitution (Section 4, Algorithm 1) and the stable grouping of the
// surviving assignments by expert.
//
// Tokens are processed in tiles of TILE_T = 32.  One workgroup owns one tile:
// its waves split the hidden dimension for the router product (MFMA for bf16,
// fp32 FMA for fp32), the partial logits meet in LDS, then each wave ranks
// whole tokens (one expert per lane), 32 lanes walk Algorithm 1 for the 32
// tokens, and the tile's per-expert histogram goes to global memory.  A
// one-workgroup scan turns the histograms into group offsets, per-tile bases
// and the row-tile table of the grouped GEMMs; a scatter kernel then places
// every assignment (rank inside the tile by counting earlier equal keys, so
// the order is the stable one and no atomics decide a position).
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

__device__ __forceinline__ void remap_token(int K, int E, int R, int H, bool unique,
                                            const uint64_t *bitmap, const int32_t *table,
                                            const int32_t *ids_in, int32_t *ids_out, float *w,
                                            int &n_miss, int &n_sub, int &n_drop) {
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
            for (int r = 0; r < H; ++r) {
                const int b = row[r];
                const bool bvalid = (unsigned)b < (unsigned)E;
                const int bc = bvalid ? b : 0;
                bool ok = bvalid && ((bitmap[bc >> 6] >> (bc & 63)) & 1ull);
                ok = ok && !(unique && test_bit4(used, bc));
                out = (ok && !found) ? b : out;
                found = found || ok;
            }
            if (found) { ++n_sub; set_bit4(used, out); } else { ++n_drop; }
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
    int32_t stats[4];
    uint64_t bitmap[4];
};

// Ranks the tile's tokens from the logits in LDS and finishes the tile.
// logits: [TILE_T][stride] fp32, bias already added.  The logits region is
// reused for the buddy table once ranking is done (cap = its size in ints).
__device__ void tile_epilogue(const FrontParams &p, float *logits, int stride, int cap_ints,
                              FrontLds &s, int tile) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    const int t0 = tile * TILE_T;
    const int ntok = min(TILE_T, p.T - t0);
    const int E = p.E, K = p.K;
    const int ec = (E + 63) >> 6;

    for (int i = wave; i < ntok; i += nw) {
        float vals[4], orig[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int e = lane + 64 * c;
            vals[c] = (c < ec && e < E) ? logits[i * stride + e] : -INFINITY;
            orig[c] = vals[c];
        }
        float my_z = -INFINITY;
        int my_id = -1;
        for (int k = 0; k < K; ++k) {
            float bv = vals[0];
            int bi = lane;
#pragma unroll
            for (int c = 1; c < 4; ++c) {
                if (vals[c] > bv) { bv = vals[c]; bi = lane + 64 * c; }   // lower index wins ties
            }
            wave_argmax(bv, bi);
            if ((bi & 63) == lane) {
#pragma unroll
                for (int c = 0; c < 4; ++c) if ((bi >> 6) == c) vals[c] = -INFINITY;
            }
            if (lane == k) { my_z = bv; my_id = bi; }
        }
        const float zmax = __shfl(my_z, 0, WAVE);
        const float pk = (lane < K) ? expf(my_z - zmax) : 0.0f;
        float denom;
        if (p.flags & BM_RENORM_TOPK) {
            denom = wave_sum(pk);
        } else {
            float acc = 0.0f;
#pragma unroll
            for (int c = 0; c < 4; ++c) acc += (orig[c] == -INFINITY) ? 0.0f : expf(orig[c] - zmax);
            denom = wave_sum(acc);
        }
        if (lane < K) {
            p.ids[(size_t)(t0 + i) * K + lane] = my_id;
            s.ids[i * K + lane] = my_id;
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
    const bool tab_in_lds = E * p.R <= cap_ints;
    int32_t *s_table = reinterpret_cast<int32_t *>(logits);
    if (tab_in_lds)
        for (int idx = tid; idx < E * p.R; idx += blockDim.x) s_table[idx] = p.table[idx];
    for (int idx = tid; idx < BM_MAX_E; idx += blockDim.x) s.counts[idx] = 0;
    if (tid < 4) { s.bitmap[tid] = (tid < ec) ? p.bitmap[tid] : 0ull; s.stats[tid] = 0; }
    __syncthreads();

    if (tid < ntok) {
        int n_miss = 0, n_sub = 0, n_drop = 0;
        int32_t *tok_ids = &s.ids[tid * K];
        float *tok_w = &s.w[tid * K];
        remap_token(K, E, p.R, p.H, (p.flags & BM_REMAP_UNIQUE) != 0, s.bitmap,
                    tab_in_lds ? s_table : p.table, tok_ids, tok_ids, tok_w, n_miss, n_sub, n_drop);
        if (n_miss) atomicAdd(&s.stats[0], n_miss);
        if (n_sub) atomicAdd(&s.stats[1], n_sub);
        if (n_drop) atomicAdd(&s.stats[2], n_drop);
        for (int k = 0; k < K; ++k) {
            const int e = tok_ids[k];
            if (e >= 0) atomicAdd(&s.counts[e], 1);
        }
    }
    __syncthreads();

    for (int idx = tid; idx < n; idx += blockDim.x) {
        p.ids2[(size_t)t0 * K + idx] = s.ids[idx];
        p.w[(size_t)t0 * K + idx] = s.w[idx];
    }
    for (int e = tid; e < E; e += blockDim.x) p.tile_counts[(size_t)tile * E + e] = s.counts[e];
    if (tid < 3) p.tile_stats[tile * 4 + tid] = s.stats[tid];
}

// ---------------------------------------------------------------------------
// bf16 front kernel: router product on MFMA 32x32x16 (tokens x experts),
// operands read from global memory directly in the instruction's layout:
// lane l supplies row/column (l % 32) and the 8 consecutive k values starting
// at 8 * (l / 32), i.e. one 16-byte load per operand per k-step.
// NB = number of 32-expert column blocks, NW = waves per workgroup (k split).
// ---------------------------------------------------------------------------
template <int NB, int NW>
__global__ void __launch_bounds__(NW * 64) front_bf16_kernel(FrontParams p) {
    constexpr int STRIDE = NB * 32 + 1;
    __shared__ float logits[TILE_T * STRIDE];
    __shared__ FrontLds s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tile = blockIdx.x, t0 = tile * TILE_T;
    const int r32 = lane & 31, half = lane >> 5;
    const uint16_t *x = static_cast<const uint16_t *>(p.x);
    const uint16_t *wr = static_cast<const uint16_t *>(p.wr);

    const int trow = min(t0 + r32, p.T - 1);
    const uint16_t *xa = x + (size_t)trow * p.d + half * 8;
    const uint16_t *wb[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) wb[nb] = wr + (size_t)min(nb * 32 + r32, p.E - 1) * p.d + half * 8;

    f32x16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] = 0.0f;

    const int ksteps = p.d >> 4;
#pragma unroll 4
    for (int ks = wave; ks < ksteps; ks += NW) {
        const bf16x8 a = as_bf16x8(ldg128(xa + ks * 16));
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const bf16x8 b = as_bf16x8(ldg128(wb[nb] + ks * 16));
            acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[nb], 0, 0, 0);
        }
    }

    // D[i][j]: lane holds column j = l % 32 and rows i = 8*(v/4) + 4*(l/32) + v%4.
    // Waves add their partial sums in wave order, so the sum is reproducible.
    for (int w = 0; w < NW; ++w) {
        if (wave == w) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int e = nb * 32 + r32;
                const float b0 = (w == 0) ? ((p.bias != nullptr && e < p.E) ? p.bias[e] : 0.0f) : 0.0f;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int i = 8 * (v >> 2) + 4 * half + (v & 3);
                    float *q = &logits[i * STRIDE + e];
                    *q = (w == 0 ? b0 : *q) + acc[nb][v];
                }
            }
        }
        __syncthreads();
    }
    tile_epilogue(p, logits, STRIDE, TILE_T * STRIDE, s, tile);
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
    tile_epilogue(p, logits, STRIDE, TILE_T * STRIDE, s, tile);
}

// ---------------------------------------------------------------------------
// Stand-alone substitution kernel: one lane per token, bitmap and table in LDS.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) remap_kernel(RemapParams p) {
    extern __shared__ int32_t s_table[];
    __shared__ uint64_t s_bitmap[4];
    __shared__ int32_t s_stats[3];
    const int tid = threadIdx.x;
    const int ec = (p.E + 63) >> 6;
    for (int idx = tid; idx < p.E * p.R; idx += blockDim.x) s_table[idx] = p.table[idx];
    if (tid < 4) s_bitmap[tid] = (tid < ec) ? p.bitmap[tid] : 0ull;
    if (tid < 3) s_stats[tid] = 0;
    __syncthreads();
    const int t = blockIdx.x * blockDim.x + tid;
    if (t < p.T) {
        int n_miss = 0, n_sub = 0, n_drop = 0;
        const int32_t *in = p.ids_in + (size_t)t * p.K;
        int32_t *out = p.ids_out + (size_t)t * p.K;
        float *w = p.w ? p.w + (size_t)t * p.K : nullptr;
        remap_token(p.K, p.E, p.R, p.H, p.unique != 0, s_bitmap, s_table, in, out, w, n_miss, n_sub, n_drop);
        if (n_miss) atomicAdd(&s_stats[0], n_miss);
        if (n_sub) atomicAdd(&s_stats[1], n_sub);
        if (n_drop) atomicAdd(&s_stats[2], n_drop);
    }
    __syncthreads();
    if (p.stats != nullptr && tid < 3 && s_stats[tid]) atomicAdd(&p.stats[tid], s_stats[tid]);
}

__global__ void zero_ints_kernel(int32_t *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// Per-tile histogram of given ids (stand-alone grouping entry point).
__global__ void __launch_bounds__(256) count_kernel(const int32_t *ids, int T, int K, int E,
                                                    int32_t *tile_counts) {
    __shared__ int32_t counts[BM_MAX_E];
    const int tid = threadIdx.x, tile = blockIdx.x, t0 = tile * TILE_T;
    const int n = min(TILE_T, T - t0) * K;
    for (int e = tid; e < E; e += blockDim.x) counts[e] = 0;
    __syncthreads();
    for (int idx = tid; idx < n; idx += blockDim.x) {
        const int e = ids[(size_t)t0 * K + idx];
        if ((unsigned)e < (unsigned)E) atomicAdd(&counts[e], 1);
    }
    __syncthreads();
    for (int e = tid; e < E; e += blockDim.x) tile_counts[(size_t)tile * E + e] = counts[e];
}

// ---------------------------------------------------------------------------
// One-workgroup scan: tile histograms -> per-tile bases (relative to the
// group start), group offsets (routed experts, then shared experts with T
// rows each), the row-tile table of the grouped GEMMs, and the summed
// substitution statistics.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) scan_kernel(ScanParams p) {
    __shared__ int32_t total[BM_MAX_E + 8];
    __shared__ int32_t start[BM_MAX_E + 9];
    __shared__ int32_t tstart[BM_MAX_E + 9];
    const int tid = threadIdx.x;
    const int G = p.E + p.n_shared;
    for (int e = tid; e < p.E; e += blockDim.x) {
        int run = 0;
        for (int t = 0; t < p.n_tiles; ++t) {
            const int c = p.tile_counts[(size_t)t * p.E + e];
            p.tile_base[(size_t)t * p.E + e] = run;
            run += c;
        }
        total[e] = run;
    }
    for (int g = p.E + tid; g < G; g += blockDim.x) total[g] = p.T;
    __syncthreads();
    if (tid == 0) {
        int run = 0, trun = 0;
        for (int g = 0; g < G; ++g) {
            start[g] = run;
            tstart[g] = trun;
            run += total[g];
            trun += (total[g] + p.BM - 1) / p.BM;
        }
        start[G] = run;
        tstart[G] = trun;
        p.n_mtiles[0] = trun;
        p.n_mtiles[1] = run;                       // total rows
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
    if (p.stats != nullptr && tid < 3) {
        int sum = 0;
        if (p.tile_stats != nullptr)
            for (int t = 0; t < p.n_tiles; ++t) sum += p.tile_stats[t * 4 + tid];
        p.stats[tid] = sum;
    }
}

// ---------------------------------------------------------------------------
// Scatter: position of assignment a = offsets[e] + base of its tile + number
// of earlier assignments of the tile with the same expert.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) scatter_kernel(ScatterParams p) {
    __shared__ int32_t s_ids[TILE_T * BM_MAX_K];
    const int tid = threadIdx.x, tile = blockIdx.x, t0 = tile * TILE_T;
    const int K = p.K, E = p.E;
    const int ntok = min(TILE_T, p.T - t0);
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
            pos = p.offsets[e] + p.tile_base[(size_t)tile * E + e] + rank;
            p.perm[pos] = a;
            if (p.row_token) p.row_token[pos] = a / K;
        }
        p.inv_perm[a] = pos;
    }
    // positions past the live count hold -1
    for (int idx = tid; idx < TILE_T * K; idx += blockDim.x) {
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
// Host-side launchers
// ---------------------------------------------------------------------------
template <int NB, int NW>
static void launch_front_bf16(const FrontParams &p, int n_tiles, hipStream_t st) {
    hipLaunchKernelGGL((front_bf16_kernel<NB, NW>), dim3(n_tiles), dim3(NW * 64), 0, st, p);
}

int launch_front(const FrontParams &p, int dtype, hipStream_t st) {
    const int n_tiles = (p.T + TILE_T - 1) / TILE_T;
    if (n_tiles == 0) return 0;
    if (dtype == BM_F32) {
        hipLaunchKernelGGL(front_f32_kernel, dim3(n_tiles), dim3(256), 0, st, p);
    } else {
        const int nb = (p.E + 31) / 32;
        const bool small = n_tiles <= 8;   // few tiles: split the hidden dimension 16 ways
        if (nb <= 1) small ? launch_front_bf16<1, 16>(p, n_tiles, st) : launch_front_bf16<1, 4>(p, n_tiles, st);
        else if (nb <= 2) small ? launch_front_bf16<2, 16>(p, n_tiles, st) : launch_front_bf16<2, 4>(p, n_tiles, st);
        else if (nb <= 4) small ? launch_front_bf16<4, 8>(p, n_tiles, st) : launch_front_bf16<4, 4>(p, n_tiles, st);
        else launch_front_bf16<8, 4>(p, n_tiles, st);
    }
    return launch_status(__func__);
}

int launch_remap(const RemapParams &p, hipStream_t st) {
    if (p.stats) hipLaunchKernelGGL(zero_ints_kernel, dim3(1), dim3(64), 0, st, p.stats, 3);
    if (p.T > 0) {
        const size_t lds = (size_t)p.E * p.R * sizeof(int32_t);
        hipLaunchKernelGGL(remap_kernel, dim3((p.T + 255) / 256), dim3(256), lds, st, p);
    }
    return launch_status(__func__);
}

int launch_count(const int32_t *ids, int T, int K, int E, int32_t *tile_counts, hipStream_t st) {
    const int n_tiles = (T + TILE_T - 1) / TILE_T;
    if (n_tiles) hipLaunchKernelGGL(count_kernel, dim3(n_tiles), dim3(256), 0, st, ids, T, K, E, tile_counts);
    return launch_status(__func__);
}

int launch_scan(const ScanParams &p, hipStream_t st) {
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(256), 0, st, p);
    return launch_status(__func__);
}

int launch_scatter(const ScatterParams &p, hipStream_t st) {
    const int n_tiles = (p.T + TILE_T - 1) / TILE_T;
    if (n_tiles) hipLaunchKernelGGL(scatter_kernel, dim3(n_tiles), dim3(256), 0, st, p);
    return launch_status(__func__);
}

}  // namespace bm
