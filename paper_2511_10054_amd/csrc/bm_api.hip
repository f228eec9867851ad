// C ABI of the library: argument checks, workspace carving, kernel sequencing.
// Nothing here allocates or synchronises; the only state kept between calls is the
// per-device address of the built-in scratch array of bm_moe_forward_static.
#include "bm_kernels.h"
#include "bm_device_shape.h"

#include <atomic>
#include <cstdio>
#include <mutex>

// Built-in workspace of bm_moe_forward_static: every device the library runs on holds its own copy
// until the process ends.  Host code never uses this name as an address - it is a host-side stand-in;
// the device address comes from hipGetSymbolAddress (static_scratch_ptr below).
static __device__ __align__(256) unsigned char scratch[BM_STATIC_WORKSPACE_BYTES];

namespace bm {
int launch_status(const char *what) {
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return 0;
    std::fprintf(stderr, "buddymoe: %s: %s\n", what, hipGetErrorString(e));
    return -1;
}
}  // namespace bm

namespace {

using namespace bm;

constexpr size_t ALIGN = 256;
constexpr int MAX_SHARED = 8;
constexpr int SKINNY_MAX_ROWS = 256;   // total rows up to which the weight-streaming path is always used,
constexpr int SKINNY_AVG_ROWS = 16;    // ... and rows per group (averaged over all experts) likewise
constexpr int SKINNY_UNFIT_ROWS = 16;  // total rows when the widths do not fit its fast kernels but do fit the persistent tiled kernel
constexpr int SKINNY_KSPLIT = 8;

// Shapes both projections of which fit the persistent k-step-64 kernel: reduction widths that are multiples
// of 64 and at least 256, operands within 32-bit byte offsets.
bool k64_shape(const bm_layer_desc *d) {
    const unsigned long long lim = 1ull << 32;
    const int ns = d->n_shared > 0 ? d->n_shared : 0;
    const unsigned long long rows = (unsigned long long)d->T * (d->K + ns) + 256ull * (d->E + ns);
    return d->dtype == BM_BF16 && d->d % 64 == 0 && d->F % 64 == 0 && d->d >= 256 && d->F >= 256 &&
           (unsigned long long)d->T * d->d * 2 < lim && rows * d->F * 2 < lim && (unsigned long long)d->F * d->d * 2 < lim;
}

// Row tiles of a grouped projection (down: the down projection, else gate/up): TILES_MIXED, or the single
// tile height 256 / 128.  On the persistent kernel (k64_shape on a device of the expected shape) a launch
// runs both heights: a group's rows go into 256-row tiles and a rest of at most 128 rows into one 128-row
// tile, which costs 0.65 of a 256-row tile's time.  Measured against single heights, ms (gate/up, down) with
// 128- | 256-row tiles only: Mixtral-shaped layer, 5 of 8 experts resident, 384 tokens .27 .22 | .32 .19,
// 1024 tokens .55 .41 | .50 .30; DeepSeek-shaped 1024 tokens .10 .08 | .12 .08, 2048 tokens .20 .12 | .18 .12;
// Qwen3-shaped 1024 tokens .11 .07 | .13 .08, 2048 tokens .14 .10 | .16 .09: neither height wins everywhere.
// The down projection of a long reduction keeps 256 rows: its partial last round is split along the
// reduction instead (down_split_tail).  Other shapes: 256 rows when the average routed group is large, else 128.
constexpr int TILES_MIXED = 0;
int tile_mode(const bm_layer_desc *d, bool down, bool persistent) {
    if (k64_shape(d)) {
        if (!persistent) return 256;
        return (down && down_split_tail(d->F)) ? 256 : TILES_MIXED;
    }
    return ((long long)d->T * d->K / d->E >= 128) ? 256 : 128;
}

// Few rows per group: every expert group is decode-sized and the projections are bound by reading the
// weights once.  Up to 256 rows in all, or up to 16 rows per expert on average (Qwen3-shaped layer, 128
// experts, 64 / 128 / 256 tokens: 0.11 / 0.13 / 0.16 ms against 0.14 / 0.15 / 0.16 ms on the tiled path), when
// both widths fit the fast streaming kernels (multiples of 256).  Widths that do not (DeepSeek-shaped layer,
// F = 1408, whose shared experts take every token as well) leave the streaming path to its slower
// fallbacks: there the persistent tiled kernel is faster from 4 tokens on (4 / 8 / 32 tokens: 0.064 / 0.071 /
// 0.089 against 0.068 / 0.082 / 0.101 ms), so the streaming path keeps only batches of at most 16 rows.
// Mixtral-shaped layer, 8 experts, streaming | tiled, ms: 128 tokens 0.40 | 0.44, 192 tokens 0.55 | 0.47,
// 256 tokens 0.59 | 0.48 (public weight layout; 0.48 | 0.47 and 0.52 | 0.48 on the packed copies).
bool use_skinny(const bm_layer_desc *d) {
    if (d->dtype != BM_BF16) return false;
    const int ns = d->n_shared > 0 ? d->n_shared : 0;
    const long long rows = (long long)d->T * (d->K + ns);
    const bool fit = d->d % 256 == 0 && d->F % 256 == 0;
    if (!fit && k64_shape(d)) return rows <= SKINNY_UNFIT_ROWS;
    if (rows <= SKINNY_MAX_ROWS) return true;
    return fit && rows <= (long long)SKINNY_AVG_ROWS * (d->E + ns);
}
// Reduction slices of the decode down projection (each slice is a workgroup
// whose 4 waves split it once more): prefer a count that fits the
// quarter-split kernel, else up to 8 slices of at least 16 k-steps.
int skinny_ksplit(const bm_layer_desc *d) {
    // small groups: the persistent kernel splits the reduction inside one workgroup, no slices
    if ((long long)d->T * d->K <= 32 && (bm::skinny_p_ok(d->F, 14) || bm::skinny_p_ok(d->F, 8))) return 1;
    if ((long long)d->T * d->K > 32) {
        // LDS-staged kernel: the fewest slices that still give every compute unit two workgroups (64 weight
        // rows each) - longer weight streams per workgroup and fewer fp32 partial outputs beat a finer
        // split (measured on the Mixtral-shaped layer at 64 tokens: 2 slices 99 us, 4: 111, 7: 115-119, 8: 114; unsplit 147;
        // the aggregation kernel grows with the slices as well, 8 -> 11 -> 15 -> 16 us)
        const long long groups = d->E + d->n_shared < (long long)d->T * d->K ? d->E + d->n_shared : (long long)d->T * d->K;
        for (int s = 2; s <= SKINNY_KSPLIT; ++s)
            if (bm::skinny_lds_ok(d->F, s) && d->F / (512 * s) >= 2 && (d->d / 64) * groups * s >= 512) return s;
        for (int s = SKINNY_KSPLIT; s > 1; --s)
            if (bm::skinny_lds_ok(d->F, s) && d->F / (512 * s) >= 2) return s;
        if (bm::skinny_lds_ok(d->F, 1)) return 1;       // short reduction (e.g. F = 768): unsplit, still the LDS-staged kernel
    }
    for (int s = SKINNY_KSPLIT; s >= 1; --s)
        if (bm::skinny_q_ok(d->F, s)) return s;
    const int ksteps = d->F / 32;
    int s = ksteps / 16;
    return s < 1 ? 1 : (s > SKINNY_KSPLIT ? SKINNY_KSPLIT : s);
}

size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

// Workspace carving: a pure function of desc.
struct Layout {
    size_t ids, ids2, w, tile_counts, tile_base, tile_stats, offsets, perm, inv_perm, row_token;
    size_t mt_group, mt_row0, n_mtiles, mt_group_b, mt_row0_b, n_mtiles_b, mt_group_s, mt_row0_s, n_mtiles_s;
    size_t stats, probs, h, o, splitk, total;
    int n_tiles, rows_max, mtiles_max;
    bool has_splitk;
};

int check_desc(const bm_layer_desc *d, bool need_ffn) {
    if (!d) return BM_ERR_NULL;
    if (d->dtype != BM_F32 && d->dtype != BM_BF16) return BM_ERR_DTYPE;
    if (d->T < 0 || d->E <= 0 || d->K <= 0 || d->d <= 0) return BM_ERR_SHAPE;
    if (d->K > d->E || d->E > BM_MAX_E || d->K > BM_MAX_K) return BM_ERR_SHAPE;
    if ((long long)d->T * d->K > (1ll << 30)) return BM_ERR_SHAPE;
    if (d->dtype == BM_BF16 && (d->d % 32)) return BM_ERR_SHAPE;
    if (need_ffn) {
        if (d->F <= 0 || d->n_shared < 0 || d->n_shared > MAX_SHARED) return BM_ERR_SHAPE;
        if (d->dtype == BM_BF16 && (d->F % 32)) return BM_ERR_SHAPE;
        if (d->dtype == BM_F32 && (d->F > 16000 || d->d > 16000)) return BM_ERR_SHAPE;
    }
    return BM_OK;
}

int check_remap_desc(const bm_layer_desc *d) {
    if (d->R < 0 || d->R > BM_MAX_R || d->H < 0 || d->H > d->R) return BM_ERR_SHAPE;
    if ((d->flags & BM_REPLACE_BUDGET) && d->rho < 0) return BM_ERR_SHAPE;
    if ((d->flags & BM_GATE_TAE) && !(d->tae_tau == d->tae_tau)) return BM_ERR_SHAPE;            // NaN
    if ((d->flags & BM_GATE_MARGIN) && !(d->margin_gamma == d->margin_gamma)) return BM_ERR_SHAPE;
    if ((d->flags & BM_GATE_DIST) && !(d->dist_beta == d->dist_beta)) return BM_ERR_SHAPE;
    if ((d->flags & BM_PSI_TOKEN) && !(d->psi_eta >= 0.0f)) return BM_ERR_SHAPE;
    return BM_OK;
}

Layout make_layout(const bm_layer_desc *d) {
    Layout L{};
    const size_t A = (size_t)d->T * d->K;
    const int n_shared = d->n_shared > 0 ? d->n_shared : 0;
    const int G = d->E + n_shared;
    L.n_tiles = (d->T + TILE_T - 1) / TILE_T;
    const int tiles16 = (d->T + 15) / 16;          // the front kernel's tiles of small batches (per-tile arrays)
    L.rows_max = (int)(A + (size_t)n_shared * d->T);
    L.mtiles_max = L.rows_max / 128 + G;         // bound for the smaller of the two row-tile heights
    const size_t esz = d->dtype == BM_BF16 ? 2 : 4;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    L.ids = take(A * 4);
    L.ids2 = take(A * 4);
    L.w = take(A * 4);
    L.tile_counts = take((size_t)tiles16 * d->E * 4);
    L.tile_base = take((size_t)tiles16 * d->E * 4);
    L.tile_stats = take((size_t)tiles16 * 16);
    L.offsets = take((size_t)(G + 1) * 4);
    L.perm = take(A * 4);
    L.inv_perm = take(A * 4);
    L.row_token = take((size_t)L.rows_max * 4);
    L.mt_group = take((size_t)L.mtiles_max * 4);
    L.mt_row0 = take((size_t)L.mtiles_max * 4);
    L.n_mtiles = take(16);
    // the two row-tile lists of a launch that runs 256- and 128-row tiles (at most rows / 256 + G and G entries)
    const bool mixed = !use_skinny(d) && k64_shape(d);
    L.mt_group_b = take(mixed ? (size_t)L.mtiles_max * 4 : 0);
    L.mt_row0_b = take(mixed ? (size_t)L.mtiles_max * 4 : 0);
    L.n_mtiles_b = take(mixed ? 16 : 0);
    L.mt_group_s = take(mixed ? (size_t)G * 4 : 0);
    L.mt_row0_s = take(mixed ? (size_t)G * 4 : 0);
    L.n_mtiles_s = take(mixed ? 16 : 0);
    L.stats = take(32);
    // every expert's probability per token: only when the substitution runs apart from the router kernel
    L.probs = take(((d->flags & BM_PSI_TOKEN) && (d->flags & BM_GATE_DIST)) ? (size_t)d->T * d->E * 4 : 0);
    const size_t F = d->F > 0 ? d->F : 0;
    L.h = take((size_t)L.rows_max * F * esz);
    L.o = take(use_skinny(d) ? (size_t)skinny_ksplit(d) * L.rows_max * d->d * 4 : (size_t)L.rows_max * d->d * esz);
    // fp32 partial tiles of the down projection's split tail: one 256 x 256 tile per workgroup of the launch
    L.has_splitk = !use_skinny(d) && k64_shape(d) && down_split_tail(d->F);
    L.splitk = take(L.has_splitk ? (size_t)K64_CUS * 256 * 256 * 4 : 0);   // a launch has at most K64_CUS workgroups
    L.total = off;
    return L;
}

// Argument checks of the whole-layer entry points (everything but the workspace).
int check_moe_args(const bm_layer_desc *desc, const void *x, const bm_weights *wt, const uint64_t *residency_bitmap,
                   const int32_t *buddy_table, const void *y) {
    int rc = check_desc(desc, true);
    if (rc) return rc;
    rc = check_remap_desc(desc);
    if (rc) return rc;
    if (desc->T == 0) return BM_OK;
    if (!x || !wt || !residency_bitmap || !y || (!buddy_table && desc->R > 0)) return BM_ERR_NULL;
    if (!wt->w_router || !wt->w_gate || !wt->w_up || !wt->w_down) return BM_ERR_NULL;
    if (desc->n_shared > 0 && (!wt->ws_gate || !wt->ws_up || !wt->ws_down)) return BM_ERR_NULL;
    if ((desc->flags & BM_PSI_TOKEN) && !wt->buddy_q) return BM_ERR_NULL;
    return BM_OK;
}

// Scratch of bm_permute_by_expert: the per-tile histograms and bases and the row-tile table the grouping
// kernels write on the way.  A pure function of T and E.
struct GroupLayout {
    size_t tile_counts, tile_base, mt_group, mt_row0, n_mtiles, total;
    int n_tiles;
};

GroupLayout make_group_layout(int T, int E) {
    GroupLayout L{};
    L.n_tiles = (T + TILE_T - 1) / TILE_T;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    L.tile_counts = take((size_t)L.n_tiles * E * 4);
    L.tile_base = take((size_t)L.n_tiles * E * 4);
    L.mt_group = take((size_t)E * 4);            // one entry per live group (the table is built with a tile height no group reaches)
    L.mt_row0 = take((size_t)E * 4);
    L.n_mtiles = take(16);
    L.total = off;
    return L;
}

int check_group_desc(const bm_layer_desc *d) {
    if (d->T < 0 || d->E <= 0 || d->K <= 0 || d->E > BM_MAX_E || d->K > BM_MAX_K || d->K > d->E) return BM_ERR_SHAPE;
    if ((long long)d->T * d->K > (1ll << 30)) return BM_ERR_SHAPE;
    return BM_OK;
}

template <typename T>
T *at(void *ws, size_t off) { return reinterpret_cast<T *>(static_cast<char *>(ws) + off); }

int check_ws(const bm_layer_desc *d, void *ws, size_t bytes, Layout &L) {
    L = make_layout(d);
    if (!ws || (reinterpret_cast<uintptr_t>(ws) % ALIGN) || bytes < L.total) return BM_ERR_WORKSPACE;
    return BM_OK;
}

__global__ void copy_ints_kernel(const int32_t *src, int32_t *dst, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

void copy_ints(const void *src, void *dst, size_t n, hipStream_t st) {
    if (n) hipLaunchKernelGGL(copy_ints_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                              static_cast<const int32_t *>(src), static_cast<int32_t *>(dst), n);
}

// Device address of `scratch` on the current device, looked up once per device.
constexpr int MAX_DEVICES = 64;
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];
std::mutex g_scratch_mutex;

int static_scratch_ptr(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return BM_ERR_HIP;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!p) {
            const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p) {
                std::fprintf(stderr, "buddymoe: hipGetSymbolAddress(scratch): %s\n", hipGetErrorString(e));
                return BM_ERR_HIP;
            }
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return BM_OK;
}

}  // namespace

extern "C" {

int bm_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream) {
    if (!sink || (bytes && !src)) return BM_ERR_NULL;
    if (bytes % 16) return BM_ERR_SHAPE;
    (void)hipGetLastError();
    return launch_stream_read(src, bytes, sink, static_cast<hipStream_t>(stream)) ? BM_ERR_HIP : BM_OK;
}

const char *bm_strerror(int status) {
    switch (status) {
        case BM_OK: return "ok";
        case BM_ERR_NULL: return "a required pointer is NULL";
        case BM_ERR_SHAPE: return "unsupported or inconsistent shape";
        case BM_ERR_DTYPE: return "unknown dtype";
        case BM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case BM_ERR_BAD_TABLE: return "buddy table entry out of range or equal to its row";
        case BM_ERR_HIP: return "kernel launch failed";
        default: return "unknown status";
    }
}

size_t bm_workspace_bytes(const bm_layer_desc *desc) {
    if (!desc) return 0;
    if (desc->d == 0 && desc->F == 0) {          // grouping only: a function of T, E and K
        if (check_group_desc(desc) != BM_OK) return 0;
        return make_group_layout(desc->T, desc->E).total;
    }
    if (check_desc(desc, false) != BM_OK) return 0;
    return make_layout(desc).total;
}

size_t bm_packed_bytes(const bm_layer_desc *desc, int which) {
    if (check_desc(desc, true) != BM_OK || desc->dtype != BM_BF16 || which < 0 || which > 3) return 0;
    const size_t per = (size_t)desc->F * desc->d * 2;            // one matrix of one expert
    const size_t n = which < 2 ? (size_t)desc->E : (size_t)desc->n_shared;
    return n * per * ((which & 1) ? 1 : 2);
}

int bm_pack_weights(const bm_layer_desc *desc, const bm_weights *wt, const uint64_t *residency_bitmap,
                    void *stream) {
    int rc = check_desc(desc, true);
    if (rc) return rc;
    if (desc->dtype != BM_BF16) return BM_ERR_DTYPE;
    if (!wt) return BM_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    int err = 0;
    if (wt->wp_gateup) {
        if (!wt->w_gate || !wt->w_up) return BM_ERR_NULL;
        err |= launch_pack(wt->w_gate, wt->w_up, const_cast<void *>(wt->wp_gateup), desc->E, desc->F, desc->d,
                           residency_bitmap, st);
    }
    if (wt->wp_down) {
        if (!wt->w_down) return BM_ERR_NULL;
        err |= launch_pack(wt->w_down, nullptr, const_cast<void *>(wt->wp_down), desc->E, desc->d, desc->F,
                           residency_bitmap, st);
    }
    if (desc->n_shared > 0 && wt->wsp_gateup) {
        if (!wt->ws_gate || !wt->ws_up) return BM_ERR_NULL;
        err |= launch_pack(wt->ws_gate, wt->ws_up, const_cast<void *>(wt->wsp_gateup), desc->n_shared, desc->F,
                           desc->d, nullptr, st);
    }
    if (desc->n_shared > 0 && wt->wsp_down) {
        if (!wt->ws_down) return BM_ERR_NULL;
        err |= launch_pack(wt->ws_down, nullptr, const_cast<void *>(wt->wsp_down), desc->n_shared, desc->d, desc->F,
                           nullptr, st);
    }
    return err ? BM_ERR_HIP : BM_OK;
}

int bm_validate_tables(const bm_layer_desc *desc, const uint64_t *bitmap_host, const int32_t *table_host) {
    if (!desc || !bitmap_host || !table_host) return BM_ERR_NULL;
    if (desc->E <= 0 || desc->E > BM_MAX_E) return BM_ERR_SHAPE;
    int rc = check_remap_desc(desc);
    if (rc) return rc;
    for (int i = 0; i < desc->E; ++i)
        for (int r = 0; r < desc->R; ++r) {
            const int32_t b = table_host[(size_t)i * desc->R + r];
            if (b < -1 || b >= desc->E || b == i) return BM_ERR_BAD_TABLE;
        }
    // bits past E must be clear
    const int words = (desc->E + 63) / 64;
    if (desc->E % 64) {
        const uint64_t tail = bitmap_host[words - 1] >> (desc->E % 64);
        if (tail) return BM_ERR_BAD_TABLE;
    }
    return BM_OK;
}

int bm_coactivation_accumulate(const bm_layer_desc *desc, const int32_t *ids, int64_t *activations,
                               int64_t *coactivations, void *stream) {
    if (!desc) return BM_ERR_NULL;
    if (desc->T < 0 || desc->E <= 0 || desc->K <= 0 || desc->E > BM_MAX_E || desc->K > BM_MAX_K) return BM_ERR_SHAPE;
    if (desc->T == 0) return BM_OK;
    if (!ids || !activations || !coactivations) return BM_ERR_NULL;
    (void)hipGetLastError();
    return launch_coactivation(ids, desc->T, desc->K, desc->E, reinterpret_cast<long long *>(activations),
                               reinterpret_cast<long long *>(coactivations), static_cast<hipStream_t>(stream))
               ? BM_ERR_HIP : BM_OK;
}

int bm_build_buddy_table(const bm_layer_desc *desc, const int64_t *coactivations, float alpha, int32_t *buddy_table,
                         int32_t *list_len, float *q, void *stream) {
    if (!desc) return BM_ERR_NULL;
    if (desc->E <= 0 || desc->E > BM_MAX_E || desc->R <= 0 || desc->R > BM_MAX_R) return BM_ERR_SHAPE;
    if (!(alpha > 0.0f && alpha <= 1.0f)) return BM_ERR_SHAPE;
    if (!coactivations || !buddy_table) return BM_ERR_NULL;
    (void)hipGetLastError();
    return launch_buddy_build(reinterpret_cast<const long long *>(coactivations), desc->E, desc->R, alpha, buddy_table,
                              list_len, q, static_cast<hipStream_t>(stream))
               ? BM_ERR_HIP : BM_OK;
}

int bm_route_topk(const bm_layer_desc *desc, const void *x, const void *w_router, const float *bias,
                  int32_t *ids, float *w, void *stream) {
    int rc = check_desc(desc, false);
    if (rc) return rc;
    if (desc->T == 0) return BM_OK;
    if (!x || !w_router || !ids || !w) return BM_ERR_NULL;
    (void)hipGetLastError();   // errors left by earlier, unrelated HIP calls are not ours
    FrontParams p{};
    p.x = x; p.wr = w_router; p.bias = bias;
    p.T = desc->T; p.d = desc->d; p.E = desc->E; p.K = desc->K; p.R = 0; p.H = 0;
    p.flags = desc->flags;
    p.ids = ids; p.w = w;
    p.bitmap = nullptr;
    p.tile_tokens = front_tile_tokens(desc->T, desc->dtype, false);
    return launch_front(p, desc->dtype, static_cast<hipStream_t>(stream)) ? BM_ERR_HIP : BM_OK;
}

int bm_buddy_remap(const bm_layer_desc *desc, const uint64_t *residency_bitmap, const int32_t *buddy_table,
                   const int32_t *ids_in, int32_t *ids_out, float *w, bm_remap_stats *stats, void *stream) {
    if (!desc) return BM_ERR_NULL;
    if (desc->T < 0 || desc->E <= 0 || desc->K <= 0 || desc->E > BM_MAX_E || desc->K > BM_MAX_K) return BM_ERR_SHAPE;
    int rc = check_remap_desc(desc);
    if (rc) return rc;
    if (!residency_bitmap || !ids_in || !ids_out || (!buddy_table && desc->R > 0)) return BM_ERR_NULL;
    if ((desc->flags & (BM_GATE_TAE | BM_GATE_MARGIN)) && !w) return BM_ERR_NULL;   // the gates read the weights
    if (desc->flags & BM_PSI_TOKEN) return BM_ERR_SHAPE;   // needs the router's probabilities: bm_moe_forward
    (void)hipGetLastError();
    RemapParams p{};
    p.T = desc->T; p.K = desc->K; p.E = desc->E; p.R = desc->R; p.H = desc->H;
    p.flags = desc->flags; p.tau = desc->tae_tau; p.gamma = desc->margin_gamma; p.rho = desc->rho;
    p.beta = desc->dist_beta;
    p.bitmap = residency_bitmap; p.table = buddy_table;
    p.ids_in = ids_in; p.ids_out = ids_out; p.w = w;
    p.stats = reinterpret_cast<int32_t *>(stats);
    return launch_remap(p, static_cast<hipStream_t>(stream)) ? BM_ERR_HIP : BM_OK;
}

int bm_permute_by_expert(const bm_layer_desc *desc, const int32_t *ids_remapped, int32_t *offsets,
                         int32_t *perm, int32_t *inv_perm, void *workspace, size_t workspace_bytes,
                         void *stream) {
    if (!desc) return BM_ERR_NULL;
    int rc = check_group_desc(desc);
    if (rc) return rc;
    if (!offsets || (desc->T > 0 && (!ids_remapped || !perm || !inv_perm))) return BM_ERR_NULL;   // empty batch: offsets only
    const int T = desc->T, K = desc->K, E = desc->E;
    const GroupLayout L = make_group_layout(T, E);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % ALIGN) || workspace_bytes < L.total) return BM_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    (void)hipGetLastError();
    int err = 0;
    if (!grouping_small((long long)T * K, E))       // the small-batch kernel counts for itself
        err = launch_count(ids_remapped, T, K, E, TILE_T, at<int32_t>(workspace, L.tile_counts), st);
    ScanParams sp{};
    sp.T = T; sp.E = E; sp.n_shared = 0; sp.n_tiles = L.n_tiles;
    sp.BM = 1 << 30;                                // one table entry per live group: the table is not an output
    sp.tile_counts = at<int32_t>(workspace, L.tile_counts);
    sp.tile_base = at<int32_t>(workspace, L.tile_base);
    sp.tile_stats = nullptr;
    sp.offsets = offsets;
    sp.mt_group = at<int32_t>(workspace, L.mt_group);
    sp.mt_row0 = at<int32_t>(workspace, L.mt_row0);
    sp.n_mtiles = at<int32_t>(workspace, L.n_mtiles);
    sp.stats = nullptr;
    ScatterParams cp{};
    cp.T = T; cp.K = K; cp.E = E; cp.n_shared = 0; cp.tile_tokens = TILE_T;
    cp.ids = ids_remapped; cp.offsets = offsets; cp.tile_base = sp.tile_base;
    cp.perm = perm; cp.inv_perm = inv_perm; cp.row_token = nullptr;
    err |= launch_grouping(sp, cp, st);
    return err ? BM_ERR_HIP : BM_OK;
}

int bm_moe_forward_static(const bm_layer_desc *desc, const void *x, const bm_weights *wt,
                          const uint64_t *residency_bitmap, const int32_t *buddy_table, void *y,
                          const bm_debug_out *dbg, void *stream) {
    int rc = check_moe_args(desc, x, wt, residency_bitmap, buddy_table, y);
    if (rc) return rc;
    if (desc->T == 0) return BM_OK;
    if (make_layout(desc).total > (size_t)BM_STATIC_WORKSPACE_BYTES) return BM_ERR_WORKSPACE;
    void *ws = nullptr;
    rc = static_scratch_ptr(&ws);
    if (rc) return rc;
    return bm_moe_forward(desc, x, wt, residency_bitmap, buddy_table, y, ws, BM_STATIC_WORKSPACE_BYTES, dbg, stream);
}

int bm_moe_forward(const bm_layer_desc *desc, const void *x, const bm_weights *wt,
                   const uint64_t *residency_bitmap, const int32_t *buddy_table, void *y, void *workspace,
                   size_t workspace_bytes, const bm_debug_out *dbg, void *stream) {
    int rc = check_moe_args(desc, x, wt, residency_bitmap, buddy_table, y);
    if (rc) return rc;
    if (desc->T == 0) return BM_OK;
    Layout L;
    rc = check_ws(desc, workspace, workspace_bytes, L);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    void *ws = workspace;
    const int T = desc->T, K = desc->K, E = desc->E, G = E + desc->n_shared;
    const bool bf16 = desc->dtype == BM_BF16;
    int err = 0;
    (void)hipGetLastError();   // errors left by earlier, unrelated HIP calls are not ours

    hipEvent_t ev[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
    if (dbg && dbg->stage_events[0])
        for (int i = 0; i < 5; ++i) {
            if (!dbg->stage_events[i]) return BM_ERR_NULL;
            ev[i] = static_cast<hipEvent_t>(dbg->stage_events[i]);
        }
    auto mark = [&](int i) { if (ev[i]) err |= (hipEventRecord(ev[i], st) != hipSuccess); };

    // 1. router, gates, substitution, per-tile histograms
    mark(0);
    FrontParams fp{};
    fp.x = x; fp.wr = wt->w_router; fp.bias = wt->router_bias;
    fp.T = T; fp.d = desc->d; fp.E = E; fp.K = K; fp.R = desc->R; fp.H = desc->H; fp.flags = desc->flags;
    fp.tau = desc->tae_tau; fp.gamma = desc->margin_gamma; fp.rho = desc->rho; fp.beta = desc->dist_beta;
    fp.q = wt->buddy_q; fp.eta = desc->psi_eta; fp.probs_out = nullptr;
    fp.ids = at<int32_t>(ws, L.ids); fp.w = at<float>(ws, L.w);
    fp.bitmap = residency_bitmap; fp.table = buddy_table;
    fp.ids2 = at<int32_t>(ws, L.ids2);
    fp.tile_counts = at<int32_t>(ws, L.tile_counts);
    fp.tile_stats = at<int32_t>(ws, L.tile_stats);
    const bool fuse = front_can_fuse(T, desc->dtype, desc->flags);
    fp.tile_tokens = front_tile_tokens(T, desc->dtype, fuse);

    // 2. offsets, tile bases, row-tile table, statistics
    ScanParams sp{};
    const bool skinny = use_skinny(desc);
    sp.T = T; sp.E = E; sp.n_shared = desc->n_shared;
    sp.n_tiles = (T + fp.tile_tokens - 1) / fp.tile_tokens;   // tiles of the front kernel (per-tile statistics)
    const bool persistent = !skinny && bf16 && persistent_device();
    const int mode_gu = skinny ? (1 << 20) : tile_mode(desc, false, persistent);   // skinny: one table entry per live group
    const int mode_dn = skinny ? (1 << 20) : tile_mode(desc, true, persistent);
    // the plain table serves whichever projection runs a single tile height (both, unless one is mixed)
    sp.BM = mode_gu != TILES_MIXED ? mode_gu : (mode_dn != TILES_MIXED ? mode_dn : 256);
    if (mode_gu == TILES_MIXED || mode_dn == TILES_MIXED) {
        sp.mixed = 1;
        sp.mt_group_b = at<int32_t>(ws, L.mt_group_b); sp.mt_row0_b = at<int32_t>(ws, L.mt_row0_b);
        sp.n_mtiles_b = at<int32_t>(ws, L.n_mtiles_b);
        sp.mt_group_s = at<int32_t>(ws, L.mt_group_s); sp.mt_row0_s = at<int32_t>(ws, L.mt_row0_s);
        sp.n_mtiles_s = at<int32_t>(ws, L.n_mtiles_s);
    }
    sp.largest_first = skinny ? 1 : 0;
    sp.tile_counts = fp.tile_counts; sp.tile_base = at<int32_t>(ws, L.tile_base);
    sp.tile_stats = fp.tile_stats;
    sp.offsets = at<int32_t>(ws, L.offsets);
    sp.mt_group = at<int32_t>(ws, L.mt_group); sp.mt_row0 = at<int32_t>(ws, L.mt_row0);
    sp.n_mtiles = at<int32_t>(ws, L.n_mtiles);
    sp.stats = at<int32_t>(ws, L.stats);

    // 3. stable placement
    ScatterParams cp{};
    cp.T = T; cp.K = K; cp.E = E; cp.n_shared = desc->n_shared; cp.tile_tokens = fp.tile_tokens;
    cp.ids = fp.ids2; cp.offsets = sp.offsets; cp.tile_base = sp.tile_base;
    cp.perm = at<int32_t>(ws, L.perm); cp.inv_perm = at<int32_t>(ws, L.inv_perm);
    cp.row_token = at<int32_t>(ws, L.row_token);
    if (fuse) {                                // decode-sized batch: one kernel does steps 1-3
        fp.fused = 1;
        fp.scan = sp;
        fp.scat = cp;
        err |= launch_front(fp, desc->dtype, st);
    } else if (desc->flags & BM_GATE_DIST) {
        // the distribution gate needs every token's routing before the first substitution: route,
        // then substitute (each workgroup derives the batch's request set itself), then count
        FrontParams rp = fp;
        rp.bitmap = nullptr;
        const bool psi = (desc->flags & BM_PSI_TOKEN) != 0;
        if (psi) rp.probs_out = at<float>(ws, L.probs);
        err |= launch_front(rp, desc->dtype, st);
        RemapParams mp{};
        mp.T = T; mp.K = K; mp.E = E; mp.R = desc->R; mp.H = desc->H;
        mp.flags = desc->flags; mp.tau = fp.tau; mp.gamma = fp.gamma; mp.rho = fp.rho; mp.beta = fp.beta;
        mp.bitmap = residency_bitmap; mp.table = buddy_table;
        mp.q = fp.q; mp.eta = fp.eta; mp.probs = psi ? at<float>(ws, L.probs) : nullptr;
        mp.ids_in = fp.ids; mp.ids_out = fp.ids2; mp.w = fp.w; mp.stats = sp.stats;
        err |= launch_remap(mp, st);
        if (!grouping_small((long long)T * K, E)) err |= launch_count(fp.ids2, T, K, E, fp.tile_tokens, fp.tile_counts, st);
        ScanParams sq = sp;
        sq.tile_stats = nullptr; sq.stats = nullptr;      // written by the substitution kernel
        err |= launch_grouping(sq, cp, st);
    } else if (desc->dtype == BM_BF16 && sp.n_tiles == 1) {
        fp.tail = 1;                           // a single tile: its workgroup finishes the grouping too
        fp.scan = sp;
        fp.scat = cp;
        err |= launch_front(fp, desc->dtype, st);
    } else {
        err |= launch_front(fp, desc->dtype, st);
        err |= launch_grouping(sp, cp, st);
    }
    mark(1);

    // 4. gate/up projection + SwiGLU, 5. down projection
    GemmParams gp{};
    gp.a = x; gp.row_map = cp.row_token; gp.a_rows = T;
    gp.b0 = wt->w_gate; gp.b1 = wt->w_up; gp.sb0 = wt->ws_gate; gp.sb1 = wt->ws_up;
    gp.c = at<void>(ws, L.h);
    gp.N = desc->F; gp.Kd = desc->d; gp.E = E; gp.n_groups = G; gp.max_mtiles = L.mtiles_max; gp.BM = sp.BM;
    gp.mt_group = sp.mt_group; gp.mt_row0 = sp.mt_row0; gp.n_mtiles = sp.n_mtiles; gp.offsets = sp.offsets;
    GemmParams dp = gp;
    auto use_mixed = [&](GemmParams &q) {
        q.mixed = 1; q.BM = 256;
        q.mt_group = sp.mt_group_b; q.mt_row0 = sp.mt_row0_b; q.n_mtiles = sp.n_mtiles_b;
        q.mt_group_s = sp.mt_group_s; q.mt_row0_s = sp.mt_row0_s; q.n_mtiles_s = sp.n_mtiles_s;
    };
    if (mode_gu == TILES_MIXED) use_mixed(gp);
    if (mode_dn == TILES_MIXED) use_mixed(dp);
    dp.a = gp.c; dp.row_map = nullptr; dp.a_rows = L.rows_max;
    dp.b0 = wt->w_down; dp.b1 = nullptr; dp.sb0 = wt->ws_down; dp.sb1 = nullptr;
    dp.c = at<void>(ws, L.o);
    dp.N = desc->d; dp.Kd = desc->F;
    dp.splitk = L.has_splitk ? at<float>(ws, L.splitk) : nullptr;
    int ksplit = 1;
    bool combined = false;                              // the down projection has written y itself
    if (skinny) {
        ksplit = skinny_ksplit(desc);
        SkinnyParams s1{};
        s1.a = x; s1.row_map = cp.row_token;
        s1.b0 = wt->w_gate; s1.b1 = wt->w_up; s1.sb0 = wt->ws_gate; s1.sb1 = wt->ws_up;
        // packed copies are used only when every group of the layer has one
        const bool pk_gu = wt->wp_gateup && (desc->n_shared == 0 || wt->wsp_gateup);
        const bool pk_dn = wt->wp_down && (desc->n_shared == 0 || wt->wsp_down);
        s1.pk = pk_gu ? wt->wp_gateup : nullptr; s1.spk = pk_gu ? wt->wsp_gateup : nullptr;
        s1.c = gp.c; s1.N = desc->F; s1.Kd = desc->d; s1.E = E;
        s1.max_groups = G < L.mtiles_max ? G : L.mtiles_max;
        s1.ksplit = 1; s1.rows_max = L.rows_max; s1.max_rows_per_group = T * K;
        // 128 rows per pass when big groups are likely (measured on the 8- and the 128-expert layer: the gate/up
        // projection gains from 8 rows per expert on average, the down projection from 16)
        s1.wide = (T > 64 && (long long)T * K >= 8ll * E) ? 1 : 0;
        s1.mt_group = sp.mt_group; s1.n_mtiles = sp.n_mtiles; s1.offsets = sp.offsets;
        SkinnyParams s2 = s1;
        s2.a = gp.c; s2.row_map = nullptr;
        s2.b0 = wt->w_down; s2.b1 = nullptr; s2.sb0 = wt->ws_down; s2.sb1 = nullptr;
        s2.pk = pk_dn ? wt->wp_down : nullptr; s2.spk = pk_dn ? wt->wsp_down : nullptr;
        s2.c = dp.c; s2.N = desc->d; s2.Kd = desc->F; s2.ksplit = ksplit;
        s2.wide = (T > 64 && (long long)T * K >= 16ll * E) ? 1 : 0;
        // small batches on a matrix as many 16-row blocks wide as the device has units: the down kernel
        // aggregates its own results (null y: it writes them out for launch_combine below)
        s2.y = y; s2.w = fp.w; s2.inv_perm = cp.inv_perm; s2.T = T; s2.K = K; s2.n_shared = desc->n_shared;
        s2.y_f32 = (desc->flags & BM_Y_F32) ? 1 : 0;
        combined = skinny_down_fuses_combine(s2);
        if (!combined) s2.y = nullptr;
        err |= launch_skinny_gateup_bf16(s1, st);
        mark(2);
        err |= launch_skinny_down_bf16(s2, st);
    } else if (bf16) {
        err |= launch_gateup_bf16(gp, st);
        mark(2);
        err |= launch_down_bf16(dp, st);
    } else {
        err |= launch_gateup_f32(gp, L.rows_max, st);
        mark(2);
        err |= launch_down_f32(dp, L.rows_max, st);
    }
    mark(3);

    // 6. aggregation
    CombineParams mp{};
    mp.T = T; mp.d = desc->d; mp.K = K; mp.E = E; mp.n_shared = desc->n_shared;
    mp.ksplit = ksplit; mp.slice_stride = (size_t)L.rows_max * desc->d;
    mp.o = dp.c; mp.w = fp.w; mp.inv_perm = cp.inv_perm; mp.offsets = sp.offsets;
    mp.y = y; mp.y_f32 = (!bf16 || (desc->flags & BM_Y_F32)) ? 1 : 0;
    if (!combined) err |= launch_combine(mp, bf16 && !skinny, st);
    mark(4);

    if (dbg) {
        const size_t A = (size_t)T * K;
        if (dbg->ids) copy_ints(fp.ids, dbg->ids, A, st);
        if (dbg->ids_remapped) copy_ints(fp.ids2, dbg->ids_remapped, A, st);
        if (dbg->w) copy_ints(fp.w, dbg->w, A, st);
        if (dbg->offsets) copy_ints(sp.offsets, dbg->offsets, (size_t)E + 1, st);
        if (dbg->perm) copy_ints(cp.perm, dbg->perm, A, st);
        if (dbg->inv_perm) copy_ints(cp.inv_perm, dbg->inv_perm, A, st);
        if (dbg->stats) copy_ints(sp.stats, dbg->stats, 6, st);
        err |= launch_status("debug copies");
    }
    return err ? BM_ERR_HIP : BM_OK;
}

}  // extern "C"
