// Internal interface between the C-ABI layer (bm_api.hip) and the kernel
// translation units.  Parameter blocks are plain structs passed by value.
#pragma once
#include "../../include/buddymoe.h"
#include "../../include/buddymoe_bench.h"
#include "bm_device.h"

namespace bm {

struct RemapParams {
    int T, K, E, R, H;
    uint32_t flags;         // BM_REMAP_UNIQUE and the gate bits
    float tau, gamma;       // TAE and margin thresholds
    int rho;                // replacement budget per token
    float beta;             // distribution-gate threshold
    const float *q;         // [E][R] q of the table entries (BM_PSI_TOKEN)
    float eta;
    const float *probs;     // [T][E] softmax probabilities of all experts (BM_PSI_TOKEN)
    const uint64_t *bitmap;
    const int32_t *table;
    const int32_t *ids_in;
    int32_t *ids_out;
    float *w;
    int32_t *stats;         // 6 ints or null
};

struct ScanParams {
    int T, E, n_shared, n_tiles, BM;
    int largest_first;            // small-batch kernel, one row tile per group: list the groups by falling row count
    const int32_t *tile_counts;   // [E][n_tiles]
    int32_t *tile_base;           // [E][n_tiles]
    const int32_t *tile_stats;    // [n_tiles][4] or null
    int32_t *offsets;             // [E + n_shared + 1]
    int32_t *mt_group, *mt_row0;  // row-tile table
    int32_t *n_mtiles;            // [2]: number of row tiles, total rows
    int mixed;                    // also write the two lists of a projection that runs 256- and 128-row tiles in one launch
    int32_t *mt_group_b, *mt_row0_b, *n_mtiles_b;   // its 256-row tiles
    int32_t *mt_group_s, *mt_row0_s, *n_mtiles_s;   // its 128-row tiles
    int32_t *stats;               // 3 ints or null
};

struct ScatterParams {
    int T, K, E, n_shared;
    int tile_tokens;              // tokens per tile of the histograms (the front kernel's or count kernel's tiles)
    const int32_t *ids;           // [T][K] after substitution
    const int32_t *offsets;       // [E + n_shared + 1]
    const int32_t *tile_base;     // [E][n_tiles]
    int32_t *perm, *inv_perm;     // [T*K]
    int32_t *row_token;           // [rows] or null
};

struct FrontParams {
    const void *x;          // [T][d]
    const void *wr;         // [E][d]
    const float *bias;      // [E] or null
    int T, d, E, K, R, H;
    uint32_t flags;
    float tau, gamma;       // TAE and margin thresholds (gate bits of flags)
    int rho;                // replacement budget per token
    float beta;             // distribution-gate threshold (BM_GATE_DIST: only when one tile holds the batch)
    const float *q;         // [E][R] q of the table entries (BM_PSI_TOKEN)
    float eta;
    float *probs_out;       // [T][E]: with BM_PSI_TOKEN, write every expert's probability (or null)
    int32_t *ids;           // [T][K] router's choice
    float *w;               // [T][K]
    const uint64_t *bitmap; // null => routing only (no substitution, no histogram)
    const int32_t *table;   // [E][R]
    int32_t *ids2;          // [T][K] after substitution
    int32_t *tile_counts;   // [E][n_tiles]
    int32_t *tile_stats;    // [n_tiles][4]
    int fused;              // one workgroup walks all tiles and also does the scan and the scatter
    int tail;               // not fused, a single tile: the workgroup also finishes the grouping (bf16 kernel)
    int tile_tokens;        // tokens per workgroup: TILE_T, or 16 for small batches (bf16 kernel, see front_tile_tokens)
    ScanParams scan;        // used when fused or tail
    ScatterParams scat;     // used when fused or tail
};


// Grouped projection C[rows][N] = A[rows][Kd] * B_g[N][Kd]^T over row tiles.
struct GemmParams {
    const void *a;                // activations: [T][Kd] gathered via row_map, or [rows][Kd]
    const int32_t *row_map;       // row -> row of a (null: identity)
    long long a_rows;             // rows of a (bound for 32-bit byte offsets)
    const void *b0, *b1;          // routed weights ([E][N][Kd]); b1 = second matrix (up) or null
    const void *sb0, *sb1;        // shared-expert weights ([n_shared][N][Kd])
    void *c;                      // [rows][N]
    int N, Kd, E;
    int n_groups;                 // E + n_shared
    int max_mtiles;               // grid bound on row tiles
    int BM;                       // rows per tile of the row-tile table: 128 or 256
    const int32_t *mt_group, *mt_row0, *n_mtiles, *offsets;
    int mixed;                    // both tile heights in one launch: the table above lists the 256-row tiles and
    const int32_t *mt_group_s, *mt_row0_s, *n_mtiles_s;   // ... this one the 128-row tiles
    float *splitk;                // scratch for the reduction-split tail of the down projection (or null)
    int splitk_stride;            // workgroups per XCD of the launch that wrote it
};

// Skinny (decode) projections: one weight-row block per wave, see bm_skinny_bf16.hip.
struct SkinnyParams {
    const void *a;                // activations [..][Kd] bf16
    const int32_t *row_map;       // row -> row of a (null: identity)
    const void *b0, *b1, *sb0, *sb1;
    const void *pk, *spk;         // fragment-major copies (routed, shared) from bm_pack_weights, or null
    void *c;                      // DUAL: bf16 [rows][N]; else fp32 [ksplit][rows_max][N]
    int N, Kd, E;
    int max_groups;               // grid bound on live groups
    int ksplit, rows_max;
    int max_rows_per_group;       // launch-time bound: T*K routed rows (or T for a shared expert)
    int wide;                     // groups of more than 64 rows are expected (more than 64 tokens): 128 rows per pass
    const int32_t *mt_group, *n_mtiles, *offsets;
    // down projection of the persistent kernel with the aggregation fused in (skinny_down_fuses_combine):
    void *y;                      // [T][N] layer output, or null: write c and leave the aggregation to launch_combine
    const float *w;               // [T][K] gate weights
    const int32_t *inv_perm;      // [T*K]
    int T, K, n_shared, y_f32;
};

struct CombineParams {
    int T, d, K, E, n_shared;
    int ksplit;                   // fp32 o: number of partial-sum slices to add (>= 1)
    size_t slice_stride;          // elements between slices
    const void *o;                // [rows][d] (bf16), or [ksplit][rows_max][d] (fp32)
    const float *w;               // [T][K]
    const int32_t *inv_perm;      // [T*K]
    const int32_t *offsets;       // [E + n_shared + 1]
    void *y;
    int y_f32;
};

// 0 if the launch just issued was accepted, -1 (and a line on stderr naming
// the kernel and the HIP error) otherwise
int launch_status(const char *what);

bool front_can_fuse(int T, int dtype, uint32_t flags);   // the batch is small enough for the one-workgroup front end
int front_tile_tokens(int T, int dtype, bool fused);   // tokens per workgroup of the front kernel
int launch_front(const FrontParams &p, int dtype, hipStream_t st);
int launch_remap(const RemapParams &p, hipStream_t st);
int launch_count(const int32_t *ids, int T, int K, int E, int tile_tokens, int32_t *tile_counts, hipStream_t st);
int launch_scan(const ScanParams &p, hipStream_t st);
int launch_scatter(const ScatterParams &p, hipStream_t st);
int launch_grouping(const ScanParams &sp, const ScatterParams &cp, hipStream_t st);   // scan + scatter (one kernel for small batches)
bool grouping_small(long long assignments, int E);   // launch_grouping takes the one-kernel path (and needs no tile histograms)

// bf16 MFMA grouped projections (row tile height p.BM, which the row-tile table was built for)
int launch_gateup_bf16(const GemmParams &p, hipStream_t st);   // c = silu(a b0^T) * (a b1^T), bf16
int launch_down_bf16(const GemmParams &p, hipStream_t st);     // c = a b0^T, bf16
bool persistent_device();       // the current device has the shape the persistent prefill kernels are laid out for
bool down_split_tail(int Kd);   // the down projection of this reduction width may use p.splitk (its split tail)

// fp32 FMA projections (one workgroup per row)
int launch_gateup_f32(const GemmParams &p, int max_rows, hipStream_t st);
int launch_down_f32(const GemmParams &p, int max_rows, hipStream_t st);

bool skinny_p_ok(int Kd, int ch);       // shape fits the persistent decode kernel with ring depth ch
bool skinny_lds_ok(int Kd, int ksplit); // shape fits the LDS-staged decode kernel
bool skinny_q_ok(int Kd, int ksplit);   // shape fits the quarter-split decode kernel
int launch_skinny_gateup_bf16(const SkinnyParams &p, hipStream_t st);
int launch_skinny_down_bf16(const SkinnyParams &p, hipStream_t st);
// launch_skinny_down_bf16(p) with p.y set will write the layer output itself (no launch_combine needed)
bool skinny_down_fuses_combine(const SkinnyParams &p);

int launch_combine(const CombineParams &p, bool o_bf16, hipStream_t st);
int launch_stream_read(const void *src, size_t bytes, uint32_t *sink, hipStream_t st);

// fragment-major repacking of n matrices [N][Kd] (two interleaved when src1 is given)
int launch_pack(const void *src0, const void *src1, void *dst, int n, int N, int Kd, const uint64_t *bitmap,
                hipStream_t st);

// profiling statistics and buddy lists (bm_profile.hip)
int launch_coactivation(const int32_t *ids, int T, int K, int E, long long *A, long long *M, hipStream_t st);
int launch_buddy_build(const long long *M, int E, int R, float alpha, int32_t *table, int32_t *list_len, float *q,
                       hipStream_t st);

}  // namespace bm
