// Grouped bf16 projections on MFMA for gfx950 (prefill-sized groups).
//
// Rows are the surviving assignments, grouped by expert; a row-tile table
// built on the device says which group each tile of BM rows belongs to.  One
// workgroup computes BM rows x 256 weight rows with fp32 accumulators (v_mfma_f32_16x16x32_bf16 in the
// main kernel - per flop it draws less power than the 32 x 32 x 16 form, and these kernels run against
// the chip's power limit - v_mfma_f32_32x32x16_bf16 in the fallbacks):
//   DUAL  : the 256 weight rows are 128 rows of W_gate and the same 128 rows
//           of W_up; the epilogue writes h = silu(g) * u as bf16.
//   !DUAL : 256 rows of W_down; the epilogue writes the product as bf16.
// Both operands have the reduction dimension contiguous, so a lane's MFMA
// operand (8 consecutive k) is one 16-byte piece of a row.
//
// Kernels, in the order the launchers prefer them:
//   grouped_gemm_mixed_k64w      persistent, k-steps of 64 with whole-line direct-to-LDS loads,
//                                v_mfma_f32_16x16x32_bf16; 256-row tiles plus one 128-row tile for a group's
//                                rest of at most 128 rows, both heights in one launch
//   grouped_gemm256_k64w         the same tile loop on 256-row tiles only, with a reduction-split tail: the
//                                down projection of long reductions
//   grouped_gemm256_dma          BM = 256, k-steps of 32 (reduction not a multiple of 64, offsets beyond
//                                32 bits, or a device that is not the full part)
//   grouped_gemm_bf16_kernel     BM = 128, 4 waves, register-staged double buffer, for groups too small
//                                for 256-row tiles on those shapes
// LDS rows of 128 bytes: the 64 banks span two rows, so piece p of row r is stored at slot
// p ^ ((r >> 1) & 7); the 16 lanes of one ds_read_b128 pass (16 rows, same p) then hit 16 distinct
// 16-byte slots (measured: zero bank-conflict cycles).
#include "bm_kernels.h"
#include "bm_device_shape.h"
#include "bm_tile_dealer.h"

namespace bm {

constexpr int G_BN = 256, G_BK = 64;

// Logical tile id -> (row tile, column tile).  The 32 workgroups that run together on one XCD (its
// 32 compute units take consecutive ids) form a block of GM row tiles x 32/GM column tiles, so they
// share GM activation tiles and 32/GM weight panels in that XCD's L2 instead of 32 + 1.
constexpr int G_GM = 4;
__device__ __forceinline__ void tile_of(int lid, int n_mt, int n_nt, int &mt, int &nt) {
    const int per_group = G_GM * n_nt;
    const int group = lid / per_group, in_group = lid - group * per_group;
    const int first = group * G_GM;
    const int gsize = min(n_mt - first, G_GM);
    nt = in_group / gsize;
    mt = first + (in_group - nt * gsize);
}

__device__ __forceinline__ int lds_slot(int row, int piece) { return row * G_BK + ((piece ^ ((row >> 1) & 7)) << 3); }

template <bool DUAL, int BM>
__global__ void __launch_bounds__(256) grouped_gemm_bf16_kernel(GemmParams p) {
    constexpr int THREADS = 256;                    // 4 waves, 2 x 2
    constexpr int WN = 2;                           // waves along the weight rows (2 along the rows)
    constexpr int AI = BM / 2 / 32;                 // 32-row blocks per wave
    constexpr int BJ = G_BN / WN / 32;              // 32-column blocks per wave
    constexpr int RSTEP = THREADS / 8;              // tile rows covered by one round of 16-byte loads
    constexpr int NA = BM / RSTEP, NB = G_BN / RSTEP;
    __shared__ __attribute__((aligned(16))) uint16_t sA[2][BM * G_BK];
    __shared__ __attribute__((aligned(16))) uint16_t sB[2][G_BN * G_BK];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int r32 = lane & 31, half = lane >> 5;

    // tile scheduling: consecutive logical tiles stay on one XCD (workgroups
    // are dealt round-robin to the 8 XCDs); see tile_of for the order inside
    const int n_mt = p.n_mtiles[0];
    const int n_nt = DUAL ? (p.N + 127) / 128 : (p.N + 255) / 256;
    const int total = n_mt * n_nt;
    const int per_xcd = (total + 7) >> 3;
    const int lid = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || lid >= total) return;
    int mt, nt;
    tile_of(lid, n_mt, n_nt, mt, nt);

    const int g = p.mt_group[mt];
    const int row0 = p.mt_row0[mt];
    const int row_end = p.offsets[g + 1];
    const int n0 = nt * (DUAL ? 128 : 256);
    const int N = p.N, Kd = p.Kd;

    const uint16_t *a = static_cast<const uint16_t *>(p.a);
    const uint16_t *b0, *b1;
    if (g < p.E) {
        b0 = static_cast<const uint16_t *>(p.b0) + (size_t)g * N * Kd;
        b1 = DUAL ? static_cast<const uint16_t *>(p.b1) + (size_t)g * N * Kd : nullptr;
    } else {
        b0 = static_cast<const uint16_t *>(p.sb0) + (size_t)(g - p.E) * N * Kd;
        b1 = DUAL ? static_cast<const uint16_t *>(p.sb1) + (size_t)(g - p.E) * N * Kd : nullptr;
    }

    // per-thread global sources and LDS destinations
    const int lrow = tid >> 3, chunk = tid & 7;
    const uint16_t *pa[NA];
    const uint16_t *pb[NB];
    int sa_off[NA], sb_off[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int r = lrow + RSTEP * i;
        const int pos = min(row0 + r, row_end - 1);
        const int src = p.row_map ? p.row_map[pos] : pos;
        pa[i] = a + (size_t)src * Kd + chunk * 8;
        sa_off[i] = lds_slot(r, chunk);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int rb = lrow + RSTEP * i;
        if (DUAL) {
            const int f = min(n0 + (rb & 127), N - 1);
            pb[i] = ((rb >> 7) ? b1 : b0) + (size_t)f * Kd + chunk * 8;
        } else {
            const int n = min(n0 + rb, N - 1);
            pb[i] = b0 + (size_t)n * Kd + chunk * 8;
        }
        sb_off[i] = lds_slot(rb, chunk);
    }

    f32x16 acc[AI][BJ];
#pragma unroll
    for (int i = 0; i < AI; ++i)
#pragma unroll
        for (int j = 0; j < BJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // operand rows of this wave inside the tile
    int a_row[AI], b_row[BJ];
#pragma unroll
    for (int i = 0; i < AI; ++i) a_row[i] = wm * (BM / 2) + i * 32 + r32;
#pragma unroll
    for (int j = 0; j < BJ; ++j)
        b_row[j] = DUAL ? ((j / (BJ / 2)) * 128 + wn * (128 / WN) + (j % (BJ / 2)) * 32 + r32)
                        : (wn * (G_BN / WN) + j * 32 + r32);

    const int KT = (Kd + G_BK - 1) / G_BK;
    u32x4 ra[NA], rb[NB];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

#define BM_LOAD_GLOBAL(kt_)                                                                        \
    {                                                                                              \
        const int k0_ = (kt_) * G_BK;                                                              \
        const bool in_ = (k0_ + chunk * 8) < Kd;                                                   \
        _Pragma("unroll") for (int i = 0; i < NA; ++i) ra[i] = in_ ? ldg128(pa[i] + k0_) : zero4;  \
        _Pragma("unroll") for (int i = 0; i < NB; ++i) rb[i] = in_ ? ldg128(pb[i] + k0_) : zero4;  \
    }
#define BM_STORE_LDS(buf_)                                                                         \
    {                                                                                              \
        _Pragma("unroll") for (int i = 0; i < NA; ++i)                                             \
            *reinterpret_cast<u32x4 *>(&sA[buf_][sa_off[i]]) = ra[i];                              \
        _Pragma("unroll") for (int i = 0; i < NB; ++i)                                             \
            *reinterpret_cast<u32x4 *>(&sB[buf_][sb_off[i]]) = rb[i];                              \
    }

    BM_LOAD_GLOBAL(0);
    BM_STORE_LDS(0);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) BM_LOAD_GLOBAL(kt + 1);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int piece = kk * 2 + half;
            bf16x8 fa[AI], fb[BJ];
#pragma unroll
            for (int i = 0; i < AI; ++i)
                fa[i] = as_bf16x8(*reinterpret_cast<const u32x4 *>(&sA[buf][lds_slot(a_row[i], piece)]));
#pragma unroll
            for (int j = 0; j < BJ; ++j)
                fb[j] = as_bf16x8(*reinterpret_cast<const u32x4 *>(&sB[buf][lds_slot(b_row[j], piece)]));
#pragma unroll
            for (int i = 0; i < AI; ++i)
#pragma unroll
                for (int j = 0; j < BJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) BM_STORE_LDS(buf ^ 1);
        __syncthreads();
    }
#undef BM_LOAD_GLOBAL
#undef BM_STORE_LDS

    // epilogue.  D[i][j]: lane holds column j = l % 32, rows 8*(v/4) + 4*(l/32) + v%4
    uint16_t *c = static_cast<uint16_t *>(p.c);
#pragma unroll
    for (int i = 0; i < AI; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = row0 + wm * (BM / 2) + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
            if (row >= row_end) continue;
            if (DUAL) {
#pragma unroll
                for (int jj = 0; jj < BJ / 2; ++jj) {
                    const int f = n0 + wn * (128 / WN) + jj * 32 + r32;
                    if (f < N)
                        stg16(&c[(size_t)row * N + f], f32_to_bf16(silu(acc[i][jj][v]) * acc[i][BJ / 2 + jj][v]));
                }
            } else {
#pragma unroll
                for (int j = 0; j < BJ; ++j) {
                    const int n = n0 + wn * (G_BN / WN) + j * 32 + r32;
                    if (n < N) stg16(&c[(size_t)row * N + n], f32_to_bf16(acc[i][j][v]));
                }
            }
        }
    }
}

// 256-row tiles with k-steps of 32: LDS rows are 64 bytes (4 pieces); the 64 banks span 4 rows, so piece p
// of row r sits at slot p ^ ((r >> 2) & 3).
constexpr int L_BK = 32, L_BM = 256, L_STAGE = (L_BM + G_BN) * L_BK;   // bf16 elements per stage

__device__ __forceinline__ int lds_slot32(int row, int piece) { return row * L_BK + ((piece ^ ((row >> 2) & 3)) << 3); }

// ---------------------------------------------------------------------------
// Fallback for reductions that are a multiple of 32 but not of 64.  256 rows x 256 weight rows per
// workgroup, 4 waves (2 x 2) with wave tiles of 128 x 128; the tiles go from global memory straight into
// LDS (global_load_lds_dwordx4: each lane's 16 bytes land at M0 + 16 * lane, so
// one instruction fills 16 tile rows of 64 bytes; the swizzle is applied by
// choosing which piece a lane fetches).  No staging registers, no LDS-write
// instructions, and a 5-stage ring over the whole 160 KB of LDS: the loads of
// tile kt+4 are issued in iteration kt and first needed three iterations later.
// Its 64-byte row pieces use half of every cache line they fetch, which is what
// the k-step-64 kernels below avoid.
//   iteration kt:  wait until tile kt+1 has landed (at most the 16 loads of tiles
//   kt+2, kt+3 outstanding) -> barrier (every wave's part of tile kt+1 is in LDS
//   and every wave is done with stage (kt-1)%5) -> issue tile kt+4 into stage
//   (kt+4)%5 -> MFMAs on stage kt%5, reading the first fragments of tile kt+1
//   under the last MFMAs.
// The compiler does not order LDS reads after these loads by itself, so the
// waits are explicit s_waitcnt vmcnt(n) and the barrier is a bare s_barrier.
// Needs Kd divisible by 32.
// ---------------------------------------------------------------------------
#define BM_LDS __attribute__((address_space(3)))
// s_waitcnt with only vmcnt set (gfx9 encoding: vmcnt[3:0] | expcnt 7 << 4 | lgkmcnt 15 << 8 | vmcnt[5:4] << 14)
#define BM_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))
#define BM_BARE_BARRIER() asm volatile("s_barrier" ::: "memory")

template <bool DUAL>
__global__ void __launch_bounds__(256) grouped_gemm256_dma_bf16_kernel(GemmParams p) {
    __shared__ __attribute__((aligned(1024))) uint16_t smem[5 * L_STAGE];        // 160 KB: the whole LDS
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r32 = lane & 31, half = lane >> 5;

    const int n_mt = p.n_mtiles[0];
    const int n_nt = DUAL ? (p.N + 127) / 128 : (p.N + 255) / 256;
    const int total = n_mt * n_nt;
    const int per_xcd = (total + 7) >> 3;
    const int lid = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || lid >= total) return;
    int mt, nt;
    tile_of(lid, n_mt, n_nt, mt, nt);

    const int g = p.mt_group[mt];
    const int row0 = p.mt_row0[mt];
    const int row_end = p.offsets[g + 1];
    const int n0 = nt * (DUAL ? 128 : 256);
    const int N = p.N, Kd = p.Kd;

    const uint16_t *a = static_cast<const uint16_t *>(p.a);
    const uint16_t *b0, *b1;
    if (g < p.E) {
        b0 = static_cast<const uint16_t *>(p.b0) + (size_t)g * N * Kd;
        b1 = DUAL ? static_cast<const uint16_t *>(p.b1) + (size_t)g * N * Kd : nullptr;
    } else {
        b0 = static_cast<const uint16_t *>(p.sb0) + (size_t)(g - p.E) * N * Kd;
        b1 = DUAL ? static_cast<const uint16_t *>(p.sb1) + (size_t)(g - p.E) * N * Kd : nullptr;
    }

    // Load instruction j of this wave fills the 1 KB block (4*j + wave) of a stage: blocks 0..15 are
    // the A tile (16 rows each), 16..31 the B tile.  Lane i supplies row 16*block + i/4, LDS slot i%4,
    // i.e. global piece (i%4) ^ ((row >> 2) & 3) = (i & 3) ^ ((i >> 4) & 3).
    const int piece = (lane & 3) ^ ((lane >> 4) & 3);
    const uint16_t *ps[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = 16 * (4 * j + wave) + (lane >> 2);         // row inside the 256-row tile
        const int pos = min(row0 + r, row_end - 1);
        const int src = p.row_map ? p.row_map[pos] : pos;
        ps[j] = a + (size_t)src * Kd + piece * 8;
        if (DUAL) {
            const int f = min(n0 + (r & 127), N - 1);
            ps[4 + j] = ((r >> 7) ? b1 : b0) + (size_t)f * Kd + piece * 8;
        } else {
            const int n = min(n0 + r, N - 1);
            ps[4 + j] = b0 + (size_t)n * Kd + piece * 8;
        }
    }

    int fa_off[2][4], fb_off[2][4];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ar = wm * 128 + i * 32 + r32;
            const int br = DUAL ? ((i >> 1) * 128 + wn * 64 + (i & 1) * 32 + r32) : (wn * 128 + i * 32 + r32);
            fa_off[kk][i] = lds_slot32(ar, kk * 2 + half);
            fb_off[kk][i] = L_BM * L_BK + lds_slot32(br, kk * 2 + half);
        }

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int KT = Kd / L_BK;
    bf16x8 f0a[4], f0b[4], f1a[4], f1b[4];

// tile_ -> stage_: 8 direct-to-LDS loads per wave
#define BM_DMA(stage_, tile_)                                                                      \
    {                                                                                              \
        const int k0_ = min((tile_), KT - 1) * L_BK;                                               \
        uint16_t *st_ = smem + (stage_) * L_STAGE + wave * 512;                                    \
        _Pragma("unroll") for (int j = 0; j < 8; ++j)                                              \
            __builtin_amdgcn_global_load_lds((const BM_GLOBAL void *)(ps[j] + k0_),                \
                                             (BM_LDS void *)(st_ + ((j >> 2) * 16 + 4 * (j & 3)) * 512), 16, 0, 0); \
    }
#define BM_FREAD(fa_, fb_, stage_, kk_)                                                    \
    {                                                                                      \
        const uint16_t *st_ = smem + (stage_) * L_STAGE;                                   \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                      \
            fa_[i] = as_bf16x8(*reinterpret_cast<const u32x4 *>(st_ + fa_off[kk_][i]));    \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                      \
            fb_[i] = as_bf16x8(*reinterpret_cast<const u32x4 *>(st_ + fb_off[kk_][i]));    \
    }
#define BM_MFMA16(fa_, fb_)                                                                \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                          \
        _Pragma("unroll") for (int j = 0; j < 4; ++j)                                      \
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa_[i], fb_[j], acc[i][j], 0, 0, 0);

    // prologue: tiles 0..3 in flight, tile 0 landed, its first fragments loaded
    BM_DMA(0, 0);
    BM_DMA(1, 1);
    BM_DMA(2, 2);
    BM_DMA(3, 3);
    BM_WAIT_VMCNT(24);
    BM_BARE_BARRIER();
    BM_FREAD(f0a, f0b, 0, 0);

    int s_cur = 0, s_nxt = 1, s_wr = 4;                // stage being multiplied, the next one, the free one
    for (int kt = 0; kt < KT; ++kt) {
        BM_WAIT_VMCNT(16);                             // tile kt+1 has landed (this wave's part)
        BM_BARE_BARRIER();                             // ... and everybody's; stage s_wr is free
        BM_FREAD(f1a, f1b, s_cur, 1);
        BM_DMA(s_wr, kt + 4);
        BM_MFMA16(f0a, f0b);
        BM_FREAD(f0a, f0b, s_nxt, 0);
        BM_MFMA16(f1a, f1b);
        _Pragma("unroll") for (int q = 0; q < 8; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read (f1)
        }
        _Pragma("unroll") for (int q = 0; q < 8; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // direct-to-LDS load
        }
        _Pragma("unroll") for (int q = 0; q < 8; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read (next f0)
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
        s_wr = s_cur;
        s_cur = s_nxt;
        s_nxt = (s_nxt == 4) ? 0 : s_nxt + 1;
    }
    BM_WAIT_VMCNT(0);                                  // no load may land in LDS after this workgroup is gone
#undef BM_DMA
#undef BM_FREAD
#undef BM_MFMA16

    uint16_t *c = static_cast<uint16_t *>(p.c);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = row0 + wm * 128 + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
            if (row >= row_end) continue;
            if (DUAL) {
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const int f = n0 + wn * 64 + jj * 32 + r32;
                    if (f < N) stg16(&c[(size_t)row * N + f], f32_to_bf16(silu(acc[i][jj][v]) * acc[i][2 + jj][v]));
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int n = n0 + wn * 128 + j * 32 + r32;
                    if (n < N) stg16(&c[(size_t)row * N + n], f32_to_bf16(acc[i][j][v]));
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// 256 x 256 tile with k-steps of 64 and direct-to-LDS loads that fetch whole
// 128-byte lines.  The vector cache moves one 128-byte line per two cycles
// whether a load uses all of it or half, so the 64-byte row pieces of a k-step
// of 32 cost twice the cache time of the MFMAs' data and leave the matrix cores
// waiting on load issue; here one load instruction covers 8 rows x 128 bytes.
// A k-step of 64 is two parts of 32 KB (the activation rows, the weight rows)
// and LDS holds five parts as a ring, ordered B(0) A(0) B(1) A(1) B(2) ...:
//   during k-step kt the slots hold B(kt) A(kt) B(kt+1) A(kt+1) B(kt+2).
//   One barrier per k-step, before its last 16 MFMAs (every wave has read its
//   last fragments of B(kt), A(kt) by then, and B(kt+1), A(kt+1) have landed);
//   after it A(kt+2) goes into B(kt)'s slot under the last 16 MFMAs, and B(kt+3)
//   into A(kt)'s slot spread under the next k-step's first 48 (bursts of loads
//   hold up a wave's MFMAs at issue: every instruction is hand-placed and fenced).
// LDS rows are 128 bytes, piece p of row r at slot p ^ ((r >> 1) & 7) (applied
// by choosing which global piece a lane fetches): conflict-free fragment reads.
// Needs Kd divisible by 64.
// ---------------------------------------------------------------------------
constexpr int P_PART = 256 * 64;                       // bf16 elements per part
// vmcnt and lgkmcnt in one s_waitcnt
#define BM_WAIT_VM_LGKM(vm, lgkm) \
    __builtin_amdgcn_s_waitcnt(((vm) & 15) | (7 << 4) | ((lgkm) << 8) | (((vm) >> 4) << 14))

// The tail of the persistent schedule.  An XCD's workgroups (stride of them) take its tiles round by
// round; when the last round is not full its `rem` tiles would keep rem workgroups busy for a whole tile
// time while the others idle.  For the down projection (long reduction, few rounds) each of those tiles
// is instead cut along the reduction into S = stride / rem chunks, one per workgroup; the chunks leave
// fp32 partial tiles in scratch memory and splitk_fixup_kernel adds them in chunk order.
struct TailSplit {
    int full;     // tiles of this XCD done in complete rounds
    int rem;      // tiles left for the last, partial round
    int S;        // chunks per tail tile (1: not split)
};
__device__ __forceinline__ TailSplit tail_split(int total, int per_xcd, int xcd, int stride, int KT, bool allowed) {
    TailSplit t;
    const int valid = max(0, min(per_xcd, total - xcd * per_xcd));
    t.full = valid / stride * stride;
    t.rem = valid - t.full;
    t.S = 1;
    // worth it only for long reductions: a chunk costs a 256 KB partial tile written and read back, which
    // a tile of fewer than 64 k-steps does not take long enough to repay
    if (allowed && t.rem > 0 && KT >= 64) {
        t.S = min(stride / t.rem, 8);
        while (t.S > 1 && KT / t.S < 16) --t.S;
        if (t.S < 1) t.S = 1;
    }
    return t;
}
constexpr int SPLIT_TILE_FLOATS = 256 * 256;

// table[idx] for a wave-uniform idx through the scalar cache.  Written out by hand because the compiler
// uses scalar loads only for memory it can prove unwritten since the kernel began; behind the first
// output store it reads such tables with vector loads, and waiting for one of those means waiting for
// every direct-to-LDS load issued before it.  The tables are written by an earlier launch.
__device__ __forceinline__ int scalar_load_i32(const int32_t *table, int idx) {
    int v;
    const int off = __builtin_amdgcn_readfirstlane(idx) * 4;
    // (early clobber: the result register is none of the address registers, as a replayed load would need)
    asm volatile("s_load_dword %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=&s"(v) : "s"(table), "s"(off) : "memory");
    return v;
}

// SPLIT: compile the reduction-split tail in (kept out of the other instantiations: its write-out of raw
// accumulators costs registers that short tiles cannot afford to spill around)
// MI: 16-row blocks per wave.  MI = 8 is the 256-row tile described above; MI = 4 is a 128-row tile on the
// same ring (the activation part fills half of its slot: four loads per wave and k-step instead of eight,
// 32 MFMAs per k slice instead of 64, the weight part unchanged), for layers whose groups are mostly
// smaller than a 256-row tile.
//
// PHASE: 0 - every row tile of the table has the height of this instantiation.  1 and 2 - one launch runs
// both heights (grouped_gemm_mixed_k64w_bf16_kernel): a group's rows are cut into 256-row tiles, and a rest
// of at most 128 rows becomes a 128-row tile; every workgroup first takes its share of the 256-row tiles
// (phase 1, the plain persistent order), then its share of the 128-row tiles (phase 2), which are dealt out
// so that the workgroups that got one 256-row tile fewer catch up first (next_small_tile).
__shared__ __attribute__((aligned(1024))) uint16_t k64w_smem[5 * P_PART];        // 160 KB: the whole LDS

template <bool DUAL, bool SPLIT, int MI, int PHASE>
__device__ __forceinline__ void k64w_body(const GemmParams &p) {
    uint16_t *const smem = k64w_smem;
    static_assert(MI == 8 || MI == 4, "tile height is 256 or 128 rows");
    static_assert(PHASE == 0 || (!SPLIT && MI == (PHASE == 1 ? 8 : 4)), "mixed heights: 256-row tiles first, then 128-row tiles");
    static_assert(!SPLIT || MI == 8, "the reduction-split tail exists for 256-row tiles only");
    constexpr int TM = MI * 32;                            // rows per tile
    constexpr int NM = MI * 8;                             // MFMAs per k slice of 32
    constexpr int NR = MI + 8;                             // fragment reads per k slice
    const int tid = threadIdx.x, lane = tid & 63;
    // the wave index as a scalar: everything derived from it (LDS targets of the loads, tile halves) then
    // stays in scalar registers and costs no vector instructions in the main loop
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int r16 = lane & 15, quad = lane >> 4;           // MFMA 16x16x32: row (or column) and k eighth

    // Persistent: workgroup b serves the XCD it was dealt to (b % 8) and walks that XCD's share of the
    // logical tiles with stride (workgroups per XCD), so the workgroups that run together on an XCD work
    // on consecutive logical tiles (see tile_of) and a workgroup keeps its compute unit: the next tile's
    // first loads fly while the finished tile is written out, and nothing is relaunched.
    const int32_t *const mt_group = PHASE == 2 ? p.mt_group_s : p.mt_group;
    const int32_t *const mt_row0 = PHASE == 2 ? p.mt_row0_s : p.mt_row0;
    const int n_mt = PHASE == 2 ? p.n_mtiles_s[0] : p.n_mtiles[0];
    const int n_nt = DUAL ? (p.N + 127) / 128 : (p.N + 255) / 256;
    const int total = n_mt * n_nt;
    const int per_xcd = (total + 7) >> 3;
    const int xcd = blockIdx.x & 7, stride = gridDim.x >> 3, slot = blockIdx.x >> 3;
    const int N = p.N, Kd = p.Kd;
    const int KT = Kd / 64;
    const TailSplit ts = tail_split(total, per_xcd, xcd, stride, KT, SPLIT && p.splitk != nullptr);
    SmallTileDealer dealer;
    if (PHASE == 2) {
        const int total_big = p.n_mtiles[0] * n_nt, per_xcd_big = (total_big + 7) >> 3;
        dealer.init(max(0, min(per_xcd_big, total_big - xcd * per_xcd_big)), max(0, min(per_xcd, total - xcd * per_xcd)),
                    stride, slot);
    }
    int idx = slot;                                    // next tile of the complete rounds
    bool tail_pending = ts.rem > 0;
    int kbeg = 0, kend = KT;                           // k-steps of the item whose loads are being issued
    bool partial = false;                              // that item is a chunk of a split tile
    int item_tile = 0;
// next work item of this workgroup -> item_tile, kbeg, kend, partial; false when there is none
#define BM_NEXT_ITEM(ok_)                                                                          \
    {                                                                                              \
        ok_ = false;                                                                               \
        if (PHASE == 2) {                                                                          \
            ok_ = dealer.next(item_tile);                                                          \
            kbeg = 0; kend = KT; partial = false;                                                  \
        } else if (idx < ts.full) {                                                                       \
            item_tile = idx; kbeg = 0; kend = KT; partial = false; idx += stride; ok_ = true;      \
        } else if (tail_pending) {                                                                 \
            tail_pending = false;                                                                  \
            if (ts.S >= 2) {                                                                       \
                if (slot < ts.rem * ts.S) {                                                        \
                    const int c_ = slot % ts.S;                                                    \
                    item_tile = ts.full + slot / ts.S;                                             \
                    kbeg = c_ * KT / ts.S; kend = (c_ + 1) * KT / ts.S; partial = true; ok_ = true; \
                }                                                                                  \
            } else if (slot < ts.rem) {                                                            \
                item_tile = ts.full + slot; kbeg = 0; kend = KT; partial = false; ok_ = true;      \
            }                                                                                      \
        }                                                                                          \
    }
    bool have;
    BM_NEXT_ITEM(have);
    if (!have) return;
    const uint16_t *a = static_cast<const uint16_t *>(p.a);
    uint16_t *c = static_cast<uint16_t *>(p.c);

    // fragment offsets inside a part, per 32-wide k slice s: row (.. + r16), piece 4*s + quad
    int fa_off[2], fb_off[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int pc = ((4 * s + quad) ^ ((r16 >> 1) & 7)) << 3;
        fa_off[s] = (wm * (MI * 16) + r16) * 64 + pc;
        fb_off[s] = (DUAL ? (wn * 64 + r16) : (wn * 128 + r16)) * 64 + pc;
    }

    f32x4 acc[MI][8];                                  // 16 x 16 tiles: rows i*16.., columns j*16..
    bf16x8 f0a[MI], f0b[8], f1a[MI], f1b[8];
    // Load addresses are (uniform base + k offset) + a 32-bit byte offset per lane, so that the k advance
    // is scalar arithmetic and a load needs no vector address computation.
    uint32_t oa[8], ob[8];
    const uint16_t *base_b0, *base_b1;
    int row0, row_end, n0;                             // of the tile whose loads are being issued
    int g_n, row0_n, row_end_n, n0_n;                  // of the tile looked up last (BM_LOOKUP)
                                                       // (the source rows of its activation loads: in v255)
    bool n_more = false, n_partial = false;            // the item the loads move on to next, found a k-step
    int n_kbeg = 0, n_kend = 0;                        // before they do

// Load instruction j of a wave fills the 1 KB block (4*j + wave) of a part: 8 tile rows of 128 bytes.  Lane i
// supplies row 8*block + i/8 and LDS slot i%8 of it, i.e. global piece (i % 8) ^ ((row >> 1) & 7).
// Moving the loads on to another tile takes two steps, a k-step apart:
// BM_LOOKUP(lid_): the tables of logical tile lid_ (scalar loads) and the source rows of the wave's
//   activation loads: 64 tile rows per wave, one per lane (lane l: the row load l/8 fetches for lanes
//   8 * (l%8) ..), ONE vector load of row_map.  Nothing the running loads use is touched.
// BM_ADOPT(): the load addresses of the tile looked up last; every lane picks up its eight source rows
//   from the lanes that loaded them (a lane permute; it moves data through the LDS crossbar and uses no
//   LDS memory).
// The row_map load is an assembly statement into a register the compiler does not manage (v255, named as
// clobbered so that it is allocated to the kernel; the compiler's own values stay far below it), i.e. the
// compiler neither waits for the result nor moves it.  Vector memory operations complete in issue order, so
// a wait for this load is a wait for every direct-to-LDS load issued before it; left to the compiler,
// look-up and use drained the load pipeline up to three times per tile (tile index -> group -> rows,
// dependent round trips), and given a k-step of distance it copied the pending value out of the result
// register at once and waited at the top of EVERY k-step.  By hand nothing waits at all: the look-up runs
// at the end of k-step kend - 4, BM_ADOPT at the end of k-step kend - 3, whose own wait in the middle (at
// most the 8 weight loads of its first half outstanding) has covered the row_map load.
// The lane index goes through an empty assembly statement in both: otherwise the compiler keeps the sixteen
// per-load row numbers of a lane alive across the whole tile loop, and spills them.
#define BM_LOOKUP(lid_)                                                                            \
    {                                                                                              \
        int mt_, nt_;                                                                              \
        tile_of((lid_), n_mt, n_nt, mt_, nt_);                                                     \
        g_n = scalar_load_i32(mt_group, mt_);                                                      \
        row0_n = scalar_load_i32(mt_row0, mt_);                                                    \
        row_end_n = scalar_load_i32(p.offsets, g_n + 1);                                           \
        n0_n = __builtin_amdgcn_readfirstlane(nt_) * (DUAL ? 128 : 256);                           \
        int lane_ = lane;                                                                          \
        asm volatile("" : "+v"(lane_));                                                            \
        const int r_ = 8 * (4 * (lane_ >> 3) + wave) + (lane_ & 7);                                \
        const int pos_ = min(row0_n + r_, row_end_n - 1);                                          \
        if (p.row_map)                                                                             \
            asm volatile("global_load_dword v255, %0, %1" : : "v"(pos_ * 4), "s"(p.row_map) : "v255", "memory"); \
        else                                                                                       \
            asm volatile("v_mov_b32 v255, %0" : : "v"(pos_) : "v255");                             \
    }
#define BM_ADOPT()                                                                                 \
    {                                                                                              \
        row0 = row0_n; row_end = row_end_n; n0 = n0_n;                                             \
        if (g_n < p.E) {                                                                           \
            base_b0 = static_cast<const uint16_t *>(p.b0) + (size_t)g_n * N * Kd;                  \
            base_b1 = DUAL ? static_cast<const uint16_t *>(p.b1) + (size_t)g_n * N * Kd : base_b0; \
        } else {                                                                                   \
            base_b0 = static_cast<const uint16_t *>(p.sb0) + (size_t)(g_n - p.E) * N * Kd;         \
            base_b1 = DUAL ? static_cast<const uint16_t *>(p.sb1) + (size_t)(g_n - p.E) * N * Kd : base_b0; \
        }                                                                                          \
        int lane_ = lane, rmv_;                                                                    \
        asm volatile("" : "+v"(lane_));                                                            \
        asm volatile("v_mov_b32 %0, v255" : "=v"(rmv_));                                           \
        _Pragma("unroll") for (int j = 0; j < 8; ++j) {                                            \
            const int r_ = 8 * (4 * j + wave) + (lane_ >> 3);                                      \
            const int piece_ = (lane_ & 7) ^ ((r_ >> 1) & 7);                                      \
            if (j < MI) {                                                                          \
                const int src_ = __builtin_amdgcn_ds_bpermute(4 * (8 * j + (lane_ >> 3)), rmv_);   \
                oa[j] = ((uint32_t)src_ * (uint32_t)Kd + piece_ * 8) * 2u;                         \
            }                                                                                      \
            /* DUAL: rows 0-127 of the part are W_gate rows (loads 0-3), rows 128-255 W_up rows (4-7) */ \
            const int n_ = DUAL ? min(n0 + (r_ & 127), N - 1) : min(n0 + r_, N - 1);               \
            ob[j] = ((uint32_t)n_ * (uint32_t)Kd + piece_ * 8) * 2u;                               \
        }                                                                                          \
    }
// load j_ of the activation part (A) / weight part (B) of k-step tile_ into slot_
#define BM_DMA_AT(base_, off_, slot_, tile_, j_)                                                   \
    __builtin_amdgcn_global_load_lds(                                                              \
        (const BM_GLOBAL void *)(reinterpret_cast<const char *>((base_) + min((tile_), kend - 1) * 64) + (off_)), \
        (BM_LDS void *)(smem + (slot_) * P_PART + wave * 512 + (j_) * 2048), 16, 0, 0)
#define BM_DMA_A(slot_, tile_, j_) BM_DMA_AT(a, oa[j_], slot_, tile_, j_)
#define BM_DMA_B(slot_, tile_, j_) BM_DMA_AT(((j_) < 4 ? base_b0 : base_b1), ob[j_], slot_, tile_, j_)
// B(0) A(0) B(1) A(1) of the tile set up last into slots 0..3
#define BM_PROLOGUE()                                                                              \
    {                                                                                              \
        _Pragma("unroll") for (int j = 0; j < 8; ++j) BM_DMA_B(0, kbeg, j);                        \
        _Pragma("unroll") for (int j = 0; j < MI; ++j) BM_DMA_A(1, kbeg, j);                       \
        _Pragma("unroll") for (int j = 0; j < 8; ++j) BM_DMA_B(2, kbeg + 1, j);                    \
        _Pragma("unroll") for (int j = 0; j < MI; ++j) BM_DMA_A(3, kbeg + 1, j);                   \
    }
#define BM_LD(ptr_) as_bf16x8(*reinterpret_cast<const u32x4 *>(ptr_))
// weight fragment j of 8: 16 weight rows; DUAL: fragments 0-3 are W_gate rows, 4-7 the same rows of W_up
#define BM_BOFF(j_) (DUAL ? (((j_) >> 2) * 8192 + ((j_) & 3) * 1024) : (j_) * 1024)
// fragment read d_ of NR, in the order the MFMAs need them: a0 b0..b7 a1..a(MI-1)
#define BM_RD(d_, fa_, fb_, sa_, sb_)                                                              \
    {                                                                                              \
        if ((d_) == 0) fa_[0] = BM_LD(sa_);                                                        \
        else if ((d_) <= 8) fb_[(d_) - 1] = BM_LD((sb_) + BM_BOFF((d_) - 1));                      \
        else fa_[(d_) - 8] = BM_LD((sa_) + ((d_) - 8) * 1024);                                     \
    }
// The MFMA is written as an assembly statement with the accumulator tied to an AGPR tile as input and
// output.  With the builtin the register allocator lets accumulator tiles change registers across the loop
// (down projection: a loop full of copies, measured 70 % slower) and copies all 256 accumulator values to
// vector registers where the loop ends (gate/up projection: up to 48 registers spilled around the
// write-out, and every reload from scratch memory waits for all loads and stores in flight).  The
// compiler's hazard recogniser does not see inside the statement, so the two distances it would otherwise
// guarantee are put in by hand, as s_nop statements that carry a data dependency on the accumulator
// concerned (an instruction-scheduling fence in those places makes the register allocator spill about 200
// registers):
//   - accumulator zeroing (VALU writes of the AGPRs) -> first MFMA, which reads acc[0][0] as its third
//     operand: at most 2 wait states are required on this family; 8 are inserted behind the zeroing
//     (a barrier and the first 16 fragment reads follow before that MFMA can issue anyway).  The zeroing of
//     the other accumulators cannot move closer to their first MFMA than that because the k-steps of a tile
//     form ONE loop and the zeroing stays in front of it.  Do not peel the first k-step off that loop: in
//     straight-line code the compiler sinks each accumulator's zeroing to right in front of its first MFMA,
//     which then reads the stale register (every 128-row tile came out wrong when this was tried; tying a
//     wait to all 64 accumulators instead made the allocator spill 128 registers);
//   - last MFMA of a tile (acc[MI - 1][7]) -> first read of an accumulator by another instruction (write-out,
//     partial-tile store): an 8-pass MFMA result needs 11 wait states (18 for a 16-pass one); 32 are
//     inserted where the write-out starts.  Every other accumulator's MFMA is at least 16 cycles older.
// Inside the loop an accumulator is next touched by its own MFMA 63 instructions later (same register as
// destination and third operand), which the MFMA pipeline interlocks by itself.
// Down projection: the weight fragment is the first operand, so the product comes out transposed, i.e. a
// lane holds four consecutive output columns (4 * quad ...) of one output row (r16), which pack into 8
// contiguous bytes (3-9 % faster through the shorter write-out; the gate/up projection measured 1-3 %
// slower with that order and keeps activations first).
#define BM_MFMA1(m_, fa_, fb_)                                                                     \
    {                                                                                              \
        if (DUAL)                                                                                  \
            asm("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0"                                          \
                : "+a"(acc[(m_) >> 3][(m_) & 7]) : "v"(fa_[(m_) >> 3]), "v"(fb_[(m_) & 7]));       \
        else                                                                                       \
            asm("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0"                                          \
                : "+a"(acc[(m_) >> 3][(m_) & 7]) : "v"(fb_[(m_) & 7]), "v"(fa_[(m_) >> 3]));       \
    }

    BM_LOOKUP(xcd * per_xcd + item_tile);
    BM_WAIT_VM_LGKM(0, 0);                             // the row_map load, which the compiler does not wait for
    BM_ADOPT();
    BM_PROLOGUE();
    // The ring runs on across tiles: during the last two k-steps of a tile the loads already fetch the
    // first two k-steps of the workgroup's next item (instead of repeats of the last k-step), so a new
    // tile starts with its operands in LDS and nothing is drained in between.
    int sB = 0, sA = 1, sAp = 4;                       // slots of B(kt), A(kt), and of A(kt-1) (free)
    // first tile: B(0) and A(0) have landed - vector memory operations complete in issue order and only
    // the loads of B(1), A(1) are younger
    BM_WAIT_VMCNT(8 + MI);
    for (;;) {
        const int t_row0 = row0, t_row_end = row_end, t_n0 = n0;    // the tile being multiplied
        const bool t_partial = partial;
        const int t_kbeg = kbeg, t_kend = kend;
        bool more = false;                             // the loads have moved on to a next item (uniform)
        // One tile: accumulators cleared, then the k-steps.  Written as a macro so that the down projection
        // can also instantiate it without the matrix work (COMPUTE_ = false, see below); the steps, in order:
        //  - barrier: every wave's part of B(0), A(0) is in LDS (first tile: the wait above; later tiles: they
        //    were waited for in the middle of the previous tile's last k-step), and every wave is done with the
        //    write-out staging in the slot the first loads of this tile will fill; first fragments read.
        //  - per k-step, kl = the k-step its loads fetch: two ahead, in the next item once this one is through.
        //  - first k slice of 32: 64 MFMAs; the second slice's fragments are read under MFMAs 0-31 (one read
        //    per two MFMAs), the 8 loads of B(kt+2) go into the slot A(kt-1) has left, one under every eighth
        //    MFMA (spread evenly: bunched loads hold up the MFMAs behind them at issue; measured 5 % on the
        //    whole kernel).
        //  - wait + barrier: every fragment of B(kt), A(kt) is in registers; A(kt+1), B(kt+1) have landed (this
        //    wave's part: at most the 8 loads of B(kt+2) are outstanding - whatever was issued before them, the
        //    previous tile's stores included, is complete); after the barrier both hold for every wave.
        //  - second slice: A(kt+2) goes into the slot B(kt) has left, one load under every eighth MFMA; the
        //    first fragments of k-step kt+1 are read under the first half, so that none of them is still in
        //    flight when the next k-step starts (after the last k-step of a tile they are the next tile's and
        //    are read again at its start: no register stays live across the write-out).
        //  - three k-steps before the end the loads of this item are all issued: from here on they fetch the
        //    next one, which was looked up a k-step earlier (BM_LOOKUP, BM_ADOPT).
#define BM_TILE_LOOP(COMPUTE_)                                                                                        \
    {                                                                                                                 \
        if (COMPUTE_) {                                                                                               \
            _Pragma("unroll") for (int i = 0; i < MI; ++i)                                                            \
                _Pragma("unroll") for (int j = 0; j < 8; ++j)                                                         \
                    _Pragma("unroll") for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.0f;                                \
            asm volatile("s_nop 7" : "+a"(acc[0][0]));  /* acc[0][0]: the first MFMA's accumulator */       \
        }                                                                                                             \
        BM_BARE_BARRIER();                                                                                            \
        {                                                                                                             \
            const uint16_t *sa_ = smem + sA * P_PART + fa_off[0];                                                     \
            const uint16_t *sb_ = smem + sB * P_PART + fb_off[0];                                                     \
        _Pragma("unroll")                                                                                             \
            for (int d = 0; (COMPUTE_) && d < NR; ++d) BM_RD(d, f0a, f0b, sa_, sb_)                                   \
        }                                                                                                             \
        for (int kt = t_kbeg; kt < t_kend; ++kt) {                                                                    \
            const int kl = more ? kbeg + (kt + 2 - t_kend) : kt + 2;                                                  \
            /* no LDS read is pending here (the last ones were issued half a k-step ago); said explicitly,  */        \
            /* because the compiler otherwise puts its own wait for the loop-carried fragments behind this */        \
            /* k-step's first read and the first MFMA stalls for an LDS round trip */                                 \
            BM_WAIT_VM_LGKM(63, 0);                                                                                   \
            {                                                                                                         \
                const uint16_t *sa_ = smem + sA * P_PART + fa_off[1];                                                 \
                const uint16_t *sb_ = smem + sB * P_PART + fb_off[1];                                                 \
        _Pragma("unroll")                                                                                             \
                for (int m = 0; m < NM; ++m) {                                                                        \
                    if (COMPUTE_) BM_MFMA1(m, f0a, f0b);                                                              \
                    if ((COMPUTE_) && m < 2 * NR && (m & 1) == 0) BM_RD(m >> 1, f1a, f1b, sa_, sb_)                   \
                    if (MI == 8 ? (m & 7) == 5 : (m & 3) == 1) BM_DMA_B(sAp, kl, MI == 8 ? m >> 3 : m >> 2);          \
                    __builtin_amdgcn_sched_barrier(0);                                                                \
                }                                                                                                     \
            }                                                                                                         \
            BM_WAIT_VM_LGKM(8, 0);                                                                                    \
            BM_BARE_BARRIER();                                                                                        \
            const int sBn = sB >= 3 ? sB - 3 : sB + 2, sAn = sA >= 3 ? sA - 3 : sA + 2;                               \
            {                                                                                                         \
                const uint16_t *sa_ = smem + sAn * P_PART + fa_off[0];                                                \
                const uint16_t *sb_ = smem + sBn * P_PART + fb_off[0];                                                \
        _Pragma("unroll")                                                                                             \
                for (int m = 0; m < NM; ++m) {                                                                        \
                    if (COMPUTE_) BM_MFMA1(m, f1a, f1b);                                                              \
                    if ((m & 7) == 1) BM_DMA_A(sB, kl, m >> 3);                                                       \
                    if ((COMPUTE_) && m < 2 * NR && (m & 1) == 0) BM_RD(m >> 1, f0a, f0b, sa_, sb_)                   \
                    __builtin_amdgcn_sched_barrier(0);                                                                \
                }                                                                                                     \
            }                                                                                                         \
            sAp = sA;                                                                                                 \
            sB = sBn;                                                                                                 \
            sA = sAn;                                                                                                 \
            if (kt == t_kend - 3) {                                                                                   \
                more = n_more;                                                                                        \
                if (more) {                                                                                           \
                    kbeg = n_kbeg; kend = n_kend; partial = n_partial;                                                \
                    BM_ADOPT();                                                                                       \
                }                                                                                                     \
            } else if (kt == t_kend - 4) {    /* every item has at least 4 k-steps */                                  \
                const int kb_ = kbeg, ke_ = kend;                                                                     \
                const bool pa_ = partial;                                                                             \
                BM_NEXT_ITEM(n_more);                                                                                 \
                n_kbeg = kbeg; n_kend = kend; n_partial = partial;                                                    \
                kbeg = kb_; kend = ke_; partial = pa_;                                                                \
                if (n_more) BM_LOOKUP(xcd * per_xcd + item_tile);                                                     \
            }                                                                                                         \
        }                                                                                                             \
    }
        // Down projection: a tile of at most 128 rows leaves the two waves of the lower row half nothing but
        // padding.  They keep their share of the loads, the waits and the barriers - the same instruction
        // stream minus every MFMA and fragment read - and skip the write-out: the chip runs these kernels
        // against its power limit, and what the idle matrix cores do not draw lets the others clock higher
        // (Qwen3-shaped layer, 41 % padding: down projection -6 %).  The gate/up instantiation keeps the single
        // loop (a second copy costs it registers and 2 % of its time).
        const bool live = DUAL || !(wm == 1 && t_row_end - t_row0 <= MI * 16);
        if (DUAL || live) BM_TILE_LOOP(true)
        else BM_TILE_LOOP(false)
#undef BM_TILE_LOOP
        // The tile is done.  The slot A(last k-step) sat in is free for every wave since the barrier in
        // the middle of that k-step; it stages the write-out while the next tile's loads land elsewhere.

        if (!live) {                                   // nothing but padding rows: nothing to write
            if (!more) break;
            continue;
        }
        // last MFMA of the tile -> first read of an accumulator (see BM_MFMA1): acc[MI - 1][7] is the last MFMA's
        // accumulator, every other one is at least one MFMA (16 cycles) older
        asm volatile("s_nop 15\n\ts_nop 15" : "+a"(acc[MI - 1][7]));
        if (SPLIT && t_partial) {
            // chunk of a split tile: the fp32 accumulators go to this workgroup's scratch tile as they are
            // (accumulator tile, lane: 16-byte stores, contiguous over the lanes)
            // (the address advances store by store behind an optimisation barrier: 64 addresses computed
            // up front cost registers, and the spills land in the main loop)
            float *dst = p.splitk + (size_t)(xcd * stride + slot) * SPLIT_TILE_FLOATS + wave * (64 * 256) + lane * 4;
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    *(BM_GLOBAL f32x4 *)dst = acc[i][j];
                    dst += 256;
                    asm volatile("" : "+v"(dst));
                }
            if (!more) break;
            continue;
        }

        // Write-out through the free slot (8 KB per wave).  Gate/up: an accumulator tile holds, per lane, four
        // rows of one column; 16 rows at a time are laid out row-major in LDS as bf16 - neighbouring lanes
        // swap one value so that every lane writes a packed pair - and read back as 16-byte pieces, so a
        // store instruction writes whole 128-byte lines.  A wave uses only its own region and LDS
        // operations of a wave stay in order.
        if (DUAL) {
            // gate/up: accumulator tiles are (row 4 * quad + v, column r16) - four rows of one column per lane
            constexpr int OC = 4;                       // 16-column output blocks per wave
            constexpr int SD = 36;                      // LDS row stride in dwords (padded against conflicts)
            constexpr int PR = OC * 2;                  // 16-byte pieces per output row
            uint32_t *stage = reinterpret_cast<uint32_t *>(smem + sAp * P_PART) + wave * 2048;
            // The accumulators are read one pair of values at a time, by hand and behind scheduling fences:
            // left to itself the compiler copies all 256 of them to vector registers where the loop ends
            // and spills what does not fit, and every reload waits for all stores issued so far.  The lane
            // index is hidden from it for the same reason (its derived constants stayed live across tiles).
            int lane_w = lane;
            asm volatile("" : "+v"(lane_w));
            const int r16 = lane_w & 15, quad = lane_w >> 4;
            const bool odd = lane_w & 1;
#pragma unroll
            for (int i = 0; i < MI; ++i) {
#pragma unroll
                for (int j = 0; j < OC; ++j) {
#pragma unroll
                    for (int v = 0; v < 4; v += 2) {
                        float g0, g1, u0, u1;
                        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(g0) : "a"(acc[i][j][v]));
                        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(g1) : "a"(acc[i][j][v + 1]));
                        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(u0) : "a"(acc[i][4 + j][v]));
                        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(u1) : "a"(acc[i][4 + j][v + 1]));
                        const float x0 = silu(g0) * u0;
                        const float x1 = silu(g1) * u1;
                        // even lane keeps row v and gets the right-hand neighbour's value of that row;
                        // odd lane keeps row v+1 and gets the left-hand neighbour's
                        const float send = odd ? x0 : x1;
                        const float recv = __builtin_bit_cast(
                            float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, true));
                        const uint32_t pk = odd ? pack_bf16x2(recv, x1) : pack_bf16x2(x0, recv);
                        const int lrow = 4 * quad + v + (odd ? 1 : 0);
                        stage[lrow * SD + j * 8 + (r16 >> 1)] = pk;
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int t = 0; t < PR / 4; ++t) {
                    const int q = lane_w + 64 * t;
                    const int lrow = q / PR, pc = q % PR;
                    const u32x4 val = *reinterpret_cast<const u32x4 *>(stage + lrow * SD + pc * 4);
                    const int row = t_row0 + wm * (MI * 16) + i * 16 + lrow;
                    const int col = t_n0 + wn * (OC * 16) + pc * 8;
                    if (row < t_row_end && col < N) stg128(&c[(size_t)row * N + col], val);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            // Down projection (weights as the first MFMA operand): an accumulator tile holds, per lane, four
            // consecutive columns of one row (row r16, columns 4 * quad ...), i.e. 8 contiguous bytes of
            // bf16: one LDS write per accumulator tile and no lane exchange.
            constexpr int OC = 8;                       // 16-column output blocks per wave
            constexpr int SD = 68;                      // LDS row stride in dwords (16-byte aligned, rows 4 banks apart)
            constexpr int PR = OC * 2;                  // 16-byte pieces per output row
            uint32_t *stage = reinterpret_cast<uint32_t *>(smem + sAp * P_PART) + wave * 2048;
#pragma unroll
            for (int i = 0; i < MI; ++i) {
#pragma unroll
                for (int j = 0; j < OC; ++j) {
                    float x[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v) x[v] = acc[i][j][v];
                    u32x2 pk;
                    pk[0] = pack_bf16x2(x[0], x[1]);
                    pk[1] = pack_bf16x2(x[2], x[3]);
                    *reinterpret_cast<u32x2 *>(stage + r16 * SD + j * 8 + 2 * quad) = pk;
                }
#pragma unroll
                for (int t = 0; t < PR / 4; ++t) {
                    const int q = lane + 64 * t;
                    const int lrow = q / PR, pc = q % PR;
                    const u32x4 val = *reinterpret_cast<const u32x4 *>(stage + lrow * SD + pc * 4);
                    const int row = t_row0 + wm * (MI * 16) + i * 16 + lrow;
                    const int col = t_n0 + wn * (OC * 16) + pc * 8;
                    if (row < t_row_end && col < N) stg128(&c[(size_t)row * N + col], val);
                }
            }
        }
        if (!more) break;
    }
    // the last tile's loads ran past its end (repeats of its last k-step): nothing may still be landing in
    // LDS when the workgroup ends
    BM_WAIT_VM_LGKM(0, 0);
#undef BM_LOOKUP
#undef BM_ADOPT
#undef BM_NEXT_ITEM
#undef BM_PROLOGUE
#undef BM_DMA_AT
#undef BM_DMA_A
#undef BM_DMA_B
#undef BM_LD
#undef BM_BOFF
#undef BM_RD
#undef BM_MFMA1
}

template <bool DUAL, bool SPLIT, int MI = 8>
__global__ void __launch_bounds__(256) grouped_gemm256_k64w_bf16_kernel(GemmParams p) {
    k64w_body<DUAL, SPLIT, MI, 0>(p);
}

// Both tile heights in one launch (see k64w_body): p.mt_group / mt_row0 / n_mtiles list the 256-row tiles,
// p.mt_group_s / mt_row0_s / n_mtiles_s the 128-row tiles.
template <bool DUAL>
__global__ void __launch_bounds__(256) grouped_gemm_mixed_k64w_bf16_kernel(GemmParams p) {
    // A 128-row tile is the only user of its weight panel (a group has at most one), so it streams from
    // memory at a third of a 256-row tile's arithmetic intensity.  When there are many of them (at least a
    // quarter of the 256-row tiles' number) every other workgroup takes its 128-row tiles first, so that the
    // streaming is spread over the launch instead of bunched at its end (Qwen3-shaped layer, 2048 tokens:
    // gate/up 141 -> 133 us); with few of them that order only delays 256-row tiles (Mixtral-shaped prefill
    // + 1 %, 1024 tokens + 3 %).
    const bool small_first = p.n_mtiles_s[0] * 4 >= p.n_mtiles[0] && ((blockIdx.x >> 3) & 1);
    if (small_first) {
        k64w_body<DUAL, false, 4, 2>(p);
        __syncthreads();      // the last write-out's staging area becomes the next phase's first load target
        k64w_body<DUAL, false, 8, 1>(p);
    } else {
        k64w_body<DUAL, false, 8, 1>(p);
        __syncthreads();
        k64w_body<DUAL, false, 4, 2>(p);
    }
}

// Adds the chunks of every split tail tile in chunk order and writes the bf16 result (see TailSplit).
// Grid (16 tail tiles, 8 XCDs, 16 slices of a tile): a workgroup handles one sixteenth of a tile - the
// accumulator tiles (i, j) with i * 8 + j in [4 * blockIdx.z, 4 * blockIdx.z + 4) - with the chunk
// writers' thread -> element mapping, so that the reduction itself is spread over the chip.
__global__ void __launch_bounds__(256) splitk_fixup_kernel(GemmParams p) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, r16 = lane & 15, quad = lane >> 4;
    const int n_mt = p.n_mtiles[0];
    const int n_nt = (p.N + 255) / 256;
    const int total = n_mt * n_nt;
    const int per_xcd = (total + 7) >> 3;
    const int xcd = blockIdx.y, stride = p.splitk_stride, t = blockIdx.x;
    const TailSplit ts = tail_split(total, per_xcd, xcd, stride, p.Kd / 64, true);
    if (ts.S < 2 || t >= ts.rem) return;
    int mt, nt;
    tile_of(xcd * per_xcd + ts.full + t, n_mt, n_nt, mt, nt);
    const int g = p.mt_group[mt];
    const int row0 = p.mt_row0[mt], row_end = p.offsets[g + 1], n0 = nt * 256, N = p.N;
    uint16_t *c = static_cast<uint16_t *>(p.c);
    const float *src = p.splitk + (size_t)(xcd * stride + t * ts.S) * SPLIT_TILE_FLOATS + wave * (64 * 256) + lane * 4;
    // all loads of the workgroup's share go out before the first sum (S <= 8 chunks, tail_split): one
    // round trip to memory instead of one per chunk
    f32x4 part[4][8];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int ch = 0; ch < 8; ++ch)
            if (ch < ts.S)
                part[q][ch] = *(const BM_GLOBAL f32x4 *)(src + (size_t)ch * SPLIT_TILE_FLOATS + (blockIdx.z * 4 + q) * 256);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int ij = blockIdx.z * 4 + q, i = ij >> 3, j = ij & 7;
        f32x4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int ch = 0; ch < 8; ++ch)
            if (ch < ts.S) sum += part[q][ch];
        // transposed accumulator tiles: the lane holds columns 4 * quad .. + 3 of row r16
        const int n = n0 + wn * 128 + j * 16 + 4 * quad;
        const int row = row0 + wm * 128 + i * 16 + r16;
        if (row < row_end && n < N) {
            u32x2 pk;
            pk[0] = pack_bf16x2(sum[0], sum[1]);
            pk[1] = pack_bf16x2(sum[2], sum[3]);
            *(BM_GLOBAL u32x2 *)(&c[(size_t)row * N + n]) = pk;
        }
    }
}

static int grid_for(const GemmParams &p, bool dual) {
    const int n_nt = dual ? (p.N + 127) / 128 : (p.N + 255) / 256;
    const int total = p.max_mtiles * n_nt;
    return ((total + 7) / 8) * 8;
}

// One workgroup per compute unit (a workgroup takes a whole unit's LDS), fewer when there are fewer tiles;
// always a multiple of 8 so that every XCD gets the same number.
static int persistent_grid(const GemmParams &p, bool dual) {
    const int g = grid_for(p, dual);
    return g < K64_CUS ? g : K64_CUS;
}

// compute units and XCDs of the current device (0, 0 if the queries fail)
static void device_shape(int &cus, int &xcds) {
    int dev = 0;
    cus = xcds = 0;
    if (hipGetDevice(&dev) != hipSuccess) return;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 0;
    if (hipDeviceGetAttribute(&xcds, hipDeviceAttributeNumberOfXccs, dev) != hipSuccess) xcds = 0;
}

bool persistent_device() {
    int cus, xcds;
    device_shape(cus, xcds);
    return persistent_schedule_fits(cus, xcds);
}

// the k-step-64 kernel addresses rows by 32-bit byte offsets from a uniform base, and its schedule is laid
// out for the full part (see bm_device_shape.h)
static bool k64_ok(const GemmParams &p) {
    const unsigned long long lim = 1ull << 32;
    if (!persistent_device()) return false;
    // (and hands the loads over to the next tile three k-steps before a tile ends)
    return p.BM == 256 && p.Kd % 64 == 0 && p.Kd >= 256 && (unsigned long long)p.a_rows * p.Kd * 2 < lim &&
           (unsigned long long)p.N * p.Kd * 2 < lim;
}

int launch_gateup_bf16(const GemmParams &p, hipStream_t st) {
    if (p.mixed && k64_ok(p))
        hipLaunchKernelGGL((grouped_gemm_mixed_k64w_bf16_kernel<true>), dim3(persistent_grid(p, true)), dim3(256), 0, st, p);
    else if (p.mixed)
        return -1;                // the caller asks for both tile heights only where the persistent kernel runs
    else if (p.BM == 256)
        hipLaunchKernelGGL((grouped_gemm256_dma_bf16_kernel<true>), dim3(grid_for(p, true)), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL((grouped_gemm_bf16_kernel<true, 128>), dim3(grid_for(p, true)), dim3(256), 0, st, p);
    return launch_status(__func__);
}

// the reduction-split tail (see TailSplit) pays only for long reductions
bool down_split_tail(int Kd) { return Kd / 64 >= 64; }

int launch_down_bf16(const GemmParams &p, hipStream_t st) {
    if (p.mixed && k64_ok(p)) {
        hipLaunchKernelGGL((grouped_gemm_mixed_k64w_bf16_kernel<false>), dim3(persistent_grid(p, false)), dim3(256), 0, st, p);
    } else if (p.mixed) {
        return -1;
    } else if (p.BM == 256 && p.splitk != nullptr && down_split_tail(p.Kd) && k64_ok(p)) {
        GemmParams q = p;
        q.splitk_stride = persistent_grid(p, false) >> 3;
        hipLaunchKernelGGL((grouped_gemm256_k64w_bf16_kernel<false, true>), dim3(persistent_grid(p, false)), dim3(256), 0, st, q);
        hipLaunchKernelGGL(splitk_fixup_kernel, dim3(16, 8, 16), dim3(256), 0, st, q);
    } else if (p.BM == 256) {
        hipLaunchKernelGGL((grouped_gemm256_dma_bf16_kernel<false>), dim3(grid_for(p, false)), dim3(256), 0, st, p);
    } else {
        hipLaunchKernelGGL((grouped_gemm_bf16_kernel<false, 128>), dim3(grid_for(p, false)), dim3(256), 0, st, p);
    }
    return launch_status(__func__);
}

}  // namespace bm
