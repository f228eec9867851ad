// Grouped bf16 projections on MFMA for gfx950 (prefill-sized groups).
//
// Rows are the surviving assignments, grouped by expert; a row-tile table
// built on the device says which group each tile of BM rows belongs to.  One
// workgroup (4 waves, 2x2) computes BM=128 rows x 256 weight rows with
// v_mfma_f32_32x32x16_bf16 and fp32 accumulators:
//   DUAL  : the 256 weight rows are 128 rows of W_gate and the same 128 rows
//           of W_up; the epilogue writes h = silu(g) * u as bf16.
//   !DUAL : 256 rows of W_down; the epilogue writes the product as bf16.
// Both operands have the reduction dimension contiguous, so a lane's MFMA
// operand (8 consecutive k) is one 16-byte piece of a row.  Tiles of BK=64
// are staged through LDS (16-byte pieces XOR-swizzled by row so that the
// 32-row operand reads are conflict-free), double-buffered, with the next
// tile's global loads in flight while the current one is multiplied.
#include "bm_kernels.h"

namespace bm {

constexpr int G_BM = 128, G_BN = 256, G_BK = 64, G_THREADS = 256;

int gemm_bf16_bm() { return G_BM; }

template <bool DUAL>
__global__ void __launch_bounds__(G_THREADS) grouped_gemm_bf16_kernel(GemmParams p) {
    __shared__ __attribute__((aligned(16))) uint16_t sA[2][G_BM * G_BK];
    __shared__ __attribute__((aligned(16))) uint16_t sB[2][G_BN * G_BK];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r32 = lane & 31, half = lane >> 5;

    // tile scheduling: consecutive logical tiles stay on one XCD (workgroups
    // are dealt round-robin to the 8 XCDs), row tiles vary fastest so that
    // the workgroups sharing one weight panel run together on one L2
    const int n_mt = p.n_mtiles[0];
    const int n_nt = DUAL ? (p.N + 127) / 128 : (p.N + 255) / 256;
    const int total = n_mt * n_nt;
    const int per_xcd = (total + 7) >> 3;
    const int lid = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || lid >= total) return;
    const int nt = lid / n_mt, mt = lid - nt * n_mt;

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

    // per-thread global sources: 4 pieces of the A tile, 8 of the B tile
    const int lrow = tid >> 3, chunk = tid & 7;
    const uint16_t *pa[4];
    const uint16_t *pb[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int pos = min(row0 + lrow + 32 * i, row_end - 1);
        int src = p.row_map ? p.row_map[pos] : pos;
        pa[i] = a + (size_t)src * Kd + chunk * 8;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int rb = lrow + 32 * i;
        if (DUAL) {
            const int f = min(n0 + (rb & 127), N - 1);
            pb[i] = ((rb >> 7) ? b1 : b0) + (size_t)f * Kd + chunk * 8;
        } else {
            const int n = min(n0 + rb, N - 1);
            pb[i] = b0 + (size_t)n * Kd + chunk * 8;
        }
    }
    // LDS destinations (swizzled): row r, piece (chunk ^ (r & 7))
    int sa_off[4], sb_off[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) { const int r = lrow + 32 * i; sa_off[i] = r * G_BK + ((chunk ^ (r & 7)) << 3); }
#pragma unroll
    for (int i = 0; i < 8; ++i) { const int r = lrow + 32 * i; sb_off[i] = r * G_BK + ((chunk ^ (r & 7)) << 3); }

    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // operand rows of this wave inside the tile
    int a_row[2], b_row[4];
#pragma unroll
    for (int i = 0; i < 2; ++i) a_row[i] = wm * 64 + i * 32 + r32;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        b_row[j] = DUAL ? ((j >> 1) * 128 + wn * 64 + (j & 1) * 32 + r32) : (wn * 128 + j * 32 + r32);

    const int KT = (Kd + G_BK - 1) / G_BK;
    u32x4 ra[4], rb[8];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

#define BM_LOAD_GLOBAL(kt_)                                                                         \
    {                                                                                              \
        const int k0_ = (kt_) * G_BK;                                                              \
        const bool in_ = (k0_ + chunk * 8) < Kd;                                                   \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                              \
            ra[i] = in_ ? ldg128(pa[i] + k0_) : zero4;                                            \
        _Pragma("unroll") for (int i = 0; i < 8; ++i)                                              \
            rb[i] = in_ ? ldg128(pb[i] + k0_) : zero4;                                            \
    }
#define BM_STORE_LDS(buf_)                                                                         \
    {                                                                                              \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                              \
            *reinterpret_cast<u32x4 *>(&sA[buf_][sa_off[i]]) = ra[i];                              \
        _Pragma("unroll") for (int i = 0; i < 8; ++i)                                              \
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
            bf16x8 fa[2], fb[4];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                fa[i] = as_bf16x8(*reinterpret_cast<const u32x4 *>(&sA[buf][a_row[i] * G_BK + ((piece ^ (a_row[i] & 7)) << 3)]));
#pragma unroll
            for (int j = 0; j < 4; ++j)
                fb[j] = as_bf16x8(*reinterpret_cast<const u32x4 *>(&sB[buf][b_row[j] * G_BK + ((piece ^ (b_row[j] & 7)) << 3)]));
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
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
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = row0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
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

static int grid_for(const GemmParams &p, bool dual) {
    const int n_nt = dual ? (p.N + 127) / 128 : (p.N + 255) / 256;
    const int total = p.max_mtiles * n_nt;
    return ((total + 7) / 8) * 8;
}

int launch_gateup_bf16(const GemmParams &p, hipStream_t st) {
    hipLaunchKernelGGL(grouped_gemm_bf16_kernel<true>, dim3(grid_for(p, true)), dim3(G_THREADS), 0, st, p);
    return launch_status(__func__);
}

int launch_down_bf16(const GemmParams &p, hipStream_t st) {
    hipLaunchKernelGGL(grouped_gemm_bf16_kernel<false>, dim3(grid_for(p, false)), dim3(G_THREADS), 0, st, p);
    return launch_status(__func__);
}

}  // namespace bm
