// Decode-sized groups (a handful of rows per expert): the projections are
// bound by streaming the weights from HBM once.  Each wave owns 16 weight rows
// and walks the reduction dimension; a weight row block is loaded from global
// memory straight into the A operand of v_mfma_f32_16x16x32_bf16 (lane l
// supplies row l % 16 and the 8 consecutive k starting at 8 * (l / 16): one
// 16-byte load, 64 contiguous bytes per row per instruction) and is used
// exactly once, so it never passes through LDS.  The few activation rows are
// the B operand (lane l: row l % 16, same k piece) and come from L2.
//   DUAL  : W_gate and W_up rows of the same f range, epilogue h = silu(g)*u
//   !DUAL : W_down rows, the reduction dimension is split over `ksplit`
//           workgroups that write fp32 partial sums, added up in slice order
//           by the aggregation kernel (deterministic, no atomics).
#include "bm_kernels.h"

namespace bm {

typedef __attribute__((ext_vector_type(4))) uint16_t u16x4;

__device__ __forceinline__ u32x4 ldg128_stream(const void *p) {
    return __builtin_nontemporal_load((const BM_GLOBAL u32x4 *)p);
}

// One pass over up to 16*NBT activation rows.  The reduction loop handles U
// k-steps (of 32) per trip: all loads of the trip are issued first, so each
// wave keeps U * (1 or 2) KB of weights in flight, then the MFMAs drain them.
template <bool DUAL, int NBT, int U>
__device__ __forceinline__ void skinny_pass(const SkinnyParams &p, const uint16_t *w0, const uint16_t *w1,
                                            int row_begin, int row_end, int k_begin, int k_end, int n0,
                                            int kslice, int rot) {
    const int lane = threadIdx.x & 63, lr = lane & 15, lk = lane >> 4;
    const uint16_t *a = static_cast<const uint16_t *>(p.a);
    const uint16_t *xa[NBT];
#pragma unroll
    for (int tb = 0; tb < NBT; ++tb) {
        const int pos = min(row_begin + tb * 16 + lr, row_end - 1);
        const int src = p.row_map ? ldg_i32(p.row_map + pos) : pos;
        xa[tb] = a + (size_t)src * p.Kd + lk * 8;
    }
    f32x4 acc0[NBT], acc1[NBT];
#pragma unroll
    for (int tb = 0; tb < NBT; ++tb) {
        acc0[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc1[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // Trips are visited in rotated order, a different phase per wave: weight
    // rows are a multiple of the memory-channel interleave apart, so waves
    // marching in step at the same k would all queue on the same channels.
    const int ntrips = (k_end - k_begin) / (U * 32);
    int trip = ntrips ? rot % ntrips : 0;
    for (int it = 0; it < ntrips; ++it) {
        const int k = k_begin + trip * (U * 32);
        trip = (trip + 1 == ntrips) ? 0 : trip + 1;
        u32x4 rw0[U], rw1[U], rx[NBT][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            rw0[u] = ldg128_stream(w0 + k + u * 32);
            if (DUAL) rw1[u] = ldg128_stream(w1 + k + u * 32);
        }
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb)
#pragma unroll
            for (int u = 0; u < U; ++u) rx[tb][u] = ldg128(xa[tb] + k + u * 32);
        __builtin_amdgcn_sched_barrier(0);            // keep every load of the trip ahead of the first MFMA
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb) {
                acc0[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(rw0[u]), as_bf16x8(rx[tb][u]), acc0[tb], 0, 0, 0);
                if (DUAL)
                    acc1[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(rw1[u]), as_bf16x8(rx[tb][u]), acc1[tb], 0, 0, 0);
            }
    }
    for (int k = k_begin + ntrips * (U * 32); k < k_end; k += 32) {   // tail: fewer than U k-steps left
        const bf16x8 a0 = as_bf16x8(ldg128_stream(w0 + k));
        bf16x8 a1;
        if (DUAL) a1 = as_bf16x8(ldg128_stream(w1 + k));
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb) {
            const bf16x8 xb = as_bf16x8(ldg128(xa[tb] + k));
            acc0[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, xb, acc0[tb], 0, 0, 0);
            if (DUAL) acc1[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, xb, acc1[tb], 0, 0, 0);
        }
    }
    // D[i][j]: lane holds column j = l % 16 (activation row) and rows i = 4*(l/16) + 0..3 (weight rows)
#pragma unroll
    for (int tb = 0; tb < NBT; ++tb) {
        const int pos = row_begin + tb * 16 + lr;
        if (pos >= row_end) continue;
        const int n = n0 + lk * 4;
        if (DUAL) {
            u16x4 h;
#pragma unroll
            for (int i = 0; i < 4; ++i) h[i] = f32_to_bf16(silu(acc0[tb][i]) * acc1[tb][i]);
            *(BM_GLOBAL u16x4 *)(static_cast<uint16_t *>(p.c) + (size_t)pos * p.N + n) = h;
        } else {
            float *c = static_cast<float *>(p.c) + ((size_t)kslice * p.rows_max + pos) * p.N + n;
            *(BM_GLOBAL f32x4 *)c = acc0[tb];
        }
    }
}

// grid.x = n-blocks of 64 weight rows (4 waves x 16), grid.y = live-group slots, grid.z = k slices
// MAXNBT bounds the 16-row blocks one pass can hold (a launch-time bound from
// T and K, so small batches do not carry the registers of the widest pass).
template <bool DUAL, int MAXNBT>
__global__ void __launch_bounds__(256) skinny_bf16_kernel(SkinnyParams p) {
    const int gi = blockIdx.y;
    if (gi >= p.n_mtiles[0]) return;                 // the row-tile table lists each live group once
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lr = lane & 15, lk = lane >> 4;
    const int n0 = (blockIdx.x * 4 + wave) * 16;
    if (n0 >= p.N) return;
    const int g = p.mt_group[gi];
    const int row_begin = p.offsets[g], row_end = p.offsets[g + 1];
    const int kslice = blockIdx.z;
    const int ksteps = p.Kd >> 5;
    const int per = (ksteps + p.ksplit - 1) / p.ksplit;
    const int k_begin = kslice * per * 32, k_end = min(p.Kd, (kslice + 1) * per * 32);

    const size_t gofs = (size_t)(g < p.E ? g : g - p.E) * p.N * p.Kd;
    const uint16_t *b0 = static_cast<const uint16_t *>(g < p.E ? p.b0 : p.sb0) + gofs;
    const uint16_t *w0 = b0 + (size_t)(n0 + lr) * p.Kd + lk * 8;
    const uint16_t *w1 = nullptr;
    if (DUAL) {
        const uint16_t *b1 = static_cast<const uint16_t *>(g < p.E ? p.b1 : p.sb1) + gofs;
        w1 = b1 + (size_t)(n0 + lr) * p.Kd + lk * 8;
    }
    const int rot = (n0 >> 4) * 5 + gi * 3 + kslice;
    constexpr int PASS_ROWS = 16 * MAXNBT;
    for (int rb = row_begin; rb < row_end; rb += PASS_ROWS) {
        const int re = min(row_end, rb + PASS_ROWS);
        const int n_rows = re - rb;
        if (MAXNBT == 1 || n_rows <= 16) skinny_pass<DUAL, 1, 8>(p, w0, w1, rb, re, k_begin, k_end, n0, kslice, rot);
        else if (MAXNBT == 2 || n_rows <= 32) skinny_pass<DUAL, 2, 4>(p, w0, w1, rb, re, k_begin, k_end, n0, kslice, rot);
        else skinny_pass<DUAL, 4, 4>(p, w0, w1, rb, re, k_begin, k_end, n0, kslice, rot);
    }
}

template <bool DUAL>
static void launch_skinny(const SkinnyParams &p, dim3 grid, hipStream_t st) {
    if (p.max_rows_per_group <= 16) hipLaunchKernelGGL((skinny_bf16_kernel<DUAL, 1>), grid, dim3(256), 0, st, p);
    else if (p.max_rows_per_group <= 32) hipLaunchKernelGGL((skinny_bf16_kernel<DUAL, 2>), grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL((skinny_bf16_kernel<DUAL, 4>), grid, dim3(256), 0, st, p);
}

int launch_skinny_gateup_bf16(const SkinnyParams &p, hipStream_t st) {
    dim3 grid((p.N / 16 + 3) / 4, p.max_groups, 1);
    launch_skinny<true>(p, grid, st);
    return launch_status(__func__);
}

int launch_skinny_down_bf16(const SkinnyParams &p, hipStream_t st) {
    dim3 grid((p.N / 16 + 3) / 4, p.max_groups, p.ksplit);
    launch_skinny<false>(p, grid, st);
    return launch_status(__func__);
}

}  // namespace bm
