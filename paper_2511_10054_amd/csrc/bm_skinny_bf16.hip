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

// Hides a pointer's value from the optimiser at this point.  A kernel below inlines three instances
// of its pass (for 16, 32 and 64 activation rows); without this the address arithmetic of all of them
// is computed up front and kept live, which costs registers the two-workgroups-per-unit limit lacks.
#define BM_OPAQUE_PTR(ptr_) asm volatile("" : "+v"(ptr_))

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

// ---------------------------------------------------------------------------
// Main decode kernel.  One workgroup = 16 weight rows (of each matrix); its 4
// waves split the reduction into 4 contiguous quarters and meet in LDS at the
// end (partials added in wave order).  Work items are therefore small (a
// quarter of a row block per wave) and numerous, so the last round of
// workgroups on the chip is short - with whole row blocks per wave the tail
// round cost up to a third of the kernel.  No barrier inside the main loop.
// Weights and activations run through a rotating set of CH register slots: a
// slot is refilled with the k-step CH ahead right after the MFMAs that
// consumed it, so CH-1 of every CH slots are in flight.
// Needs (Kd / 32) divisible by 4 * CH * ksplit; other shapes use the kernel above.
// ---------------------------------------------------------------------------
constexpr int QCH = 8;

template <bool DUAL, int NBT>
__device__ __forceinline__ void skinny_q_pass(const SkinnyParams &p, const uint16_t *w0, const uint16_t *w1,
                                              f32x4 *red, int row_begin, int row_end, int k_begin, int k_end,
                                              int n0, int kslice) {
    constexpr int CH = QCH;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lr = lane & 15, lk = lane >> 4;
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
    u32x4 s0[CH], s1[CH], sx[NBT][CH];
#pragma unroll
    for (int u = 0; u < CH; ++u) {
        s0[u] = ldg128_stream(w0 + k_begin + u * 32);
        if (DUAL) s1[u] = ldg128_stream(w1 + k_begin + u * 32);
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb) sx[tb][u] = ldg128(xa[tb] + k_begin + u * 32);
    }
    // steady state: unconditional refills (branches around the loads would make the
    // order of outstanding loads ambiguous to the wait-count insertion)
    int k = k_begin;
    for (; k + 2 * CH * 32 <= k_end; k += CH * 32) {
#pragma unroll
        for (int u = 0; u < CH; ++u) {
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb) {
                acc0[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(s0[u]), as_bf16x8(sx[tb][u]), acc0[tb], 0, 0, 0);
                if (DUAL)
                    acc1[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(s1[u]), as_bf16x8(sx[tb][u]), acc1[tb], 0, 0, 0);
            }
            const int kn = k + (CH + u) * 32;
            s0[u] = ldg128_stream(w0 + kn);
            if (DUAL) s1[u] = ldg128_stream(w1 + kn);
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb) sx[tb][u] = ldg128(xa[tb] + kn);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // last chunk: drain
#pragma unroll
    for (int u = 0; u < CH; ++u)
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb) {
            acc0[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(s0[u]), as_bf16x8(sx[tb][u]), acc0[tb], 0, 0, 0);
            if (DUAL)
                acc1[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(s1[u]), as_bf16x8(sx[tb][u]), acc1[tb], 0, 0, 0);
        }

    // reduction over the 4 reduction quarters, in wave order
    if (wave > 0) {
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb) {
            red[((wave - 1) * NBT + tb) * 2 * 64 + lane] = acc0[tb];
            if (DUAL) red[((wave - 1) * NBT + tb) * 2 * 64 + 64 + lane] = acc1[tb];
        }
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb) {
#pragma unroll
            for (int w = 0; w < 3; ++w) {
                acc0[tb] += red[(w * NBT + tb) * 2 * 64 + lane];
                if (DUAL) acc1[tb] += red[(w * NBT + tb) * 2 * 64 + 64 + lane];
            }
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
}

// grid.x = 16-row blocks of the weight matrix, grid.y = live-group slots, grid.z = reduction slices
template <bool DUAL, int MAXNBT>
__global__ void __launch_bounds__(256) skinny_q_bf16_kernel(SkinnyParams p) {
    __shared__ f32x4 red[3 * MAXNBT * 2 * 64];
    const int gi = blockIdx.y;
    if (gi >= p.n_mtiles[0]) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lr = lane & 15, lk = lane >> 4;
    const int n0 = blockIdx.x * 16;
    const int g = p.mt_group[gi];
    const int row_begin = p.offsets[g], row_end = p.offsets[g + 1];
    const int kslice = blockIdx.z;
    const int per_wave = p.Kd / (4 * p.ksplit);        // host guarantees a multiple of 32 * QCH
    const int k_begin = (kslice * 4 + wave) * per_wave, k_end = k_begin + per_wave;

    const size_t gofs = (size_t)(g < p.E ? g : g - p.E) * p.N * p.Kd;
    const uint16_t *b0 = static_cast<const uint16_t *>(g < p.E ? p.b0 : p.sb0) + gofs;
    const uint16_t *w0 = b0 + (size_t)(n0 + lr) * p.Kd + lk * 8;
    const uint16_t *w1 = nullptr;
    if (DUAL) {
        const uint16_t *b1 = static_cast<const uint16_t *>(g < p.E ? p.b1 : p.sb1) + gofs;
        w1 = b1 + (size_t)(n0 + lr) * p.Kd + lk * 8;
    }
    constexpr int PASS_ROWS = 16 * MAXNBT;
    for (int rb = row_begin; rb < row_end; rb += PASS_ROWS) {
        const int re = min(row_end, rb + PASS_ROWS);
        const int n_rows = re - rb;
        if (MAXNBT == 1 || n_rows <= 16) skinny_q_pass<DUAL, 1>(p, w0, w1, red, rb, re, k_begin, k_end, n0, kslice);
        else if (MAXNBT == 2 || n_rows <= 32) skinny_q_pass<DUAL, 2>(p, w0, w1, red, rb, re, k_begin, k_end, n0, kslice);
        else skinny_q_pass<DUAL, 4>(p, w0, w1, red, rb, re, k_begin, k_end, n0, kslice);
        __syncthreads();                               // the next pass reuses the reduction buffer
    }
}

bool skinny_q_ok(int Kd, int ksplit) { return Kd % (4 * ksplit * 32 * QCH) == 0; }

template <bool DUAL>
static void launch_skinny_q(const SkinnyParams &p, hipStream_t st) {
    dim3 grid(p.N / 16, p.max_groups, p.ksplit);
    if (p.max_rows_per_group <= 16) hipLaunchKernelGGL((skinny_q_bf16_kernel<DUAL, 1>), grid, dim3(256), 0, st, p);
    else if (p.max_rows_per_group <= 32) hipLaunchKernelGGL((skinny_q_bf16_kernel<DUAL, 2>), grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL((skinny_q_bf16_kernel<DUAL, 4>), grid, dim3(256), 0, st, p);
}

// ---------------------------------------------------------------------------
// Decode kernel for larger groups (up to 64 rows per pass).  A workgroup's 4
// waves own 4 different 16-row weight blocks and walk the whole reduction
// together; the activation rows are staged by the workgroup in LDS in chunks
// of CH k-steps, already in MFMA B-operand order (one 1 KB fragment per
// k-step and 16-row block: contiguous ds_read_b128), double-buffered, so they
// cost each wave a quarter of the loads and no ring registers.  Weights run
// through the same rotating register ring as above.
// Needs Kd divisible by 256 * ksplit (chunks of 8 k-steps).
// ---------------------------------------------------------------------------
template <int NBT> struct SkinnyChunk { static constexpr int CH = 8; };
constexpr int KUNIT = 256;                             // one chunk: SkinnyChunk::CH k-steps of 32

// PACKED: the weights come from bm_pack_weights' fragment-major copy, where the 1 KB operand
// fragment of every (16-row block, k-step) is contiguous (gate and up fragments interleaved), so a
// wave's stream is one contiguous run; otherwise from the public row-major layout.
// Public layout (!PACKED): w0 / w1 point at weight row n0, and the rows are fetched as whole 128-byte lines
// - ring slots 2v and 2v + 1 hold rows 0-7 and 8-15 of line v (two k-steps) of the chunk, lane l row l / 8,
// 16-byte piece l % 8 - and turned into the two k-steps' operand fragments through `wst`, 2 KB of LDS per
// wave and matrix (pieces of a row rotated by the row index against bank conflicts; only the writing wave
// reads it, and a wave's LDS operations stay in order).  Loading the fragments directly, 16 rows x 64
// bytes per instruction, touches twice the cache lines, which bounds the kernel: 252 us against 191 us for
// the gate/up projection of the Mixtral-shaped layer at 64 tokens.
template <bool DUAL, int NBT, bool PACKED>
__device__ __forceinline__ void skinny_lds_pass(const SkinnyParams &p, const uint16_t *w0, const uint16_t *w1,
                                                u32x4 *xs, u32x4 *wst, int row_begin, int row_end, int k_begin,
                                                int k_end, int n0, int kslice, bool active) {
    constexpr int CH = SkinnyChunk<NBT>::CH;
    constexpr int KSTEP = 512 * (DUAL ? 2 : 1);         // packed copy: weight elements between consecutive k-steps
    constexpr int XW = CH / 4;                          // k-steps of a chunk each wave stages
    BM_OPAQUE_PTR(w0);
    BM_OPAQUE_PTR(w1);
    static_assert(XW % 2 == 0, "a wave stages whole 128-byte lines (two k-steps) of every activation row");
    constexpr int XL = XW / 2;                          // lines per row and chunk a wave stages
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lr = lane & 15, lk = lane >> 4;
    // public layout: this lane's place in the line loads (row 8j + l / 8, piece l % 8) and in the LDS area
    const uint16_t *wl0[2], *wl1[2];
    int wwr[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = 8 * j + (lane >> 3);
        wl0[j] = PACKED ? w0 : w0 + (size_t)r * p.Kd + (lane & 7) * 8;
        wl1[j] = (PACKED || !DUAL) ? w1 : w1 + (size_t)r * p.Kd + (lane & 7) * 8;
        wwr[j] = r * 8 + ((lane & 7) ^ (r & 7));
    }
    // ring slot u of the chunk that starts at reduction index kb_
#define BM_LOADW(wp_, wl_, u_, kb_)                                                        \
    (PACKED ? ldg128_stream((wp_) + ((kb_) >> 5) * KSTEP + (u_) * KSTEP)                   \
            : ldg128_stream((wl_)[(u_) & 1] + (kb_) + ((u_) >> 1) * 64))
    const uint16_t *a = static_cast<const uint16_t *>(p.a);
    // Staging loads are issued in whole lines: instruction j of row block tb reads rows 8j..8j+7, lane l
    // row 8j + l / 8 and 16-byte piece l % 8 of the line, i.e. k-step (l % 8) / 4 and quarter l % 4 of
    // that k-step.  (With the operand layout itself, 16 rows x 64 bytes per instruction, these loads
    // cost the vector memory path as much time as the weight stream they accompany.)
    const int q8 = lane >> 3, p8 = lane & 7;
    const uint16_t *xa[NBT][2];
#pragma unroll
    for (int tb = 0; tb < NBT; ++tb)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int pos = min(row_begin + tb * 16 + 8 * j + q8, row_end - 1);
            const int src = p.row_map ? ldg_i32(p.row_map + pos) : pos;
            xa[tb][j] = a + (size_t)src * p.Kd + (XW * wave) * 32 + p8 * 8;
        }
    // Place of (row r, quarter c) inside a 1 KB operand fragment in LDS: rows 64 bytes apart, the
    // quarters of a row rotated by the row's index / 4, so that neither the staging stores (8 rows x
    // 4 quarters) nor the operand reads (16 rows, one quarter) meet in a bank.
    int wslot[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = 8 * j + q8;
        wslot[j] = (p8 >> 2) * NBT * 64 + r * 4 + ((p8 & 3) ^ ((r >> 2) & 3));
    }
    const int rslot = lr * 4 + (lk ^ ((lr >> 2) & 3));
    f32x4 acc0[NBT], acc1[NBT];
#pragma unroll
    for (int tb = 0; tb < NBT; ++tb) {
        acc0[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc1[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    u32x4 s0[CH], s1[CH], xr[XL * 2 * NBT];
    const int nch = (k_end - k_begin) / (CH * 32);

#define BM_LOAD_X(k_)                                                                      \
    _Pragma("unroll") for (int li = 0; li < XL; ++li)                                      \
        _Pragma("unroll") for (int j = 0; j < 2; ++j)                                      \
            _Pragma("unroll") for (int tb = 0; tb < NBT; ++tb)                             \
                xr[(li * 2 + j) * NBT + tb] = ldg128(xa[tb][j] + (k_) + li * 64);
#define BM_STORE_X(buf_)                                                                   \
    _Pragma("unroll") for (int li = 0; li < XL; ++li)                                      \
        _Pragma("unroll") for (int j = 0; j < 2; ++j)                                      \
            _Pragma("unroll") for (int tb = 0; tb < NBT; ++tb)                             \
                xs[(((buf_) * CH + XW * wave + 2 * li) * NBT + tb) * 64 + wslot[j]] = xr[(li * 2 + j) * NBT + tb];

    BM_LOAD_X(k_begin);
#pragma unroll
    for (int u = 0; u < CH; ++u) {
        s0[u] = BM_LOADW(w0, wl0, u, k_begin);
        if (DUAL) s1[u] = BM_LOADW(w1, wl1, u, k_begin);
    }
    BM_STORE_X(0);
    __syncthreads();

// one chunk: consume slot u, then (REFILL_) refill it with the k-step CH ahead; the refill is
// unconditional inside the steady-state loop (see the note on wait counts in the kernel above)
#define BM_CHUNK(c_, REFILL_)                                                                        \
    {                                                                                                \
        const int kn_ = k_begin + ((c_) + 1) * (CH * 32);                                            \
        if (REFILL_) { BM_LOAD_X(kn_); }                                                             \
        {                                                                                            \
            const u32x4 *xc = xs + (size_t)((c_) & 1) * CH * NBT * 64 + rslot;                       \
            _Pragma("unroll") for (int u = 0; u < CH; ++u) {                                         \
                bf16x8 xb[NBT], wa, wb;                                                              \
                if (!PACKED && (u & 1) == 0) {      /* a line's two row groups -> LDS */            \
                    _Pragma("unroll") for (int j = 0; j < 2; ++j) {                                  \
                        wst[wwr[j]] = s0[u + j];                                                     \
                        if (DUAL) wst[128 + wwr[j]] = s1[u + j];                                     \
                    }                                                                                \
                }                                                                                    \
                if (PACKED) {                                                                        \
                    wa = as_bf16x8(s0[u]);                                                           \
                    wb = as_bf16x8(s1[DUAL ? u : 0]);                                                \
                } else {                                                                             \
                    const int rs_ = lr * 8 + ((((u) & 1) * 4 + lk) ^ (lr & 7));                      \
                    wa = as_bf16x8(wst[rs_]);                                                        \
                    wb = as_bf16x8(wst[(DUAL ? 128 : 0) + rs_]);                                     \
                }                                                                                    \
                _Pragma("unroll") for (int tb = 0; tb < NBT; ++tb)                                   \
                    xb[tb] = as_bf16x8(xc[(u * NBT + tb) * 64]);                                     \
                _Pragma("unroll") for (int tb = 0; tb < NBT; ++tb) {                                 \
                    acc0[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, xb[tb], acc0[tb], 0, 0, 0); \
                    if (DUAL)                                                                        \
                        acc1[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb, xb[tb], acc1[tb], 0, 0, 0); \
                }                                                                                    \
                if (REFILL_ && (PACKED || (u & 1) == 1)) {     /* public layout: both slots of the line */ \
                    _Pragma("unroll") for (int v = PACKED ? u : u - 1; v <= u; ++v) {                \
                        s0[v] = BM_LOADW(w0, wl0, v, kn_);                                           \
                        if (DUAL) s1[v] = BM_LOADW(w1, wl1, v, kn_);                                 \
                    }                                                                                \
                }                                                                                    \
                __builtin_amdgcn_sched_barrier(0);                                                   \
            }                                                                                        \
        }                                                                                            \
        if (REFILL_) { BM_STORE_X(((c_) + 1) & 1); }                                                 \
        __syncthreads();                                                                             \
    }

    for (int c = 0; c + 1 < nch; ++c) BM_CHUNK(c, true);
    BM_CHUNK(nch - 1, false);
#undef BM_CHUNK
#undef BM_LOAD_X
#undef BM_STORE_X
#undef BM_LOADW
    if (!active) return;
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

// One item of the kernel below: 64 weight rows (a 16-row block per wave) of group g over reduction slice kslice.
template <bool DUAL, int MAXNBT, bool PACKED>
__device__ __forceinline__ void skinny_lds_item(const SkinnyParams &p, u32x4 *xs, u32x4 *wstage, int g, int blk, int kslice) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n0w = (blk * 4 + wave) * 16;
    const bool active = n0w < p.N;                    // a wave past the last weight row recomputes block 0 and stores nothing
    const int n0 = active ? n0w : 0;
    const int row_begin = p.offsets[g], row_end = p.offsets[g + 1];
    const int per = (p.Kd / KUNIT) / p.ksplit;        // the host picks ksplit as a divisor
    const int k_begin = kslice * per * KUNIT, k_end = k_begin + per * KUNIT;

    const int gl = g < p.E ? g : g - p.E;             // index inside the routed or the shared stack
    const uint16_t *w0, *w1 = nullptr;
    if (PACKED) {
        constexpr int NM = DUAL ? 2 : 1;
        const uint16_t *base = static_cast<const uint16_t *>(g < p.E ? p.pk : p.spk);
        w0 = base + ((size_t)gl * (p.N >> 4) + (n0 >> 4)) * (size_t)(p.Kd >> 5) * (512 * NM) + lane * 8;
        if (DUAL) w1 = w0 + 512;
    } else {
        const size_t gofs = (size_t)gl * p.N * p.Kd;        // row n0 of the block; the pass adds the lane's place
        w0 = static_cast<const uint16_t *>(g < p.E ? p.b0 : p.sb0) + gofs + (size_t)n0 * p.Kd;
        if (DUAL) w1 = static_cast<const uint16_t *>(g < p.E ? p.b1 : p.sb1) + gofs + (size_t)n0 * p.Kd;
    }
    u32x4 *wst = wstage + (PACKED ? 0 : wave * (DUAL ? 256 : 128));
    constexpr int PASS_ROWS = 16 * MAXNBT;
    for (int rb = row_begin; rb < row_end; rb += PASS_ROWS) {
        const int re = min(row_end, rb + PASS_ROWS);
        const int n_rows = re - rb;
        if (MAXNBT == 1 || n_rows <= 16) skinny_lds_pass<DUAL, 1, PACKED>(p, w0, w1, xs, wst, rb, re, k_begin, k_end, n0, kslice, active);
        else if (MAXNBT == 2 || n_rows <= 32) skinny_lds_pass<DUAL, 2, PACKED>(p, w0, w1, xs, wst, rb, re, k_begin, k_end, n0, kslice, active);
        else if (MAXNBT == 4 || n_rows <= 64) skinny_lds_pass<DUAL, 4, PACKED>(p, w0, w1, xs, wst, rb, re, k_begin, k_end, n0, kslice, active);
        else skinny_lds_pass<DUAL, MAXNBT, PACKED>(p, w0, w1, xs, wst, rb, re, k_begin, k_end, n0, kslice, active);
        __syncthreads();                              // the next pass restages the LDS buffers
    }
}

// grid.x = 64-row blocks of the weight matrix, grid.y = reduction slices, grid.z = live-group slots,
// so workgroups are handed out group by group with the slices of a group next to each other.
// Two workgroups fit a compute unit (registers, 64 KB of LDS).  Measured on MI355X, down projection
// of the Mixtral-shaped layer at 64 tokens (640 workgroups of 0.9 MB): 99 us in this order, 111 us
// with the slice index outermost, 108 us with one workgroup per unit.  A fixed grid of two
// workgroups per unit walking the items with a stride took 117 us: the items left for its second
// round sit on a quarter of the units, and a unit's streaming rate is capped.
template <bool DUAL, int MAXNBT, bool PACKED>
__global__ void __launch_bounds__(256, MAXNBT <= 4 ? 2 : 1) skinny_lds_bf16_kernel(SkinnyParams p) {
    __shared__ u32x4 xs[2 * SkinnyChunk<MAXNBT>::CH * MAXNBT * 64];
    __shared__ u32x4 wstage[PACKED ? 1 : 4 * (DUAL ? 256 : 128)];    // public layout: 2 KB per wave and matrix
    const int gi = blockIdx.z;
    if (gi >= p.n_mtiles[0]) return;
    skinny_lds_item<DUAL, MAXNBT, PACKED>(p, xs, wstage, p.mt_group[gi], blockIdx.x, blockIdx.y);
}

bool skinny_lds_ok(int Kd, int ksplit) { return Kd % (KUNIT * ksplit) == 0; }

template <bool DUAL>
static void launch_skinny_lds(const SkinnyParams &p, hipStream_t st) {
    dim3 grid((p.N / 16 + 3) / 4, p.ksplit, p.max_groups);
    // groups of more than 64 rows (more than 64 tokens): 128 rows per pass over the weights, at one workgroup
    // per compute unit (128 KB of staged activations), instead of two passes of 64
    if (p.wide && p.pk != nullptr) hipLaunchKernelGGL((skinny_lds_bf16_kernel<DUAL, 8, true>), grid, dim3(256), 0, st, p);
    else if (p.wide) hipLaunchKernelGGL((skinny_lds_bf16_kernel<DUAL, 8, false>), grid, dim3(256), 0, st, p);
    else if (p.pk != nullptr) hipLaunchKernelGGL((skinny_lds_bf16_kernel<DUAL, 4, true>), grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL((skinny_lds_bf16_kernel<DUAL, 4, false>), grid, dim3(256), 0, st, p);
}

// ---------------------------------------------------------------------------
// Persistent decode kernel for small groups (at most 16*NBT rows each).
// Measured on MI355X, a streaming read is capped per compute unit (about
// 24 GB/s each, 6 TB/s over 256), so the bytes must be spread evenly: one
// workgroup of 8 waves per compute unit walks items (group, 16-row block of
// the weight matrix) with stride gridDim.x; the 8 waves split the reduction
// into contiguous eighths.  The register ring (CH k-steps of weights and
// activation fragments, refilled right after use) runs across item
// boundaries, so the stream never drains; at the end of an item the eight
// partial tiles meet in a double-buffered LDS area, are added in wave order,
// and each wave finishes an eighth of the 16 x 16*NBT outputs.
// Needs Kd divisible by 8 * 32 * CH.
// ---------------------------------------------------------------------------
struct PItem {
    const uint16_t *w0, *w1;
    int g, row_begin, row_end, n0;
};

template <bool DUAL, bool PACKED>
__device__ __forceinline__ PItem p_setup(const SkinnyParams &p, int it, int NRB, int lr, int lk, int k0) {
    PItem r;
    const int gi = it / NRB, rb = it - gi * NRB;
    r.g = p.mt_group[gi];
    r.row_begin = p.offsets[r.g];
    r.row_end = p.offsets[r.g + 1];
    r.n0 = rb * 16;
    const int gl = r.g < p.E ? r.g : r.g - p.E;
    if (PACKED) {
        constexpr int NM = DUAL ? 2 : 1;
        const uint16_t *base = static_cast<const uint16_t *>(r.g < p.E ? p.pk : p.spk);
        r.w0 = base + (((size_t)gl * NRB + rb) * (size_t)(p.Kd >> 5) + (k0 >> 5)) * (512 * NM) + (lk * 16 + lr) * 8;
        r.w1 = DUAL ? r.w0 + 512 : nullptr;
    } else {
        const size_t rofs = (size_t)gl * p.N * p.Kd + (size_t)r.n0 * p.Kd + k0;    // row n0; the kernel adds the lane's place
        r.w0 = static_cast<const uint16_t *>(r.g < p.E ? p.b0 : p.sb0) + rofs;
        r.w1 = DUAL ? static_cast<const uint16_t *>(r.g < p.E ? p.b1 : p.sb1) + rofs : nullptr;
    }
    return r;
}

// COMBINE (down projection only; the grid is as wide as the matrix has 16-row blocks, or divides that
// number): the stride of the item walk is then a multiple of the blocks per group, so a workgroup meets the
// same 16-row blocks - 16 columns of the layer output each - in every live group.  It keeps its finished
// 16-column slices of every row in LDS instead of writing them out, and once through adds them up per token
// the way combine_kernel does (slot order, then the shared experts: the same operations in the same order,
// so the same bits) and writes the layer output: no launch, and no round trip through memory, for the
// aggregation.
constexpr int P_COMB_ROWS = 160;                       // rows (assignments + shared-expert rows) the fused form holds
constexpr int P_COMB_BLOCKS = 2;                       // 16-row blocks per workgroup it holds

template <bool DUAL, int NBT, int CH, bool PACKED, bool COMBINE = false>
__global__ void __launch_bounds__(512) skinny_p_kernel(SkinnyParams p) {
    static_assert(!COMBINE || !DUAL, "the aggregation follows the down projection");
    constexpr int NM = DUAL ? 2 : 1;
    constexpr int KSTEP = PACKED ? 512 * NM : 32;              // weight elements between consecutive k-steps
    constexpr int RED = 2 * 8 * NBT * NM * 64;                 // f32x4 entries of the reduction area
    constexpr int WST = PACKED ? 0 : 8 * NM * 128;             // public layout: 2 KB per wave and matrix
    constexpr int PAD = (RED + WST) * 16 < 84 * 1024 ? (84 * 1024 - (RED + WST) * 16) / 16 : 0;
    __shared__ f32x4 red[RED + PAD];                           // > half the LDS: one workgroup per compute unit
    __shared__ u32x4 wstage[PACKED ? 1 : WST];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lr = lane & 15, lk = lane >> 4;
    // Public layout: the weights come in as whole 128-byte lines - ring slots 2v and 2v + 1 hold rows 0-7 and
    // 8-15 of line v of the chunk, lane l row l / 8, piece l % 8 - and reach the operand layout through the
    // wave's own LDS area, as in the LDS-staged kernel above.
    u32x4 *wst = wstage + (PACKED ? 0 : wave * NM * 128);
    int lofs[2], wwr[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r = 8 * j + (lane >> 3);
        lofs[j] = PACKED ? 0 : r * p.Kd + (lane & 7) * 8;
        wwr[j] = r * 8 + ((lane & 7) ^ (r & 7));
    }
    const int rrd = lr * 8, rx7 = lr & 7;
#define BM_PW(wp_, u_) (PACKED ? (wp_) + (u_) * KSTEP : (wp_) + lofs[(u_) & 1] + ((u_) >> 1) * 64)
    const int NRB = p.N >> 4;
    const int n_items = p.n_mtiles[0] * NRB;
    __shared__ float comb[COMBINE ? P_COMB_BLOCKS * P_COMB_ROWS * 16 : 1];   // [block][row][16 columns]
// the layer output for this workgroup's 16-column blocks from the slices in comb (see combine_kernel)
#define BM_COMBINE_OUT(HAVE_)                                                                           \
    {                                                                                                   \
        const int nbl_ = NRB / (int)gridDim.x;                                                          \
        for (int idx = threadIdx.x; idx < nbl_ * p.T * 16; idx += blockDim.x) {                         \
            const int col = idx & 15, t = (idx >> 4) % p.T, bl = (idx >> 4) / p.T;                      \
            float acc = 0.0f;                                                                           \
            for (int k = 0; (HAVE_) && k < p.K + p.n_shared; ++k) {                                     \
                const int pos = k < p.K ? p.inv_perm[(size_t)t * p.K + k] : p.offsets[p.E + (k - p.K)] + t; \
                if (pos < 0) continue;                                                                  \
                const float wk = k < p.K ? p.w[(size_t)t * p.K + k] : 1.0f;                             \
                const float o = 0.0f + comb[(bl * P_COMB_ROWS + pos) * 16 + col];                       \
                acc = fmaf(wk, o, acc);                                                                 \
            }                                                                                           \
            const size_t at = (size_t)t * p.N + ((size_t)blockIdx.x + (size_t)bl * gridDim.x) * 16 + col; \
            if (p.y_f32) static_cast<float *>(p.y)[at] = acc;                                           \
            else stg16(static_cast<uint16_t *>(p.y) + at, f32_to_bf16(acc));                            \
        }                                                                                               \
    }
    if ((int)blockIdx.x >= n_items) {
        if (COMBINE) BM_COMBINE_OUT(false)             // no live group at all: the output is zero
        return;
    }
    const int my_items = (n_items - 1 - (int)blockIdx.x) / (int)gridDim.x + 1;
    const int kq = p.Kd >> 3;
    const int k0 = wave * kq;
    const int cpi = kq / (CH * 32);                            // chunks per item
    const int total = my_items * cpi;
    const uint16_t *a = static_cast<const uint16_t *>(p.a);

    int it = blockIdx.x;
    PItem cur = p_setup<DUAL, PACKED>(p, it, NRB, lr, lk, k0);
    const uint16_t *xa[NBT];
#pragma unroll
    for (int tb = 0; tb < NBT; ++tb) {
        const int pos = min(cur.row_begin + tb * 16 + lr, cur.row_end - 1);
        const int src = p.row_map ? ldg_i32(p.row_map + pos) : pos;
        xa[tb] = a + (size_t)src * p.Kd + lk * 8 + k0;
    }
    f32x4 acc0[NBT], acc1[NBT];
#pragma unroll
    for (int tb = 0; tb < NBT; ++tb) {
        acc0[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc1[tb] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    u32x4 s0[CH], s1[CH], sx[NBT][CH];
#pragma unroll
    for (int u = 0; u < CH; ++u) {
        s0[u] = ldg128_stream(BM_PW(cur.w0, u));
        if (DUAL) s1[u] = ldg128_stream(BM_PW(cur.w1, u));
#pragma unroll
        for (int tb = 0; tb < NBT; ++tb) sx[tb][u] = ldg128(xa[tb] + u * 32);
    }

#define BM_CONSUME(u_)                                                                                  \
    {                                                                                                   \
        bf16x8 wa, wb;                                                                                  \
        if (!PACKED && ((u_) & 1) == 0) {                                                               \
            _Pragma("unroll") for (int j = 0; j < 2; ++j) {                                             \
                wst[wwr[j]] = s0[(u_) + j];                                                             \
                if (DUAL) wst[128 + wwr[j]] = s1[(u_) + j];                                             \
            }                                                                                           \
        }                                                                                               \
        if (PACKED) {                                                                                   \
            wa = as_bf16x8(s0[u_]);                                                                     \
            wb = as_bf16x8(s1[DUAL ? (u_) : 0]);                                                        \
        } else {                                                                                        \
            const int rs_ = rrd + ((((u_) & 1) * 4 + lk) ^ rx7);                                        \
            wa = as_bf16x8(wst[rs_]);                                                                   \
            wb = as_bf16x8(wst[(DUAL ? 128 : 0) + rs_]);                                                \
        }                                                                                               \
        _Pragma("unroll") for (int tb = 0; tb < NBT; ++tb) {                                            \
            acc0[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, as_bf16x8(sx[tb][u_]), acc0[tb], 0, 0, 0); \
            if (DUAL)                                                                                   \
                acc1[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wb, as_bf16x8(sx[tb][u_]), acc1[tb], 0, 0, 0); \
        }                                                                                               \
    }
// partial tiles -> LDS, barrier, every wave adds up and finishes an eighth of the outputs
#define BM_FINALIZE()                                                                                   \
    {                                                                                                   \
        f32x4 *rbuf = red + par * (8 * NBT * NM * 64);                                                  \
        _Pragma("unroll") for (int tb = 0; tb < NBT; ++tb) {                                            \
            rbuf[((wave * NBT + tb) * NM + 0) * 64 + lane] = acc0[tb];                                  \
            if (DUAL) rbuf[((wave * NBT + tb) * NM + 1) * 64 + lane] = acc1[tb];                        \
            acc0[tb] = f32x4{0.f, 0.f, 0.f, 0.f};                                                       \
            acc1[tb] = f32x4{0.f, 0.f, 0.f, 0.f};                                                       \
        }                                                                                               \
        __syncthreads();                                                                                \
        if (lane < 8 * NBT) {                                                                           \
            const int q = wave * 8 * NBT + lane, tb = q >> 6, ln = q & 63;                              \
            f32x4 t0 = f32x4{0.f, 0.f, 0.f, 0.f}, t1 = f32x4{0.f, 0.f, 0.f, 0.f};                       \
            _Pragma("unroll") for (int sw = 0; sw < 8; ++sw) {                                          \
                t0 += rbuf[((sw * NBT + tb) * NM + 0) * 64 + ln];                                       \
                if (DUAL) t1 += rbuf[((sw * NBT + tb) * NM + 1) * 64 + ln];                             \
            }                                                                                           \
            const int pos = cur.row_begin + tb * 16 + (ln & 15);                                        \
            const int n = cur.n0 + (ln >> 4) * 4;                                                       \
            if (pos < cur.row_end) {                                                                    \
                if (DUAL) {                                                                             \
                    u16x4 h;                                                                            \
                    _Pragma("unroll") for (int i = 0; i < 4; ++i) h[i] = f32_to_bf16(silu(t0[i]) * t1[i]); \
                    *(BM_GLOBAL u16x4 *)(static_cast<uint16_t *>(p.c) + (size_t)pos * p.N + n) = h;     \
                } else if (COMBINE) {                                                                   \
                    const int bl_ = (cur.n0 >> 4) / (int)gridDim.x;                                     \
                    *reinterpret_cast<f32x4 *>(&comb[(bl_ * P_COMB_ROWS + pos) * 16 + (ln >> 4) * 4]) = t0; \
                } else {                                                                                \
                    *(BM_GLOBAL f32x4 *)(static_cast<float *>(p.c) + (size_t)pos * p.N + n) = t0;       \
                }                                                                                       \
            }                                                                                           \
        }                                                                                               \
        par ^= 1;                                                                                       \
    }

    int c_in_item = 0, par = 0;
    for (int j = 0; j + 1 < total; ++j) {
        // where chunk j+1 comes from: the same item, or the first chunk of this workgroup's next item
        const bool last_in_item = (c_in_item + 1 == cpi);
        PItem nxt = cur;
        const uint16_t *rw0, *rw1, *rx[NBT];
        if (last_in_item) {
            nxt = p_setup<DUAL, PACKED>(p, it + gridDim.x, NRB, lr, lk, k0);
            rw0 = nxt.w0;
            rw1 = nxt.w1;
            if (nxt.g != cur.g) {                       // rare: the next item belongs to another group
#pragma unroll
                for (int tb = 0; tb < NBT; ++tb) {
                    const int pos = min(nxt.row_begin + tb * 16 + lr, nxt.row_end - 1);
                    const int src = p.row_map ? ldg_i32(p.row_map + pos) : pos;
                    xa[tb] = a + (size_t)src * p.Kd + lk * 8 + k0;
                }
            }
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb) rx[tb] = xa[tb];
        } else {
            const int ofs = (c_in_item + 1) * (CH * 32);
            rw0 = cur.w0 + (c_in_item + 1) * (CH * KSTEP);
            rw1 = DUAL ? cur.w1 + (c_in_item + 1) * (CH * KSTEP) : nullptr;
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb) rx[tb] = xa[tb] + ofs;
        }
        // consume slot u, refill it with the k-step CH ahead (always: a branch around the refills
        // would make the order of outstanding loads ambiguous and drain the ring)
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            BM_CONSUME(u);
            if (PACKED || (u & 1) == 1) {               // public layout: both slots of a line once it is used up
#pragma unroll
                for (int v = PACKED ? u : u - 1; v <= u; ++v) {
                    s0[v] = ldg128_stream(BM_PW(rw0, v));
                    if (DUAL) s1[v] = ldg128_stream(BM_PW(rw1, v));
                }
            }
#pragma unroll
            for (int tb = 0; tb < NBT; ++tb) sx[tb][u] = ldg128(rx[tb] + u * 32);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (last_in_item) {
            BM_FINALIZE();
            it += gridDim.x;
            cur = nxt;
            c_in_item = 0;
        } else {
            ++c_in_item;
        }
    }
    // last chunk of the last item: drain the ring
#pragma unroll
    for (int u = 0; u < CH; ++u) { BM_CONSUME(u); }
    BM_FINALIZE();
    if (COMBINE) {
        __syncthreads();
        BM_COMBINE_OUT(true)
    }
#undef BM_COMBINE_OUT
#undef BM_CONSUME
#undef BM_FINALIZE
#undef BM_PW
}

bool skinny_p_ok(int Kd, int ch) { return ch % 2 == 0 && Kd % (8 * 32 * ch) == 0; }

static int device_cus() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return 0;
    return cus;
}

// the persistent kernel takes the down projection of this call and can hold every row's slices (see COMBINE)
bool skinny_down_fuses_combine(const SkinnyParams &p) {
    const int cus = device_cus();
    return p.y != nullptr && p.ksplit == 1 && p.max_rows_per_group <= 32 && (skinny_p_ok(p.Kd, 14) || skinny_p_ok(p.Kd, 8)) &&
           cus > 0 && (p.N / 16) % cus == 0 && (p.N / 16) / cus <= P_COMB_BLOCKS && p.rows_max <= P_COMB_ROWS && p.T > 0;
}

// launches the persistent kernel if a ring depth fits the shape; false otherwise
template <bool DUAL>
static bool launch_skinny_p(const SkinnyParams &p, hipStream_t st) {
    if (p.max_rows_per_group > 32) return false;
    const int cus = device_cus();
    if (cus <= 0) return false;
    const dim3 grid(cus), block(512);
    const bool one = p.max_rows_per_group <= 16;
    const bool comb = !DUAL && skinny_down_fuses_combine(p);
#define BM_LAUNCH_P(D_, NBT_, CH_)                                                                         \
    {                                                                                                      \
        if (!D_ && comb) {                                                                                 \
            if (p.pk != nullptr) hipLaunchKernelGGL((skinny_p_kernel<false, NBT_, CH_, true, true>), grid, block, 0, st, p); \
            else hipLaunchKernelGGL((skinny_p_kernel<false, NBT_, CH_, false, true>), grid, block, 0, st, p); \
        } else if (p.pk != nullptr) hipLaunchKernelGGL((skinny_p_kernel<D_, NBT_, CH_, true>), grid, block, 0, st, p); \
        else hipLaunchKernelGGL((skinny_p_kernel<D_, NBT_, CH_, false>), grid, block, 0, st, p);           \
    }
    if (DUAL) {
        if (one && skinny_p_ok(p.Kd, 8)) BM_LAUNCH_P(true, 1, 8)
        else if (!one && skinny_p_ok(p.Kd, 8)) BM_LAUNCH_P(true, 2, 8)
        else return false;
    } else {
        if (one && skinny_p_ok(p.Kd, 14)) BM_LAUNCH_P(false, 1, 14)
        else if (one && skinny_p_ok(p.Kd, 8)) BM_LAUNCH_P(false, 1, 8)
        else if (!one && skinny_p_ok(p.Kd, 14)) BM_LAUNCH_P(false, 2, 14)
        else if (!one && skinny_p_ok(p.Kd, 8)) BM_LAUNCH_P(false, 2, 8)
        else return false;
    }
#undef BM_LAUNCH_P
    return true;
}

template <bool DUAL>
static void launch_skinny(const SkinnyParams &p, dim3 grid, hipStream_t st) {
    if (p.max_rows_per_group <= 16) hipLaunchKernelGGL((skinny_bf16_kernel<DUAL, 1>), grid, dim3(256), 0, st, p);
    else if (p.max_rows_per_group <= 32) hipLaunchKernelGGL((skinny_bf16_kernel<DUAL, 2>), grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL((skinny_bf16_kernel<DUAL, 4>), grid, dim3(256), 0, st, p);
}

int launch_skinny_gateup_bf16(const SkinnyParams &p, hipStream_t st) {
    if (launch_skinny_p<true>(p, st)) {
    } else if (p.max_rows_per_group > 32 && skinny_lds_ok(p.Kd, 1)) {
        launch_skinny_lds<true>(p, st);
    } else if (skinny_q_ok(p.Kd, 1)) {
        launch_skinny_q<true>(p, st);
    } else {
        dim3 grid((p.N / 16 + 3) / 4, p.max_groups, 1);
        launch_skinny<true>(p, grid, st);
    }
    return launch_status(__func__);
}

int launch_skinny_down_bf16(const SkinnyParams &p, hipStream_t st) {
    if (p.ksplit == 1 && launch_skinny_p<false>(p, st)) {
    } else if (p.max_rows_per_group > 32 && skinny_lds_ok(p.Kd, p.ksplit)) {
        launch_skinny_lds<false>(p, st);
    } else if (skinny_q_ok(p.Kd, p.ksplit)) {
        launch_skinny_q<false>(p, st);
    } else {
        dim3 grid((p.N / 16 + 3) / 4, p.max_groups, p.ksplit);
        launch_skinny<false>(p, grid, st);
    }
    return launch_status(__func__);
}

}  // namespace bm
