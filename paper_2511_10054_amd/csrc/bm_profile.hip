// Profiling statistics and buddy-list construction on the device.
//
//   coact_kernel        per-expert activation counts A and pairwise co-activation counts M of a batch
//                       of routed ids, added to running totals
//   buddy_build_kernel  per pivot: peers ranked by conditional co-activation, cut at the cumulative
//                       frequency threshold
//
// Both are exact integer work up to one fp64 comparison per list entry.
#include "bm_kernels.h"

namespace bm {

// index of the pair (i < j) in a row-major strict upper triangle of an E x E matrix
__device__ __forceinline__ int tri_index(int i, int j, int E) { return i * (2 * E - i - 1) / 2 + (j - i - 1); }

// One wave per token.  Lane k holds slot k's expert; a repeated or out-of-range id is dropped (an expert
// counts once per token).  Counts are gathered in LDS (strict upper triangle, one int per pair) and added
// to the global int64 totals once per workgroup, so the global atomics are per touched pair, not per token.
template <int EMAX>
__global__ void __launch_bounds__(256) coact_kernel(const int32_t *ids, int T, int K, int E, int tokens_per_wg,
                                                    unsigned long long *A, unsigned long long *M) {
    __shared__ int32_t s_pair[EMAX * (EMAX - 1) / 2];
    __shared__ int32_t s_act[EMAX];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_pair = E * (E - 1) / 2;
    for (int i = tid; i < n_pair; i += blockDim.x) s_pair[i] = 0;
    for (int i = tid; i < E; i += blockDim.x) s_act[i] = 0;
    __syncthreads();
    const int t_begin = blockIdx.x * tokens_per_wg, t_end = min(T, t_begin + tokens_per_wg);
    for (int t = t_begin + wave; t < t_end; t += (int)(blockDim.x >> 6)) {
        int e = lane < K ? ids[(size_t)t * K + lane] : -1;
        bool valid = (unsigned)e < (unsigned)E;
        for (int k = 0; k < K; ++k) {                      // drop repeats: keep the first occurrence
            const int ek = __shfl(e, k, WAVE);
            if (lane > k && ek == e) valid = false;
        }
        if (valid) atomicAdd(&s_act[e], 1);
        for (int k = 0; k < K; ++k) {
            const int ek = __shfl(e, k, WAVE);
            const bool vk = __shfl((int)valid, k, WAVE) != 0;
            if (vk && valid && lane > k) atomicAdd(&s_pair[tri_index(min(e, ek), max(e, ek), E)], 1);
        }
    }
    __syncthreads();
    for (int i = tid; i < E; i += blockDim.x)
        if (s_act[i]) atomicAdd(&A[i], (unsigned long long)s_act[i]);
    for (int idx = tid; idx < E * E; idx += blockDim.x) {
        const int i = idx / E, j = idx - i * E;
        if (i >= j) continue;
        const int v = s_pair[tri_index(i, j, E)];
        if (v) {
            atomicAdd(&M[(size_t)i * E + j], (unsigned long long)v);
            atomicAdd(&M[(size_t)j * E + i], (unsigned long long)v);
        }
    }
}

// One wave per pivot i.  Lane l owns peers l, l+64, ...; a peer's rank is the number of peers with a
// larger count, or the same count and a lower index (the order of q = count / row sum); peers of rank r
// form the sequence pi_i.  Lane 0 then walks the prefix sums: the list ends at the first t with
//   count(pi_i(1..t)) >= alpha * row sum         (one fp64 product, one comparison)
// cut to at most R entries, at least one if the row sum is positive.
__global__ void __launch_bounds__(64) buddy_build_kernel(const long long *M, int E, int R, float alpha,
                                                         int32_t *table, int32_t *list_len, float *q_out) {
    __shared__ long long s_cnt[BM_MAX_E];
    __shared__ int32_t s_order[BM_MAX_E];
    const int i = blockIdx.x, lane = threadIdx.x;
    long long total = 0;
    for (int j = lane; j < E; j += WAVE) {
        const long long c = (j == i) ? 0 : M[(size_t)i * E + j];
        s_cnt[j] = c;
        total += c;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) total += __shfl_xor(total, m, WAVE);
    for (int j = lane; j < E; j += WAVE) s_order[j] = -1;
    __syncthreads();
    for (int j = lane; j < E; j += WAVE) {
        const long long c = s_cnt[j];
        if (c <= 0) continue;
        int rank = 0;
        for (int o = 0; o < E; ++o) {
            const long long co = s_cnt[o];
            rank += (co > c) || (co == c && o < j);
        }
        s_order[rank] = j;
    }
    __syncthreads();
    if (lane == 0) {
        int t_i = 0;
        long long cum = 0;
        const double need = (double)alpha * (double)total;
        for (int r = 0; r < E && s_order[r] >= 0; ++r) {
            cum += s_cnt[s_order[r]];
            t_i = r + 1;
            if ((double)cum >= need) break;
        }
        if (t_i > R) t_i = R;
        for (int r = 0; r < R; ++r) {
            table[(size_t)i * R + r] = r < t_i ? s_order[r] : -1;
            if (q_out) q_out[(size_t)i * R + r] = r < t_i ? (float)((double)s_cnt[s_order[r]] / (double)total) : 0.0f;
        }
        if (list_len) list_len[i] = t_i;
    }
}

int launch_coactivation(const int32_t *ids, int T, int K, int E, long long *A, long long *M, hipStream_t st) {
    if (T > 0) {
        // enough workgroups to fill the chip, enough tokens per workgroup to amortise the LDS flush
        int per = (T + 511) / 512;
        if (per < 64) per = 64;
        const int grid = (T + per - 1) / per;
        unsigned long long *a = reinterpret_cast<unsigned long long *>(A), *m = reinterpret_cast<unsigned long long *>(M);
        if (E <= 64) hipLaunchKernelGGL(coact_kernel<64>, dim3(grid), dim3(256), 0, st, ids, T, K, E, per, a, m);
        else if (E <= 128) hipLaunchKernelGGL(coact_kernel<128>, dim3(grid), dim3(256), 0, st, ids, T, K, E, per, a, m);
        else hipLaunchKernelGGL(coact_kernel<256>, dim3(grid), dim3(256), 0, st, ids, T, K, E, per, a, m);
    }
    return launch_status(__func__);
}

int launch_buddy_build(const long long *M, int E, int R, float alpha, int32_t *table, int32_t *list_len, float *q,
                       hipStream_t st) {
    hipLaunchKernelGGL(buddy_build_kernel, dim3(E), dim3(64), 0, st, M, E, R, alpha, table, list_len, q);
    return launch_status(__func__);
}

}  // namespace bm
