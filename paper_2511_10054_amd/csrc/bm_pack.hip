// One-time repacking of expert weights for the decode kernels: the public
// layout keeps the reduction dimension contiguous ([N][Kd] per matrix), the
// packed copy is fragment-major - for every block of 16 weight rows and every
// k-step of 32 the 1 KB MFMA operand fragment (lane l: row l % 16, the 8
// values from k = 8 * (l / 16)) is contiguous, fragments of one row block
// follow each other along k, and for the gate/up pair the two fragments of a
// k-step are interleaved.  A wave then streams its row block as one contiguous
// run of full cache lines (measured: a contiguous read stream reaches
// 6.8-7.0 TB/s on MI355X, the 16-rows-by-64-bytes pattern of the public layout
// 6.0 TB/s).
#include "bm_kernels.h"

namespace bm {

struct PackParams {
    const uint16_t *src0, *src1;   // [n][N][Kd]; src1 = second matrix (up) or null
    uint16_t *dst;                 // [n][N/16][Kd/32][NM][64][8]
    int n, N, Kd, NM;
    const uint64_t *bitmap;        // experts to pack (null: all)
};

__global__ void __launch_bounds__(256) pack_kernel(PackParams p) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;     // one 16-byte piece
    const int KB = p.Kd >> 5, NRB = p.N >> 4;
    const size_t total = (size_t)p.n * NRB * KB * p.NM * 64;
    if (idx >= total) return;
    const int lane = (int)(idx & 63);
    size_t r = idx >> 6;
    const int m = (int)(r % p.NM); r /= p.NM;
    const int kb = (int)(r % KB); r /= KB;
    const int nb = (int)(r % NRB);
    const int e = (int)(r / NRB);
    if (p.bitmap != nullptr && !((p.bitmap[e >> 6] >> (e & 63)) & 1ull)) return;
    const uint16_t *src = (m ? p.src1 : p.src0) + ((size_t)e * p.N + nb * 16 + (lane & 15)) * p.Kd + kb * 32 + (lane >> 4) * 8;
    stg128(p.dst + idx * 8, ldg128(src));
}

int launch_pack(const void *src0, const void *src1, void *dst, int n, int N, int Kd, const uint64_t *bitmap,
                hipStream_t st) {
    PackParams p{static_cast<const uint16_t *>(src0), static_cast<const uint16_t *>(src1),
                 static_cast<uint16_t *>(dst), n, N, Kd, src1 ? 2 : 1, bitmap};
    const size_t total = (size_t)n * (N >> 4) * (Kd >> 5) * p.NM * 64;
    if (total) hipLaunchKernelGGL(pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, p);
    return launch_status(__func__);
}

}  // namespace bm
