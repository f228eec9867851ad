// Device-side helpers shared by the gfx950 kernels: bf16 storage, wave64
// reductions, MFMA operand types.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bm {

constexpr int WAVE = 64;
constexpr int TILE_T = 32;      // tokens per front-end tile (one MFMA row block)

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;   // one 16-byte piece
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;   // four bf16 values
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}

// fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32: one instruction for two values, NaN stays NaN)
typedef float bm_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bm_bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const bm_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bm_bf16x2));
}

__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return (uint16_t)(pack_bf16x2(f, 0.0f) & 0xffffu); }

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Loads and stores through an explicit global-memory pointer.  Pointers that
// arrive inside a by-value parameter struct are generic to the compiler; the
// explicit address space turns flat_load/flat_store into global_load/store,
// which do not tie up the LDS counter.
#define BM_GLOBAL __attribute__((address_space(1)))
__device__ __forceinline__ u32x4 ldg128(const void *p) { return *(const BM_GLOBAL u32x4 *)p; }
__device__ __forceinline__ void stg128(void *p, u32x4 v) { *(BM_GLOBAL u32x4 *)p = v; }
__device__ __forceinline__ void stg16(void *p, uint16_t v) { *(BM_GLOBAL uint16_t *)p = v; }
__device__ __forceinline__ int ldg_i32(const void *p) { return *(const BM_GLOBAL int *)p; }
__device__ __forceinline__ float ldg_f32(const void *p) { return *(const BM_GLOBAL float *)p; }

// x * sigmoid(x) with the hardware exponential and reciprocal (both within 1 ulp; the result is rounded
// to bf16 or feeds an fp32 product)
__device__ __forceinline__ float silu(float a) { return a * __builtin_amdgcn_rcpf(1.0f + __expf(-a)); }

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (WAVE - 1)); }

// butterfly sum over the 64 lanes; every lane ends with the same value and
// the association order is fixed, so the result is reproducible
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, WAVE);
    return v;
}

// Largest 32-bit key over the wave, returned to every lane as a wave-uniform value.  Within a row of
// 16 lanes: four DPP exchanges (lane ^ 1, lane ^ 2, mirror inside a half row, mirror inside the row);
// the four row results are then read with v_readlane and compared on the scalar side.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#define BM_DPP_MAX(ctrl_)                                                                             \
    {                                                                                                 \
        const uint32_t o_ = (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, ctrl_, 0xF, 0xF, false); \
        v = o_ > v ? o_ : v;                                                                          \
    }
    BM_DPP_MAX(0xB1)     // quad_perm [1, 0, 3, 2]
    BM_DPP_MAX(0x4E)     // quad_perm [2, 3, 0, 1]
    BM_DPP_MAX(0x141)    // row_half_mirror
    BM_DPP_MAX(0x140)    // row_mirror
#undef BM_DPP_MAX
    uint32_t best = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint32_t o = (uint32_t)__builtin_amdgcn_readlane((int)v, 16 * r);
        best = o > best ? o : best;
    }
    return best;
}

// Order-preserving map of finite floats (and infinities) to unsigned integers, and back.  -0 is mapped
// like +0, so keys of equal floats are equal.
__device__ __forceinline__ uint32_t float_to_ordered(float f) {
    const uint32_t u = __builtin_bit_cast(uint32_t, f == 0.0f ? 0.0f : f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ordered_to_float(uint32_t k) {
    return __builtin_bit_cast(float, (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

}  // namespace bm
