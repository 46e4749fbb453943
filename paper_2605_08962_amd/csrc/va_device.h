// Device-side helpers for the gfx950 kernels: vector types, MFMA, LDS transposing reads,
// cross-half exchange.  Lane layouts used throughout (wave64, v_mfma_f32_32x32x16_bf16):
//   A operand: lane l holds A[m = l % 32][k = 8*(l/32) .. 8*(l/32)+7]
//   B operand: lane l holds B[k = 8*(l/32) .. +7][n = l % 32]
//   C/D      : lane l, register r holds C[m = 8*(r/4) + 4*(l/32) + r%4][n = l % 32]
// A C tile X[m][n] therefore already is the B operand of a product that contracts over m,
// provided the A operand enumerates k in the order  k(l/32, e) = 8*(e/4) + 4*(l/32) + e%4
// per 16-wide step (registers 0..7 = step 0, 8..15 = step 1).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace va {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define VA_LDS __attribute__((address_space(3)))

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// max / sum of x between lane l and lane l ^ 32 (v_permlane32_swap exchanges the upper half of
// its first operand with the lower half of its second).
__device__ __forceinline__ float xhalf_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// ds_read_b64_tr_b16: inside each group of 16 lanes, lane 4*k + j supplies the LDS address of
// elements [row k][cols 4j .. 4j+3] of a 4 x 16 block of 16-bit values; lane i receives
// [rows 0..3][col i].  Two of them give one 8-deep MFMA A operand of a row-major tile read
// "down the columns".
__device__ __forceinline__ bf16x4 lds_read_tr(const unsigned char* p) {
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 VA_LDS*)(p));
    return __builtin_bit_cast(bf16x4, r);
}
__device__ __forceinline__ bf16x8 cat4(bf16x4 a, bf16x4 b) {
    return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}
// Per-lane byte offset, inside a row-major LDS tile with `stride` bytes per row, of the address
// this lane supplies to lds_read_tr for the block whose origin is (row 0, col 0) for lanes 0..15,
// col 16 for lanes 16..31, and 4 rows further down for lanes 32..63.
__device__ __forceinline__ int tr_lane_offset(int lane, int stride) {
    return (4 * (lane >> 5) + ((lane & 15) >> 2)) * stride + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
}

__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3, float a4, float a5, float a6, float a7) {
    bf16x8 r;
    r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
    r[4] = (__bf16)a4; r[5] = (__bf16)a5; r[6] = (__bf16)a6; r[7] = (__bf16)a7;
    return r;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kMaskedScore = -1.0e30f;  // finite stand-in for -inf: keeps 0 * score finite

}  // namespace va
