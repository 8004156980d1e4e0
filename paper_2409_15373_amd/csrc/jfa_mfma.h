// gfx950 matrix-core and cross-lane helpers shared by the bf16 kernels.
//
// Register layouts of v_mfma_f32_32x32x16_bf16 (D = A[32x16] * B[16x32] + C), lane l in a 64-wide wave:
//   A operand  8 x bf16 : row  l % 32, contraction slots 8 * (l / 32) + 0..7
//   B operand  8 x bf16 : col  l % 32, contraction slots 8 * (l / 32) + 0..7
//   C/D       16 x fp32 : col  l % 32, rows (v / 4) * 8 + (l / 32) * 4 + v % 4 for v = 0..15
// The contraction index is a dummy: any assignment of "slots" to real indices is valid as long as
// both operands use the same one.  The kernels exploit this so that an accumulator tile can be fed
// back as the next product's operand without any cross-lane shuffle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace jfa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ inline f32x16 mfma_32x32x16(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row (l % 32, l / 32) of an accumulator tile for register v.
__device__ inline int acc_row(int v, int half) { return (v >> 2) * 8 + half * 4 + (v & 3); }

// max / sum of x over the lane pair {l, l ^ 32} (one v_permlane32_swap + one VALU op).
__device__ inline float pair_max(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float pair_sum(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 16-byte LDS read as an MFMA operand.
__device__ inline bf16x8 lds_read_b128(const char *p) { return *reinterpret_cast<const bf16x8 *>(p); }

// ds_read_b64_tr_b16: inside each block of 16 lanes, lane i receives element (i % 4) of the four
// 8-byte chunks addressed by lanes (i / 4), 4 + (i / 4), 8 + (i / 4), 12 + (i / 4).  With source lane s
// pointing at row (s / 4) and column 4 * (s % 4) of a row-major 16-bit matrix, destination lane i gets
// column i of rows 0..3: a 4 x 16 tile delivered transposed.
__device__ inline bf16x4 lds_read_tr16(const char *p) {
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4 *)(__attribute__((address_space(3))) char *)(const_cast<char *>(p)));
    return __builtin_bit_cast(bf16x4, r);
}

__device__ inline bf16x8 concat(bf16x4 a, bf16x4 b) { return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7); }

// Eight fp32 accumulator registers acc[first .. first+7] rounded to bf16 (round to nearest even).
__device__ inline bf16x8 pack_bf16(const f32x16 &acc, int first) {
    bf16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (__bf16)acc[first + e];
    return r;
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ inline float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

}  // namespace jfa
