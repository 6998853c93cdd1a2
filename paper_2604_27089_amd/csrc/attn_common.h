// Device-side building blocks shared by the attention kernels: vector types,
// the bf16 MFMA wrapper and its operand / accumulator lane layouts.
//
// v_mfma_f32_32x32x16_bf16 computes C[32x32] += A[32x16] * B[16x32] per wave.
// With lane l, lo = l % 32, hi = l / 32:
//   A operand: lane holds A[lo][8*hi + e], e = 0..7   (8 bf16 = 16 bytes)
//   B operand: lane holds B[8*hi + e][lo], e = 0..7
//   C/D      : lane holds C[8*(r/4) + 4*hi + r%4][lo] in register r = 0..15
// The contraction index only has to be paired consistently between A and B,
// which the kernels use to feed an accumulator straight back in as an operand:
// registers r = 8c .. 8c+7 of a C tile are rows {16c + 4*hi + e, 16c + 8 + 4*hi + e}.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ u32x4 as_u32x4(bf16x8 v) { return __builtin_bit_cast(u32x4, v); }

// two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    f32x2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

// registers [first, first+8) of an accumulator tile as a bf16 MFMA operand
__device__ __forceinline__ bf16x8 acc_to_operand(const f32x16& c, int first) {
    u32x4 r;
    r[0] = pack_bf16(c[first + 0], c[first + 1]);
    r[1] = pack_bf16(c[first + 2], c[first + 3]);
    r[2] = pack_bf16(c[first + 4], c[first + 5]);
    r[3] = pack_bf16(c[first + 6], c[first + 7]);
    return as_bf16x8(r);
}

// Position of a 4-row group inside its 16-row block in the "operand order" used
// for transposed LDS tiles: [0-3, 8-11, 4-7, 12-15], so that lane half `hi`
// reads its 8 contraction slots {4*hi + e, 8 + 4*hi + e} as one 16-byte load at
// offset 8*hi.
__device__ __forceinline__ int operand_pos4(int group4) {  // group4 = row/4
    const int blk = group4 >> 2, q4 = group4 & 3;
    const int pb = (q4 == 1) ? 2 : (q4 == 2) ? 1 : q4;
    return 16 * blk + 4 * pb;
}

// exchange with the other 32-lane half of the wave
__device__ __forceinline__ float xhalf(float x) { return __shfl_xor(x, 32, 64); }

// Transpose a 4 (rows) x 8 (cols) bf16 block held as four 16-byte row vectors
// into eight 8-byte column vectors (4 rows each).
__device__ __forceinline__ void transpose4x8(const u32x4 (&row)[4], u32x2 (&col)[8]) {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        col[2 * w][0] = (row[0][w] & 0xffffu) | (row[1][w] << 16);
        col[2 * w][1] = (row[2][w] & 0xffffu) | (row[3][w] << 16);
        col[2 * w + 1][0] = (row[0][w] >> 16) | (row[1][w] & 0xffff0000u);
        col[2 * w + 1][1] = (row[2][w] >> 16) | (row[3][w] & 0xffff0000u);
    }
}

}  // namespace sp
