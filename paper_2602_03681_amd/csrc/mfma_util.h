// MFMA fragment helpers for gfx950 (wave64), internal header.
//
// v_mfma_f32_16x16x32_f16 lane layout (lane l of 64):
//   A fragment: row  m = l % 16, contraction slots k = 8*(l/16) + j, j = 0..7
//   B fragment: col  n = l % 16, contraction slots k = 8*(l/16) + j
//   C/D       : rows 4*(l/16) + j (j = 0..3), col l % 16
// so both operands are read as 8 consecutive fp16 (16 bytes) from a buffer that is
// contiguous along the contraction index, and a result tile hands every lane four
// consecutive rows of one column.
//
// MFMA operands are fp16 with fp32 accumulation: bf16 tensors convert exactly
// (8 significant bits, values clamped to the fp16 range), and intermediates rounded to
// fp16 carry 2^-12 relative error instead of bf16's 2^-9, which the parity bar needs.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nats {

typedef _Float16 half_t;
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte word held in registers

__device__ __forceinline__ f32x4 mfma16(half8 a, half8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ half_t f32_to_half_sat(float f) {
    return (half_t)__builtin_amdgcn_fmed3f(f, -65504.f, 65504.f);
}

// 8 consecutive bf16 (one 16-byte word) -> 8 fp16, exact inside the fp16 range
__device__ __forceinline__ half8 bf16x8_to_half8(u32x4 u) {
    half8 h;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        h[2 * i] = f32_to_half_sat(__uint_as_float(u[i] << 16));
        h[2 * i + 1] = f32_to_half_sat(__uint_as_float(u[i] & 0xffff0000u));
    }
    return h;
}

__device__ __forceinline__ half8 bf16x8_to_half8(uint4 w) { return bf16x8_to_half8(u32x4{w.x, w.y, w.z, w.w}); }

__device__ __forceinline__ half8 lds_read8(const half_t* p) { return *reinterpret_cast<const half8*>(p); }
__device__ __forceinline__ half4 lds_read4(const half_t* p) { return *reinterpret_cast<const half4*>(p); }

__device__ __forceinline__ half4 to_half4(f32x4 v) {
    half4 h;
    h[0] = f32_to_half_sat(v[0]); h[1] = f32_to_half_sat(v[1]);
    h[2] = f32_to_half_sat(v[2]); h[3] = f32_to_half_sat(v[3]);
    return h;
}

// Conversions to fp16 without the explicit clamp, for kernels that have switched the hardware's fp16 overflow
// mode on (fp16_saturate_on): a result beyond the fp16 range then becomes +-65504 instead of infinity, at no
// instruction cost (the clamp costs one vector instruction per element, a fifth of the vector work of the
// recurrence kernel).
__device__ __forceinline__ void fp16_saturate_on() {
    // MODE register (hardware register 1), bit 23, one bit wide: FP16_OVFL
    __builtin_amdgcn_s_setreg(1 | (23 << 6) | (0 << 11), 1);
}
__device__ __forceinline__ half4 to_half4_hw(f32x4 v) {
    half4 h;
    h[0] = (half_t)v[0]; h[1] = (half_t)v[1]; h[2] = (half_t)v[2]; h[3] = (half_t)v[3];
    return h;
}

// ---- fp32 matrix instruction v_mfma_f32_16x16x4_f32: out[m][n] += sum_kk A[m][kk] B[kk][n]; lane (l16, lq) gives
// A[m = l16][kk = lq], B[kk = lq][n = l16] and holds out[m = 4 lq + j][n = l16], j = 0..3.  mac16 contracts over 16
// indices in four instructions, instruction j over the indices 4 lq + j: a lane's A operands are then four
// consecutive elements of a row, and a result tile can be the B operand of a next product as it sits in registers.
__device__ __forceinline__ f32x4 mac16(const float4 a, const float4 b, f32x4 c) {
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, b.x, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, b.y, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, b.z, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, b.w, c, 0, 0, 0);
    return c;
}
__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
// four elements of one column, rows r0 .. r0 + 3 (row stride rs)
__device__ __forceinline__ float4 ld4col(const float* p, int rs) { return make_float4(p[0], p[rs], p[2 * rs], p[3 * rs]); }
// the same two reads from a buffer of bf16 (raw 16 bits; p 8-byte aligned for ldb4)
__device__ __forceinline__ float4 ldb4(const uint16_t* p) {
    const uint2 w = *reinterpret_cast<const uint2*>(p);
    return make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16),
                       __uint_as_float(w.y & 0xffff0000u));
}
__device__ __forceinline__ float4 ldbcol(const uint16_t* p, int rs) {
    return make_float4(__uint_as_float((uint32_t)p[0] << 16), __uint_as_float((uint32_t)p[rs] << 16),
                       __uint_as_float((uint32_t)p[2 * rs] << 16), __uint_as_float((uint32_t)p[3 * rs] << 16));
}

constexpr int LDS_PAD = 8;  // fp16 elements added to every LDS row: 16-byte reads of 16 rows hit distinct banks

}  // namespace nats
