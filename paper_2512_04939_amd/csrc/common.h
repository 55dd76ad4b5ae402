// Shared device helpers for the gfx950 kernels (wave64, CDNA4).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lv {

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(8))) int i32x8;

constexpr int kWave = 64;
constexpr int kXcd = 8;      // MI355X: 8 XCDs, workgroups are dealt to them round-robin

// bf16 <-> fp32 on raw bit patterns
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// two floats -> packed bf16 pair (round to nearest even; v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 b = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// Sum over the 64 lanes with DPP moves only (no LDS round trips): butterflies inside each row of
// 16 lanes (quad permutes, half-row mirror, row mirror), then lane 15 of a row broadcast into the
// next row and lane 31 into rows 2 and 3; lane 63 holds the total, returned as a uniform value.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ float dpp_take(float v) {   // 0 where the row is masked out
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, kRowMask, 0xF, false));
}
__device__ __forceinline__ float wave_sum_uniform(float v) {
  v += dpp_take<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
  v += dpp_take<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
  v += dpp_take<0x141, 0xF>(v);   // row_half_mirror
  v += dpp_take<0x140, 0xF>(v);   // row_mirror: every lane holds its row's sum
  v += dpp_take<0x142, 0xA>(v);   // row_bcast15 into rows 1 and 3
  v += dpp_take<0x143, 0xC>(v);   // row_bcast31 into rows 2 and 3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64));
  return v;
}

// Workgroup id -> logical id such that each XCD (own L2) gets a contiguous range of
// logical ids: hardware deals workgroup b to XCD b % 8.
__device__ __forceinline__ uint32_t xcd_contiguous(uint32_t b, uint32_t n) {
  uint32_t per = (n + kXcd - 1) / kXcd;
  return (b % kXcd) * per + b / kXcd;   // may be >= n: caller skips
}

// LDS address (byte offset in the workgroup's LDS) of a __shared__ object
__device__ __forceinline__ uint32_t lds_addr(const void *p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}
// Four 16-byte LDS reads at addr + 0, 1, 2, 3 KB, issued here and NOT waited for: the compiler
// does not know that dst is still in flight, so every use of dst must come after an lds_wait
// on the same registers.
__device__ __forceinline__ void lds_read4_async(u32x4 (&dst)[4], uint32_t addr) {
  asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:1024\n\t"
               "ds_read_b128 %2, %4 offset:2048\n\tds_read_b128 %3, %4 offset:3072"
               : "=&v"(dst[0]), "=&v"(dst[1]), "=&v"(dst[2]), "=&v"(dst[3])
               : "v"(addr)
               : "memory");
}
// Two such reads, at addr and addr + 1 KB.
__device__ __forceinline__ void lds_read2_async(u32x4 (&dst)[2], uint32_t addr) {
  asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:1024"
               : "=&v"(dst[0]), "=&v"(dst[1])
               : "v"(addr)
               : "memory");
}

// two 16-byte pieces side by side: an 8-register MFMA operand
__device__ __forceinline__ i32x8 cat8(const u32x4 a, const u32x4 b) {
  return i32x8{(int)a.x, (int)a.y, (int)a.z, (int)a.w, (int)b.x, (int)b.y, (int)b.z, (int)b.w};
}

// FP8 E4M3 (OCP "fn": bias 7, largest value 448, no infinities), round to nearest even
constexpr float kFp8Max = 448.0f;

__device__ __forceinline__ uint32_t cvt4_fp8(float a, float b, float c, float d) {
  uint32_t w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0u, false);
  return __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
}
__device__ __forceinline__ float clamp448(float x) { return fminf(fmaxf(x, -kFp8Max), kFp8Max); }
// 8 bf16 values scaled by r and quantised to 8 fp8 bytes
__device__ __forceinline__ u32x2 quant8(const u32x4 w, float r) {
  return u32x2{cvt4_fp8(clamp448(bf16_lo(w.x) * r), clamp448(bf16_hi(w.x) * r),
                        clamp448(bf16_lo(w.y) * r), clamp448(bf16_hi(w.y) * r)),
               cvt4_fp8(clamp448(bf16_lo(w.z) * r), clamp448(bf16_hi(w.z) * r),
                        clamp448(bf16_lo(w.w) * r), clamp448(bf16_hi(w.w) * r))};
}
__device__ __forceinline__ float absmax8(const u32x4 w) {
  const float a = fmaxf(fmaxf(fabsf(bf16_lo(w.x)), fabsf(bf16_hi(w.x))), fmaxf(fabsf(bf16_lo(w.y)), fabsf(bf16_hi(w.y))));
  const float b = fmaxf(fmaxf(fabsf(bf16_lo(w.z)), fabsf(bf16_hi(w.z))), fmaxf(fabsf(bf16_lo(w.w)), fabsf(bf16_hi(w.w))));
  return fmaxf(a, b);
}
__device__ __forceinline__ float fp8_scale_inv(uint32_t amax_bits) {   // 448 / amax (1 if amax = 0)
  const float a = __uint_as_float(amax_bits);
  return a > 0.f ? kFp8Max / a : 1.0f;
}

}  // namespace lv

#define LV_HIP_CHECK_LAUNCH()                                  \
  do {                                                         \
    if (hipGetLastError() != hipSuccess) return LV_ERR_HIP;    \
  } while (0)
