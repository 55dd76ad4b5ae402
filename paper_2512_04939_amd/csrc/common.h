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

}  // namespace lv

#define LV_HIP_CHECK_LAUNCH()                                  \
  do {                                                         \
    if (hipGetLastError() != hipSuccess) return LV_ERR_HIP;    \
  } while (0)
