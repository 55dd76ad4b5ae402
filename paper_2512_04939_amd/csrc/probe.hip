// Measurement aids, no part of the method: what the GPU sustains on the resources the
// rooflines of the kernels are quoted against (matrix pipes, HBM), with nothing else in the way.
// The benchmark runs them next to the hot path so that a fraction of the published peak can be
// read against what the same box delivers to the simplest possible kernel.
#include "common.h"
#include "internal.h"

namespace lv {

constexpr int kProbeGroups = 2048;     // workgroups of 512 threads: 8 per CU, several rounds
constexpr int kProbeOperandWords = 32768;

// Eight independent accumulator tiles per wave, operands loaded once from memory (real data:
// with constant operands the pipes draw less power and the clock stays higher than any kernel
// with changing data sees), two waves per SIMD.  FP8: v_mfma_f32_32x32x64_f8f6f4 with both
// formats E4M3 and no block scales; bf16: v_mfma_f32_32x32x16_bf16.
template <bool FP8>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_probe_mfma(
    const uint32_t *__restrict__ operands, int iters, float *__restrict__ out) {
  constexpr int W = FP8 ? 8 : 4;   // operand words per lane
  uint32_t a[2][W], b[4][W];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int i = 0; i < W; ++i) a[j][i] = operands[(threadIdx.x * W + i + 4096 * j) & (kProbeOperandWords - 1)];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < W; ++i) b[j][i] = operands[(threadIdx.x * W + i + 4096 * j + 7777) & (kProbeOperandWords - 1)];
  f32x16 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if constexpr (FP8) {
        const i32x8 va = {(int)a[j & 1][0], (int)a[j & 1][1], (int)a[j & 1][2], (int)a[j & 1][3],
                          (int)a[j & 1][4], (int)a[j & 1][5], (int)a[j & 1][6], (int)a[j & 1][7]};
        const i32x8 vb = {(int)b[j >> 1][0], (int)b[j >> 1][1], (int)b[j >> 1][2], (int)b[j >> 1][3],
                          (int)b[j >> 1][4], (int)b[j >> 1][5], (int)b[j >> 1][6], (int)b[j >> 1][7]};
        acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va, vb, acc[j], 0, 0, 0, 0, 0, 0);
      } else {
        const u32x4 va = {a[j & 1][0], a[j & 1][1], a[j & 1][2], a[j & 1][3]};
        const u32x4 vb = {b[j >> 1][0], b[j >> 1][1], b[j >> 1][2], b[j >> 1][3]};
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va),
                                                        __builtin_bit_cast(bf16x8, vb), acc[j], 0, 0, 0);
      }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// 16 bytes per lane and access, grid-stride; dst == nullptr: read only (the sum keeps the loads)
__global__ __launch_bounds__(256) void k_probe_stream(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                      size_t n16, uint32_t *__restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  uint32_t s = 0;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
    const u32x4 v = src[i];
    if (dst) dst[i] = v;
    else s += v.x ^ v.y ^ v.z ^ v.w;
  }
  if (!dst && s == 0x9e3779b9u) *sink = s;   // practically never: the loads stay, no write traffic
}

// rows of `row16` 16-byte pieces read whole, one row per wave and step, in the order `order`
// gives them (the access pattern of a merge: 2 KB token rows gathered through an index); eight
// rows in flight per wave, nothing written
__global__ __launch_bounds__(256) void k_probe_gather(const u32x4 *__restrict__ src, int row16,
                                                      const int32_t *__restrict__ order, int64_t n_rows,
                                                      uint32_t *__restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), n_waves = (int64_t)gridDim.x * 4;
  uint32_t s = 0;
  for (int64_t r0 = wave * 8; r0 < n_rows; r0 += n_waves * 8) {
    int32_t idx[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) idx[u] = r0 + u < n_rows ? order[r0 + u] : -1;
    for (int c = lane; c < row16; c += 64) {
      u32x4 w[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) w[u] = idx[u] >= 0 ? src[(size_t)idx[u] * row16 + c] : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
      for (int u = 0; u < 8; ++u) s += w[u].x ^ w[u].y ^ w[u].z ^ w[u].w;
    }
  }
  if (s == 0x9e3779b9u) *sink = s;   // practically never: the loads stay, no write traffic
}

}  // namespace lv

using namespace lv;

extern "C" double litevggt_probe_mfma_flop(int dtype, int iters) {
  if (iters < 0 || (dtype != LV_ATTN_BF16 && dtype != LV_ATTN_FP8_E4M3)) return 0.0;
  const double k = dtype == LV_ATTN_FP8_E4M3 ? 64.0 : 16.0;
  return (double)kProbeGroups * 8.0 * (double)iters * 8.0 * 2.0 * 32.0 * 32.0 * k;
}

extern "C" int litevggt_probe_mfma(int dtype, const void *operands, int iters, float *out, void *stream) {
  if (!operands || !out) return LV_ERR_NULL;
  if (iters < 1 || iters > (1 << 20)) return LV_ERR_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == LV_ATTN_BF16)
    hipLaunchKernelGGL(k_probe_mfma<false>, dim3(kProbeGroups), dim3(512), 0, st, (const uint32_t *)operands, iters, out);
  else if (dtype == LV_ATTN_FP8_E4M3)
    hipLaunchKernelGGL(k_probe_mfma<true>, dim3(kProbeGroups), dim3(512), 0, st, (const uint32_t *)operands, iters, out);
  else
    return LV_ERR_DTYPE;
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

extern "C" int litevggt_probe_stream(const void *src, void *dst, size_t bytes, void *sink, void *stream) {
  if (!src || !sink) return LV_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0 || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return LV_ERR_SHAPE;
  hipLaunchKernelGGL(k_probe_stream, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const u32x4 *)src,
                     (u32x4 *)dst, bytes / 16, (uint32_t *)sink);
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

extern "C" int litevggt_probe_gather(const void *src, size_t row_bytes, const int32_t *order, int64_t n_rows,
                                     void *sink, void *stream) {
  if (!src || !order || !sink) return LV_ERR_NULL;
  if (n_rows < 1 || row_bytes == 0 || row_bytes % 16 != 0 || row_bytes > (1u << 20) || ((uintptr_t)src & 15))
    return LV_ERR_SHAPE;
  const int64_t groups = (n_rows + 31) / 32;
  hipLaunchKernelGGL(k_probe_gather, dim3((unsigned)(groups < 16384 ? groups : 16384)), dim3(256), 0,
                     (hipStream_t)stream, (const u32x4 *)src, (int)(row_bytes / 16), order, n_rows, (uint32_t *)sink);
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}
