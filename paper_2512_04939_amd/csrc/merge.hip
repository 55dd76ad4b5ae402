// Merge (Sec. 3.4 merge equation) and unmerge (Sec. 3.4 "Token Unmerging").
// Both are pure HBM streaming: every token row (dim bf16 values, 2 KB at dim 1024) is
// read or written exactly once with 16-byte accesses per lane, whole rows per wave.
#include "common.h"
#include "internal.h"

namespace lv {

__device__ __forceinline__ void acc8(float (&a)[8], const u32x4 w) {
  a[0] += bf16_lo(w.x);
  a[1] += bf16_hi(w.x);
  a[2] += bf16_lo(w.y);
  a[3] += bf16_hi(w.y);
  a[4] += bf16_lo(w.z);
  a[5] += bf16_hi(w.z);
  a[6] += bf16_lo(w.w);
  a[7] += bf16_hi(w.w);
}

// One wave per merged slot; lane l owns the 16-byte chunks l, l+64, ... of the row.
// Members are summed in ascending token order (the CSR order), so the result does not
// depend on scheduling.  Four member rows are in flight per lane.
template <int CPL>
__global__ __launch_bounds__(256) void k_merge(const uint16_t *__restrict__ x,
                                               const int32_t *__restrict__ group_off,
                                               const int32_t *__restrict__ group_mem, int M,
                                               int C, uint16_t *__restrict__ z) {
  const int lane = threadIdx.x & 63;
  const int nch = C >> 3;
  const int wpb = blockDim.x >> 6;
  for (int m = blockIdx.x * wpb + (threadIdx.x >> 6); m < M; m += gridDim.x * wpb) {
    const int mu = __builtin_amdgcn_readfirstlane(m);
    const int b = group_off[mu], e = group_off[mu + 1];
    float a[CPL][8];
#pragma unroll
    for (int c = 0; c < CPL; ++c)
#pragma unroll
      for (int i = 0; i < 8; ++i) a[c][i] = 0.f;
    int j = b;
    for (; j + 4 <= e; j += 4) {
      const int r0 = group_mem[j], r1 = group_mem[j + 1], r2 = group_mem[j + 2],
                r3 = group_mem[j + 3];
      u32x4 w[4][CPL];
#pragma unroll
      for (int c = 0; c < CPL; ++c) {
        const int ch = lane + 64 * c;
        if (ch < nch) {
          w[0][c] = ((const u32x4 *)(x + (size_t)r0 * C))[ch];
          w[1][c] = ((const u32x4 *)(x + (size_t)r1 * C))[ch];
          w[2][c] = ((const u32x4 *)(x + (size_t)r2 * C))[ch];
          w[3][c] = ((const u32x4 *)(x + (size_t)r3 * C))[ch];
        } else {
          w[0][c] = w[1][c] = w[2][c] = w[3][c] = u32x4{0u, 0u, 0u, 0u};
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc8(a[c], w[u][c]);
    }
    for (; j < e; ++j) {
      const int r0 = group_mem[j];
#pragma unroll
      for (int c = 0; c < CPL; ++c) {
        const int ch = lane + 64 * c;
        if (ch < nch) acc8(a[c], ((const u32x4 *)(x + (size_t)r0 * C))[ch]);
      }
    }
    const float inv = 1.0f / (float)(e - b);
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
      const int ch = lane + 64 * c;
      if (ch < nch) {
        u32x4 o;
        o.x = pack_bf16(a[c][0] * inv, a[c][1] * inv);
        o.y = pack_bf16(a[c][2] * inv, a[c][3] * inv);
        o.z = pack_bf16(a[c][4] * inv, a[c][5] * inv);
        o.w = pack_bf16(a[c][6] * inv, a[c][7] * inv);
        ((u32x4 *)(z + (size_t)mu * C))[ch] = o;
      }
    }
  }
}

int launch_merge(const uint16_t *x, const Dims &d, int64_t M, const litevggt_index &ix,
                 uint16_t *z, hipStream_t st) {
  const int cpl = (d.C / 8 + 63) / 64;
  const unsigned grid = (unsigned)((M + 3) / 4);
#define LV_MERGE(CPL)                                                                       \
  hipLaunchKernelGGL(k_merge<CPL>, dim3(grid), dim3(256), 0, st, x, ix.group_off, ix.group_mem, \
                     (int)M, d.C, z)
  switch (cpl) {
    case 1: LV_MERGE(1); break;
    case 2: LV_MERGE(2); break;
    case 3: LV_MERGE(3); break;
    case 4: LV_MERGE(4); break;
    default: return LV_ERR_SHAPE;
  }
#undef LV_MERGE
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

// out[i] = y[slot_of[i]] (+ residual[i]); one wave per token row, grid-stride over rows.
template <bool RES>
__global__ __launch_bounds__(256) void k_unmerge(const uint16_t *__restrict__ y,
                                                 const int32_t *__restrict__ slot_of,
                                                 const uint16_t *residual, int64_t N, int C,
                                                 uint16_t *out) {
  const int lane = threadIdx.x & 63;
  const int nch = C >> 3;
  const int wpb = blockDim.x >> 6;
  for (int64_t i = (int64_t)blockIdx.x * wpb + (threadIdx.x >> 6); i < N;
       i += (int64_t)gridDim.x * wpb) {
    const int s = slot_of[i];
    const u32x4 *src = (const u32x4 *)(y + (size_t)s * C);
    u32x4 *dst = (u32x4 *)(out + (size_t)i * C);
    for (int ch = lane; ch < nch; ch += 64) {
      u32x4 w = src[ch];
      if (RES) {
        const u32x4 r = ((const u32x4 *)(residual + (size_t)i * C))[ch];
        w.x = pack_bf16(bf16_lo(w.x) + bf16_lo(r.x), bf16_hi(w.x) + bf16_hi(r.x));
        w.y = pack_bf16(bf16_lo(w.y) + bf16_lo(r.y), bf16_hi(w.y) + bf16_hi(r.y));
        w.z = pack_bf16(bf16_lo(w.z) + bf16_lo(r.z), bf16_hi(w.z) + bf16_hi(r.z));
        w.w = pack_bf16(bf16_lo(w.w) + bf16_lo(r.w), bf16_hi(w.w) + bf16_hi(r.w));
      }
      __builtin_nontemporal_store(w, dst + ch);
    }
  }
}

int launch_unmerge(const uint16_t *y, const Dims &d, const litevggt_index &ix,
                   const uint16_t *residual, uint16_t *out, hipStream_t st) {
  const int64_t want = (d.N + 3) / 4;
  const unsigned grid = (unsigned)(want < 256 * 64 ? want : 256 * 64);
  if (residual)
    hipLaunchKernelGGL(k_unmerge<true>, dim3(grid), dim3(256), 0, st, y, ix.slot_of, residual, d.N,
                       d.C, out);
  else
    hipLaunchKernelGGL(k_unmerge<false>, dim3(grid), dim3(256), 0, st, y, ix.slot_of, residual,
                       d.N, d.C, out);
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

}  // namespace lv
