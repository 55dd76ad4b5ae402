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

#ifndef LV_MERGE_COOP
#define LV_MERGE_COOP 64
#endif
constexpr int kCoopSize = LV_MERGE_COOP;   // groups larger than this are summed by all 4 waves of a workgroup

// acc += rows group_mem[lo..hi) of x, this lane's chunks; R member rows in flight per lane.
// Rows are taken in batches of R; the last batch is masked (lo, hi are wave-uniform), so its
// loads are issued together as well.  The member indices of a batch are fetched while the rows
// of the batch before it are in flight, so a batch costs one memory round trip, not two.
template <int CPL, int R>
__device__ __forceinline__ void sum_rows(const uint16_t *__restrict__ x,
                                         const int32_t *__restrict__ group_mem, int lo, int hi,
                                         int C, int nch, int lane, float (&a)[CPL][8]) {
  int r[R];
#pragma unroll
  for (int u = 0; u < R; ++u) r[u] = lo + u < hi ? group_mem[lo + u] : -1;
  for (int j = lo; j < hi; j += R) {
    u32x4 w[R][CPL];
#pragma unroll
    for (int u = 0; u < R; ++u)
#pragma unroll
      for (int c = 0; c < CPL; ++c) {
        const int ch = lane + 64 * c;
        w[u][c] = (r[u] >= 0 && ch < nch) ? ((const u32x4 *)(x + (size_t)r[u] * C))[ch] : u32x4{0u, 0u, 0u, 0u};
      }
#pragma unroll
    for (int u = 0; u < R; ++u) r[u] = j + R + u < hi ? group_mem[j + R + u] : -1;
#pragma unroll
    for (int u = 0; u < R; ++u)
#pragma unroll
      for (int c = 0; c < CPL; ++c) acc8(a[c], w[u][c]);
  }
}

template <int CPL>
__device__ __forceinline__ void store_mean(uint16_t *__restrict__ z, int m, int C, int nch, int lane,
                                           const float (&a)[CPL][8], float inv) {
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const int ch = lane + 64 * c;
    if (ch < nch) {
      u32x4 o;
      o.x = pack_bf16(a[c][0] * inv, a[c][1] * inv);
      o.y = pack_bf16(a[c][2] * inv, a[c][3] * inv);
      o.z = pack_bf16(a[c][4] * inv, a[c][5] * inv);
      o.w = pack_bf16(a[c][6] * inv, a[c][7] * inv);
      ((u32x4 *)(z + (size_t)m * C))[ch] = o;
    }
  }
}

// Slots with at most kCoopSize members are summed by one wave each, in ascending member
// order (a workgroup takes 4 consecutive slots).  Larger groups (a heavy tail: a few percent of
// the slots hold most of the tokens once the features have been through some layers) are
// summed by all 4 waves of a workgroup, each taking a contiguous quarter of the members, and
// the four partial sums are added in wave order -- the order of additions depends only on the
// group size, so results are reproducible.  The large groups are the long jobs, so they are
// started first: workgroups 0 .. nb0-1 scan kScan slots each (nb0 apart) and sum the large
// groups among them, workgroups nb0 .. take the small ones behind them.
constexpr int kScan = 64;

template <int CPL>
__global__ __launch_bounds__(256) void k_merge(const uint16_t *__restrict__ x,
                                               const int32_t *__restrict__ group_off,
                                               const int32_t *__restrict__ group_mem, int M,
                                               int C, int nb0, uint16_t *__restrict__ z) {
  __shared__ float part[3][CPL * 64 * 8];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nch = C >> 3;
  if ((int)blockIdx.x < nb0) {           // cooperative pass over the large groups of kScan slots
    // strided: neighbouring slots (the all-dst first frame) hold the largest groups
    const int64_t ms = (int64_t)blockIdx.x + (int64_t)lane * nb0;
    const int bl = ms < M ? group_off[ms] : 0, el = ms < M ? group_off[ms + 1] : 0;
    uint64_t big = __builtin_amdgcn_ballot_w64(el - bl > kCoopSize);   // same in every wave
    while (big) {
      const int s = __builtin_ctzll(big);
      big &= big - 1;
      const int m = (int)(blockIdx.x + (int64_t)s * nb0);   // < M: its lane passed the range check
      const int b = __builtin_amdgcn_readlane(bl, s), e = __builtin_amdgcn_readlane(el, s), n = e - b;
      const int per = (n + 3) >> 2;
      const int lo = min(b + wave * per, e), hi = min(lo + per, e);
      float a[CPL][8];
#pragma unroll
      for (int c = 0; c < CPL; ++c)
#pragma unroll
        for (int i = 0; i < 8; ++i) a[c][i] = 0.f;
      sum_rows<CPL, 16>(x, group_mem, lo, hi, C, nch, lane, a);
      if (wave > 0) {
#pragma unroll
        for (int c = 0; c < CPL; ++c)
#pragma unroll
          for (int i = 0; i < 8; ++i) part[wave - 1][(c * 8 + i) * 64 + lane] = a[c][i];
      }
      __syncthreads();
      if (wave == 0) {
#pragma unroll
        for (int w = 0; w < 3; ++w)
#pragma unroll
          for (int c = 0; c < CPL; ++c)
#pragma unroll
            for (int i = 0; i < 8; ++i) a[c][i] += part[w][(c * 8 + i) * 64 + lane];
        store_mean<CPL>(z, m, C, nch, lane, a, 1.0f / (float)n);
      }
      __syncthreads();
    }
    return;
  }
  const int m = ((int)blockIdx.x - nb0) * 4 + wave;   // own slot, if small
  if (m < M) {
    const int b = group_off[m], e = group_off[m + 1];
    if (e - b <= kCoopSize) {
      float a[CPL][8];
#pragma unroll
      for (int c = 0; c < CPL; ++c)
#pragma unroll
        for (int i = 0; i < 8; ++i) a[c][i] = 0.f;
      sum_rows<CPL, 8>(x, group_mem, b, e, C, nch, lane, a);
      store_mean<CPL>(z, m, C, nch, lane, a, 1.0f / (float)(e - b));
    }
  }
}

int launch_merge(const uint16_t *x, const Dims &d, int64_t M, const litevggt_index &ix,
                 uint16_t *z, hipStream_t st) {
  const int cpl = (d.C / 8 + 63) / 64;
  const int nb0 = (int)((M + kScan - 1) / kScan);
  const unsigned grid = (unsigned)(nb0 + (M + 3) / 4);
#define LV_MERGE(CPL)                                                                       \
  hipLaunchKernelGGL(k_merge<CPL>, dim3(grid), dim3(256), 0, st, x, ix.group_off, ix.group_mem, \
                     (int)M, d.C, nb0, z)
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

#ifndef LV_UNMERGE_ROWS
#define LV_UNMERGE_ROWS 2
#endif
// out[i] = y[slot_of[i]] (+ residual[i]); a wave moves LV_UNMERGE_ROWS token rows per step
// (all loads of a step are issued before its stores), grid-stride over row groups.
template <bool RES>
__global__ __launch_bounds__(256) void k_unmerge(const uint16_t *__restrict__ y,
                                                 const int32_t *__restrict__ slot_of,
                                                 const uint16_t *residual, int64_t N, int C,
                                                 uint16_t *out) {
  constexpr int R = LV_UNMERGE_ROWS;
  const int lane = threadIdx.x & 63;
  const int nch = C >> 3;
  const int wpb = blockDim.x >> 6;
  for (int64_t i0 = ((int64_t)blockIdx.x * wpb + (threadIdx.x >> 6)) * R; i0 < N;
       i0 += (int64_t)gridDim.x * wpb * R) {
    int slot[R];
#pragma unroll
    for (int r = 0; r < R; ++r) slot[r] = slot_of[min(i0 + r, N - 1)];
    for (int ch = lane; ch < nch; ch += 64) {
      u32x4 w[R], res[R];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        w[r] = ((const u32x4 *)(y + (size_t)slot[r] * C))[ch];
        if (RES) res[r] = ((const u32x4 *)(residual + (size_t)min(i0 + r, N - 1) * C))[ch];
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        if (i0 + r >= N) break;
        u32x4 v = w[r];
        if (RES) {
          v.x = pack_bf16(bf16_lo(v.x) + bf16_lo(res[r].x), bf16_hi(v.x) + bf16_hi(res[r].x));
          v.y = pack_bf16(bf16_lo(v.y) + bf16_lo(res[r].y), bf16_hi(v.y) + bf16_hi(res[r].y));
          v.z = pack_bf16(bf16_lo(v.z) + bf16_lo(res[r].z), bf16_hi(v.z) + bf16_hi(res[r].z));
          v.w = pack_bf16(bf16_lo(v.w) + bf16_lo(res[r].w), bf16_hi(v.w) + bf16_hi(res[r].w));
        }
        __builtin_nontemporal_store(v, (u32x4 *)(out + (size_t)(i0 + r) * C) + ch);
      }
    }
  }
}

int launch_unmerge(const uint16_t *y, const Dims &d, const litevggt_index &ix,
                   const uint16_t *residual, uint16_t *out, hipStream_t st) {
  const int64_t want = (d.N + 4 * LV_UNMERGE_ROWS - 1) / (4 * LV_UNMERGE_ROWS);
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
