// Token partition (Sec. 3.4 "GA Token Partitioning"): one workgroup per frame keeps the
// frame's scores in LDS, picks one dst token per grid cell (lowest score), the GA tokens
// (highest scores among the rest) by rank counting, and writes the ascending index lists
// with a block-wide prefix sum.  All per-frame counts are closed-form, so every frame
// knows its output offsets without any cross-frame communication.
#include "common.h"
#include "internal.h"

namespace lv {

// fp32 score -> uint32 key with the same order (-0 folded onto +0; key 0 is reserved).
__device__ __forceinline__ uint32_t order_key(float s) {
  uint32_t b = __float_as_uint(s + 0.0f);
  uint32_t k = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
  return k == 0u ? 1u : k;
}

struct Tri {
  int k, d, s;
};
__device__ __forceinline__ Tri operator+(Tri a, Tri b) { return {a.k + b.k, a.d + b.d, a.s + b.s}; }

__global__ __launch_bounds__(256) void k_select(
    const float *__restrict__ score, int H, int W, int S, int cell, int n_ga, int n_dst_pf,
    int n_src_pf, uint8_t *__restrict__ role_out, int32_t *__restrict__ kept_idx,
    int32_t *__restrict__ dst_idx, int32_t *__restrict__ src_idx,
    int32_t *__restrict__ anchor_of, int32_t *__restrict__ slot_of) {
  extern __shared__ uint32_t smem[];
  const int P = H * W, T = P + S, f = blockIdx.x;
  uint32_t *key = smem;                       // [P] order keys
  uint32_t *cand = smem + P;                  // [P] key of non-dst tokens, 0 for dst tokens
  uint8_t *role = (uint8_t *)(smem + 2 * P);  // [P]
  __shared__ Tri wtot[4];
  const int tid = threadIdx.x;
  const bool all_dst = (f == 0) || (n_src_pf == 0);

  for (int t = tid; t < P; t += blockDim.x) {
    uint32_t k = order_key(score[(size_t)f * P + t]);
    key[t] = k;
    cand[t] = k;
    role[t] = all_dst ? LV_ROLE_DST : LV_ROLE_SRC;
  }
  __syncthreads();
  if (!all_dst) {
    const int ncw = (W + cell - 1) / cell, nch = (H + cell - 1) / cell;
    for (int c = tid; c < nch * ncw; c += blockDim.x) {
      const int ci = (c / ncw) * cell, cj = (c % ncw) * cell;
      uint32_t best = 0xffffffffu;
      int bt = -1;
      for (int i = ci; i < min(H, ci + cell); ++i)
        for (int j = cj; j < min(W, cj + cell); ++j) {
          uint32_t k = key[i * W + j];
          if (bt < 0 || k < best) {
            best = k;
            bt = i * W + j;
          }
        }
      role[bt] = LV_ROLE_DST;
      cand[bt] = 0u;
    }
    __syncthreads();
    if (n_ga > 0) {
      for (int t = tid; t < P; t += blockDim.x) {
        const uint32_t k = cand[t];
        if (k == 0u) continue;
        int rank = 0;
        for (int u = 0; u < P; ++u) {
          uint32_t ku = cand[u];
          rank += (ku > k) || (ku == k && u < t);
        }
        if (rank < n_ga) role[t] = LV_ROLE_PROTECTED;
      }
    }
    __syncthreads();
  }

  // prefix sums of (kept, dst, src) flags over the frame's T tokens, chunk per thread
  const int per = (T + blockDim.x - 1) / blockDim.x;
  const int t0 = min(tid * per, T), t1 = min(t0 + per, T);
  Tri mine = {0, 0, 0};
  for (int t = t0; t < t1; ++t) {
    int r = t < S ? LV_ROLE_PROTECTED : role[t - S];
    mine.k += r != LV_ROLE_SRC;
    mine.d += r == LV_ROLE_DST;
    mine.s += r == LV_ROLE_SRC;
  }
  Tri inc = mine;
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    Tri n = {__shfl_up(inc.k, o, 64), __shfl_up(inc.d, o, 64), __shfl_up(inc.s, o, 64)};
    if (lane >= o) inc = inc + n;
  }
  if (lane == 63) wtot[wave] = inc;
  __syncthreads();
  Tri base = {0, 0, 0};
  for (int w = 0; w < wave; ++w) base = base + wtot[w];
  Tri pos = {base.k + inc.k - mine.k, base.d + inc.d - mine.d, base.s + inc.s - mine.s};

  const int K = n_dst_pf + n_ga;
  const int64_t kb = f == 0 ? 0 : (int64_t)T + (int64_t)(f - 1) * (S + K);
  const int64_t db = f == 0 ? 0 : (int64_t)P + (int64_t)(f - 1) * n_dst_pf;
  const int64_t sb = f == 0 ? 0 : (int64_t)(f - 1) * n_src_pf;
  for (int t = t0; t < t1; ++t) {
    const int r = t < S ? LV_ROLE_PROTECTED : role[t - S];
    const int64_t g = (int64_t)f * T + t;
    role_out[g] = (uint8_t)r;
    if (r != LV_ROLE_SRC) {
      kept_idx[kb + pos.k] = (int32_t)g;
      slot_of[g] = (int32_t)(kb + pos.k);
      anchor_of[g] = (int32_t)g;
      ++pos.k;
    }
    if (r == LV_ROLE_DST) dst_idx[db + pos.d++] = (int32_t)g;
    if (r == LV_ROLE_SRC) src_idx[sb + pos.s++] = (int32_t)g;
  }
}

int launch_select(const float *score, const Dims &d, const litevggt_plan_t &pl,
                  const litevggt_index &ix, hipStream_t st) {
  size_t lds = (size_t)d.P * 9;
  lds = align_up(lds, 16);
  if (lds > 60 * 1024) return LV_ERR_SHAPE;
  hipLaunchKernelGGL(k_select, dim3((unsigned)d.F), dim3(256), lds, st, score, d.H, d.W, d.S,
                     pl.cell, pl.n_ga_per_frame, pl.n_dst_per_frame, pl.n_src_per_frame, ix.role,
                     ix.kept_idx, ix.dst_idx, ix.src_idx, ix.anchor_of, ix.slot_of);
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

}  // namespace lv
