// Geometry-aware map (Sec. 3.4 "Geometry-aware Feature Map"): Sobel gradient map,
// local token-variance map, per-frame min-max normalisation and fusion.
// All three kernels are HBM-bound streaming passes; arithmetic is fp32.
#include "common.h"
#include "internal.h"

namespace lv {

// ---------------------------------------------------------------------------------
// Psi_g.  One workgroup per (frame, patch row): the patch+2 luma rows it needs are
// built once in LDS (border pixels replicated), then each wave reduces whole patches.
// ---------------------------------------------------------------------------------
template <typename PixT>
__global__ __launch_bounds__(256) void k_grad_map(const PixT *__restrict__ img, int H, int W,
                                                  int patch, float *__restrict__ psi_g) {
  extern __shared__ float luma[];            // [(patch+2)][Wi+2]
  const int Hi = H * patch, Wi = W * patch, LW = Wi + 2;
  const int f = blockIdx.x / H, ph = blockIdx.x % H;
  const size_t plane = (size_t)Hi * Wi;
  const PixT *base = img + (size_t)f * 3 * plane;
  const float unit = sizeof(PixT) == 1 ? (1.0f / 255.0f) : 1.0f;
  for (int i = threadIdx.x; i < (patch + 2) * LW; i += blockDim.x) {
    int rr = i / LW, cc = i - rr * LW;
    int y = min(max(ph * patch + rr - 1, 0), Hi - 1);
    int x = min(max(cc - 1, 0), Wi - 1);
    size_t o = (size_t)y * Wi + x;
    float r = (float)base[o] * unit, g = (float)base[plane + o] * unit,
          b = (float)base[2 * plane + o] * unit;
    luma[i] = 0.299f * r + 0.587f * g + 0.114f * b;
  }
  __syncthreads();
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
  const int pp = patch * patch;
  for (int pw = wave; pw < W; pw += nw) {
    float acc = 0.f;
    for (int i = lane; i < pp; i += 64) {
      int py = i / patch, px = i - py * patch;
      const float *c = luma + (py + 1) * LW + pw * patch + px + 1;
      float tl = c[-LW - 1], tc = c[-LW], tr = c[-LW + 1];
      float ml = c[-1], mr = c[1];
      float bl = c[LW - 1], bc = c[LW], br = c[LW + 1];
      float gx = (tr + 2.f * mr + br) - (tl + 2.f * ml + bl);
      float gy = (bl + 2.f * bc + br) - (tl + 2.f * tc + tr);
      acc += sqrtf(gx * gx + gy * gy);
    }
    acc = wave_sum(acc);
    if (lane == 0) psi_g[((size_t)f * H + ph) * W + pw] = acc / (float)pp;
  }
}

int launch_grad_map(const void *images, int img_dtype, const Dims &d, int patch, float *psi_g,
                    hipStream_t st) {
  size_t lds = (size_t)(patch + 2) * (d.W * patch + 2) * sizeof(float);
  if (lds > 64 * 1024) return LV_ERR_SHAPE;
  dim3 grid((unsigned)(d.F * d.H));
  if (img_dtype == LV_IMG_F32)
    hipLaunchKernelGGL(k_grad_map<float>, grid, dim3(256), lds, st, (const float *)images, d.H,
                       d.W, patch, psi_g);
  else
    hipLaunchKernelGGL(k_grad_map<uint8_t>, grid, dim3(256), lds, st, (const uint8_t *)images,
                       d.H, d.W, patch, psi_g);
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

// ---------------------------------------------------------------------------------
// Psi_v.  One workgroup (2 waves) per (frame, grid row); thread t owns channels 8t..8t+7 (+1024k).
// The workgroup slides along the row: for every grid column it loads the K tokens of that
// column (rows i-R..i+R, clipped) once and keeps their per-channel sum and sum of squares
// for the last K columns in registers; the window of an output column is the sum of those K
// column partials, its variance E[d^2] - E[d]^2 in fp32 with d = x - (the frame's first patch
// token), so that the cancellation costs ~1e-7 of the spread and not of a channel's offset.
// Workgroups of consecutive grid rows are placed on the same XCD so the two neighbouring rows
// they share are found in that XCD's L2.
// ---------------------------------------------------------------------------------
template <int K>
__global__ __launch_bounds__(128) void k_var_map(const uint16_t *__restrict__ x, int F, int H,
                                                 int W, int S, int C, float *__restrict__ psi_v) {
  extern __shared__ float part[];            // [W][2 waves]
  const uint32_t nblk = (uint32_t)F * H;
  const uint32_t lb = xcd_contiguous(blockIdx.x, nblk);
  if (lb >= nblk) return;
  const int f = lb / H, i = lb % H;
  constexpr int R = K / 2;
  const int T = H * W + S;
  const uint16_t *frame = x + ((size_t)f * T + S) * C;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i0 = max(i - R, 0), i1 = min(i + R, H - 1);
  const int nrow = i1 - i0 + 1;
  for (int c0 = threadIdx.x * 8, pass = 0; c0 < (C + 1023) / 1024 * 1024; c0 += 1024, ++pass) {
    const bool on = c0 < C;                  // every thread walks every pass: part[] is per wave
    float s1[K][8], s2[K][8];                // column partials of the last K columns; slot = column % K
#pragma unroll
    for (int u = 0; u < K; ++u)
#pragma unroll
      for (int e = 0; e < 8; ++e) s1[u][e] = s2[u][e] = 0.f;
    // Sums are taken of x - pivot, the pivot being the frame's first patch token: the variance
    // does not change, and a channel that sits at a large offset (mean >> spread) no longer loses
    // its spread in the rounding of E[x^2] - E[x]^2.
    const u32x4 pbits = on ? *(const u32x4 *)(frame + c0) : u32x4{0u, 0u, 0u, 0u};
    const float pv[8] = {bf16_lo(pbits.x), bf16_hi(pbits.x), bf16_lo(pbits.y), bf16_hi(pbits.y),
                         bf16_lo(pbits.z), bf16_hi(pbits.z), bf16_lo(pbits.w), bf16_hi(pbits.w)};
    // the K tokens of a column are requested one column ahead of their use
    auto load_col = [&](int jj, u32x4(&w)[K]) {
#pragma unroll
      for (int a = 0; a < K; ++a) {          // rows outside the grid read as the pivot: they add nothing
        const int ii = i - R + a;
        w[a] = pbits;
        if (on && jj < W && ii >= i0 && ii <= i1) w[a] = *(const u32x4 *)(frame + ((size_t)ii * W + jj) * C + c0);
      }
    };
    u32x4 wcur[K], wnext[K];
    load_col(0, wcur);
    for (int jb = 0; jb < W + R; jb += K) {
#pragma unroll
      for (int u = 0; u < K; ++u) {
        const int jj = jb + u;               // column entering the window; output column is jj - R
        load_col(jj + 1, wnext);
        float a1[8], a2[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) a1[e] = a2[e] = 0.f;
#pragma unroll
        for (int a = 0; a < K; ++a) {        // (the pivot beyond the row end)
          const float v[8] = {bf16_lo(wcur[a].x), bf16_hi(wcur[a].x), bf16_lo(wcur[a].y), bf16_hi(wcur[a].y),
                              bf16_lo(wcur[a].z), bf16_hi(wcur[a].z), bf16_lo(wcur[a].w), bf16_hi(wcur[a].w)};
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float dlt = v[e] - pv[e];
            a1[e] += dlt;
            a2[e] = __builtin_fmaf(dlt, dlt, a2[e]);
          }
        }
#pragma unroll
        for (int a = 0; a < K; ++a) wcur[a] = wnext[a];
#pragma unroll
        for (int e = 0; e < 8; ++e) {        // columns beyond the row end enter as zeros of x - pivot
          s1[u][e] = a1[e];
          s2[u][e] = a2[e];
        }
        const int j = jj - R;
        if (j >= 0 && j < W) {
          const int j0 = max(j - R, 0), j1 = min(j + R, W - 1);
          const float inv_cnt = 1.0f / (float)(nrow * (j1 - j0 + 1));
          float tot = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            float t1 = 0.f, t2 = 0.f;
#pragma unroll
            for (int q = 0; q < K; ++q) {
              t1 += s1[q][e];
              t2 += s2[q][e];
            }
            const float m = t1 * inv_cnt;
            tot += __builtin_fmaf(-m, m, t2 * inv_cnt);
          }
          tot = wave_sum(tot);
          if (lane == 0) part[j * 2 + wave] = (pass ? part[j * 2 + wave] : 0.f) + tot;
        }
      }
    }
  }
  __syncthreads();
  for (int j = threadIdx.x; j < W; j += blockDim.x)
    psi_v[((size_t)f * H + i) * W + j] = (part[j * 2] + part[j * 2 + 1]) / (float)C;
}

// ---------------------------------------------------------------------------------
// Psi_v for the 3 x 3 window, every token row read once (plus a one-column halo on each side
// of a strip).  A workgroup (2 waves, lane = 8 channels, wave = 512 channels) owns a strip of
// kSeg grid columns of one frame and walks down the grid rows.  When row i arrives the window
// sums of output row i - 1 follow from
//   sum_c var_c = (1/n) sum_window e  -  (1/n^2) sum_c (sum_window d_c)^2,
// d = x - (the frame's first patch token), e = sum_c d_c^2 of one token: only the first moment
// needs per-channel window sums, the second moment is a window sum of one number per token.
// Per column the lane keeps d of row i-1 and the pair sum d(i-1) + d(i-2) in fp32, so every
// token is widened once: vertical sum = d(i) + pair, then pair <- d(i) + d(i-1); the horizontal
// 3-sum slides over the strip's columns.  Cells outside the grid are fed as the pivot token
// (d = 0) and n counts the cells inside.  The bits of row i+1 are requested into a column's
// registers as soon as that column of row i has been widened.
// ---------------------------------------------------------------------------------
#ifndef LV_VAR_SEG
#define LV_VAR_SEG 4
#endif
constexpr int kSeg = LV_VAR_SEG;
constexpr int kVarWaves = 2;                   // waves per workgroup: 512 channels each, 8 per lane

__global__ __launch_bounds__(64 * kVarWaves) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_var_map3(
    const uint16_t *__restrict__ x, int F, int H, int W, int S, int C, int nseg, float *__restrict__ psi_v) {
  constexpr int NC = kSeg + 2;               // columns a strip reads: its own and one on each side
  __shared__ float comb[2][kVarWaves][kSeg]; // the waves' partial sums of a grid row, by row parity
  const uint32_t nblk = (uint32_t)F * nseg;
  const uint32_t lb = xcd_contiguous(blockIdx.x, nblk);   // neighbouring strips share an L2
  if (lb >= nblk) return;
  const int f = lb / nseg, j0 = (int)(lb % nseg) * kSeg;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int T = H * W + S;
  const uint16_t *frame = x + ((size_t)f * T + S) * C;
  float *out = psi_v + (size_t)f * H * W;
  const float inv_c = 1.0f / (float)C;
  for (int cbase = 0; cbase < C; cbase += 512 * kVarWaves) {
    const int c0 = cbase + wave * 512 + lane * 8;
    const bool on = c0 < C;
    const u32x4 pbits = on ? *(const u32x4 *)(frame + c0) : u32x4{0u, 0u, 0u, 0u};
    const float pv[8] = {bf16_lo(pbits.x), bf16_hi(pbits.x), bf16_lo(pbits.y), bf16_hi(pbits.y),
                         bf16_lo(pbits.z), bf16_hi(pbits.z), bf16_lo(pbits.w), bf16_hi(pbits.w)};
    u32x4 raw[2][NC];                          // bits of rows i and i+1, by row parity; a column's
                                               // registers are refilled with row i+2 once used
    float d1[NC][8], pair[NC][8];              // d(i-1) and d(i-1) + d(i-2) per column
    float e1[NC], epair[NC];                   // the same for this lane's share of e
    auto fetch = [&](int i, int a, u32x4 &dst) {   // column a of the strip in grid row i, or the pivot
      const int jj = j0 - 1 + a;
      dst = pbits;
      if (on && i < H && jj >= 0 && jj < W) dst = *(const u32x4 *)(frame + ((size_t)i * W + jj) * C + c0);
    };
#pragma unroll
    for (int a = 0; a < NC; ++a) {
      fetch(0, a, raw[0][a]);
      fetch(1, a, raw[1][a]);
      e1[a] = epair[a] = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) d1[a][e] = pair[a][e] = 0.f;
    }
    auto step = [&](auto parity, int i) {      // grid row i arrives, output row i - 1 leaves
      u32x4(&rw)[NC] = raw[decltype(parity)::value];
      const int io = i - 1;
      const int nrow = min(io + 1, H - 1) - max(io - 1, 0) + 1;
      const float inv_r = nrow == 3 ? (1.0f / 3.0f) : nrow == 2 ? 0.5f : 1.0f;
      float v0[8], v1[8], v2[8];               // vertical sums of the last three columns
      float ve0 = 0.f, ve1 = 0.f, ve2 = 0.f;
      float res[kSeg];
#pragma unroll
      for (int e = 0; e < 8; ++e) v0[e] = v1[e] = v2[e] = 0.f;
#pragma unroll
      for (int a = 0; a < NC; ++a) {
        const u32x4 w = rw[a];
        const float xv[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                             bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
        fetch(i + 2, a, rw[a]);
        float e_new = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {          // slide: columns a - 2, a - 1 stay
          v0[e] = v1[e];
          v1[e] = v2[e];
          const float dn = xv[e] - pv[e];
          e_new = __builtin_fmaf(dn, dn, e_new);
          v2[e] = dn + pair[a][e];
          pair[a][e] = dn + d1[a][e];
          d1[a][e] = dn;
        }
        ve0 = ve1;
        ve1 = ve2;
        ve2 = e_new + epair[a];
        epair[a] = e_new + e1[a];
        e1[a] = e_new;
        if (a >= 2) {                          // output column j0 + a - 2
          const int jo = j0 + a - 2;
          const int ncol = min(jo + 1, W - 1) - max(jo - 1, 0) + 1;
          const float inv_n = (ncol == 3 ? (1.0f / 3.0f) : ncol == 2 ? 0.5f : 1.0f) * inv_r;   // scalar work
          float sq = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float h = v0[e] + v1[e] + v2[e];
            sq = __builtin_fmaf(h, h, sq);
          }
          const float m2 = (ve0 + ve1 + ve2) * inv_n;
          res[a - 2] = __builtin_fmaf(-sq * inv_n, inv_n, m2);
        }
      }
      // every lane holds its 8 channels' share of the strip's kSeg outputs of row io
#pragma unroll
      for (int q = 0; q < kSeg; ++q) res[q] = wave_sum_uniform(res[q]);
      float r = res[0];
#pragma unroll
      for (int q = 1; q < kSeg; ++q) r = lane == q ? res[q] : r;
      if (lane < kSeg) comb[i & 1][wave][lane] = r;
      __syncthreads();
      if (wave == 0 && lane < kSeg && io >= 0 && io < H && j0 + lane < W) {
        r = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < kVarWaves; ++w2) r += comb[i & 1][w2][lane];
        r *= inv_c;
        float *o = out + (size_t)io * W + j0 + lane;
        *o = cbase ? *o + r : r;
      }
    };
    // rows 0 .. H; row H is a row of pivots that flushes output row H - 1 (a step beyond it sees
    // pivots only and writes nothing)
    for (int i = 0; i <= H; i += 2) {
      step(std::integral_constant<int, 0>{}, i);
      step(std::integral_constant<int, 1>{}, i + 1);
    }
    __syncthreads();                           // comb is reused by the next channel pass
  }
}

int launch_var_map(const uint16_t *x, const Dims &d, int pool, float *psi_v, hipStream_t st) {
  if (pool == 3) {
    const int nseg = (d.W + kSeg - 1) / kSeg;
    hipLaunchKernelGGL(k_var_map3, dim3((unsigned)align_up((size_t)d.F * nseg, kXcd)), dim3(64 * kVarWaves), 0, st, x, d.F,
                       d.H, d.W, d.S, d.C, nseg, psi_v);
    LV_HIP_CHECK_LAUNCH();
    return LV_OK;
  }
  dim3 grid((unsigned)(align_up((size_t)d.F * d.H, kXcd)));
  size_t lds = (size_t)d.W * 2 * sizeof(float);
  switch (pool) {
    case 1:
      hipLaunchKernelGGL(k_var_map<1>, grid, dim3(128), lds, st, x, d.F, d.H, d.W, d.S, d.C, psi_v);
      break;
    case 5:
      hipLaunchKernelGGL(k_var_map<5>, grid, dim3(128), lds, st, x, d.F, d.H, d.W, d.S, d.C, psi_v);
      break;
    default:
      return LV_ERR_PARAM;
  }
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

// ---------------------------------------------------------------------------------
// Fusion: one workgroup per frame finds min/max of both maps, then writes
// alpha*norm(Psi_g) + beta*norm(Psi_v).
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_ga_fuse(const float *__restrict__ psi_g,
                                                 const float *__restrict__ psi_v, int P,
                                                 float alpha, float beta,
                                                 float *__restrict__ score) {
  __shared__ float red[4][4];
  const float *g = psi_g + (size_t)blockIdx.x * P, *v = psi_v + (size_t)blockIdx.x * P;
  float glo = INFINITY, ghi = -INFINITY, vlo = INFINITY, vhi = -INFINITY;
  for (int t = threadIdx.x; t < P; t += blockDim.x) {
    float a = g[t], b = v[t];
    glo = fminf(glo, a);
    ghi = fmaxf(ghi, a);
    vlo = fminf(vlo, b);
    vhi = fmaxf(vhi, b);
  }
  glo = wave_min(glo);
  ghi = wave_max(ghi);
  vlo = wave_min(vlo);
  vhi = wave_max(vhi);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane == 0) {
    red[wave][0] = glo;
    red[wave][1] = ghi;
    red[wave][2] = vlo;
    red[wave][3] = vhi;
  }
  __syncthreads();
  glo = fminf(fminf(red[0][0], red[1][0]), fminf(red[2][0], red[3][0]));
  ghi = fmaxf(fmaxf(red[0][1], red[1][1]), fmaxf(red[2][1], red[3][1]));
  vlo = fminf(fminf(red[0][2], red[1][2]), fminf(red[2][2], red[3][2]));
  vhi = fmaxf(fmaxf(red[0][3], red[1][3]), fmaxf(red[2][3], red[3][3]));
  const float gr = ghi - glo, vr = vhi - vlo;
  for (int t = threadIdx.x; t < P; t += blockDim.x) {
    float ng = gr > 0.f ? (g[t] - glo) / gr : 0.f;
    float nv = vr > 0.f ? (v[t] - vlo) / vr : 0.f;
    score[(size_t)blockIdx.x * P + t] = alpha * ng + beta * nv;
  }
}

int launch_ga_fuse(const float *psi_g, const float *psi_v, const Dims &d, float alpha, float beta,
                   float *score, hipStream_t st) {
  hipLaunchKernelGGL(k_ga_fuse, dim3((unsigned)d.F), dim3(256), 0, st, psi_g, psi_v, d.P, alpha,
                     beta, score);
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

// Scores of the geometry-blind partitions (Sec. 3.2 "Naive Token Merging"): a fixed
// low-discrepancy pattern over the token index, or an independent hash per (frame, token).
// 24-bit values, exact in fp32.
__global__ __launch_bounds__(256) void k_naive_score(int F, int P, int policy, uint32_t seed,
                                                     float *__restrict__ score) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)F * P) return;
  const uint32_t f = (uint32_t)(idx / P), t = (uint32_t)(idx % P);
  uint32_t hsh;
  if (policy == LV_POLICY_FIXED) {
    hsh = (t + 1u) * 2654435769u;                 // multiplicative hash by 2^32 / golden ratio
  } else {
    hsh = seed ^ (f * 0x9E3779B9u) ^ (t * 0x85EBCA6Bu);
    hsh ^= hsh >> 16;                             // 32-bit finaliser of MurmurHash3
    hsh *= 0x85EBCA6Bu;
    hsh ^= hsh >> 13;
    hsh *= 0xC2B2AE35u;
    hsh ^= hsh >> 16;
  }
  score[idx] = (float)(hsh >> 8) * (1.0f / 16777216.0f);
}

int launch_naive_score(const Dims &d, int policy, uint32_t seed, float *score, hipStream_t st) {
  const int64_t n = (int64_t)d.F * d.P;
  hipLaunchKernelGGL(k_naive_score, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, d.F, d.P,
                     policy, seed, score);
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

}  // namespace lv

// ---------------------------------------------------------------------------------
// Scratch for callers that cannot hand over a workspace (litevggt_importance_static): the
// variance map of one call lives in this file-scope device array.  Every GPU holds its own
// copy at its own address, so the address is looked up once per device, with that device
// current, and host code only ever uses the looked-up pointer (the array's name is a host-side
// stand-in, not a device address).
// ---------------------------------------------------------------------------------
namespace lv {

static __device__ __align__(256) float g_static_psi_v[kStaticScoreFloats];

int static_importance_scratch(float **out) {
  static std::atomic<float *> per_device[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return LV_ERR_HIP;
  if (dev < 0 || dev >= 64) return LV_ERR_HIP;
  float *p = per_device[dev].load(std::memory_order_acquire);
  if (!p) {
    void *sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(g_static_psi_v)) != hipSuccess || !sym) return LV_ERR_HIP;
    p = (float *)sym;
    per_device[dev].store(p, std::memory_order_release);   // the same value from every thread
  }
  *out = p;
  return LV_OK;
}

}  // namespace lv
