// Full (unmasked) self-attention over the merged sequence of all frames, per head
// (Sec. 3.1 "Bottleneck Analysis": every token attends to every token of every frame).
//
// Flash-style: scores never leave registers, softmax is computed online in fp32.
// Layout choices for CDNA4 (wave64, v_mfma_f32_32x32x16_bf16):
//   * the score tile is computed transposed, S^T = K Q^T, so that a lane owns one query
//     column: row max / row sum are in-lane reductions plus one exchange between the two
//     lane halves, and the exponentiated tile is already in the B-operand layout of the
//     second contraction O^T += V^T P^T -- probabilities go from accumulator registers
//     to MFMA operands without touching LDS;
//   * K and V are re-laid out once per call into "fragment-major" order (each MFMA A
//     operand is 1 KB contiguous), V with the key permutation that the accumulator layout
//     of S^T induces.  A K/V tile is then a straight 16 KB copy into LDS, read back
//     conflict-free with ds_read_b128;
//   * a wave owns 64 queries (two 32-wide MFMA column blocks) so every K/V fragment read
//     from LDS feeds two MFMAs; a workgroup owns 256 queries;
//   * workgroups are dealt to the 8 XCDs round-robin by hardware, so the grid is ordered
//     to give each XCD whole heads: all CUs of an XCD stream the same K/V through one L2.
#include "common.h"
#include "internal.h"

namespace lv {

constexpr int kKT = 32;              // keys per MFMA tile
constexpr int kKV = 64;              // keys per LDS stage (2 MFMA tiles)
constexpr int kQW = 64;              // queries per wave
constexpr int kQB = 256;             // queries per workgroup
constexpr int kFragU4 = 64;          // one fragment = 64 lanes x 16 B

constexpr float kQkEps = 1e-6f;
constexpr float kRaise = 8.0f;       // log2 headroom before the softmax reference is raised

// RMS-normalise a 64-value head row that is spread over 2^log2_lanes neighbouring lanes (8
// bf16 values each, or several such chunks per lane): returns this lane's chunk scaled by
// 1/sqrt(mean(x^2) + eps), rounded to bf16.
__device__ __forceinline__ float sumsq8(const u32x4 w) {
  const float a0 = bf16_lo(w.x), a1 = bf16_hi(w.x), a2 = bf16_lo(w.y), a3 = bf16_hi(w.y);
  const float a4 = bf16_lo(w.z), a5 = bf16_hi(w.z), a6 = bf16_lo(w.w), a7 = bf16_hi(w.w);
  return ((a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3)) + ((a4 * a4 + a5 * a5) + (a6 * a6 + a7 * a7));
}
__device__ __forceinline__ u32x4 scale8(const u32x4 w, float r) {
  return u32x4{pack_bf16(bf16_lo(w.x) * r, bf16_hi(w.x) * r), pack_bf16(bf16_lo(w.y) * r, bf16_hi(w.y) * r),
               pack_bf16(bf16_lo(w.z) * r, bf16_hi(w.z) * r), pack_bf16(bf16_lo(w.w) * r, bf16_hi(w.w) * r)};
}
__device__ __forceinline__ u32x4 rms_scale8(const u32x4 w, int log2_lanes) {
  float ss = sumsq8(w);
  for (int o = 1; o < (1 << log2_lanes); o <<= 1) ss += __shfl_xor(ss, o, 64);
  return scale8(w, 1.0f / sqrtf(ss * (1.0f / 64.0f) + kQkEps));
}

// K -> [head][key tile][k-step s][lane] : lane (h*32+r) holds K[tile*32+r][16s+8h .. +8]
// V -> [head][key tile][u][dt][lane]    : lane (h*32+dr) holds, for e = 0..7,
//      V[tile*32 + 16u + 8(e/4) + 4h + e%4][32dt + dr]   (the key order in which a lane of
//      the S^T accumulator holds its rows, so P needs no shuffle before the second MFMA)
__global__ __launch_bounds__(256) void k_attn_pack(const uint16_t *__restrict__ k,
                                                   const uint16_t *__restrict__ v, int64_t n,
                                                   int heads, int n_kt, int qk_norm,
                                                   u32x4 *__restrict__ kp,
                                                   u32x4 *__restrict__ vp) {
  __shared__ __attribute__((aligned(16))) uint16_t vt[kKT][72];
  const int kt = blockIdx.x, head = blockIdx.y, t = threadIdx.x;
  const int C = heads * 64;
  const int key = t >> 3, chunk = t & 7;
  const int64_t row = (int64_t)kt * kKT + key;
  u32x4 wk = {0u, 0u, 0u, 0u}, wv = {0u, 0u, 0u, 0u};
  if (row < n) {
    wk = *(const u32x4 *)(k + (size_t)row * C + head * 64 + chunk * 8);
    wv = *(const u32x4 *)(v + (size_t)row * C + head * 64 + chunk * 8);
  }
  if (qk_norm) wk = rms_scale8(wk, 3);   // the 8 lanes that share a key hold its 64 values
  const size_t tile = ((size_t)head * n_kt + kt) * 4 * kFragU4;
  kp[tile + (chunk >> 1) * kFragU4 + (chunk & 1) * 32 + key] = wk;
  *(u32x4 *)&vt[key][chunk * 8] = wv;
  __syncthreads();
  const int u = t >> 7, dt = (t >> 6) & 1, lane = t & 63, h = lane >> 5, dr = lane & 31;
  uint32_t w[4];
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    const int k0 = 16 * u + 8 * (e >> 2) + 4 * h + (e & 3);
    w[e >> 1] = (uint32_t)vt[k0][32 * dt + dr] | ((uint32_t)vt[k0 + 1][32 * dt + dr] << 16);
  }
  vp[tile + (u * 2 + dt) * kFragU4 + lane] = u32x4{w[0], w[1], w[2], w[3]};
}

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

template <bool RAGGED_UNUSED = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_attn_bf16(
    const uint16_t *__restrict__ q, const u32x4 *__restrict__ kp, const u32x4 *__restrict__ vp,
    uint16_t *__restrict__ o, int64_t n, int heads, int n_kt, int nqb, float c, int qk_norm) {
  __shared__ u32x4 ks[2][8 * kFragU4];
  __shared__ u32x4 vs[2][8 * kFragU4];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, h = lane >> 5, ql = lane & 31;
  const int C = heads * 64;
  int head, qb;
  if ((heads & 7) == 0) {
    const int hp = heads >> 3, xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    head = xcd * hp + local / nqb;
    qb = local % nqb;
  } else {
    head = blockIdx.x / nqb;
    qb = blockIdx.x % nqb;
  }
  const int64_t q0 = (int64_t)qb * kQB + wave * kQW;

  // Q^T fragments (B operand): lane (h*32+ql) holds Q[q0+32*sub+ql][16s+8h .. +8]
  bf16x8 qf[2][4];
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const int64_t row = min(q0 + sub * 32 + ql, n - 1);
    const uint16_t *qp = q + (size_t)row * C + head * 64 + 8 * h;
    u32x4 w[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) w[s] = *(const u32x4 *)(qp + 16 * s);
    if (qk_norm) {   // this lane holds 32 of the row's 64 values, lane^32 the other 32
      float ss = (sumsq8(w[0]) + sumsq8(w[1])) + (sumsq8(w[2]) + sumsq8(w[3]));
      ss += __shfl_xor(ss, 32, 64);
      const float r = 1.0f / sqrtf(ss * (1.0f / 64.0f) + kQkEps);
#pragma unroll
      for (int s = 0; s < 4; ++s) w[s] = scale8(w[s], r);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) qf[sub][s] = __builtin_bit_cast(bf16x8, w[s]);
  }

  f32x16 oacc[2][2];
#pragma unroll
  for (int sub = 0; sub < 2; ++sub)
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[sub][dt][r] = 0.f;
  float mref[2] = {-INFINITY, -INFINITY}, mc[2] = {0.f, 0.f}, lrow[2] = {0.f, 0.f};
  const bf16x2 kOnes = {(__bf16)1.0f, (__bf16)1.0f};

  const int nkv = n_kt >> 1;
  const u32x4 *kh = kp + (size_t)head * n_kt * 4 * kFragU4;
  const u32x4 *vh = vp + (size_t)head * n_kt * 4 * kFragU4;
  u32x4 rk[2], rv[2];
  rk[0] = kh[tid];
  rk[1] = kh[256 + tid];
  rv[0] = vh[tid];
  rv[1] = vh[256 + tid];
  ks[0][tid] = rk[0];
  ks[0][256 + tid] = rk[1];
  vs[0][tid] = rv[0];
  vs[0][256 + tid] = rv[1];
  __syncthreads();

  for (int it = 0; it < nkv; ++it) {
    const int buf = it & 1;
    if (it + 1 < nkv) {
      const size_t off = (size_t)(it + 1) * 8 * kFragU4;
      rk[0] = kh[off + tid];
      rk[1] = kh[off + 256 + tid];
      rv[0] = vh[off + tid];
      rv[1] = vh[off + 256 + tid];
    }
    // ---- S^T = K Q^T for the 64 keys of this stage
    f32x16 sacc[2][2];   // [key tile][query block]
#pragma unroll
    for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[kt2][sub][r] = 0.f;
#pragma unroll
    for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, ks[buf][(kt2 * 4 + s) * kFragU4 + lane]);
        sacc[kt2][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0][s], sacc[kt2][0], 0, 0, 0);
        sacc[kt2][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[1][s], sacc[kt2][1], 0, 0, 0);
      }
    if (it == nkv - 1) {   // keys beyond the sequence end in the last stage
      const int64_t kbase = (int64_t)it * kKV;
      if (kbase + kKV > n) {
#pragma unroll
        for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int64_t key = kbase + kt2 * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
            if (key >= n) {
              sacc[kt2][0][r] = -INFINITY;
              sacc[kt2][1][r] = -INFINITY;
            }
          }
      }
    }
    // ---- online softmax, one query column per lane.  The running reference mref is only
    // raised (and O, l rescaled) when some lane's tile maximum exceeds it by more than
    // kRaise in log2 units, so weights stay below 2^kRaise and rescaling is rare.
    u32x4 pb[2][2][2];   // [query block][key tile][u]
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      float mx = -INFINITY;
#pragma unroll
      for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
        for (int r = 0; r < 16; r += 2) mx = max3(mx, sacc[kt2][sub][r], sacc[kt2][sub][r + 1]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      if (__builtin_amdgcn_ballot_w64((mx - mref[sub]) * c > kRaise) != 0) {
        const float mnew = fmaxf(mref[sub], mx);
        const float alpha = __builtin_amdgcn_exp2f((mref[sub] - mnew) * c);
        mref[sub] = mnew;
        mc[sub] = mnew * c;
        lrow[sub] *= alpha;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[sub][dt][r] *= alpha;
      }
      float ls = lrow[sub];
#pragma unroll
      for (int kt2 = 0; kt2 < 2; ++kt2) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r)
          p[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kt2][sub][r], c, -mc[sub]));
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          uint32_t w[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            w[e] = pack_bf16(p[8 * u + 2 * e], p[8 * u + 2 * e + 1]);
            // row sum of the bf16-rounded weights (what the second MFMA really multiplies)
            ls = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w[e]), kOnes, ls, false);
          }
          pb[sub][kt2][u] = u32x4{w[0], w[1], w[2], w[3]};
        }
      }
      lrow[sub] = ls;
    }
    // ---- O^T += V^T P^T
#pragma unroll
    for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
          const bf16x8 a = __builtin_bit_cast(bf16x8, vs[buf][((kt2 * 2 + u) * 2 + dt) * kFragU4 + lane]);
          oacc[0][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              a, __builtin_bit_cast(bf16x8, pb[0][kt2][u]), oacc[0][dt], 0, 0, 0);
          oacc[1][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              a, __builtin_bit_cast(bf16x8, pb[1][kt2][u]), oacc[1][dt], 0, 0, 0);
        }
    if (it + 1 < nkv) {
      ks[buf ^ 1][tid] = rk[0];
      ks[buf ^ 1][256 + tid] = rk[1];
      vs[buf ^ 1][tid] = rv[0];
      vs[buf ^ 1][256 + tid] = rv[1];
    }
    __syncthreads();
  }

  // ---- normalise and store: lane holds query column ql, rows d = 32dt + 8g + 4h + i
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const float l = lrow[sub] + __shfl_xor(lrow[sub], 32, 64);
    const float inv = 1.0f / l;
    const int64_t row = q0 + sub * 32 + ql;
    if (row < n) {
      uint16_t *op = o + (size_t)row * C + head * 64 + 4 * h;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 w = {pack_bf16(oacc[sub][dt][4 * g] * inv, oacc[sub][dt][4 * g + 1] * inv),
                     pack_bf16(oacc[sub][dt][4 * g + 2] * inv, oacc[sub][dt][4 * g + 3] * inv)};
          *(u32x2 *)(op + 32 * dt + 8 * g) = w;
        }
    }
  }
}

static int n_key_tiles(int64_t n) { return (int)(2 * ((n + kKV - 1) / kKV)); }

size_t attn_ws_bytes(int heads, int64_t n_tokens, int attn_dtype) {
  (void)attn_dtype;
  const size_t per = (size_t)heads * n_key_tiles(n_tokens) * 4 * kFragU4 * sizeof(u32x4);
  return 2 * align_up(per, 256);
}

int launch_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v, uint16_t *o,
                int64_t n, int heads, float scale, int attn_dtype, int qk_norm, void *ws,
                hipStream_t st, hipEvent_t after_pack) {
  if (attn_dtype != LV_ATTN_BF16) return LV_ERR_DTYPE;
  const int n_kt = n_key_tiles(n);
  const size_t per = align_up((size_t)heads * n_kt * 4 * kFragU4 * sizeof(u32x4), 256);
  u32x4 *kp = (u32x4 *)ws;
  u32x4 *vp = (u32x4 *)((char *)ws + per);
  hipLaunchKernelGGL(k_attn_pack, dim3((unsigned)n_kt, (unsigned)heads), dim3(256), 0, st, k, v, n,
                     heads, n_kt, qk_norm, kp, vp);
  if (after_pack && hipEventRecord(after_pack, st) != hipSuccess) return LV_ERR_HIP;
  const int nqb = (int)((n + kQB - 1) / kQB);
  const float c = scale * 1.4426950408889634f;
  hipLaunchKernelGGL(k_attn_bf16<false>, dim3((unsigned)(nqb * heads)), dim3(256), 0, st, q, kp, vp,
                     o, n, heads, n_kt, nqb, c, qk_norm);
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

}  // namespace lv
