// Cosine matching of src tokens to dst tokens (Sec. 3.4 "Cached Token Merging") and the
// construction of the merge index (CSR groups).
//
// The similarity is a dense contraction dst[n_dst,C] x src[n_src,C]^T that is never
// materialised: a workgroup keeps 64 src rows resident in LDS as ready-made MFMA B
// fragments, its waves stream 64-row blocks of the (pre-packed, fragment-major) dst matrix
// straight from L2 into registers as A fragments, run v_mfma_f32_32x32x16_bf16 over the
// whole channel dimension, and fold each finished 32x32 tile into a per-lane running
// (best, second best) pair.  With dst as the MFMA row dimension every lane owns one src
// column, so the running arg-max needs no cross-lane traffic until the very end.
// bf16 x bf16 products are exact in fp32, only the accumulation order differs from an
// exact dot product; rows whose two best candidates are closer than kRescoreGap are
// re-decided from float64 dot products in a cheap second kernel.
#include "common.h"
#include "internal.h"

namespace lv {

constexpr int kSrcTile = 64;         // src rows resident per workgroup
#ifndef LV_MATCH_WAVES
#define LV_MATCH_WAVES 12
#endif
#ifndef LV_MATCH_DEPTH
#define LV_MATCH_DEPTH 2
#endif
#ifndef LV_MATCH_PANEL_GROUPS
#define LV_MATCH_PANEL_GROUPS 11   /* 11 groups x 768 rows x 2 KB = 16.5 MB of dst per launch */
#endif
constexpr int kMatchWaves = LV_MATCH_WAVES;   // 12 = 3 waves per SIMD (measured best)
constexpr int kDepth = LV_MATCH_DEPTH;        // register ring: chunks of dst fragments in flight per wave
constexpr float kRescoreGap = 2e-4f; // similarity gap below which float64 decides

struct Top2 {
  float v1;
  int i1;
  float v2;
  int i2;
};

// inv[i] = 1 / max(|x_i|, 1e-12), norm accumulated in float64.  One wave per row.
__global__ __launch_bounds__(256) void k_inv_norm(const uint16_t *__restrict__ x, int64_t N, int C,
                                                  float *__restrict__ inv) {
  const int lane = threadIdx.x & 63, wpb = blockDim.x >> 6, nch = C >> 3;
  for (int64_t i = (int64_t)blockIdx.x * wpb + (threadIdx.x >> 6); i < N;
       i += (int64_t)gridDim.x * wpb) {
    double ss = 0.0;
    for (int ch = lane; ch < nch; ch += 64) {
      u32x4 w = ((const u32x4 *)(x + (size_t)i * C))[ch];
      double a0 = bf16_lo(w.x), a1 = bf16_hi(w.x), a2 = bf16_lo(w.y), a3 = bf16_hi(w.y);
      double a4 = bf16_lo(w.z), a5 = bf16_hi(w.z), a6 = bf16_lo(w.w), a7 = bf16_hi(w.w);
      ss += a0 * a0 + a1 * a1 + a2 * a2 + a3 * a3 + a4 * a4 + a5 * a5 + a6 * a6 + a7 * a7;
    }
    ss = wave_sum(ss);
    if (lane == 0) inv[i] = (float)(1.0 / fmax(sqrt(ss), 1e-12));
  }
}

// Gather dst rows into fragment-major order: fragment (tile t of 32 rows, k-step s of 16
// channels) is 1 KB contiguous, lane (h*32 + r) holds row r, channels 16s+8h .. 16s+8h+7.
// Rows beyond n_dst are zero.
__global__ __launch_bounds__(256) void k_pack_dst(const uint16_t *__restrict__ x,
                                                  const int32_t *__restrict__ dst_idx,
                                                  const float *__restrict__ inv, int n_dst,
                                                  int n_dst_pad, int C, u32x4 *__restrict__ packed,
                                                  float *__restrict__ invd,
                                                  int32_t *__restrict__ belt) {
  const int nch = C >> 3, KS = C >> 4;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < kXcd) belt[idx] = 0;   // sweep positions of the matching kernel start at 0
  if (idx >= (int64_t)n_dst_pad * nch) return;
  const int j = (int)(idx / nch), c = (int)(idx % nch);
  u32x4 w = {0u, 0u, 0u, 0u};
  int row = -1;
  if (j < n_dst) {
    row = dst_idx[j];
    w = ((const u32x4 *)(x + (size_t)row * C))[c];
  }
  const int t = j >> 5, r = j & 31, s = c >> 1, h = c & 1;
  packed[((size_t)t * KS + s) * 64 + h * 32 + r] = w;
  if (c == 0) invd[j] = row >= 0 ? inv[row] : 0.f;
}

__device__ __forceinline__ void top2_insert_ordered(Top2 &t, float v, int i) {
  // candidates arrive in ascending index order: strict > keeps the lowest index on ties
  if (v > t.v1) {
    t.v2 = t.v1;
    t.i2 = t.i1;
    t.v1 = v;
    t.i1 = i;
  } else if (v > t.v2) {
    t.v2 = v;
    t.i2 = i;
  }
}
__device__ __forceinline__ void top2_insert_any(Top2 &t, float v, int i) {
  if (i < 0) return;
  if (v > t.v1 || (v == t.v1 && (t.i1 < 0 || i < t.i1))) {
    t.v2 = t.v1;
    t.i2 = t.i1;
    t.v1 = v;
    t.i1 = i;
  } else if (v > t.v2 || (v == t.v2 && (t.i2 < 0 || i < t.i2))) {
    t.v2 = v;
    t.i2 = i;
  }
}

__global__ __launch_bounds__(kMatchWaves * 64) void k_match(
    const uint16_t *__restrict__ x, const int32_t *__restrict__ src_idx, int n_src,
    const u32x4 *__restrict__ dstp, const float *__restrict__ invd, int n_dst, int g_first,
    int n_groups, int C, Top2 *__restrict__ top2, int32_t *belt) {
  extern __shared__ u32x4 frag[];   // [2 src tiles][KS][64 lanes]
  __shared__ int g_start;
  const int KS = C >> 4, nch = C >> 3, NCHUNK = KS >> 2;
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // keeps address math scalar
  // All workgroups of an XCD share one L2.  They sweep the dst matrix circularly and a new
  // workgroup joins the sweep where its XCD's others currently are (belt[xcd], a hint that
  // wave 0 keeps publishing), so the same dst rows are requested by many CUs while they
  // are still resident in that L2 instead of each CU streaming them from memory.
  const int xcd = __builtin_amdgcn_s_getreg((3 << 11) | 20) & (kXcd - 1);   // XCC_ID[3:0]
  if (tid == 0) {
    int g = __atomic_load_n(&belt[xcd], __ATOMIC_RELAXED);
    g_start = (g >= 0 && g < n_groups) ? g : 0;
  }
  const int src0 = blockIdx.x * kSrcTile;

  for (int idx = tid; idx < kSrcTile * nch; idx += blockDim.x) {
    const int row = idx / nch, c = idx - row * nch;
    const int srow = min(src0 + row, n_src - 1);
    const u32x4 w = ((const u32x4 *)(x + (size_t)src_idx[srow] * C))[c];
    frag[((row >> 5) * KS + (c >> 1)) * 64 + (c & 1) * 32 + (row & 31)] = w;
  }
  __syncthreads();

  Top2 best[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) best[b] = Top2{-INFINITY, -1, -INFINITY, -1};

  // A group is kMatchWaves consecutive tile pairs (64 dst rows each), one per wave.  This
  // wave's K-chunks (4 k-steps = 8 fragments) over all groups form one flat stream that is
  // prefetched kDepth-1 chunks ahead through a register ring, across tile-pair boundaries,
  // so that enough bytes are in flight to cover L2 latency.
  const int g0 = g_start;
  const int total = n_groups * NCHUNK;
  const size_t a1off = (size_t)KS * 64;
  u32x4 ring[kDepth][8];
  int pgrp = g0, psb = 0, pg = 0;            // next chunk to fetch: group, chunk, flat index
  auto fetch = [&](u32x4(&buf)[8]) {
    const int ptp = (g_first + pgrp) * kMatchWaves + wave;
    const u32x4 *ap = dstp + ((size_t)(2 * ptp) * KS + (size_t)psb * 4) * 64 + lane;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      buf[ks] = ap[(size_t)ks * 64];
      buf[4 + ks] = ap[a1off + (size_t)ks * 64];
    }
    ++pg;
    if (++psb == NCHUNK) {
      psb = 0;
      if (++pgrp == n_groups) pgrp = 0;
    }
  };
  f32x16 acc[2][2];
  auto clear_acc = [&]() {
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
  };
  clear_acc();
#pragma unroll
  for (int j = 0; j < kDepth - 1; ++j)
    if (pg < total) fetch(ring[j]);
  int grp = g0, sb = 0;                      // chunk being computed
  for (int f0 = 0; f0 < total; f0 += kDepth) {
#pragma unroll
    for (int j = 0; j < kDepth; ++j) {
      if (f0 + j < total) {
        if (pg < total) fetch(ring[(j + kDepth - 1) % kDepth]);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const int s = sb * 4 + ks;
          const bf16x8 a0 = __builtin_bit_cast(bf16x8, ring[j][ks]);
          const bf16x8 a1 = __builtin_bit_cast(bf16x8, ring[j][4 + ks]);
#ifdef LV_MATCH_NOLDS   /* timing experiment only: wrong results */
          const bf16x8 b0 = a1, b1 = a0;
          (void)s;
#else
          const bf16x8 b0 = __builtin_bit_cast(bf16x8, frag[(size_t)s * 64 + lane]);
          const bf16x8 b1 = __builtin_bit_cast(bf16x8, frag[(size_t)(KS + s) * 64 + lane]);
#endif
          acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[0][0], 0, 0, 0);
          acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc[0][1], 0, 0, 0);
          acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc[1][0], 0, 0, 0);
          acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[1][1], 0, 0, 0);
        }
        if (++sb == NCHUNK) {
          // fold the four finished 32x32 tiles into the running top-2 of this lane's columns
          const int tp = (g_first + grp) * kMatchWaves + wave;
#pragma unroll
          for (int a = 0; a < 2; ++a) {
            const int row0 = (2 * tp + a) * 32 + h * 4;
            const f32x4 *ip = (const f32x4 *)(invd + row0);
            f32x4 iv[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) iv[g] = ip[2 * g];
#pragma unroll
            for (int b = 0; b < 2; ++b) {
              float v[16];
              float m = -INFINITY;
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                v[r] = acc[a][b][r] * iv[r >> 2][r & 3];
                m = fmaxf(m, v[r]);
              }
              if (__builtin_amdgcn_ballot_w64(m > best[b].v2) != 0) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                  const int j2 = row0 + (r >> 2) * 8 + (r & 3);
                  if (j2 < n_dst) top2_insert_any(best[b], v[r], j2);   // sweep order is circular
                }
              }
            }
          }
          clear_acc();
          sb = 0;
          if (++grp == n_groups) grp = 0;
          if (wave == 0 && lane == 0) __atomic_store_n(&belt[xcd], grp, __ATOMIC_RELAXED);
        }
      }
    }
  }

  __syncthreads();   // everyone is done with the resident fragments: reuse LDS
  Top2 *cand = (Top2 *)frag;
#pragma unroll
  for (int b = 0; b < 2; ++b) cand[(wave * 2 + b) * 64 + lane] = best[b];
  __syncthreads();
  if (tid < kSrcTile) {
    const int b = tid >> 5, q = tid & 31;
    Top2 t = Top2{-INFINITY, -1, -INFINITY, -1};
    for (int w = 0; w < kMatchWaves; ++w)
      for (int hh = 0; hh < 2; ++hh) {
        const Top2 c = cand[(w * 2 + b) * 64 + hh * 32 + q];
        top2_insert_any(t, c.v1, c.i1);
        top2_insert_any(t, c.v2, c.i2);
      }
    if (src0 + tid < n_src) {
      if (g_first > 0) {   // earlier launches covered the dst rows before this panel
        const Top2 prev = top2[src0 + tid];
        top2_insert_any(t, prev.v1, prev.i1);
        top2_insert_any(t, prev.v2, prev.i2);
      }
      top2[src0 + tid] = t;
    }
  }
}

// Final decision per src row (one wave each).  Rows whose two best fp32 similarities are
// closer than kRescoreGap recompute both in float64 and decide on the fp32-rounded values,
// lowest token index on a tie.
__global__ __launch_bounds__(256) void k_match_finish(
    const uint16_t *__restrict__ x, const int32_t *__restrict__ src_idx,
    const int32_t *__restrict__ dst_idx, const float *__restrict__ inv,
    const Top2 *__restrict__ top2, int n_src, int C, int32_t *__restrict__ anchor_of,
    int32_t *slot_of, float *__restrict__ best_sim) {
  const int lane = threadIdx.x & 63, wpb = blockDim.x >> 6, nch = C >> 3;
  for (int p = blockIdx.x * wpb + (threadIdx.x >> 6); p < n_src; p += gridDim.x * wpb) {
    const Top2 t = top2[p];
    const int s = src_idx[p];
    const float invs = inv[s];
    int choose = t.i1 < 0 ? 0 : t.i1;
    float sim = t.i1 < 0 ? 0.f : t.v1 * invs;
    if (t.i1 >= 0 && t.i2 >= 0 && (t.v1 - t.v2) * invs < kRescoreGap) {
      const int d1 = dst_idx[t.i1], d2 = dst_idx[t.i2];
      double ss = 0, n1 = 0, n2 = 0, p1 = 0, p2 = 0;
      for (int ch = lane; ch < nch; ch += 64) {
        const u32x4 ws = ((const u32x4 *)(x + (size_t)s * C))[ch];
        const u32x4 w1 = ((const u32x4 *)(x + (size_t)d1 * C))[ch];
        const u32x4 w2 = ((const u32x4 *)(x + (size_t)d2 * C))[ch];
        const uint32_t us[4] = {ws.x, ws.y, ws.z, ws.w}, u1[4] = {w1.x, w1.y, w1.z, w1.w},
                       u2[4] = {w2.x, w2.y, w2.z, w2.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const double sl = bf16_lo(us[k]), sh = bf16_hi(us[k]);
          const double al = bf16_lo(u1[k]), ah = bf16_hi(u1[k]);
          const double bl = bf16_lo(u2[k]), bh = bf16_hi(u2[k]);
          ss += sl * sl + sh * sh;
          n1 += al * al + ah * ah;
          n2 += bl * bl + bh * bh;
          p1 += sl * al + sh * ah;
          p2 += sl * bl + sh * bh;
        }
      }
      ss = wave_sum(ss);
      n1 = wave_sum(n1);
      n2 = wave_sum(n2);
      p1 = wave_sum(p1);
      p2 = wave_sum(p2);
      const double is = 1.0 / fmax(sqrt(ss), 1e-12);
      const float s1 = (float)(p1 * is * (1.0 / fmax(sqrt(n1), 1e-12)));
      const float s2 = (float)(p2 * is * (1.0 / fmax(sqrt(n2), 1e-12)));
      if (s2 > s1 || (s2 == s1 && d2 < d1)) {
        choose = t.i2;
        sim = s2;
      } else {
        sim = s1;
      }
    }
    if (lane == 0) {
      const int a = dst_idx[choose];
      anchor_of[s] = a;
      slot_of[s] = slot_of[a];
      if (best_sim) best_sim[p] = sim;
    }
  }
}

// ---------------------------------------------------------------------------------
// CSR groups: a stable LSD radix sort of (slot_of[i], i) gives the members of every slot
// in ascending token order.  One wave per 1024-element chunk keeps the scatter stable.
// ---------------------------------------------------------------------------------
constexpr int kSortChunk = 1024;

__global__ __launch_bounds__(64) void k_radix_hist(const uint32_t *__restrict__ keys, int64_t N,
                                                   int shift, int nchunks,
                                                   uint32_t *__restrict__ hist) {
  __shared__ uint32_t h[256];
  const int lane = threadIdx.x;
  for (int d = lane; d < 256; d += 64) h[d] = 0;
  __syncthreads();
  const int64_t b = (int64_t)blockIdx.x * kSortChunk;
  for (int i = lane; i < kSortChunk; i += 64)
    if (b + i < N) atomicAdd(&h[(keys[b + i] >> shift) & 255u], 1u);
  __syncthreads();
  for (int d = lane; d < 256; d += 64) hist[(size_t)d * nchunks + blockIdx.x] = h[d];
}

// exclusive prefix sum over hist[256*nchunks] in place (digit-major), single workgroup
__global__ __launch_bounds__(1024) void k_radix_scan(uint32_t *__restrict__ hist, int64_t n) {
  __shared__ uint32_t wtot[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t per = (n + 1023) / 1024;
  const int64_t b = min((int64_t)tid * per, n), e = min(b + per, n);
  uint32_t sum = 0;
  for (int64_t i = b; i < e; ++i) sum += hist[i];
  uint32_t inc = sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t v = __shfl_up(inc, o, 64);
    if (lane >= o) inc += v;
  }
  if (lane == 63) wtot[wave] = inc;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += wtot[w];
  uint32_t run = base + inc - sum;
  for (int64_t i = b; i < e; ++i) {
    uint32_t v = hist[i];
    hist[i] = run;
    run += v;
  }
}

__global__ __launch_bounds__(64) void k_radix_scatter(const uint32_t *__restrict__ keys,
                                                      const int32_t *__restrict__ vals, int64_t N,
                                                      int shift, int nchunks,
                                                      const uint32_t *__restrict__ hist,
                                                      uint32_t *__restrict__ keys_out,
                                                      int32_t *__restrict__ vals_out) {
  __shared__ uint32_t base[256];
  const int lane = threadIdx.x;
  for (int d = lane; d < 256; d += 64) base[d] = hist[(size_t)d * nchunks + blockIdx.x];
  __syncthreads();
  const int64_t b = (int64_t)blockIdx.x * kSortChunk;
  const uint64_t lt = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  for (int i0 = 0; i0 < kSortChunk; i0 += 64) {
    const int64_t g = b + i0 + lane;
    const bool ok = g < N;
    const uint32_t key = ok ? keys[g] : 0u;
    const int32_t val = ok ? (vals ? vals[g] : (int32_t)g) : 0;
    const uint32_t d = (key >> shift) & 255u;
    uint64_t peers = __builtin_amdgcn_ballot_w64(ok);
#pragma unroll
    for (int bit = 0; bit < 8; ++bit) {
      const uint64_t bal = __builtin_amdgcn_ballot_w64((d >> bit) & 1u);
      peers &= ((d >> bit) & 1u) ? bal : ~bal;
    }
    const uint32_t rank = (uint32_t)__popcll(peers & lt);
    const uint32_t cnt = (uint32_t)__popcll(peers);
    uint32_t pos = 0;
    if (ok) pos = base[d] + rank;
    __syncthreads();
    if (ok && rank == cnt - 1) base[d] += cnt;   // one lane per digit present
    __syncthreads();
    if (ok) {
      keys_out[pos] = key;
      vals_out[pos] = val;
    }
  }
}

__global__ __launch_bounds__(256) void k_csr_finish(const uint32_t *__restrict__ keys,
                                                    const int32_t *__restrict__ vals, int64_t N,
                                                    int64_t M, int32_t *__restrict__ group_off,
                                                    int32_t *__restrict__ group_mem) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= N) return;
  group_mem[j] = vals[j];
  const uint32_t k = keys[j];
  if ((j == 0 || keys[j - 1] != k) && (int64_t)k < M) group_off[k] = (int32_t)j;
  if (j == N - 1) group_off[M] = (int32_t)N;
}

// ---------------------------------------------------------------------------------
struct MatchWs {
  float *inv;
  u32x4 *dstp;
  float *invd;
  Top2 *top2;
  uint32_t *keys[2];
  int32_t *vals[2];
  uint32_t *hist;
  int32_t *belt;
  size_t bytes;
  int n_dst_pad, nchunks;
};

static MatchWs carve(const Dims &d, const litevggt_plan_t &pl, char *base) {
  MatchWs w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char *p = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  w.n_dst_pad = (int)align_up((size_t)pl.n_dst, 64 * kMatchWaves);   // whole groups
  w.nchunks = (int)((d.N + kSortChunk - 1) / kSortChunk);
  w.inv = (float *)take((size_t)d.N * 4);
  w.dstp = (u32x4 *)take((size_t)w.n_dst_pad * d.C * 2);
  w.invd = (float *)take((size_t)w.n_dst_pad * 4);
  w.top2 = (Top2 *)take(align_up((size_t)pl.n_src, 64) * sizeof(Top2));
  for (int i = 0; i < 2; ++i) {
    w.keys[i] = (uint32_t *)take((size_t)d.N * 4);
    w.vals[i] = (int32_t *)take((size_t)d.N * 4);
  }
  w.hist = (uint32_t *)take((size_t)256 * w.nchunks * 4);
  w.belt = (int32_t *)take(kXcd * sizeof(int32_t));
  w.bytes = off;
  return w;
}

size_t match_ws_bytes(const Dims &d, const litevggt_plan_t &pl) { return carve(d, pl, nullptr).bytes; }

int launch_match(const uint16_t *x, const Dims &d, const litevggt_plan_t &pl,
                 const litevggt_index &ix, float *best_sim, void *ws, hipStream_t st) {
  MatchWs w = carve(d, pl, (char *)ws);
  const int n_src = (int)pl.n_src, n_dst = (int)pl.n_dst;
  if (n_src > 0) {
    size_t lds = (size_t)2 * (d.C / 16) * 64 * 16;     // resident src fragments
    const size_t cand = (size_t)kMatchWaves * 2 * 64 * sizeof(Top2);   // reused at the end
    if (lds < cand) lds = cand;
    if (lds > 160 * 1024 - 1024) return LV_ERR_SHAPE;
    static size_t lds_set = 0;
    if (lds > lds_set) {
      if (hipFuncSetAttribute((const void *)k_match, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)lds) != hipSuccess)
        return LV_ERR_HIP;
      lds_set = lds;
    }
    const unsigned rows_grid = (unsigned)(((d.N + 3) / 4) < 16384 ? ((d.N + 3) / 4) : 16384);
    hipLaunchKernelGGL(k_inv_norm, dim3(rows_grid), dim3(256), 0, st, x, d.N, d.C, w.inv);
    const int64_t pk = (int64_t)w.n_dst_pad * (d.C / 8);
    hipLaunchKernelGGL(k_pack_dst, dim3((unsigned)((pk + 255) / 256)), dim3(256), 0, st, x,
                       ix.dst_idx, w.inv, n_dst, w.n_dst_pad, d.C, w.dstp, w.invd, w.belt);
    // The dst matrix is processed in panels small enough to stay resident in every XCD's L2
    // (one launch per panel, all workgroups of a launch stream the same panel); the running
    // top-2 of each src row is carried from launch to launch in `top2`.
    const int groups = w.n_dst_pad / (64 * kMatchWaves);
    const int per_panel = LV_MATCH_PANEL_GROUPS > 0 ? LV_MATCH_PANEL_GROUPS : groups;
    for (int g = 0; g < groups; g += per_panel)
      hipLaunchKernelGGL(k_match, dim3((unsigned)((n_src + kSrcTile - 1) / kSrcTile)),
                         dim3(kMatchWaves * 64), lds, st, x, ix.src_idx, n_src, w.dstp, w.invd,
                         n_dst, g, (groups - g < per_panel ? groups - g : per_panel), d.C, w.top2,
                         w.belt);
    const unsigned fin = (unsigned)(((n_src + 3) / 4) < 16384 ? ((n_src + 3) / 4) : 16384);
    hipLaunchKernelGGL(k_match_finish, dim3(fin), dim3(256), 0, st, x, ix.src_idx, ix.dst_idx,
                       w.inv, w.top2, n_src, d.C, ix.anchor_of, ix.slot_of, best_sim);
    LV_HIP_CHECK_LAUNCH();
  }
  // CSR groups by stable radix sort of slot_of
  int bits = 1;
  while (((int64_t)1 << bits) < pl.M) ++bits;
  const int passes = (bits + 7) / 8;
  const uint32_t *kin = (const uint32_t *)ix.slot_of;
  const int32_t *vin = nullptr;
  for (int p = 0; p < passes; ++p) {
    uint32_t *kout = w.keys[p & 1];
    int32_t *vout = w.vals[p & 1];
    hipLaunchKernelGGL(k_radix_hist, dim3((unsigned)w.nchunks), dim3(64), 0, st, kin, d.N, 8 * p,
                       w.nchunks, w.hist);
    hipLaunchKernelGGL(k_radix_scan, dim3(1), dim3(1024), 0, st, w.hist,
                       (int64_t)256 * w.nchunks);
    hipLaunchKernelGGL(k_radix_scatter, dim3((unsigned)w.nchunks), dim3(64), 0, st, kin, vin, d.N,
                       8 * p, w.nchunks, w.hist, kout, vout);
    kin = kout;
    vin = vout;
  }
  hipLaunchKernelGGL(k_csr_finish, dim3((unsigned)((d.N + 255) / 256)), dim3(256), 0, st, kin, vin,
                     d.N, pl.M, ix.group_off, ix.group_mem);
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

}  // namespace lv
