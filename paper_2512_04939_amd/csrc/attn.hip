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
constexpr int kQB = 512;             // queries per workgroup (8 waves)
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
// With several sequences of n tokens each in one call (frame attention: one per frame) the
// second grid dimension runs over (sequence, head) pairs and so do the packed arrays.
__global__ __launch_bounds__(256) void k_attn_pack(const uint16_t *__restrict__ k,
                                                   const uint16_t *__restrict__ v, int64_t n,
                                                   int heads, int n_kt, int qk_norm,
                                                   u32x4 *__restrict__ kp,
                                                   u32x4 *__restrict__ vp) {
  __shared__ __attribute__((aligned(16))) uint16_t vt[kKT][72];
  const int kt = blockIdx.x, t = threadIdx.x;
  const int seq = blockIdx.y / heads, head = blockIdx.y - seq * heads;
  const int C = heads * 64;
  k += (size_t)seq * n * C;
  v += (size_t)seq * n * C;
  const int key = t >> 3, chunk = t & 7;
  const int64_t row = (int64_t)kt * kKT + key;
  u32x4 wk = {0u, 0u, 0u, 0u}, wv = {0u, 0u, 0u, 0u};
  if (row < n) {
    wk = *(const u32x4 *)(k + (size_t)row * C + head * 64 + chunk * 8);
    wv = *(const u32x4 *)(v + (size_t)row * C + head * 64 + chunk * 8);
  }
  if (qk_norm) wk = rms_scale8(wk, 3);   // the 8 lanes that share a key hold its 64 values
  const size_t tile = ((size_t)blockIdx.y * n_kt + kt) * 4 * kFragU4;
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

constexpr int kKSlots = 2;           // LDS ring slots of 64-key K tiles
constexpr int kVSlots = 3;           // LDS ring slots of 64-key V tiles

// One workgroup = 8 waves = two groups of 4 (one wave of each group per SIMD), 512 queries.
// A wave alternates between a matrix phase (O^T += V^T P^T of the previous key tile, then the
// scores K Q^T of the next one) and a vector phase (softmax of those scores: exp2, bf16 pack,
// row sums).  The two groups run exactly one phase apart, with a workgroup barrier at every
// phase boundary, so on every SIMD one wave feeds the matrix pipe while the other feeds the
// VALU -- deterministically, not by luck of the wave scheduler.
__global__ __launch_bounds__(512) void k_attn_bf16(
    const uint16_t *q, const u32x4 *__restrict__ kp, const u32x4 *__restrict__ vp, uint16_t *o,
    const uint16_t *res, int64_t n, int heads, int n_seq, int n_kt, int nqb, float c,
    int qk_norm, const uint32_t *__restrict__ redo) {
  __shared__ u32x4 ks[kKSlots][8 * kFragU4];
  __shared__ u32x4 vs[kVSlots][8 * kFragU4];
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, ql = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;           // phase group
  const int C = heads * 64;
  int sh, qb;   // (sequence, head) pair and query block; each XCD gets whole pairs
  if (((heads * n_seq) & 7) == 0) {
    const int hp = (heads * n_seq) >> 3, xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    sh = xcd * hp + local / nqb;
    qb = local % nqb;
  } else {
    sh = blockIdx.x / nqb;
    qb = blockIdx.x % nqb;
  }
  // second pass behind the per-row-reference kernel: only the query blocks it left undone (one
  // flag per 256 queries; the whole workgroup takes the same branch, before any barrier)
  if (redo && redo[(size_t)sh * (2 * nqb) + 2 * qb] == 0u && redo[(size_t)sh * (2 * nqb) + 2 * qb + 1] == 0u) return;
  const int seq = sh / heads, head = sh - seq * heads;
  q += (size_t)seq * n * C;
  o += (size_t)seq * n * C;
  if (res) res += (size_t)seq * n * C;
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

  f32x16 oacc[2][2];   // [query block][d tile]
#pragma unroll
  for (int sub = 0; sub < 2; ++sub)
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[sub][dt][r] = 0.f;
  float mref[2] = {-INFINITY, -INFINITY}, lrow[2] = {0.f, 0.f};
  const bf16x2 kOnes = {(__bf16)1.0f, (__bf16)1.0f};

  const int nkv = n_kt >> 1;           // 64-key tiles
  const u32x4 *kh = kp + (size_t)sh * n_kt * 4 * kFragU4;
  const u32x4 *vh = vp + (size_t)sh * n_kt * 4 * kFragU4;
  u32x4 rk, rv;
  auto g2r = [&](int j) {              // global -> registers, 64-key tile j (16 B of K and V per thread)
    const size_t off = (size_t)j * 8 * kFragU4;
    rk = kh[off + tid];
    rv = vh[off + tid];
  };
  auto r2s = [&](int j) {              // registers -> LDS ring slots of tile j
    ks[j % kKSlots][tid] = rk;
    vs[j % kVSlots][tid] = rv;
  };

  f32x16 sacc[2][2];   // [key half][query block]: scores of one 64-key tile
  u32x4 pb[2][2][2];   // [query block][key half][u]: its bf16 weights

  // ---- matrix phase j: PV of tile j-1 (if any), scores of tile j (if any).  All LDS
  // fragment reads of a half-phase are issued before its MFMAs so that LDS latency is paid
  // once, not once per fragment.
  auto phase_m = [&](int j) {
    __builtin_amdgcn_sched_barrier(0);
    if (j > 0) {
      const u32x4 *vt = &vs[(j - 1) % kVSlots][lane];
      u32x4 vf[8];
#pragma unroll
      for (int f = 0; f < 8; ++f) vf[f] = vt[f * kFragU4];
#pragma unroll
      for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int dt = 0; dt < 2; ++dt) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, vf[(kt2 * 2 + u) * 2 + dt]);
            oacc[0][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                a, __builtin_bit_cast(bf16x8, pb[0][kt2][u]), oacc[0][dt], 0, 0, 0);
            oacc[1][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                a, __builtin_bit_cast(bf16x8, pb[1][kt2][u]), oacc[1][dt], 0, 0, 0);
          }
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (j < nkv) {
      const u32x4 *kt = &ks[j % kKSlots][lane];
      u32x4 kf[8];
#pragma unroll
      for (int f = 0; f < 8; ++f) kf[f] = kt[f * kFragU4];
#pragma unroll
      for (int kt2 = 0; kt2 < 2; ++kt2) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
          for (int r = 0; r < 16; ++r) sacc[kt2][sub][r] = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const bf16x8 a = __builtin_bit_cast(bf16x8, kf[kt2 * 4 + s]);
          sacc[kt2][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0][s], sacc[kt2][0], 0, 0, 0);
          sacc[kt2][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[1][s], sacc[kt2][1], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
    }
    // The phase discipline only works if this phase's MFMAs are really issued here: make
    // their results opaque so that nothing is sunk past the barrier into the vector phase.
    asm volatile("" : "+v"(sacc[0][0]), "+v"(sacc[0][1]), "+v"(sacc[1][0]), "+v"(sacc[1][1]),
                 "+v"(oacc[0][0]), "+v"(oacc[0][1]), "+v"(oacc[1][0]), "+v"(oacc[1][1]));
    __builtin_amdgcn_sched_barrier(0);
  };
  // ---- vector phase j: online softmax of tile j, one query column per lane.  The running
  // reference mref is only raised (and O, l rescaled) when some lane's tile maximum exceeds
  // it by more than kRaise in log2 units, so weights stay below 2^kRaise and rescaling is rare.
  auto phase_v = [&](int j) {
    __builtin_amdgcn_sched_barrier(0);
    if (j == nkv - 1) {   // keys beyond the sequence end in the last tile
      const int64_t kbase = (int64_t)j * kKV;
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
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      {
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
          lrow[sub] *= alpha;
#pragma unroll
          for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[sub][dt][r] *= alpha;
        }
      }
      float ls = lrow[sub];
#pragma unroll
      for (int kt2 = 0; kt2 < 2; ++kt2) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          uint32_t w[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float s0 = sacc[kt2][sub][8 * u + 2 * e], s1 = sacc[kt2][sub][8 * u + 2 * e + 1];
            // the difference first: scores are of any size here, and c * s - c * mref with the
            // second product rounded is off by 2^-24 of it, i.e. by thousands once scores reach 1e11
            const float p0 = __builtin_amdgcn_exp2f((s0 - mref[sub]) * c);
            const float p1 = __builtin_amdgcn_exp2f((s1 - mref[sub]) * c);
            w[e] = pack_bf16(p0, p1);
            // row sum of the bf16-rounded weights (what the second MFMA really multiplies)
            ls = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w[e]), kOnes, ls, false);
          }
          pb[sub][kt2][u] = u32x4{w[0], w[1], w[2], w[3]};
        }
      }
      lrow[sub] = ls;
    }
    // likewise the weights must exist before the barrier, not be recomputed lazily after it
    asm volatile("" : "+v"(pb[0][0][0]), "+v"(pb[0][0][1]), "+v"(pb[0][1][0]), "+v"(pb[0][1][1]),
                 "+v"(pb[1][0][0]), "+v"(pb[1][0][1]), "+v"(pb[1][1][0]), "+v"(pb[1][1][1]),
                 "+v"(lrow[0]), "+v"(lrow[1]));
    __builtin_amdgcn_sched_barrier(0);
  };

  g2r(0);
  r2s(0);
  __syncthreads();
  // Global phases p = 0 .. 2*nkv+1; group g works on local phase p-g: even local phases are
  // matrix phases, odd ones vector phases.  Every wave passes every barrier (2 per j, for
  // j = 0 .. nkv).  Tile j+1 is fetched during phase 2j and written to LDS during phase
  // 2j+1: its K slot held tile j-1 (last read in phase 2j-1) and its V slot tile j-2 (last
  // read in phase 2j-1).  The two groups run separate copies of the loop so that each is
  // straight-line code for the register allocator.
  if (grp == 0) {
    for (int j = 0; j < nkv; ++j) {
      if (j + 1 < nkv) g2r(j + 1);
      phase_m(j);                        // phase 2j
      __syncthreads();
      if (j + 1 < nkv) r2s(j + 1);
      phase_v(j);                        // phase 2j+1
      __syncthreads();
    }
    phase_m(nkv);                        // phase 2*nkv: last PV
    __syncthreads();
    __syncthreads();
  } else {
    if (nkv > 1) g2r(1);
    __syncthreads();                     // phase 0: idle
    if (nkv > 1) r2s(1);
    phase_m(0);                          // phase 1
    __syncthreads();
    for (int j = 1; j < nkv; ++j) {
      if (j + 1 < nkv) g2r(j + 1);
      phase_v(j - 1);                    // phase 2j
      __syncthreads();
      if (j + 1 < nkv) r2s(j + 1);
      phase_m(j);                        // phase 2j+1
      __syncthreads();
    }
    phase_v(nkv - 1);                    // phase 2*nkv
    __syncthreads();
    phase_m(nkv);                        // phase 2*nkv+1: last PV
    __syncthreads();
  }

  // ---- normalise and store: lane holds query column ql, rows d = 32dt + 8g + 4h + i
  // second pass: the 256-query half that the first pass completed keeps its rows (with a fused
  // residual in place they already hold the sum)
  const bool mine = !redo || redo[(size_t)sh * (2 * nqb) + 2 * qb + grp] != 0u;
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const float l = lrow[sub] + __shfl_xor(lrow[sub], 32, 64);
    const float inv = 1.0f / l;
    const int64_t row = q0 + sub * 32 + ql;
    if (row < n && mine) {
      uint16_t *op = o + (size_t)row * C + head * 64 + 4 * h;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float r0 = oacc[sub][dt][4 * g] * inv, r1 = oacc[sub][dt][4 * g + 1] * inv;
          float r2 = oacc[sub][dt][4 * g + 2] * inv, r3 = oacc[sub][dt][4 * g + 3] * inv;
          if (res) {   // out = res + attention, one rounding (res may be the output buffer)
            const u32x2 x = *(const u32x2 *)(res + (size_t)row * C + head * 64 + 4 * h + 32 * dt + 8 * g);
            r0 += bf16_lo(x.x);
            r1 += bf16_hi(x.x);
            r2 += bf16_lo(x.y);
            r3 += bf16_hi(x.y);
          }
          const u32x2 w = {pack_bf16(r0, r1), pack_bf16(r2, r3)};
          *(u32x2 *)(op + 32 * dt + 8 * g) = w;
        }
    }
  }
}

// ---------------------------------------------------------------------------------------
// The main attention kernel.  A wave owns two 32-query blocks that run half a 32-key step
// apart, which gives every stretch of the instruction stream independent VALU (exp2, bf16
// pack, row sum of one block) and MFMA work (PV and next scores of the other):
//   A(t): weights of block 0, tile t   ||  PV of block 1, tile t-1;  scores of block 1, tile t
//   B(t): weights of block 1, tile t   ||  PV of block 0, tile t;    scores of block 0, tile t+1
// The MFMAs are interleaved with the VALU work by an explicit scheduling recipe.
//
// The softmax scale (in log2 units) is folded into q before its one bf16 rounding, so a
// score leaves the MFMA ready for exp2.  What the exponent is taken against:
//   ONLINE = false (unit-RMS q and k whose scores cannot exceed 64 in log2 units): nothing;
//     softmax is invariant to the reference and exp2 of a bounded score cannot overflow.  The
//     loop has no maximum, no subtraction, no rescale and no branch.
//   ONLINE = true: online softmax with one running reference R per wave, raised lazily.  The
//     score accumulators start from -R (the MFMA's C operand), so the steady state costs the
//     same instructions plus one compare and branch per phase: a tile whose weights push a row
//     sum beyond 2^40 (some score more than ~40 above R, or not finite) triggers a raise: R
//     moves to that tile's maximum, O and the row sums of both blocks are rescaled by 2^-(R' - R),
//     the scores still pending are re-based, the tile's weights are recomputed.  fp32 covers
//     rows up to ~100 binades apart in one wave; a 256-query block in which some row ends with a
//     sum below 2^-60 (all its scores far below its wave's reference), or whose reference grows
//     beyond kRefUseful (where the bf16 rounding of the scaled q no longer resolves the
//     scores), writes nothing, sets its flag, and the per-row kernel k_attn_bf16 redoes it.
// ---------------------------------------------------------------------------------------
// waits until every LDS operation issued so far has completed
__device__ __forceinline__ void lds_wait(u32x4 (&a)[4], u32x4 (&b)[4]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]),
                 "+v"(b[3])
               :
               : "memory");
}

constexpr int kBQB = 256;            // queries per workgroup (4 waves)
constexpr float kRefUseful = 256.0f; // largest reference (log2 units) the folded scale resolves scores against
constexpr float kSumRaise = 1.0995116e12f;   // 2^40: a row sum beyond it raises the wave's reference
constexpr int kBStages = 4;          // LDS ring of 64-key K/V stages


// PACKED (one sequence, no residual, not ONLINE): `o` is a linear layer's activation operand
// buffer and receives the output rows in that layer's fragment order, [row / 32][k-step of 16
// channels][lane = row % 32 + 32 * (second 8 of the 16)], 16 bytes each.
template <bool ONLINE, bool PACKED = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_attn_bf16_main(
    const uint16_t *q, const u32x4 *__restrict__ kp, const u32x4 *__restrict__ vp, uint16_t *o,
    const uint16_t *res, int64_t n, int heads, int n_seq, int n_kt, int nqb, float c, int qk_norm,
    uint32_t *__restrict__ redo, int redo_stride) {
  __shared__ u32x4 ks[kBStages][8 * kFragU4];
  __shared__ u32x4 vs[kBStages][8 * kFragU4];
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, ql = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int C = heads * 64;
  int sh, qb;   // (sequence, head) pair and query block; each XCD gets whole pairs
  if (((heads * n_seq) & 7) == 0) {
    const int hp = (heads * n_seq) >> 3, xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    sh = xcd * hp + local / nqb;
    qb = local % nqb;
  } else {
    sh = blockIdx.x / nqb;
    qb = blockIdx.x % nqb;
  }
  const int seq = sh / heads, head = sh - seq * heads;
  q += (size_t)seq * n * C;
  o += (size_t)seq * n * C;
  if (res) res += (size_t)seq * n * C;
  const int64_t q0 = (int64_t)qb * kBQB + wave * kQW;

  const int nkv = n_kt >> 1, nkt = n_kt;
  const u32x4 *kh = kp + (size_t)sh * n_kt * 4 * kFragU4;
  const u32x4 *vh = vp + (size_t)sh * n_kt * 4 * kFragU4;
  // Stage `stage` of this head's packed K and V (64 keys, 8 KB each) goes from global memory
  // straight into its ring slot, 1 KB per wave and instruction (global_load_lds_dwordx4: lane l
  // of a wave lands at the wave's LDS base + 16 l).  No registers are staged, so a stage can be
  // fetched three iterations before its first use.  Completion is per wave (vmcnt) and is
  // published to the workgroup by the barrier of the steady-state loop.
  auto fetch = [&](int stage) {
    const int slot = stage & (kBStages - 1);
    const size_t off = (size_t)stage * 8 * kFragU4 + tid;
    __builtin_amdgcn_global_load_lds(kh + off, &ks[slot][wave * 64], 16, 0, 0);
    __builtin_amdgcn_global_load_lds(kh + off + 256, &ks[slot][256 + wave * 64], 16, 0, 0);
    __builtin_amdgcn_global_load_lds(vh + off, &vs[slot][wave * 64], 16, 0, 0);
    __builtin_amdgcn_global_load_lds(vh + off + 256, &vs[slot][256 + wave * 64], 16, 0, 0);
  };
  // the first two stages are requested before q is loaded and normalised: one memory round
  // trip for both (short sequences, e.g. frame attention, have few stages to hide it behind)
  fetch(0);
  fetch(min(1, nkv - 1));

  // Q^T fragments with the softmax scale (log2 units) folded in, RMS-normalised per head when
  // qk_norm is set
  bf16x8 qf[2][4];
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const int64_t row = min(q0 + sub * 32 + ql, n - 1);
    const uint16_t *qp = q + (size_t)row * C + head * 64 + 8 * h;
    u32x4 w[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) w[s] = *(const u32x4 *)(qp + 16 * s);
    float ss = (sumsq8(w[0]) + sumsq8(w[1])) + (sumsq8(w[2]) + sumsq8(w[3]));
    ss += __shfl_xor(ss, 32, 64);
    const float r = qk_norm ? c / sqrtf(ss * (1.0f / 64.0f) + kQkEps) : c;
#pragma unroll
    for (int s = 0; s < 4; ++s) qf[sub][s] = __builtin_bit_cast(bf16x8, scale8(w[s], r));
  }

  f32x16 oacc[2][2];   // [query block][d tile]
#pragma unroll
  for (int sub = 0; sub < 2; ++sub)
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[sub][dt][r] = 0.f;
  float lrow[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
  // what the score accumulators start from: 0, or minus the wave's running reference (16
  // registers that stay live through the loop; one per query block would not fit, a subtraction
  // per score would cost a fifth of the kernel's VALU time)
  f32x16 s_start = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float ref_run = 0.f;         // ONLINE: the reference R (uniform over the wave)
  bool over = false;           // ONLINE: R went beyond kRefUseful
  float lnew[2] = {0.f, 0.f};  // ONLINE: row sums including the tile whose weights were just taken

  f32x16 sacc[2];      // [query block]: scores of its current 32-key tile
  u32x4 pb[2][2];      // [query block][u]: bf16 weights of its current 32-key tile
  // Fragments held in registers feed both query blocks: fv[t & 1] = V fragments of tile t
  // (used in B(t), A(t+1)), fk[t & 1] = K fragments of tile t (used in B(t-1), A(t)).
  u32x4 fv[2][4], fk[2][4];

  auto load_v = [&](int t, u32x4(&dst)[4]) {
    const u32x4 *vt = &vs[(t >> 1) & (kBStages - 1)][(t & 1) * 4 * kFragU4 + lane];
#pragma unroll
    for (int f = 0; f < 4; ++f) dst[f] = vt[f * kFragU4];
  };
  auto load_k = [&](int t, u32x4(&dst)[4]) {
    const u32x4 *kt = &ks[(t >> 1) & (kBStages - 1)][(t & 1) * 4 * kFragU4 + lane];
#pragma unroll
    for (int f = 0; f < 4; ++f) dst[f] = kt[f * kFragU4];
  };
  auto mma_s = [&](int sub, const u32x4(&kf)[4]) {
    f32x16 acc = s_start;
#pragma unroll
    for (int s = 0; s < 4; ++s)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[s]), qf[sub][s],
                                                    acc, 0, 0, 0);
    sacc[sub] = acc;
  };
  auto mma_pv = [&](int sub, const u32x4(&vf)[4]) {
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
        oacc[sub][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, vf[u * 2 + dt]), __builtin_bit_cast(bf16x8, pb[sub][u]),
            oacc[sub][dt], 0, 0, 0);
  };
  auto mask_tail = [&](int t, int sub) {   // keys beyond the sequence end
    if ((int64_t)(t + 1) * kKT > n) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t key = (int64_t)t * kKT + (r >> 2) * 8 + h * 4 + (r & 3);
        if (key >= n) sacc[sub][r] = -INFINITY;
      }
    }
  };
  // exp2 of the scaled scores, bf16 pack, row sums.  The sums are plain fp32 adds of the
  // unrounded weights in two chains: v_dot2c_f32_bf16 on the packed pairs would halve the
  // instruction count, but it does not overlap with MFMAs (measured: a phase with dot2 row sums
  // takes as long as its MFMA and VALU parts one after the other, with adds it takes 1.1x its
  // MFMA part).
  auto weights = [&](int sub) {
    float l0 = lrow[sub][0], l1 = lrow[sub][1];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float p0 = __builtin_amdgcn_exp2f(sacc[sub][8 * u + 2 * e]);
        const float p1 = __builtin_amdgcn_exp2f(sacc[sub][8 * u + 2 * e + 1]);
        w[e] = pack_bf16(p0, p1);
        l0 += p0;
        l1 += p1;
      }
      pb[sub][u] = u32x4{w[0], w[1], w[2], w[3]};
    }
    if (ONLINE) {      // held back until settle() has seen them
      lnew[0] = l0;
      lnew[1] = l1;
    } else {
      lrow[sub][0] = l0;
      lrow[sub][1] = l1;
    }
  };
  // ONLINE, at the end of the phase that took the weights of block `sub`: accept the new row
  // sums, or raise the reference first.  At this point the other block's weights have been
  // consumed (its PV was issued in this phase), its scores of the next tile are pending, and no
  // MFMA of `sub`'s tile has been issued yet.
  auto settle = [&](int sub) {
    if (!ONLINE) return;
    __builtin_amdgcn_sched_barrier(0);
    if (__builtin_amdgcn_ballot_w64(!(lnew[0] + lnew[1] <= kSumRaise)) != 0) {
      // fragment reads issued by hand may be in flight: let them land before anything else
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      float mx = sacc[sub][0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[sub][r]);
      const float delta = fmaxf(wave_max(mx), 0.f);      // how far the tile's maximum lies above R
      const float alpha = __builtin_amdgcn_exp2f(-delta);
      ref_run += delta;
      over |= !(ref_run <= kRefUseful);
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        lrow[b][0] *= alpha;
        lrow[b][1] *= alpha;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[b][dt][r] *= alpha;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[b][r] -= delta;   // own tile: redone below; other block: pending scores
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) s_start[r] = -ref_run;
      weights(sub);
    }
    lrow[sub][0] = lnew[0];
    lrow[sub][1] = lnew[1];
    __builtin_amdgcn_sched_barrier(0);
  };
  // One phase = 8 MFMAs + the weights of 16 scores per lane (16 exp2, 8 pack, 16 add).  The
  // recipe asks the scheduler to spread the MFMAs over the VALU work; A phases re-fill fv
  // after their 4 PV MFMAs and fk after their 4 score MFMAs.  (Forcing a strict
  // exp2/exp2/MFMA/pack/sum order with opaque pins was measured slower than this.)
  auto recipe = [&]() {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);   // 2 exp2
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // 1 MFMA
      __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);   // pack + 2 adds
    }
  };
  // In the steady state the fragment reads are issued by hand (lds_read4_async): V(t) and
  // K(t+1) at the start of A(t); B(t) is their first user and waits for them a whole phase
  // later.  Both are double-buffered, so the registers a read overwrites were last used by
  // MFMAs a whole phase before it is issued.
  const uint32_t ks_lane = lds_addr(&ks[0][lane]), vs_lane = lds_addr(&vs[0][lane]);
  auto frag_off = [&](int t) {   // byte offset of tile t's four fragments in a ring array
    return (uint32_t)((((t >> 1) & (kBStages - 1)) * 8 + (t & 1) * 4) * kFragU4 * 16);
  };
  // A(t), t >= 1: weights of block 0 || PV(t-1) and scores(t) of block 1
  int fslot = 0;       // ring slot and source offset of the stage being fetched
  size_t foff = 0;
  auto fetch1 = [&](int q) {   // one of the four fetch instructions of a stage
    const u32x4 *src = (q < 2 ? kh : vh) + foff + (q & 1) * 256;
    u32x4 *dst = (q < 2 ? &ks[fslot][0] : &vs[fslot][0]) + (q & 1) * 256 + wave * 64;
    __builtin_amdgcn_global_load_lds(src, dst, 16, 0, 0);
  };
  auto phase_a = [&](int t, const u32x4(&v_prev)[4], u32x4(&v_cur)[4], const u32x4(&k_cur)[4],
                     u32x4(&k_next)[4], int fq = -1) {
    lds_read4_async(v_cur, vs_lane + frag_off(t));
    lds_read4_async(k_next, ks_lane + frag_off(t + 1));   // past the last tile: a stale slot, never used
    if (fq >= 0) fetch1(fq);
    __builtin_amdgcn_sched_barrier(0);
    weights(0);
    mma_pv(1, v_prev);
    mma_s(1, k_cur);
    recipe();
    settle(0);
  };
  // B(t), t <= nkt-2: weights of block 1 || PV(t) and scores(t+1) of block 0
  auto phase_b = [&](u32x4(&v_cur)[4], u32x4(&k_next)[4], int fq = -1) {
    __builtin_amdgcn_sched_barrier(0);     // the work of A(t) stays ahead of the wait
    lds_wait(v_cur, k_next);
    if (fq >= 0) {
      fetch1(fq);
      __builtin_amdgcn_sched_barrier(0);
    }
    weights(1);
    mma_pv(0, v_cur);
    mma_s(0, k_next);
    recipe();
    settle(1);
  };

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  fetch(min(2, nkv - 1));                  // in flight during the prologue and the first iteration
  if (q0 >= n) {
    // All 64 queries of this wave lie beyond the sequence end (the ragged last block: 1374
    // tokens per frame are 5.4 blocks).  The wave only moves its share of the K/V stages and
    // keeps the workgroup's barriers company, leaving both pipes of its SIMD to the other
    // workgroup resident there.
    if (ONLINE && __syncthreads_or(0)) {     // the other waves' first-tile check
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      return;
    }
    for (int i = 0; i < nkv - 2; ++i) {
      fslot = (i + 3) & (kBStages - 1);
      foff = (size_t)min(i + 3, nkv - 1) * 8 * kFragU4 + tid;
      fetch1(0);
      fetch1(1);
      fetch1(2);
      asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      fetch1(3);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (ONLINE) __syncthreads_or(0);         // the other waves' final check
    return;
  }
  // prologue: scores of tile 0 for both blocks, weights of block 0, then V(0) and K(1)
  load_k(0, fk[0]);
  mma_s(0, fk[0]);
  mask_tail(0, 0);
  if (ONLINE) {
    // the reference starts at the largest score of the first tile (both blocks)
    mma_s(1, fk[0]);
    mask_tail(0, 1);
    float mx = fmaxf(sacc[0][0], sacc[1][0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(sacc[0][r], sacc[1][r]));
    ref_run = wave_max(mx);
    // A reference this large cannot serve (and one that is not finite cannot at all): the block
    // goes to the second pass without being computed here first.
    if (__syncthreads_or(!(ref_run <= kRefUseful))) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the stages already requested land before the workgroup ends
      if (tid == 0) redo[(size_t)sh * redo_stride + qb] = 1u;
      return;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      s_start[r] = -ref_run;
      sacc[0][r] -= ref_run;
      sacc[1][r] -= ref_run;
    }
    weights(0);
    lrow[0][0] = lnew[0];
    lrow[0][1] = lnew[1];
  } else {
    weights(0);
    mma_s(1, fk[0]);
  }
  load_v(0, fv[0]);
  load_k(1, fk[1]);
  if (!ONLINE && nkv == 1) mask_tail(0, 1);
  // steady state: stage i holds tiles 2i, 2i+1; iteration i reads stages i and i+1, stage i+2
  // is in flight since the previous iteration and stage i+3 is fetched now, into the slot of
  // stage i-1, which every wave finished reading before the previous barrier.  (Past the end
  // the last stage is fetched again into a slot nobody reads: the loop body has no branches.)
  for (int i = 0; i < nkv - 2; ++i) {
    // one fetch instruction at the head of each phase
    fslot = (i + 3) & (kBStages - 1);
    foff = (size_t)min(i + 3, nkv - 1) * 8 * kFragU4 + tid;
    phase_b(fv[0], fk[1], 0);                           // B(2i)
    phase_a(2 * i + 1, fv[0], fv[1], fk[1], fk[0], 1);  // A(2i+1)
    phase_b(fv[1], fk[0], 2);                           // B(2i+1)
    // this wave's part of stage i+2 has landed (the three newest loads, of stage i+3, may still
    // be in flight); after the barrier all of stage i+2 is readable: first read in A(2i+3)
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    phase_a(2 * i + 2, fv[1], fv[0], fk[0], fk[1], 3);  // A(2i+2)
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // nothing may land after the workgroup ends
  if (nkv >= 2) {                          // stage nkv-2; it enters the last stage, whose tiles may be ragged
    const int i = nkv - 2;
    phase_b(fv[0], fk[1]);
    phase_a(2 * i + 1, fv[0], fv[1], fk[1], fk[0]);
    phase_b(fv[1], fk[0]);
    mask_tail(2 * i + 2, 0);
    phase_a(2 * i + 2, fv[1], fv[0], fk[0], fk[1]);
    mask_tail(2 * i + 2, 1);
  }
  // last stage: tiles nkt-2, nkt-1
  phase_b(fv[0], fk[1]);                   // B(nkt-2)
  mask_tail(nkt - 1, 0);
  phase_a(nkt - 1, fv[0], fv[1], fk[1], fk[0]);   // A(nkt-1)
  mask_tail(nkt - 1, 1);
  lds_wait(fv[1], fk[0]);
  weights(1);
  mma_pv(0, fv[1]);
  settle(1);
  mma_pv(1, fv[1]);

  float lsub[2];
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const float lsum = lrow[sub][0] + lrow[sub][1];
    lsub[sub] = lsum + __shfl_xor(lsum, 32, 64);
  }
  if (ONLINE) {
    // A row whose scores all lie ~60 binades or more below its wave's reference has lost its
    // weights to underflow, and a reference beyond kRefUseful is not resolved: the whole
    // 256-query block is left to the per-row kernel, and nothing of it is written here (the
    // output may alias the residual).
    bool low = over;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) low |= q0 + sub * 32 + ql < n && !(lsub[sub] >= 8.67e-19f);   // 2^-60
    if (__syncthreads_or(low)) {
      if (tid == 0) redo[(size_t)sh * redo_stride + qb] = 1u;
      return;
    }
  }
  if constexpr (PACKED) {
    // a lane holds channels 8g + 4h .. + 3 of its query per group of four registers: lanes l and
    // l + 32 trade halves (first operand's lanes 32-63 <-> second operand's lanes 0-31), after
    // which lane l has channels 0-7 and lane l + 32 channels 8-15 of a k-step: 1 KB per store
    u32x4 *op = (u32x4 *)o;
    const int KS = C >> 4;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const bool live = q0 + sub * 32 + ql < n;
      const float inv = live ? 1.0f / lsub[sub] : 0.f;
      const size_t base = ((size_t)((q0 + sub * 32) >> 5) * KS + head * 4) * 64 + lane;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int gp = 0; gp < 2; ++gp) {
          float r[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) r[i] = live ? oacc[sub][dt][8 * gp + i] * inv : 0.f;
          const auto s0 = __builtin_amdgcn_permlane32_swap(pack_bf16(r[0], r[1]), pack_bf16(r[4], r[5]), false, false);
          const auto s1 = __builtin_amdgcn_permlane32_swap(pack_bf16(r[2], r[3]), pack_bf16(r[6], r[7]), false, false);
          op[base + (size_t)(dt * 2 + gp) * 64] = u32x4{s0[0], s1[0], s0[1], s1[1]};
        }
    }
    return;
  }
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const float l = lsub[sub];
    const float inv = 1.0f / l;
    const int64_t row = q0 + sub * 32 + ql;
    if (row < n) {
      uint16_t *op = o + (size_t)row * C + head * 64 + 4 * h;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float r0 = oacc[sub][dt][4 * g] * inv, r1 = oacc[sub][dt][4 * g + 1] * inv;
          float r2 = oacc[sub][dt][4 * g + 2] * inv, r3 = oacc[sub][dt][4 * g + 3] * inv;
          if (res) {   // out = res + attention, one rounding (res may be the output buffer)
            const u32x2 x = *(const u32x2 *)(res + (size_t)row * C + head * 64 + 4 * h + 32 * dt + 8 * g);
            r0 += bf16_lo(x.x);
            r1 += bf16_hi(x.x);
            r2 += bf16_lo(x.y);
            r3 += bf16_hi(x.y);
          }
          const u32x2 w = {pack_bf16(r0, r1), pack_bf16(r2, r3)};
          *(u32x2 *)(op + 32 * dt + 8 * g) = w;
        }
    }
  }
}

// ---------------------------------------------------------------------------------------
// FP8 (E4M3, OCP "fn": bias 7, max 448) variant: q, k, v are quantised per tensor with
// scale = amax/448 taken in the same call, the softmax weights with a fixed scale 2^8; the
// MFMAs are v_mfma_f32_32x32x64_f8f6f4, everything else (scores, max, sums, O) stays fp32.
// ---------------------------------------------------------------------------------------
constexpr float kFp8PShift = 8.0f;   // weights are stored as 2^8 * p, p <= 1 at the reference
constexpr float kFp8Raise = 0.75f;   // 2^(8 + 0.75) < 448: the reference follows the maximum closely

// bf16 values of w scaled by r and rounded to bf16 (the normalised q/k as the bf16 path sees them)
__device__ __forceinline__ u32x4 norm8(const u32x4 w, float ss_head, int qk_norm) {
  return qk_norm ? scale8(w, 1.0f / sqrtf(ss_head * (1.0f / 64.0f) + kQkEps)) : w;
}

__global__ __launch_bounds__(256) void k_zero_words(uint32_t *p, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

__global__ void k_attn_amax_zero(uint32_t *amax) {
  if (threadIdx.x < 4) amax[threadIdx.x] = 0u;
}

// amax[0..2] = max |q^|, |k^|, |v| over the call's tensors (q^, k^ normalised when qk_norm).
// One thread per 8-value chunk; the 8 lanes of a (row, head) combine their sums of squares.
__global__ __launch_bounds__(256) void k_attn_amax(const uint16_t *__restrict__ q,
                                                   const uint16_t *__restrict__ k,
                                                   const uint16_t *__restrict__ v, int64_t n, int C,
                                                   int qk_norm, uint32_t *__restrict__ amax) {
  __shared__ float red[3][4];
  const int64_t nchunks = n * (C >> 3);
  float mq = 0.f, mk = 0.f, mv = 0.f;
  // the 8 lanes that share a (row, head) hold consecutive chunk indices, so they enter and
  // leave this loop together and the xor-shuffles below only read lanes that are active
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nchunks;
       i += (int64_t)gridDim.x * blockDim.x) {
    const u32x4 wq = ((const u32x4 *)q)[i], wk = ((const u32x4 *)k)[i], wv = ((const u32x4 *)v)[i];
    float sq = sumsq8(wq), sk = sumsq8(wk);
    for (int o = 1; o < 8; o <<= 1) {
      sq += __shfl_xor(sq, o, 64);
      sk += __shfl_xor(sk, o, 64);
    }
    mq = fmaxf(mq, absmax8(norm8(wq, sq, qk_norm)));
    mk = fmaxf(mk, absmax8(norm8(wk, sk, qk_norm)));
    mv = fmaxf(mv, absmax8(wv));
  }
  mq = wave_max(mq);
  mk = wave_max(mk);
  mv = wave_max(mv);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane == 0) {
    red[0][wave] = mq;
    red[1][wave] = mk;
    red[2][wave] = mv;
  }
  __syncthreads();
  if (threadIdx.x < 3) {
    const float m = fmaxf(fmaxf(red[threadIdx.x][0], red[threadIdx.x][1]),
                          fmaxf(red[threadIdx.x][2], red[threadIdx.x][3]));
    atomicMax(&amax[threadIdx.x], __float_as_uint(m));   // non-negative floats order like uints
  }
}

// fp8 counterpart of k_attn_pack: same fragment-major orders with 8 bytes per lane.
__global__ __launch_bounds__(256) void k_attn_pack_fp8(const uint16_t *__restrict__ k,
                                                       const uint16_t *__restrict__ v, int64_t n,
                                                       int heads, int n_kt, int qk_norm,
                                                       const uint32_t *__restrict__ amax,
                                                       const uint32_t *__restrict__ gate,
                                                       u32x2 *__restrict__ kp, u32x2 *__restrict__ vp) {
  __shared__ __attribute__((aligned(8))) uint8_t vt[kKT][72];
  if (gate && *gate == 0u) return;   // second pass with nothing flagged: no one will read the result
  const int kt = blockIdx.x, head = blockIdx.y, t = threadIdx.x;
  const int C = heads * 64;
  const int key = t >> 3, chunk = t & 7;
  const int64_t row = (int64_t)kt * kKT + key;
  u32x4 wk = {0u, 0u, 0u, 0u}, wv = {0u, 0u, 0u, 0u};
  if (row < n) {
    wk = *(const u32x4 *)(k + (size_t)row * C + head * 64 + chunk * 8);
    wv = *(const u32x4 *)(v + (size_t)row * C + head * 64 + chunk * 8);
  }
  float ss = sumsq8(wk);
  for (int o = 1; o < 8; o <<= 1) ss += __shfl_xor(ss, o, 64);
  wk = norm8(wk, ss, qk_norm);
  const size_t tile = ((size_t)head * n_kt + kt) * 4 * kFragU4;
  kp[tile + (chunk >> 1) * kFragU4 + (chunk & 1) * 32 + key] = quant8(wk, fp8_scale_inv(amax[1]));
  *(u32x2 *)&vt[key][chunk * 8] = quant8(wv, fp8_scale_inv(amax[2]));
  __syncthreads();
  const int u = t >> 7, dt = (t >> 6) & 1, lane = t & 63, h = lane >> 5, dr = lane & 31;
  uint32_t w[2] = {0u, 0u};
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int k0 = 16 * u + 8 * (e >> 2) + 4 * h + (e & 3);
    w[e >> 2] |= (uint32_t)vt[k0][32 * dt + dr] << (8 * (e & 3));
  }
  vp[tile + (u * 2 + dt) * kFragU4 + lane] = u32x2{w[0], w[1]};
}

// four 8-byte operand pieces side by side: the 32-byte operand of v_mfma_f32_32x32x64_f8f6f4
__device__ __forceinline__ i32x8 cat_fp8(u32x2 a, u32x2 b, u32x2 c, u32x2 d) {
  return i32x8{(int)a.x, (int)a.y, (int)b.x, (int)b.y, (int)c.x, (int)c.y, (int)d.x, (int)d.y};
}

// Same structure as k_attn_bf16 (two phase groups, lazily raised reference) on fp8 operands.
// Each contraction is one v_mfma_f32_32x32x64_f8f6f4 (contraction length 64: all channels of a
// head for the scores, all keys of a stage for the output), which runs at twice the rate of the
// 32x32x16 fp8 form; the order of the 64 contraction indices inside an operand is the same for
// both operands (piece p of the packed fragments = indices 16p .. 16p+15 in fragment order).
__global__ __launch_bounds__(512) void k_attn_fp8(
    const uint16_t *__restrict__ q, const u32x2 *__restrict__ kp, const u32x2 *__restrict__ vp,
    uint16_t *__restrict__ o, int64_t n, int heads, int n_kt, int nqb, float c_in, int qk_norm,
    const uint32_t *__restrict__ amax, const uint32_t *__restrict__ redo) {
  __shared__ u32x2 ks[kKSlots][8 * kFragU4];
  __shared__ u32x2 vs[kVSlots][8 * kFragU4];
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, ql = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;
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
  // second pass behind the bounded kernel: only the query blocks it has flagged (one flag per
  // 256 queries; the whole workgroup takes the same branch, before any barrier)
  if (redo && redo[(size_t)head * (2 * nqb) + 2 * qb] == 0u && redo[(size_t)head * (2 * nqb) + 2 * qb + 1] == 0u)
    return;
  const int64_t q0 = (int64_t)qb * kQB + wave * kQW;
  const float inv_sq = fp8_scale_inv(amax[0]);
  // scores come out in units of scale_q*scale_k; fold both into the exponent scale
  const float c = c_in * (1.0f / inv_sq) * (1.0f / fp8_scale_inv(amax[1]));
  const float out_scale = 1.0f / fp8_scale_inv(amax[2]);

  i32x8 qf8[2];
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const int64_t row = min(q0 + sub * 32 + ql, n - 1);
    const uint16_t *qp = q + (size_t)row * C + head * 64 + 8 * h;
    u32x4 w[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) w[s] = *(const u32x4 *)(qp + 16 * s);
    float ss = (sumsq8(w[0]) + sumsq8(w[1])) + (sumsq8(w[2]) + sumsq8(w[3]));
    ss += __shfl_xor(ss, 32, 64);
    u32x2 q8[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) q8[s] = quant8(norm8(w[s], ss, qk_norm), inv_sq);
    qf8[sub] = cat_fp8(q8[0], q8[1], q8[2], q8[3]);
  }

  f32x16 oacc[2][2];
#pragma unroll
  for (int sub = 0; sub < 2; ++sub)
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[sub][dt][r] = 0.f;
  float mref[2] = {-INFINITY, -INFINITY}, lrow[2] = {0.f, 0.f};

  const int nkv = n_kt >> 1;
  const u32x2 *kh = kp + (size_t)head * n_kt * 4 * kFragU4;
  const u32x2 *vh = vp + (size_t)head * n_kt * 4 * kFragU4;
  u32x2 rk, rv;
  auto g2r = [&](int j) {
    const size_t off = (size_t)j * 8 * kFragU4;
    rk = kh[off + tid];
    rv = vh[off + tid];
  };
  auto r2s = [&](int j) {
    ks[j % kKSlots][tid] = rk;
    vs[j % kVSlots][tid] = rv;
  };

  f32x16 sacc[2][2];
  u32x2 pb[2][2][2];

  auto phase_m = [&](int j) {
    __builtin_amdgcn_sched_barrier(0);
    if (j > 0) {
      const u32x2 *vt = &vs[(j - 1) % kVSlots][lane];
      u32x2 vf[8];
#pragma unroll
      for (int f = 0; f < 8; ++f) vf[f] = vt[f * kFragU4];
      // one MFMA per (query block, d tile) over all 64 keys: the operands are the four 16-key
      // pieces (kt2, u) side by side, in the same order for V and for the weights
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        const i32x8 a = cat_fp8(vf[0 * 2 + dt], vf[1 * 2 + dt], vf[2 * 2 + dt], vf[3 * 2 + dt]);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
          oacc[sub][dt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
              a, cat_fp8(pb[sub][0][0], pb[sub][0][1], pb[sub][1][0], pb[sub][1][1]), oacc[sub][dt], 0, 0, 0,
              0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (j < nkv) {
      const u32x2 *kt = &ks[j % kKSlots][lane];
      u32x2 kf[8];
#pragma unroll
      for (int f = 0; f < 8; ++f) kf[f] = kt[f * kFragU4];
      // one MFMA per (key tile, query block) over all 64 channels: the four k-step pieces side by side
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kt2 = 0; kt2 < 2; ++kt2) {
        const i32x8 a = cat_fp8(kf[kt2 * 4], kf[kt2 * 4 + 1], kf[kt2 * 4 + 2], kf[kt2 * 4 + 3]);
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
          sacc[kt2][sub] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, qf8[sub], zero, 0, 0, 0, 0, 0, 0);
      }
    }
    asm volatile("" : "+v"(sacc[0][0]), "+v"(sacc[0][1]), "+v"(sacc[1][0]), "+v"(sacc[1][1]),
                 "+v"(oacc[0][0]), "+v"(oacc[0][1]), "+v"(oacc[1][0]), "+v"(oacc[1][1]));
    __builtin_amdgcn_sched_barrier(0);
  };
  auto phase_v = [&](int j) {
    __builtin_amdgcn_sched_barrier(0);
    if (j == nkv - 1) {
      const int64_t kbase = (int64_t)j * kKV;
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
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      float mx = -INFINITY;
#pragma unroll
      for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
        for (int r = 0; r < 16; r += 2) mx = max3(mx, sacc[kt2][sub][r], sacc[kt2][sub][r + 1]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      if (__builtin_amdgcn_ballot_w64((mx - mref[sub]) * c > kFp8Raise) != 0) {
        const float mnew = fmaxf(mref[sub], mx);
        const float alpha = __builtin_amdgcn_exp2f((mref[sub] - mnew) * c);
        mref[sub] = mnew;
        lrow[sub] *= alpha;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[sub][dt][r] *= alpha;
      }
      float ls = lrow[sub];
      // exp2(c (s - mref) + shift).  As one fma on c * mref - shift while that product is small
      // enough to be exact to 2^-10 (this kernel is bound by its VALU instructions); beyond that
      // (scores of any size come in here) the difference is taken first.
      const float mc = mref[sub] * c - kFp8PShift;
      if (__builtin_amdgcn_ballot_w64(!(fabsf(mc) < 16384.0f)) == 0) {
#pragma unroll
        for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            float pv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              pv[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kt2][sub][8 * u + e], c, -mc));
              ls += pv[e];   // row sum of the fp32 weights, before the cast
            }
            pb[sub][kt2][u] = u32x2{cvt4_fp8(pv[0], pv[1], pv[2], pv[3]), cvt4_fp8(pv[4], pv[5], pv[6], pv[7])};
          }
      } else {
#pragma unroll
        for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            float pv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              pv[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kt2][sub][8 * u + e] - mref[sub], c, kFp8PShift));
              ls += pv[e];
            }
            pb[sub][kt2][u] = u32x2{cvt4_fp8(pv[0], pv[1], pv[2], pv[3]), cvt4_fp8(pv[4], pv[5], pv[6], pv[7])};
          }
      }
      lrow[sub] = ls;
    }
    asm volatile("" : "+v"(pb[0][0][0]), "+v"(pb[0][0][1]), "+v"(pb[0][1][0]), "+v"(pb[0][1][1]),
                 "+v"(pb[1][0][0]), "+v"(pb[1][0][1]), "+v"(pb[1][1][0]), "+v"(pb[1][1][1]),
                 "+v"(lrow[0]), "+v"(lrow[1]));
    __builtin_amdgcn_sched_barrier(0);
  };

  g2r(0);
  r2s(0);
  __syncthreads();
  if (grp == 0) {
    for (int j = 0; j < nkv; ++j) {
      if (j + 1 < nkv) g2r(j + 1);
      phase_m(j);
      __syncthreads();
      if (j + 1 < nkv) r2s(j + 1);
      phase_v(j);
      __syncthreads();
    }
    phase_m(nkv);
    __syncthreads();
    __syncthreads();
  } else {
    if (nkv > 1) g2r(1);
    __syncthreads();
    if (nkv > 1) r2s(1);
    phase_m(0);
    __syncthreads();
    for (int j = 1; j < nkv; ++j) {
      if (j + 1 < nkv) g2r(j + 1);
      phase_v(j - 1);
      __syncthreads();
      if (j + 1 < nkv) r2s(j + 1);
      phase_m(j);
      __syncthreads();
    }
    phase_v(nkv - 1);
    __syncthreads();
    phase_m(nkv);
    __syncthreads();
  }

#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const float l = lrow[sub] + __shfl_xor(lrow[sub], 32, 64);
    const float inv = out_scale / l;
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


// ---------------------------------------------------------------------------------------
// Bounded-score FP8 kernel (qk_norm).  With unit-RMS heads a score cannot exceed
// B = 73 * softmax_scale (Cauchy-Schwarz, with room for the bf16 and E4M3 roundings of the
// normalised rows), so the weights are exponentiated against the fixed reference B: stored weight =
// 2^(score - B) * 2^8.75 <= 430, no running maximum, no rescaling, no branches.  E4M3 keeps 3
// mantissa bits down to 2^-6 and flushes below 2^-10, so a row is served well when the scores
// that carry its mass are within ~15 binades of B.  The sum L of a row's stored weights
// tells: rows with L < 1 (the total mass of the row sits more than 8.75 binades below the bound,
// where single weights lose precision and nothing averages the loss out) are flagged per 256-
// query block, and k_attn_fp8 (running maximum) recomputes the flagged blocks afterwards.  With
// q = k (the layer driver) every row has the weight 2^8.75 of its own key and nothing is flagged.
//
// Structure as k_attn_bf16_main with a 64-key stage in place of a 32-key tile (the FP8 MFMA
// contracts 64 keys at once): a wave owns two 32-query blocks half a stage apart,
//   A(t): weights of block 0, stage t   ||  PV of block 1, stage t-1;  scores of block 1, stage t
//   B(t): weights of block 1, stage t   ||  PV of block 0, stage t;    scores of block 0, stage t+1
// K and V are packed so that an MFMA operand is two 16-byte pieces per lane:
//   K piece (stage, kt2, j): lane (h*32+key) holds channels 32j+8h .. +8 and 32j+16+8h .. +8 of
//                            key 64 stage + 32 kt2 + key
//   V piece (stage, dt, kt2): lane (h*32+dr) holds column 32dt+dr of the 16 keys of tile
//                            2 stage + kt2 that the lane's accumulator rows map to (u = 0, 1)
// ---------------------------------------------------------------------------------------
constexpr int kF8Stages = 4;          // LDS ring of 64-key stages (4 KB of K, 4 KB of V each)
constexpr float kF8Bound = 73.0f;     // |q.k| <= 64 (1 + 2^-8)^2 (1 + 2^-4)^2 < 73: unit-RMS rows rounded to bf16,
                                      // then to E4M3 (every element at most 2^-4 off, all in the same direction)
constexpr float kF8Top = 8.75f;       // a weight at the bound is stored as 2^8.75

__global__ __launch_bounds__(256) void k_attn_pack_fp8b(const uint16_t *__restrict__ k,
                                                        const uint16_t *__restrict__ v, int64_t n,
                                                        int heads, int n_kt,
                                                        const uint32_t *__restrict__ amax,
                                                        u32x2 *__restrict__ kp, u32x2 *__restrict__ vp) {
  __shared__ __attribute__((aligned(8))) uint8_t vt[kKT][72];
  const int kt = blockIdx.x, head = blockIdx.y, t = threadIdx.x;
  const int C = heads * 64;
  const int key = t >> 3, chunk = t & 7;
  const int64_t row = (int64_t)kt * kKT + key;
  u32x4 wk = {0u, 0u, 0u, 0u}, wv = {0u, 0u, 0u, 0u};
  if (row < n) {
    wk = *(const u32x4 *)(k + (size_t)row * C + head * 64 + chunk * 8);
    wv = *(const u32x4 *)(v + (size_t)row * C + head * 64 + chunk * 8);
  }
  float ss = sumsq8(wk);
  for (int o = 1; o < 8; o <<= 1) ss += __shfl_xor(ss, o, 64);
  wk = norm8(wk, ss, 1);
  const int stage = kt >> 1, kt2 = kt & 1;
  const size_t base = ((size_t)head * (n_kt >> 1) + stage) * 4 * 64;   // in 16-byte pieces
  const int s = chunk >> 1, hh = chunk & 1;
  kp[2 * (base + (size_t)(kt2 * 2 + (s >> 1)) * 64 + hh * 32 + key) + (s & 1)] = quant8(wk, fp8_scale_inv(amax[1]));
  *(u32x2 *)&vt[key][chunk * 8] = quant8(wv, fp8_scale_inv(amax[2]));
  __syncthreads();
  const int u = t >> 7, dt = (t >> 6) & 1, lane = t & 63, h = lane >> 5, dr = lane & 31;
  uint32_t w[2] = {0u, 0u};
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int k0 = 16 * u + 8 * (e >> 2) + 4 * h + (e & 3);
    w[e >> 2] |= (uint32_t)vt[k0][32 * dt + dr] << (8 * (e & 3));
  }
  vp[2 * (base + (size_t)(dt * 2 + kt2) * 64 + lane) + u] = u32x2{w[0], w[1]};
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_attn_fp8_bounded(
    const uint16_t *__restrict__ q, const u32x4 *__restrict__ kp, const u32x4 *__restrict__ vp,
    uint16_t *__restrict__ o, int64_t n, int heads, int nkv, int nqb, float c_in,
    const uint32_t *__restrict__ amax, uint32_t *__restrict__ redo, int redo_stride,
    uint32_t *__restrict__ redo_any) {
  __shared__ u32x4 ks[kF8Stages][4 * 64];
  __shared__ u32x4 vs[kF8Stages][4 * 64];
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, ql = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
  const int64_t q0 = (int64_t)qb * kBQB + wave * kQW;
  // The score MFMA delivers log2-domain scores minus the reference directly: its accumulator
  // starts at -ref, and the factor between a product of codes and a log2-domain score, c / (scale
  // of q * scale of k), is made a power of two 2^e by quantising q with a scale up to 2x smaller
  // than 448 / amax (same relative precision, floating point); 2^e is the MFMA's block scale.
  const float inv_sk = fp8_scale_inv(amax[1]);
  const float e_f = fminf(fmaxf(ceilf(log2f(c_in / (fp8_scale_inv(amax[0]) * inv_sk))), -100.f), 100.f);
  const float inv_sq = c_in / (inv_sk * exp2f(e_f));
  const int scale_k = 127 + (int)e_f;       // E8M0: 2^(scale_k - 127), applied to the K operand
  const float ref = kF8Bound * c_in - kF8Top;
  const float out_scale = 1.0f / fp8_scale_inv(amax[2]);

  i32x8 qf8[2];
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const int64_t row = min(q0 + sub * 32 + ql, n - 1);
    const uint16_t *qp = q + (size_t)row * C + head * 64 + 8 * h;
    u32x4 w[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) w[s] = *(const u32x4 *)(qp + 16 * s);
    float ss = (sumsq8(w[0]) + sumsq8(w[1])) + (sumsq8(w[2]) + sumsq8(w[3]));
    ss += __shfl_xor(ss, 32, 64);
    u32x2 q8[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) q8[s] = quant8(norm8(w[s], ss, 1), inv_sq);
    qf8[sub] = cat_fp8(q8[0], q8[1], q8[2], q8[3]);
  }

  f32x16 oacc[2][2];
#pragma unroll
  for (int sub = 0; sub < 2; ++sub)
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[sub][dt][r] = 0.f;
  // Row sums come from the matrix pipe as well: a V fragment of ones (E4M3 1.0 = 0x38) makes
  // every accumulator row the sum of the E4M3 weights of the lane's query.  The normaliser is
  // then the sum of exactly the weights that multiply V: with a fixed reference the largest
  // weight of a row is not a power of two (as it is relative to a running maximum) and carries
  // up to 3 % rounding error, which cancels in this ratio and would not against the fp32 sum.
  f32x16 lacc[2];
#pragma unroll
  for (int sub = 0; sub < 2; ++sub)
#pragma unroll
    for (int r = 0; r < 16; ++r) lacc[sub][r] = 0.f;
  const int kOne = 0x38383838;
  const i32x8 ones8 = {kOne, kOne, kOne, kOne, kOne, kOne, kOne, kOne};
  const float nr = -ref;
  const f32x16 kStart = {nr, nr, nr, nr, nr, nr, nr, nr, nr, nr, nr, nr, nr, nr, nr, nr};

  const u32x4 *kh = kp + (size_t)head * nkv * 4 * 64;
  const u32x4 *vh = vp + (size_t)head * nkv * 4 * 64;
  // one stage = 256 pieces of K and 256 of V: one direct-to-LDS load of each per thread
  // (stage `src` goes to the ring slot of stage `as`: past the end the last stage is fetched
  // again, into a slot nobody reads, so that the loop body has no branches)
  auto fetch_k = [&](int src, int as) {
    __builtin_amdgcn_global_load_lds(kh + (size_t)src * 256 + tid, &ks[as & (kF8Stages - 1)][wave * 64], 16, 0, 0);
  };
  auto fetch_v = [&](int src, int as) {
    __builtin_amdgcn_global_load_lds(vh + (size_t)src * 256 + tid, &vs[as & (kF8Stages - 1)][wave * 64], 16, 0, 0);
  };

  f32x16 sacc[2];      // [32-key half]: the scores in flight (of one query block at a time)
  i32x8 pb[2];         // [query block]: E4M3 weights of its current stage
  u32x4 fv[4], fk[4];  // the pieces of one stage of V and of K

  auto load4 = [&](const u32x4 *base, u32x4(&dst)[4]) {
#pragma unroll
    for (int f = 0; f < 4; ++f) dst[f] = base[f * 64];
  };
  auto mma_s = [&](int sub) {
#pragma unroll
    for (int kt2 = 0; kt2 < 2; ++kt2)
      sacc[kt2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(cat8(fk[2 * kt2], fk[2 * kt2 + 1]), qf8[sub],
                                                                  kStart, 0, 0, 0, scale_k, 0, 127);
  };
  auto mma_pv = [&](int sub) {
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
      oacc[sub][dt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(cat8(fv[2 * dt], fv[2 * dt + 1]), pb[sub],
                                                                      oacc[sub][dt], 0, 0, 0, 0, 0, 0);
    lacc[sub] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ones8, pb[sub], lacc[sub], 0, 0, 0, 0, 0, 0);
  };
  auto mask_tail = [&](int t) {   // keys beyond the sequence end
    if ((int64_t)(t + 1) * kKV > n) {
#pragma unroll
      for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t key = (int64_t)t * kKV + kt2 * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
          if (key >= n) sacc[kt2][r] = -INFINITY;
        }
    }
  };
  // exp2 against the fixed reference, E4M3 pack
  auto weights = [&](int sub) {
#pragma unroll
    for (int kt2 = 0; kt2 < 2; ++kt2)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        float pv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) pv[e] = __builtin_amdgcn_exp2f(sacc[kt2][8 * u + e]);
        pb[sub][(kt2 * 2 + u) * 2] = (int)cvt4_fp8(pv[0], pv[1], pv[2], pv[3]);
        pb[sub][(kt2 * 2 + u) * 2 + 1] = (int)cvt4_fp8(pv[4], pv[5], pv[6], pv[7]);
      }
  };
  auto wait4 = [&](u32x4(&f)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) : : "memory");
  };
  // A phase is: the MFMAs that consume what the phase before produced, the fragment read for
  // the next consumer (by hand, waited for a whole VALU part later), the VALU part (the longer
  // one: 32 exp2, 16 packs per lane against 3 + 2 MFMAs of 64 cycles), then the score
  // MFMAs whose results the next phase's VALU part turns into weights.  Scores of only one
  // query block are alive at a time, and one stage of K and of V.
  const uint32_t ks_lane = lds_addr(&ks[0][lane]), vs_lane = lds_addr(&vs[0][lane]);
  auto slot_off = [&](int t) { return (uint32_t)((t & (kF8Stages - 1)) * 4 * 64 * 16); };
  // B(t): PV(t) of block 0; read K(t+1); weights of block 1 (stage t); scores(t+1) of block 0
  auto phase_b = [&](int t, bool last) {
    __builtin_amdgcn_sched_barrier(0);
    wait4(fv);                                            // V(t), read in A(t)
    mma_pv(0);
    __builtin_amdgcn_sched_barrier(0);
    lds_read4_async(fk, ks_lane + slot_off(t + 1));
    __builtin_amdgcn_sched_barrier(0);
    weights(1);
    __builtin_amdgcn_sched_barrier(0);
    wait4(fk);
    mma_s(0);
    if (last) mask_tail(t + 1);
  };
  // A(t): PV(t-1) of block 1; read V(t); weights of block 0 (stage t); scores(t) of block 1
  auto phase_a = [&](int t, bool last) {
    __builtin_amdgcn_sched_barrier(0);
    mma_pv(1);                                            // V(t-1): waited for in B(t-1)
    __builtin_amdgcn_sched_barrier(0);
    lds_read4_async(fv, vs_lane + slot_off(t));
    __builtin_amdgcn_sched_barrier(0);
    weights(0);
    __builtin_amdgcn_sched_barrier(0);
    mma_s(1);                                             // K(t): waited for in B(t-1)
    if (last) mask_tail(t);
  };

  // stages 0, 1 complete and stage 2 in flight before the loop; iteration t fetches stage t+3
  // into the slot of stage t-1, which nobody reads any more
  fetch_k(0, 0);
  fetch_v(0, 0);
  fetch_k(min(1, nkv - 1), 1);
  fetch_v(min(1, nkv - 1), 1);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  fetch_k(min(2, nkv - 1), 2);
  fetch_v(min(2, nkv - 1), 2);
  // A(0) without a PV
  load4(&ks[0][lane], fk);
  mma_s(0);
  if (nkv == 1) mask_tail(0);
  weights(0);
  mma_s(1);
  if (nkv == 1) mask_tail(0);
  load4(&vs[0][lane], fv);
  // steady state: B(t), A(t+1) for t <= nkv-3: the stages they touch (t+1) are complete ones
  for (int t = 0; t < nkv - 2; ++t) {
    // this wave's parts of stage t+1 have landed (the two newest loads, of stage t+2, may be in
    // flight); after the barrier all of stage t+1 is readable
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    const int fs = min(t + 3, nkv - 1);
    fetch_k(fs, t + 3);
    fetch_v(fs, t + 3);
    phase_b(t, false);
    phase_a(t + 1, false);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // nothing may land after the workgroup ends
  __syncthreads();
  if (nkv >= 2) {                                         // enters the last stage, which may be ragged
    phase_b(nkv - 2, true);
    phase_a(nkv - 1, true);
  }
  // B(nkv-1) without scores of a next stage, and the last PV of block 1
  __builtin_amdgcn_sched_barrier(0);
  wait4(fv);
  mma_pv(0);
  weights(1);
  mma_pv(1);

  bool low = false;
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    const float l = lacc[sub][0];   // every row of the accumulator holds the lane's query's sum
    const float inv = out_scale / l;
    const int64_t row = q0 + sub * 32 + ql;
    if (row < n) {
      low |= !(l >= 1.0f);
      uint16_t *op = o + (size_t)row * C + head * 64 + 4 * h;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const u32x2 w = {pack_bf16(oacc[sub][dt][4 * g] * inv, oacc[sub][dt][4 * g + 1] * inv),
                           pack_bf16(oacc[sub][dt][4 * g + 2] * inv, oacc[sub][dt][4 * g + 3] * inv)};
          *(u32x2 *)(op + 32 * dt + 8 * g) = w;
        }
    }
  }
  if (redo && __builtin_amdgcn_ballot_w64(low) != 0 && lane == 0) {
    atomicOr(&redo[(size_t)head * redo_stride + qb], 1u);
    atomicOr(redo_any, 1u);
  }
}

static int n_key_tiles(int64_t n) { return (int)(2 * ((n + kKV - 1) / kKV)); }

// flags of the bounded FP8 kernel: one word per (head, 256-query block), rows padded to two per
// 512-query block of the second pass
static size_t fp8_flag_words(int heads, int64_t n) { return (size_t)heads * 2 * ((n + kQB - 1) / kQB); }

size_t attn_ws_bytes(int heads, int64_t n_tokens, int attn_dtype, int n_seq) {
  const size_t elem = attn_dtype == LV_ATTN_FP8_E4M3 ? sizeof(u32x2) : sizeof(u32x4);
  const size_t per = (size_t)heads * n_seq * n_key_tiles(n_tokens) * 4 * kFragU4 * elem;
  // [amax block][K fragments][V fragments]; FP8: a second pair of K/V arrays in the layout of
  // the second-pass kernel, and the flags
  size_t total = 256 + 2 * align_up(per, 256);
  if (attn_dtype == LV_ATTN_FP8_E4M3) total += 2 * align_up(per, 256) + align_up(fp8_flag_words(heads, n_tokens) * 4, 256);
  // bf16: the flags of the online-softmax pass (one word per 256-query block)
  else total += align_up(fp8_flag_words(heads * n_seq, n_tokens) * 4, 256);
  return total;
}

// n_seq independent sequences of n tokens each, stored one after the other (n_seq = 1: the
// global attention over the merged sequence; n_seq = frames: frame attention).  Several
// sequences and the fused residual (o = res + attention, res may be o: a workgroup reads the
// rows it writes and nothing else of them) are supported by the bf16 kernels only.
int launch_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v, uint16_t *o,
                int64_t n, int heads, float scale, int attn_dtype, int qk_norm, void *ws,
                hipStream_t st, hipEvent_t after_pack, int n_seq, const uint16_t *res,
                void *o_packed, bool *wrote_packed) {
  if (wrote_packed) *wrote_packed = false;
  if (n_seq < 1 || (int64_t)heads * n_seq > 65535) return LV_ERR_SHAPE;
  if ((n_seq > 1 || res) && attn_dtype != LV_ATTN_BF16) return LV_ERR_DTYPE;
  const int n_kt = n_key_tiles(n);
  const float c = scale * 1.4426950408889634f;
  const int nqb = (int)((n + kQB - 1) / kQB);
  uint32_t *amax = (uint32_t *)ws;
  char *frag = (char *)ws + 256;
  if (attn_dtype == LV_ATTN_FP8_E4M3) {
    const size_t per = align_up((size_t)heads * n_kt * 4 * kFragU4 * sizeof(u32x2), 256);
    u32x2 *kp = (u32x2 *)frag, *vp = (u32x2 *)(frag + per);
    const int C = heads * 64;
    const int64_t nchunks = n * (C / 8);
    const unsigned ag = (unsigned)(((nchunks + 255) / 256) < 4096 ? ((nchunks + 255) / 256) : 4096);
    hipLaunchKernelGGL(k_attn_amax_zero, dim3(1), dim3(64), 0, st, amax);
    hipLaunchKernelGGL(k_attn_amax, dim3(ag), dim3(256), 0, st, q, k, v, n, C, qk_norm, amax);
    // bounded scores (unit-RMS heads, exponent range checked like for bf16): the branch-free
    // kernel against the fixed reference first, then the running-maximum kernel on the query
    // blocks the first one flagged (normally none: its workgroups return at once)
    const bool bounded = qk_norm && kF8Bound * c <= 64.0f;
    uint32_t *redo = nullptr;
    if (bounded) {
      u32x2 *kpb = (u32x2 *)(frag + 2 * per), *vpb = (u32x2 *)(frag + 3 * per);
      redo = (uint32_t *)(frag + 4 * per);
      const size_t words = fp8_flag_words(heads, n);
      hipLaunchKernelGGL(k_zero_words, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, redo, words);
      hipLaunchKernelGGL(k_attn_pack_fp8b, dim3((unsigned)n_kt, (unsigned)heads), dim3(256), 0, st, k, v, n,
                         heads, n_kt, amax, kpb, vpb);
      if (after_pack && hipEventRecord(after_pack, st) != hipSuccess) return LV_ERR_HIP;
      const int nqb2 = (int)((n + kBQB - 1) / kBQB);
      hipLaunchKernelGGL(k_attn_fp8_bounded, dim3((unsigned)(nqb2 * heads)), dim3(256), 0, st, q,
                         (const u32x4 *)kpb, (const u32x4 *)vpb, o, n, heads, n_kt / 2, nqb2, c, amax, redo,
                         2 * nqb, amax + 3);
    }
    hipLaunchKernelGGL(k_attn_pack_fp8, dim3((unsigned)n_kt, (unsigned)heads), dim3(256), 0, st, k,
                       v, n, heads, n_kt, qk_norm, amax, bounded ? amax + 3 : (const uint32_t *)nullptr, kp, vp);
    if (!bounded && after_pack && hipEventRecord(after_pack, st) != hipSuccess) return LV_ERR_HIP;
    hipLaunchKernelGGL(k_attn_fp8, dim3((unsigned)(nqb * heads)), dim3(512), 0, st, q, kp, vp, o, n,
                       heads, n_kt, nqb, c, qk_norm, amax, redo);
    LV_HIP_CHECK_LAUNCH();
    return LV_OK;
  }
  if (attn_dtype != LV_ATTN_BF16) return LV_ERR_DTYPE;
  const size_t per = align_up((size_t)heads * n_seq * n_kt * 4 * kFragU4 * sizeof(u32x4), 256);
  u32x4 *kp = (u32x4 *)frag;
  u32x4 *vp = (u32x4 *)(frag + per);
  // two ways: q, k normalised with exponents that stay in range: the branch-free kernel with
  // no reference; otherwise (q, k as given, or a softmax scale beyond that range) the same kernel
  // as online softmax with a per-wave running reference, then the per-row kernel on the query
  // blocks the first pass flagged (normally none: its workgroups return at once)
  const bool bounded = qk_norm && 64.25f * c <= 64.0f;
  uint32_t *redo = (uint32_t *)(frag + 2 * per);
  if (!bounded) {
    const size_t words = fp8_flag_words(heads * n_seq, n);
    hipLaunchKernelGGL(k_zero_words, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, redo, words);
  }
  hipLaunchKernelGGL(k_attn_pack, dim3((unsigned)n_kt, (unsigned)(heads * n_seq)), dim3(256), 0, st,
                     k, v, n, heads, n_kt, qk_norm, kp, vp);
  if (after_pack && hipEventRecord(after_pack, st) != hipSuccess) return LV_ERR_HIP;
  const int nqb2 = (int)((n + kBQB - 1) / kBQB);
  if (bounded && o_packed && wrote_packed && n_seq == 1 && !res) {
    hipLaunchKernelGGL((k_attn_bf16_main<false, true>), dim3((unsigned)(nqb2 * heads)), dim3(256), 0,
                       st, q, kp, vp, (uint16_t *)o_packed, res, n, heads, n_seq, n_kt, nqb2, c, qk_norm,
                       (uint32_t *)nullptr, 0);
    *wrote_packed = true;
  } else if (bounded) {
    hipLaunchKernelGGL(k_attn_bf16_main<false>, dim3((unsigned)(nqb2 * heads * n_seq)), dim3(256), 0,
                       st, q, kp, vp, o, res, n, heads, n_seq, n_kt, nqb2, c, qk_norm, (uint32_t *)nullptr, 0);
  } else {
    hipLaunchKernelGGL(k_attn_bf16_main<true>, dim3((unsigned)(nqb2 * heads * n_seq)), dim3(256), 0,
                       st, q, kp, vp, o, res, n, heads, n_seq, n_kt, nqb2, c, qk_norm, redo, 2 * nqb);
    hipLaunchKernelGGL(k_attn_bf16, dim3((unsigned)(nqb * heads * n_seq)), dim3(512), 0, st, q, kp,
                       vp, o, res, n, heads, n_seq, n_kt, nqb, c, qk_norm, (const uint32_t *)redo);
  }
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

}  // namespace lv
