// Cosine matching of src tokens to dst tokens (Sec. 3.4 "Cached Token Merging") and the
// construction of the merge index (CSR groups).
//
// The similarity is a dense contraction dst[n_dst,C] x src[n_src,C]^T that is never
// materialised (see k_match_sim).  bf16 x bf16 products are exact in fp32, only the
// accumulation order differs from an exact dot product; rows whose two best candidates are
// closer than kRescoreGap are re-decided from float64 dot products in a cheap second kernel.
#include "common.h"
#include "internal.h"

namespace lv {

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

// Gather token rows into fragment-major order: fragment (tile t of 32 rows, k-step s of 16
// channels) is 1 KB contiguous, lane (h*32 + r) holds row r, channels 16s+8h .. 16s+8h+7.
// idx_of == NULL packs rows 0..n-1 in place order.  Rows beyond n are zero.  inv_out (optional)
// receives the rows' inverse norms, 0 beyond n; zero256 (optional) is a 256-word array to clear.
// A wave writes whole fragments (1 KB stores); it takes 4 consecutive k-steps of its 32 rows,
// so the 128 bytes it needs of a row are one cache line read by 4 back-to-back loads.
// Grid: (row tiles, ceil(KS / 16)); a workgroup's 4 waves take 4 k-steps each.
__global__ __launch_bounds__(256) void k_pack_rows(const uint16_t *__restrict__ x,
                                                   const int32_t *__restrict__ idx_of,
                                                   const float *__restrict__ inv, int n, int n_pad,
                                                   int C, u32x4 *__restrict__ packed,
                                                   float *__restrict__ inv_out,
                                                   uint32_t *__restrict__ zero256) {
  const int KS = C >> 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h = lane >> 5, r = lane & 31;
  const int t = blockIdx.x, j = t * 32 + r;
  if (zero256 && blockIdx.x == 0 && blockIdx.y == 0) zero256[threadIdx.x] = 0u;   // the similarity kernel's team counters
  int row = -1;
  if (j < n) row = idx_of ? idx_of[j] : j;
  if (inv_out && blockIdx.y == 0 && wave == 0 && h == 0 && j < n_pad) inv_out[j] = row >= 0 ? inv[row] : 0.f;
  const int s0 = (blockIdx.y * 4 + wave) * 4;
  u32x4 w[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    w[u] = u32x4{0u, 0u, 0u, 0u};
    if (row >= 0 && s0 + u < KS) w[u] = ((const u32x4 *)(x + (size_t)row * C))[(s0 + u) * 2 + h];
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (s0 + u < KS) packed[((size_t)t * KS + s0 + u) * 64 + lane] = w[u];
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

int launch_pack_rows(const uint16_t *x, int64_t n, int64_t n_pad, int C, void *packed, hipStream_t st) {
  if (n_pad >= ((int64_t)1 << 31) || n_pad % 32 != 0 || C % 16 != 0) return LV_ERR_SHAPE;
  hipLaunchKernelGGL(k_pack_rows, dim3((unsigned)(n_pad / 32), (unsigned)((C / 16 + 15) / 16)), dim3(256), 0, st, x,
                     (const int32_t *)nullptr, (const float *)nullptr, (int)n, (int)n_pad, C,
                     (u32x4 *)packed,
                     (float *)nullptr, (uint32_t *)nullptr);
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

// ---------------------------------------------------------------------------------
// Similarity kernel.  A workgroup (8 waves) computes 256 src x 256 dst tiles of the similarity
// matrix with the channel dimension as the inner loop: both operands come pre-packed in
// fragment-major order, go from global memory straight into a 4-stage LDS ring (2 k-steps =
// 32 KB per stage, fetched 3 stages ahead) and are read from there as MFMA fragments, so every
// byte fetched from L2 feeds 128 flop (a src-resident design with streamed dst reaches 64 and
// was bound by the L2 -> CU rate).  Wave (wd, ws) owns the 64 dst x 128 src sub-tile: dst is
// the MFMA row dimension, so a lane owns one src column per 32-column block and folds every
// finished tile into its running (best, second best) pair without cross-lane traffic.
//
// The kernel is persistent: one workgroup per CU.  The workgroups the hardware deals to one
// XCD (block index mod 8) form a team of 8 src tiles x 4 sweeps; the team takes every 8th
// super-row of 8 src tiles, and in it workgroup (src tile, sweep dl) visits the dst tiles dl,
// dl + 4, dl + 8, ...  The team moves from one dst tile to the next together (a bounded,
// advisory wait on a counter in the XCD's L2), so its 32 workgroups ask for the same 8 src
// and 4 dst tiles within a few microseconds of each other and 4 of 5 requests hit that L2.
// The four partial results of a src row are merged by k_match_finish.
// ---------------------------------------------------------------------------------
constexpr int kGTile = 256;          // src and dst rows per workgroup tile
constexpr int kGStages = 4;          // LDS ring depth
constexpr int kGStageU4 = 2 * 2 * 8 * 64;   // u32x4 per stage: [src|dst][2 k-steps][8 fragments][64 lanes]
constexpr int kTeamSpin = 512;       // polls of the team counter before a workgroup goes on alone
constexpr int kInvBufs = 8;          // per-wave LDS buffers of 64 inverse dst norms
constexpr int kGLanes = 4;           // dst tiles are dealt to this many workgroups per src tile (<= kMaxSweeps of k_match_finish)

__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_match_sim(
    const u32x4 *__restrict__ srcp, const u32x4 *__restrict__ dstp, const float *__restrict__ invd,
    int n_dst, int n_src_tiles, int n_dst_tiles, int n_lanes, int KS, int n_src_pad,
    int team_size, int spin_budget, uint32_t *team_ctr, Top2 *__restrict__ top2p) {
  extern __shared__ u32x4 ring[];    // kGStages stages
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wd = wave & 3, wsrc = wave >> 2;
  const int team = blockIdx.x & (kXcd - 1), rank = blockIdx.x >> 3;
  if (rank >= team_size) return;     // not a member of its team: nothing to do
  const int dl = rank % n_lanes, sti = rank / n_lanes, sr_tiles = team_size / n_lanes;
  const int n_super = (n_src_tiles + sr_tiles - 1) / sr_tiles;
  const int nt_max = (n_dst_tiles + n_lanes - 1) / n_lanes;
  const int nt = dl < n_dst_tiles ? (n_dst_tiles - dl + n_lanes - 1) / n_lanes : 0;   // my dst tiles
  const int SPT = KS >> 1;           // stages per tile
  const int total = nt * SPT;
  uint32_t *ctr = team_ctr + team * 32;      // one counter per team, 128 bytes apart
  uint32_t rounds = 0;                       // sweep steps of the super-rows the team has finished

  for (int sr = team; sr < n_super; sr += kXcd) {   // super-row: sr_tiles consecutive src tiles
  const int st = sr * sr_tiles + sti;
  const bool active = st < n_src_tiles && total > 0;
  Top2 best[4];
#pragma unroll
  for (int b = 0; b < 4; ++b) best[b] = Top2{-INFINITY, -1, -INFINITY, -1};

  if (active) {
    // fetch: this wave moves fragments f = 4*wave .. 4*wave+3 of a stage (f = op*16 + ks*8 + a)
    const int f_op = wave >> 2, f_ks = (wave >> 1) & 1, f_a0 = (wave & 1) * 4;
    int pf_tile = dl, pf_s = 0, pf_g = 0;      // next stage to fetch: dst tile, stage in tile, flat index
    int pf_t = 0;                              // tiles whose first stage has been requested
    // the inverse norms of this wave's 64 dst rows travel with the first stage of their tile
    // into a wave-private LDS buffer, so the fold at the end of the tile has them without a
    // memory round trip.  kInvBufs buffers in turn: stages are requested up to kGStages ahead,
    // which with one stage per tile (C = 32) is that many tiles not yet folded.
    float *inv_lds = (float *)(ring + (size_t)kGStages * kGStageU4) + wave * (kInvBufs * 64);
    // fetch_part<0>: the inverse norms and fragments 0, 1 of the stage; fetch_part<1>: fragments
    // 2, 3 and the bookkeeping.
    auto fetch_part = [&](auto part) {
      constexpr int P = decltype(part)::value;
      if (P == 0 && pf_s == 0 && pf_g < total) {
        __builtin_amdgcn_global_load_lds(invd + (size_t)pf_tile * kGTile + wd * 64 + lane,
                                         inv_lds + (pf_t & (kInvBufs - 1)) * 64, 4, 0, 0);
        ++pf_t;
      }
      const int tile = f_op ? pf_tile : st;
      const u32x4 *src = (f_op ? dstp : srcp) +
                         ((size_t)(tile * 8 + f_a0) * KS + (size_t)(pf_s * 2 + f_ks)) * 64 + lane;
      u32x4 *dst = ring + (size_t)(pf_g & (kGStages - 1)) * kGStageU4 + (size_t)(wave * 4) * 64;
#pragma unroll
      for (int i = 2 * P; i < 2 * P + 2; ++i)
        __builtin_amdgcn_global_load_lds(src + (size_t)i * KS * 64, dst + i * 64, 16, 0, 0);
      if (P == 1) {
        ++pf_g;
        // past the end the last stage is fetched again (into a free slot nobody reads)
        if (pf_g < total && ++pf_s == SPT) {
          pf_s = 0;
          pf_tile += n_lanes;
        }
      }
    };
    auto fetch = [&]() {
      fetch_part(std::integral_constant<int, 0>{});
      fetch_part(std::integral_constant<int, 1>{});
    };
    const uint32_t ring_lane = lds_addr(&ring[lane]);
    // byte offsets of this wave's fragments inside a stage, k-step 0: src (B operand) fragments
    // 4*wsrc .. +3, dst (A operand) fragments 2*wd, 2*wd+1; k-step 1 is 8 KB further
    const uint32_t b_off = (uint32_t)((0 * 16 + wsrc * 4) * 1024), a_off = (uint32_t)((16 + wd * 2) * 1024);
    u32x4 fb[2][4], fa[2][2];
    auto read_frags = [&](int g, int ks, u32x4(&b)[4], u32x4(&a)[2]) {
      const uint32_t base = ring_lane + (uint32_t)((g & (kGStages - 1)) * kGStageU4 * 16 + ks * 8 * 1024);
      lds_read4_async(b, base + b_off);
      lds_read2_async(a, base + a_off);
    };
    auto wait_frags = [&](u32x4(&b)[4], u32x4(&a)[2]) {
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]), "+v"(a[0]), "+v"(a[1])
                   :
                   : "memory");
    };
    f32x16 acc[2][4];
    auto clear_acc = [&]() {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    };
    auto mma = [&](const u32x4(&b)[4], const u32x4(&a)[2]) {
#pragma unroll
      for (int bi = 0; bi < 4; ++bi)
#pragma unroll
        for (int ai = 0; ai < 2; ++ai)
          acc[ai][bi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[ai]),
                                                               __builtin_bit_cast(bf16x8, b[bi]),
                                                               acc[ai][bi], 0, 0, 0);
    };
    auto mma_first = [&](const u32x4(&b)[4], const u32x4(&a)[2]) {   // first k-step of a tile: starts from zero
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int bi = 0; bi < 4; ++bi)
#pragma unroll
        for (int ai = 0; ai < 2; ++ai)
          acc[ai][bi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[ai]),
                                                               __builtin_bit_cast(bf16x8, b[bi]), zero, 0, 0, 0);
    };
    auto mma_pair = [&](const u32x4(&b)[4], const u32x4(&a)[2], int bi) {   // the two MFMAs of column block bi
#pragma unroll
      for (int ai = 0; ai < 2; ++ai)
        acc[ai][bi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[ai]),
                                                             __builtin_bit_cast(bf16x8, b[bi]),
                                                             acc[ai][bi], 0, 0, 0);
    };
    // Fold the eight finished 32x32 tiles into the running top-2 of this lane's four columns.
    // Almost no element beats its column's second best once a few tiles have been seen, but
    // with 64 columns per wave "some lane of the wave has such an element in this tile" is true
    // nearly always, so the test is made per element: a compare per element and one branch per
    // tile in the common case, the insertion code only for the elements that need it.
    //
    // A column's rows are spread over eight running pairs (four waves, two lane halves), each
    // of which alone would let through about 2 ln(rows / 8) elements.  The test is therefore
    // made against thr >= the largest second best any of the eight had at the end of the
    // previous tile (exchanged through LDS once per tile): an element at or below it cannot be
    // one of the column's two best, and with equal values it has the higher row index, because
    // earlier tiles hold lower rows.  Two buffers by tile parity: a wave that is already done
    // with this tile writes the other one (bounds from this tile's rows could tie with a lower
    // row that a slower wave has yet to see), and nobody is more than one tile-end barrier apart.
    float *share = (float *)(ring + (size_t)kGStages * kGStageU4) + 8 * kInvBufs * 64;   // [parity][wsrc][b][wd][column]
    float thr[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
    for (int b = 0; b < 4; ++b) {   // before the first barrier of the super-row
      share[((wsrc * 4 + b) * 4 + wd) * 32 + (lane & 31)] = -INFINITY;
      share[1024 + ((wsrc * 4 + b) * 4 + wd) * 32 + (lane & 31)] = -INFINITY;
    }
    auto fold = [&](int tile, int buf, int parity) {
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int w = 0; w < 4; ++w)
          thr[b] = fmaxf(thr[b], share[parity * 1024 + ((wsrc * 4 + b) * 4 + w) * 32 + (lane & 31)]);
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const int row0 = tile * kGTile + wd * 64 + a * 32 + h * 4;
        const f32x4 *ip = (const f32x4 *)(inv_lds + buf * 64 + a * 32 + h * 4);
        f32x4 iv[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) iv[g] = ip[2 * g];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          float v[16];
          uint64_t hit[16], any = 0;       // lanes whose element r beats their second best (scalar masks)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            v[r] = acc[a][b][r] * iv[r >> 2][r & 3];
            hit[r] = __builtin_amdgcn_ballot_w64(v[r] > thr[b]);
            any |= hit[r];
          }
          if (any != 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              if (hit[r] != 0) {   // insertions only raise the thresholds: the masks stay a superset
                const int j2 = row0 + (r >> 2) * 8 + (r & 3);
                if (j2 < n_dst) top2_insert_any(best[b], v[r], j2);
              }
            }
            thr[b] = fmaxf(thr[b], best[b].v2);
          }
        }
      }
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        thr[b] = fmaxf(thr[b], __shfl_xor(thr[b], 32, 64));   // the other half of the wave has the same column
        share[(parity ^ 1) * 1024 + ((wsrc * 4 + b) * 4 + wd) * 32 + (lane & 31)] = thr[b];
      }
    };

    clear_acc();
#pragma unroll
    for (int i = 0; i < kGStages; ++i) fetch();                // stages 0..3
    asm volatile("s_waitcnt vmcnt(12)" ::: "memory");          // stage 0 has landed (this wave's part)
    __builtin_amdgcn_s_barrier();
    read_frags(0, 0, fb[0], fa[0]);
    int tile = dl, sidx = 0, steps = 0;
    for (int g = 0; g < total; ++g) {
      // k-step 0 of stage g
      __builtin_amdgcn_sched_barrier(0);
      wait_frags(fb[0], fa[0]);
      read_frags(g, 1, fb[1], fa[1]);
      __builtin_amdgcn_sched_barrier(0);
      if (sidx == 0) mma_first(fb[0], fa[0]);
      else mma(fb[0], fa[0]);
      // k-step 1 of stage g: its fragments are in registers, so the slot of stage g is free once
      // every wave is here; stage g+1 is published by the same barrier.  The barrier, the
      // fetch instructions and the fragment reads sit between pairs of MFMAs, so that the MFMA
      // pipe still has queued work from this wave while it does them.
      __builtin_amdgcn_sched_barrier(0);
      wait_frags(fb[1], fa[1]);
      mma_pair(fb[1], fa[1], 0);
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");         // stage g+1 has landed; g+2, g+3 may be in flight
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      mma_pair(fb[1], fa[1], 1);
      __builtin_amdgcn_sched_barrier(0);
      // The stage's loads go out in two halves with an MFMA pair and the fragment reads between
      // them: eight waves issuing all five loads at once right behind the barrier was measured
      // 1 % slower.  (Anything moved ahead of the barrier, into k-step 0, costs 2-6 %.)
      fetch_part(std::integral_constant<int, 0>{});            // stage g+4 -> slot of stage g, first half
      __builtin_amdgcn_sched_barrier(0);
      mma_pair(fb[1], fa[1], 2);
      __builtin_amdgcn_sched_barrier(0);
      read_frags(g + 1, 0, fb[0], fa[0]);                      // past the end: a stale slot, never used
      __builtin_amdgcn_sched_barrier(0);
      fetch_part(std::integral_constant<int, 1>{});            // second half
      __builtin_amdgcn_sched_barrier(0);
      mma_pair(fb[1], fa[1], 3);
      if (++sidx == SPT) {
        // Team step: the workgroups of a team finish a dst tile at about the same time and
        // start the next one together, so that what one of them fetches is still in their
        // XCD's L2 when the others ask for it.  The wait is advisory: it is bounded, and no
        // result depends on it.
        if (tid == 0) __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        fold(tile, steps & (kInvBufs - 1), steps & 1);
        sidx = 0;
        tile += n_lanes;
        ++steps;
        if (tid == 0) {
          const uint32_t target = (uint32_t)team_size * (rounds + (uint32_t)steps);
          for (int spin = 0; spin < spin_budget; ++spin) {
            if (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) break;
            __builtin_amdgcn_s_sleep(8);
          }
        }
        __builtin_amdgcn_s_barrier();
      }
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");   // nothing may land in LDS any more
  }
  __syncthreads();
  // sweep steps this workgroup did not take still count for its team
  {
    const uint32_t missing = (uint32_t)(nt_max - (active ? nt : 0));
    if (tid == 0 && missing)
      __hip_atomic_fetch_add(ctr, missing, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    rounds += (uint32_t)nt_max;
  }
  if (st < n_src_tiles) {
    // merge the two half-wave copies of a column and the four dst quarters (waves wd = 0..3)
    Top2 *cand = (Top2 *)ring;
#pragma unroll
    for (int b = 0; b < 4; ++b) cand[(wave * 4 + b) * 64 + lane] = best[b];
    __syncthreads();
    if (tid < kGTile) {
      const int ws2 = tid >> 7, b = (tid >> 5) & 3, c = tid & 31;
      Top2 t = Top2{-INFINITY, -1, -INFINITY, -1};
      for (int w = 0; w < 4; ++w)
        for (int hh = 0; hh < 2; ++hh) {
          const Top2 cd = cand[((ws2 * 4 + w) * 4 + b) * 64 + hh * 32 + c];
          top2_insert_any(t, cd.v1, cd.i1);
          top2_insert_any(t, cd.v2, cd.i2);
        }
      top2p[(size_t)dl * n_src_pad + (size_t)st * kGTile + tid] = t;
    }
    __syncthreads();   // the ring is reused by the next super-row
  }
  }   // super-rows
}

// Final decision per src row (one wave each).  Every sweep hands over its two best candidates
// by fp32 similarity (up to kMaxSweeps * 2 per row).  If the runner-up is closer than
// kRescoreGap to the best, every candidate inside that gap is recomputed in float64 and the
// decision is taken on those values rounded to fp32, lowest token index on a tie: the rule the
// fp32 accumulation order cannot disturb.  A row with more near-equal candidates than one
// sweep's two best can still lose its true best inside a sweep; what it picks instead is within
// twice the fp32 accumulation error of it (C / 16 additions of exact 16-product sums).
constexpr int kMaxSweeps = 4;
static_assert(kGLanes <= kMaxSweeps, "k_match_finish reads every sweep's candidates");

__global__ __launch_bounds__(256) void k_match_finish(
    const uint16_t *__restrict__ x, const int32_t *__restrict__ src_idx,
    const int32_t *__restrict__ dst_idx, const float *__restrict__ inv,
    const Top2 *__restrict__ top2p, int n_lanes, int n_src_pad, int n_src, int C,
    int32_t *__restrict__ anchor_of, int32_t *slot_of, float *__restrict__ best_sim) {
  const int lane = threadIdx.x & 63, wpb = blockDim.x >> 6, nch = C >> 3;
  for (int p = blockIdx.x * wpb + (threadIdx.x >> 6); p < n_src; p += gridDim.x * wpb) {
    float cv[2 * kMaxSweeps];
    int ci[2 * kMaxSweeps];
    Top2 t = Top2{-INFINITY, -1, -INFINITY, -1};
#pragma unroll
    for (int l = 0; l < kMaxSweeps; ++l) {    // every sweep's candidates for this row
      Top2 o = Top2{-INFINITY, -1, -INFINITY, -1};
      if (l < n_lanes) o = top2p[(size_t)l * n_src_pad + p];
      cv[2 * l] = o.v1;
      ci[2 * l] = o.i1;
      cv[2 * l + 1] = o.v2;
      ci[2 * l + 1] = o.i2;
      top2_insert_any(t, o.v1, o.i1);
      top2_insert_any(t, o.v2, o.i2);
    }
    const int s = src_idx[p];
    const float invs = inv[s];
    int choose = t.i1 < 0 ? 0 : t.i1;
    float sim = t.i1 < 0 ? 0.f : t.v1 * invs;
    if (t.i1 >= 0 && t.i2 >= 0 && (t.v1 - t.v2) * invs < kRescoreGap) {
      double ss = 0;
      for (int ch = lane; ch < nch; ch += 64) {
        const u32x4 w = ((const u32x4 *)(x + (size_t)s * C))[ch];
        const uint32_t us[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const double sl = bf16_lo(us[q]), sh = bf16_hi(us[q]);
          ss += sl * sl + sh * sh;
        }
      }
      ss = wave_sum(ss);
      const double is = 1.0 / fmax(sqrt(ss), 1e-12);
      float bs = -INFINITY;
      int bd = 0x7fffffff, bi = choose;
#pragma unroll
      for (int c = 0; c < 2 * kMaxSweeps; ++c) {
        if (ci[c] < 0 || !((t.v1 - cv[c]) * invs < kRescoreGap)) continue;   // wave-uniform
        const int d = dst_idx[ci[c]];
        double nn = 0, pp = 0;
        for (int ch = lane; ch < nch; ch += 64) {
          const u32x4 wd = ((const u32x4 *)(x + (size_t)d * C))[ch];
          const u32x4 w = ((const u32x4 *)(x + (size_t)s * C))[ch];   // the src row again: a cache hit
          const uint32_t us[4] = {w.x, w.y, w.z, w.w}, ud[4] = {wd.x, wd.y, wd.z, wd.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const double sl = bf16_lo(us[q]), sh = bf16_hi(us[q]);
            const double al = bf16_lo(ud[q]), ah = bf16_hi(ud[q]);
            nn += al * al + ah * ah;
            pp += sl * al + sh * ah;
          }
        }
        nn = wave_sum(nn);
        pp = wave_sum(pp);
        const float sc = (float)(pp * is * (1.0 / fmax(sqrt(nn), 1e-12)));
        if (sc > bs || (sc == bs && d < bd)) {
          bs = sc;
          bd = d;
          bi = ci[c];
        }
      }
      choose = bi;
      sim = bs;
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

// exclusive prefix sum over hist[256*nchunks] in place (digit-major), single workgroup: tiles
// of 4096 elements, 4 consecutive elements per thread, the running total carried from tile to tile
__global__ __launch_bounds__(1024) void k_radix_scan(uint32_t *__restrict__ hist, int64_t n) {
  __shared__ uint32_t wtot[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t carry = 0;
  for (int64_t t0 = 0; t0 < n; t0 += 4096) {
    const int64_t i = t0 + (int64_t)tid * 4;
    uint32_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = i + u < n ? hist[i + u] : 0u;
    const uint32_t sum = v[0] + v[1] + v[2] + v[3];
    uint32_t inc = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t up = __shfl_up(inc, o, 64);
      if (lane >= o) inc += up;
    }
    if (lane == 63) wtot[wave] = inc;
    __syncthreads();
    uint32_t base = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      const uint32_t wt = wtot[w];
      if (w < wave) base += wt;
      total += wt;
    }
    uint32_t run = carry + base + inc - sum;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (i + u < n) hist[i + u] = run;
      run += v[u];
    }
    carry += total;
    __syncthreads();   // wtot is rewritten by the next tile
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
  u32x4 *dstp, *srcp;
  float *invd;
  Top2 *top2p;
  uint32_t *keys[2];
  int32_t *vals[2];
  uint32_t *hist, *team_ctr;
  size_t bytes;
  int n_dst_pad, n_src_pad, n_lanes, nchunks;
};

static MatchWs carve(const Dims &d, const litevggt_plan_t &pl, char *base) {
  MatchWs w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char *p = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  w.n_dst_pad = (int)align_up((size_t)pl.n_dst, kGTile);
  w.n_src_pad = (int)align_up((size_t)pl.n_src, kGTile);
  const int dst_tiles = w.n_dst_pad / kGTile;
  w.n_lanes = dst_tiles < kGLanes ? (dst_tiles > 0 ? dst_tiles : 1) : kGLanes;
  w.nchunks = (int)((d.N + kSortChunk - 1) / kSortChunk);
  w.inv = (float *)take((size_t)d.N * 4);
  w.dstp = (u32x4 *)take((size_t)w.n_dst_pad * d.C * 2);
  w.srcp = (u32x4 *)take((size_t)w.n_src_pad * d.C * 2);
  w.invd = (float *)take((size_t)w.n_dst_pad * 4);
  w.top2p = (Top2 *)take((size_t)w.n_lanes * w.n_src_pad * sizeof(Top2));
  for (int i = 0; i < 2; ++i) {
    w.keys[i] = (uint32_t *)take((size_t)d.N * 4);
    w.vals[i] = (int32_t *)take((size_t)d.N * 4);
  }
  w.hist = (uint32_t *)take((size_t)256 * w.nchunks * 4);
  w.team_ctr = (uint32_t *)take(256 * 4);
  w.bytes = off;
  return w;
}

size_t match_ws_bytes(const Dims &d, const litevggt_plan_t &pl) { return carve(d, pl, nullptr).bytes; }

int launch_match(const uint16_t *x, const Dims &d, const litevggt_plan_t &pl,
                 const litevggt_index &ix, float *best_sim, void *ws, hipStream_t st) {
  MatchWs w = carve(d, pl, (char *)ws);
  const int n_src = (int)pl.n_src, n_dst = (int)pl.n_dst;
  if (n_src > 0) {
    if (d.C % 32 != 0 || n_dst <= 0) return LV_ERR_SHAPE;
    // 128 KB ring (reused for the final merge) + per wave kInvBufs buffers of 64 inverse norms
    // and two buffers of 8 x 4 x 32 second-best bounds the waves of a column exchange
    const size_t lds = (size_t)kGStages * kGStageU4 * 16 + 8 * kInvBufs * 64 * sizeof(float) + 2 * 1024 * sizeof(float);
    static std::atomic<uint64_t> lds_done{0};
    if (int rc = allow_dynamic_lds((const void *)k_match_sim, lds, lds_done)) return rc;
    const unsigned rows_grid = (unsigned)(((d.N + 3) / 4) < 16384 ? ((d.N + 3) / 4) : 16384);
    hipLaunchKernelGGL(k_inv_norm, dim3(rows_grid), dim3(256), 0, st, x, d.N, d.C, w.inv);
    const unsigned ks_groups = (unsigned)((d.C / 16 + 15) / 16);
    hipLaunchKernelGGL(k_pack_rows, dim3((unsigned)(w.n_dst_pad / 32), ks_groups), dim3(256), 0, st, x,
                       ix.dst_idx, w.inv, n_dst, w.n_dst_pad, d.C, w.dstp, w.invd, w.team_ctr);
    hipLaunchKernelGGL(k_pack_rows, dim3((unsigned)(w.n_src_pad / 32), ks_groups), dim3(256), 0, st, x,
                       ix.src_idx, w.inv, n_src, w.n_src_pad, d.C, w.srcp, (float *)nullptr,
                       (uint32_t *)nullptr);
    // One workgroup per CU, all resident at once; the workgroups the hardware deals to one
    // XCD (block index mod 8) form a team of (src tiles per super-row) x (sweeps).
    const int src_tiles = w.n_src_pad / kGTile, dst_tiles = w.n_dst_pad / kGTile;
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
      return LV_ERR_HIP;
    int per_team = n_cu / kXcd;
    if (per_team < w.n_lanes) per_team = w.n_lanes;
    const int team_size = per_team / w.n_lanes * w.n_lanes;
    hipLaunchKernelGGL(k_match_sim, dim3((unsigned)(per_team * kXcd)), dim3(512), lds, st, w.srcp,
                       w.dstp, w.invd, n_dst, src_tiles, dst_tiles, w.n_lanes, d.C / 16, w.n_src_pad,
                       team_size, kTeamSpin, w.team_ctr, w.top2p);
    const unsigned fin = (unsigned)(((n_src + 3) / 4) < 16384 ? ((n_src + 3) / 4) : 16384);
    hipLaunchKernelGGL(k_match_finish, dim3(fin), dim3(256), 0, st, x, ix.src_idx, ix.dst_idx,
                       w.inv, w.top2p, w.n_lanes, w.n_src_pad, n_src, d.C, ix.anchor_of, ix.slot_of,
                       best_sim);
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
