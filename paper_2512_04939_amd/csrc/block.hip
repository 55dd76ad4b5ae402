// The transformer block around the global attention core, on the merged sequence (Sec. 3.1:
// the aggregator's global layers are standard pre-norm attention + MLP blocks; the paper does
// not restate their details and there are no trained weights here, so the block is the plain
// one with synthetic weights):
//   h  = LN(z; g1, b1)                       q|k|v = h Wqkv^T + bqkv
//   a  = Attn(q, k, v)   (q, k RMS-normalised per head when qk_norm)
//   u1 = a Wo^T + bo                         h2 = LN(z + u1; g2, b2)
//   u2 = GELU(h2 W1^T + b1m) W2^T + b2m      delta = u1 + u2        (Block(z) = z + delta)
// Every intermediate is stored as bf16; the four linear layers run on one tiled MFMA kernel,
// with bf16 operands or (supplementary "FP8 Quantization Details") with FP8 E4M3 operands
// quantised per tensor, the input's scale taken from the tensor itself or from an 80-step amax
// history (delayed scaling).
#include "common.h"
#include "internal.h"

namespace lv {

// ---------------------------------------------------------------------------------------
// LayerNorm over the channel dimension, one wave per row, statistics in fp32 (two passes over
// registers: mean, then the centred sum of squares).  `add` (optional) is added to x first.
// ---------------------------------------------------------------------------------------
constexpr float kLnEps = 1e-6f;

// one row: lane holds the 16-byte pieces lane, lane + 64, ... of x (and of add); o = the normalised row
template <int CPL>
__device__ __forceinline__ void ln_row(const u32x4 (&w)[CPL], const u32x4 (&a)[CPL],
                                       const float *__restrict__ gamma, const float *__restrict__ beta,
                                       int lane, int nch, int C, u32x4 (&o)[CPL]) {
  float v[CPL][8];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const uint32_t uw[4] = {w[c].x, w[c].y, w[c].z, w[c].w}, ua[4] = {a[c].x, a[c].y, a[c].z, a[c].w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[c][2 * i] = bf16_lo(uw[i]) + bf16_lo(ua[i]);
      v[c][2 * i + 1] = bf16_hi(uw[i]) + bf16_hi(ua[i]);
      sum += v[c][2 * i] + v[c][2 * i + 1];
    }
  }
  const float mean = wave_sum(sum) / (float)C;
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < CPL; ++c)
    if (lane + 64 * c < nch)
#pragma unroll
      for (int i = 0; i < 8; ++i) ss += (v[c][i] - mean) * (v[c][i] - mean);
  const float rstd = 1.0f / sqrtf(wave_sum(ss) / (float)C + kLnEps);
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const int ch = lane + 64 * c;
    o[c] = u32x4{0u, 0u, 0u, 0u};
    if (ch < nch) {
      const f32x4 g0 = ((const f32x4 *)gamma)[2 * ch], g1 = ((const f32x4 *)gamma)[2 * ch + 1];
      const f32x4 b0 = ((const f32x4 *)beta)[2 * ch], b1 = ((const f32x4 *)beta)[2 * ch + 1];
      o[c].x = pack_bf16((v[c][0] - mean) * rstd * g0[0] + b0[0], (v[c][1] - mean) * rstd * g0[1] + b0[1]);
      o[c].y = pack_bf16((v[c][2] - mean) * rstd * g0[2] + b0[2], (v[c][3] - mean) * rstd * g0[3] + b0[3]);
      o[c].z = pack_bf16((v[c][4] - mean) * rstd * g1[0] + b1[0], (v[c][5] - mean) * rstd * g1[1] + b1[1]);
      o[c].w = pack_bf16((v[c][6] - mean) * rstd * g1[2] + b1[2], (v[c][7] - mean) * rstd * g1[3] + b1[3]);
    }
  }
}

template <int CPL>
__device__ __forceinline__ void ln_load(const uint16_t *__restrict__ x, const uint16_t *__restrict__ add,
                                        int64_t row, int C, int lane, int nch, u32x4 (&w)[CPL], u32x4 (&a)[CPL]) {
#pragma unroll
  for (int c = 0; c < CPL; ++c) {
    const int ch = lane + 64 * c;
    w[c] = u32x4{0u, 0u, 0u, 0u};
    a[c] = u32x4{0u, 0u, 0u, 0u};
    if (ch < nch) {
      w[c] = ((const u32x4 *)(x + (size_t)row * C))[ch];
      if (add) a[c] = ((const u32x4 *)(add + (size_t)row * C))[ch];
    }
  }
}

template <int CPL>
__global__ __launch_bounds__(256) void k_layernorm(const uint16_t *__restrict__ x,
                                                   const uint16_t *__restrict__ add,
                                                   const float *__restrict__ gamma,
                                                   const float *__restrict__ beta, int64_t M, int C,
                                                   uint16_t *__restrict__ out) {
  const int lane = threadIdx.x & 63, nch = C >> 3;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  u32x4 w[CPL], a[CPL], o[CPL];
  ln_load<CPL>(x, add, row, C, lane, nch, w, a);
  ln_row<CPL>(w, a, gamma, beta, lane, nch, C, o);
#pragma unroll
  for (int c = 0; c < CPL; ++c)
    if (lane + 64 * c < nch) ((u32x4 *)(out + (size_t)row * C))[lane + 64 * c] = o[c];
}

// The same LayerNorm with the result written as a linear layer's activation operand (the
// fragment order k_pack_rows produces: [row / 32][k-step of 16 channels][lane = row % 32 + 32 *
// (second 8 of the 16)], 16 bytes each).  A workgroup owns the 32 rows of one fragment row, a
// wave 8 of them (their loads are all issued before the first row is reduced); the normalised
// rows meet in LDS (row stride C * 2 + 16 bytes: the 32 rows a wave reads back at one channel
// piece then lie in different banks) and leave as one contiguous run of 32 * C * 2 bytes.
// Rows beyond M are written as zeros.
//
// FP8: the normalised row (rounded to bf16, as if it had been stored) is quantised with the
// scale *inv to E4M3 codes and leaves in the FP8 operand order of k_quant_pack_fp8 (units of 32
// rows x 32 channels, lane h * 32 + r holds the 16 codes of channels 32u + 16h .. + 15 of row
// r); the largest |value| of the rows below M is reduced into *amax.  Row stride in LDS: C + 16
// bytes.
template <int CPL, bool FP8>
__global__ __launch_bounds__(256) void k_layernorm_packed(const uint16_t *__restrict__ x,
                                                          const uint16_t *__restrict__ add,
                                                          const float *__restrict__ gamma,
                                                          const float *__restrict__ beta, int64_t M, int C,
                                                          u32x4 *__restrict__ packed,
                                                          const uint32_t *__restrict__ inv,
                                                          uint32_t *__restrict__ amax) {
  extern __shared__ u32x4 ln_stage[];
  constexpr int RB = CPL <= 2 ? 8 : 4;   // rows whose loads are in flight together
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nch = C >> 3, stride = nch + 1;
  if constexpr (FP8) {
    const float r = __uint_as_float(*inv);
    const int stride8 = (C >> 3) + 2;   // u32x2 per row
    u32x2 *stage8 = (u32x2 *)ln_stage;
    float m = 0.f;
#pragma unroll 1
    for (int j0 = 0; j0 < 8; j0 += RB) {
      u32x4 w[RB][CPL], a[RB][CPL];
#pragma unroll
      for (int j = 0; j < RB; ++j) {
        const int64_t row = (int64_t)blockIdx.x * 32 + wave * 8 + j0 + j;
        ln_load<CPL>(x, add, row < M ? row : 0, C, lane, row < M ? nch : 0, w[j], a[j]);
      }
#pragma unroll
      for (int j = 0; j < RB; ++j) {
        const int rr = wave * 8 + j0 + j;
        u32x4 o[CPL];
        ln_row<CPL>(w[j], a[j], gamma, beta, lane, nch, C, o);
        const bool live = (int64_t)blockIdx.x * 32 + rr < M;
#pragma unroll
        for (int c = 0; c < CPL; ++c)
          if (lane + 64 * c < nch) {
            if (live) m = fmaxf(m, absmax8(o[c]));
            stage8[rr * stride8 + lane + 64 * c] = live ? quant8(o[c], r) : u32x2{0u, 0u};
          }
      }
    }
    m = wave_max(m);
    if (lane == 0 && __float_as_uint(m) > __hip_atomic_load(amax, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
      atomicMax(amax, __float_as_uint(m));
    __syncthreads();
    const int pieces = 32 * (C >> 4);   // = (C / 32) units x 64 lanes
    for (int p = threadIdx.x; p < pieces; p += 256) {
      const int u = p >> 6, lp = p & 63;
      const u32x2 *src = stage8 + (lp & 31) * stride8 + 4 * u + 2 * (lp >> 5);
      const u32x2 lo = src[0], hi = src[1];
      packed[(size_t)blockIdx.x * pieces + p] = u32x4{lo.x, lo.y, hi.x, hi.y};
    }
    return;
  }
#pragma unroll 1
  for (int j0 = 0; j0 < 8; j0 += RB) {
    u32x4 w[RB][CPL], a[RB][CPL];
#pragma unroll
    for (int j = 0; j < RB; ++j) {
      const int64_t row = (int64_t)blockIdx.x * 32 + wave * 8 + j0 + j;
      ln_load<CPL>(x, add, row < M ? row : 0, C, lane, row < M ? nch : 0, w[j], a[j]);
    }
#pragma unroll
    for (int j = 0; j < RB; ++j) {
      const int rr = wave * 8 + j0 + j;
      u32x4 o[CPL];
      ln_row<CPL>(w[j], a[j], gamma, beta, lane, nch, C, o);
      const bool live = (int64_t)blockIdx.x * 32 + rr < M;
#pragma unroll
      for (int c = 0; c < CPL; ++c)
        if (lane + 64 * c < nch) ln_stage[rr * stride + lane + 64 * c] = live ? o[c] : u32x4{0u, 0u, 0u, 0u};
    }
  }
  __syncthreads();
  const int pieces = 32 * nch;   // = (C / 16) k-steps x 64 lanes
  for (int p = threadIdx.x; p < pieces; p += 256) {
    const int ks = p >> 6, lp = p & 63;
    packed[(size_t)blockIdx.x * pieces + p] = ln_stage[(lp & 31) * stride + 2 * ks + (lp >> 5)];
  }
}

// packed: the result goes there in a linear layer's operand order (Mp rows, the ones beyond M
// zero) instead of to out; with fp8_inv / fp8_amax as E4M3 codes (scale *fp8_inv, the largest
// |value| reduced into *fp8_amax), else as bf16
static int launch_layernorm(const uint16_t *x, const uint16_t *add, const float *gamma,
                            const float *beta, int64_t M, int C, uint16_t *out, hipStream_t st,
                            u32x4 *packed = nullptr, int64_t Mp = 0, const uint32_t *fp8_inv = nullptr,
                            uint32_t *fp8_amax = nullptr) {
  const int cpl = (C / 8 + 63) / 64;
  if (C % 32 != 0 || cpl > 4) return LV_ERR_SHAPE;
  if (packed) {
    if (Mp % 32 != 0 || Mp < M || !fp8_inv != !fp8_amax) return LV_ERR_SHAPE;
    const size_t lds = (size_t)32 * (C / 8 + 1) * 16;   // the FP8 rows (C + 16 bytes) fit as well
    static std::atomic<uint64_t> lds_done[8];
    const unsigned grid = (unsigned)(Mp / 32);
    int rc;
#define LV_LNP(CPL, F8)                                                                                       \
  if ((rc = allow_dynamic_lds((const void *)k_layernorm_packed<CPL, F8>, lds, lds_done[(CPL - 1) * 2 + F8])))   \
    return rc;                                                                                                \
  hipLaunchKernelGGL((k_layernorm_packed<CPL, F8>), dim3(grid), dim3(256), lds, st, x, add, gamma, beta, M, C,  \
                     packed, fp8_inv, fp8_amax)
    if (fp8_inv) {
      switch (cpl) {
        case 1: LV_LNP(1, true); break;
        case 2: LV_LNP(2, true); break;
        case 3: LV_LNP(3, true); break;
        default: LV_LNP(4, true); break;
      }
    } else {
      switch (cpl) {
        case 1: LV_LNP(1, false); break;
        case 2: LV_LNP(2, false); break;
        case 3: LV_LNP(3, false); break;
        default: LV_LNP(4, false); break;
      }
    }
#undef LV_LNP
    LV_HIP_CHECK_LAUNCH();
    return LV_OK;
  }
  const unsigned grid = (unsigned)((M + 3) / 4);
#define LV_LN(CPL) \
  hipLaunchKernelGGL(k_layernorm<CPL>, dim3(grid), dim3(256), 0, st, x, add, gamma, beta, M, C, out)
  switch (cpl) {
    case 1: LV_LN(1); break;
    case 2: LV_LN(2); break;
    case 3: LV_LN(3); break;
    case 4: LV_LN(4); break;
    default: return LV_ERR_SHAPE;
  }
#undef LV_LN
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

// ---------------------------------------------------------------------------------------
// FP8 E4M3 operands.  Scalars of one linear layer (device memory, 8 words):
//   [0] amax of the input (bits of a non-negative float, reduced with atomic max)
//   [1] amax of the weight     [2] 448 / amax used for the input    [3] the same for the weight
//   [4] product of the two scales (what the accumulators are multiplied with)
// ---------------------------------------------------------------------------------------
constexpr int kFp8Words = 8;

__global__ void k_fp8_zero(uint32_t *sc) {
  if (threadIdx.x < kFp8Words) sc[threadIdx.x] = 0u;
}

// amax of a bf16 tensor of n16 16-byte pieces
__global__ __launch_bounds__(256) void k_amax_bf16(const u32x4 *__restrict__ x, int64_t n16,
                                                   uint32_t *__restrict__ amax) {
  __shared__ float red[4];
  float m = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
       i += (int64_t)gridDim.x * blockDim.x)
    m = fmaxf(m, absmax8(x[i]));
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0)
    atomicMax(amax, __float_as_uint(fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]))));
}

// One wave: picks the scales of a layer from the tensors' own amax (current scaling).
__global__ __launch_bounds__(64) void k_fp8_scales(uint32_t *__restrict__ sc) {
  if (threadIdx.x == 0) {
    const float ia = fp8_scale_inv(sc[0]), iw = fp8_scale_inv(sc[1]);
    sc[2] = __float_as_uint(ia);
    sc[3] = __float_as_uint(iw);
    sc[4] = __float_as_uint((1.0f / ia) * (1.0f / iw));
  }
}

// Quantise rows 0..n-1 of a row-major [n, K] bf16 matrix with the scale in *inv and store them
// fragment-major for the FP8 MFMA: a unit (32 rows x 32 consecutive k, 1 KB) holds, in lane
// (h*32 + r), the 16 codes k = 32u + 16h .. + 15 of row r; an MFMA operand of 64 k is two
// units.  (Both operands use the same k order inside an operand, which is all a dot product
// needs.)  The byte layout equals that of the bf16 packing of a matrix with K/2 columns, so
// the tiled kernel fetches and reads both types the same way.  Rows n..n_pad-1 are zero.
// A wave writes whole units (1 KB stores) and takes 4 consecutive units of its 32 rows (256
// bytes of each bf16 row).  Grid: (row tiles, ceil(units / 16)).
// amax != NULL: the largest |x| read is reduced into *amax on the way (delayed scaling needs
// it only afterwards, for the history, so no pass of its own).
__global__ __launch_bounds__(256) void k_quant_pack_fp8(const uint16_t *__restrict__ x, int n,
                                                        int K, const uint32_t *__restrict__ inv,
                                                        u32x4 *__restrict__ packed,
                                                        uint32_t *__restrict__ amax) {
  const int KS = K >> 5;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h = lane >> 5, rr = lane & 31;
  const int t = blockIdx.x, j = t * 32 + rr;
  const int s0 = (blockIdx.y * 4 + wave) * 4;
  const float r = __uint_as_float(*inv);
  u32x4 src[4][2];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    src[u][0] = src[u][1] = u32x4{0u, 0u, 0u, 0u};
    if (j < n && s0 + u < KS) {
      const u32x4 *p = (const u32x4 *)(x + (size_t)j * K) + 2 * ((s0 + u) * 2 + h);
      src[u][0] = p[0];
      src[u][1] = p[1];
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (s0 + u < KS) {
      const u32x2 lo = quant8(src[u][0], r), hi = quant8(src[u][1], r);
      packed[((size_t)t * KS + s0 + u) * 64 + lane] = u32x4{lo.x, lo.y, hi.x, hi.y};
    }
  if (amax) {   // rows and units outside the matrix were read as zeros
    float m = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) m = fmaxf(m, fmaxf(absmax8(src[u][0]), absmax8(src[u][1])));
    m = wave_max(m);
    // one word for 10^5 waves: only a wave that would raise it sends an atomic (a stale read only
    // sends one too many)
    if (lane == 0 && __float_as_uint(m) > __hip_atomic_load(amax, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
      atomicMax(amax, __float_as_uint(m));
  }
}

// ---------------------------------------------------------------------------------------
// Y[M, Nout] = A[M, K] W[Nout, K]^T + bias (optionally GELU), bf16 in and out, fp32
// accumulation.  Same machinery as the similarity kernel of the matching step: 256 x 256
// output tiles, both operands pre-packed fragment-major, fetched straight into a 4-stage LDS
// ring (2 k-steps per stage, 3 stages ahead), fragments read by hand one k-step ahead, 8 waves
// of 64 rows x 128 columns.  The finished tile goes from the accumulators straight to global
// memory (bias, optional GELU, one rounding to bf16); `addend` (optional, shaped like the
// output) is added to the rounded result on the way out.  The ring is free meanwhile, so the
// next tile's first stages are fetched during the epilogue.
// `split`: the output is Nout / split row-major blocks of [M, split] one after the other
// (split = Nout: one plain matrix; split = C for the fused q|k|v projection).
// PACKED: the output is the activation operand of a following layer with K = Nout and is
// written in that layer's operand order straight from the accumulators (bf16 fragments, or,
// with FP8, E4M3 codes quantised with *out_inv while the largest |value| goes to *out_amax).
// FP8: the same ring and the same byte traffic per stage, but a stage (two 1 KB units per
// fragment) is one k-step of 64 for v_mfma_f32_32x32x64_f8f6f4, whose operands are the two
// units of a fragment side by side in 8 registers: per stage a wave issues 8 MFMAs of twice
// the work.  The activation fragments of the next stage go to a second register set at the
// start of a stage, the weight fragments replace those of the current stage pair by pair as
// its MFMAs have been issued.  `alpha` (FP8: the product of the two scales) multiplies the
// accumulators before the bias.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void lds_read1_async(u32x4 &dst, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1" : "=&v"(dst) : "v"(addr) : "memory");
}
constexpr int kTile = 256;
constexpr int kStages = 4;
constexpr int kStageU4 = 2 * 2 * 8 * 64;     // [weights|activations][2 k-steps][8 fragments][64 lanes]

// GELU in its erf form, x * Phi(x).  erfc(|x| / sqrt 2) by the rational-times-exponential form of
// Abramowitz & Stegun 7.1.26 (absolute error <= 1.5e-7, four orders below a bf16 step); the
// negative side uses erfc itself, so nothing cancels there.  A third of erff's instructions: the
// epilogue of the first MLP layer evaluates it 65536 times per tile.
__device__ __forceinline__ float gelu_erf(float v) {
  const float x = fabsf(v) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, x, 1.0f));
  float p = __builtin_fmaf(1.061405429f, t, -1.453152027f);
  p = __builtin_fmaf(p, t, 1.421413741f);
  p = __builtin_fmaf(p, t, -0.284496736f);
  p = __builtin_fmaf(p, t, 0.254829592f);
  const float erfc_abs = p * t * __builtin_amdgcn_exp2f(-1.4426950408889634f * x * x);
  return 0.5f * v * (v < 0.f ? erfc_abs : 2.0f - erfc_abs);
}

template <bool FP8, bool PACKED>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_gemm_bt(
    const u32x4 *__restrict__ ap, const u32x4 *__restrict__ wp, int64_t M, int KS, int nt_n,
    const float *__restrict__ bias, int gelu, uint16_t *__restrict__ out, int split,
    const float *__restrict__ alpha_p, int n_tiles, const uint16_t *__restrict__ addend,
    const uint32_t *__restrict__ out_inv, uint32_t *__restrict__ out_amax) {
  extern __shared__ u32x4 ring[];
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wd = wave & 3, wn = wave >> 2;
  const int total = KS >> 1;
  // persistent: one workgroup per CU walks the tiles (a workgroup owns a whole CU's LDS, so a
  // launch per tile would pay a dispatch between any two tiles of a CU)
  // Workgroup w runs on XCD w % 8.  An XCD takes the row tiles tm = x, x + 8, ..., so an
  // activation tile is fetched into one L2 only.  Its workgroups form a block of Rb row tiles x G
  // column tiles (8 x 4 with 32 workgroups) that takes one group of G column tiles through all
  // the XCD's row tiles before it moves to the next group: the G weight tiles of a group (2 MB
  // at K = 1024) stay in that L2 meanwhile, and an activation tile is shared by G workgroups.
  const int nt_m = n_tiles / nt_n;
  const int xcd = blockIdx.x & (kXcd - 1), per_xcd = (int)gridDim.x >> 3;
  const int G = nt_n < 4 ? nt_n : 4, Rb = per_xcd / G;
  const bool by_xcd = (gridDim.x & (kXcd - 1)) == 0 && Rb >= 1;
  const int my_rows = by_xcd ? (nt_m - xcd + kXcd - 1) / kXcd : 0;   // row tiles of this XCD
  const int n_rb = by_xcd ? (my_rows + Rb - 1) / Rb : 0, n_cg = (nt_n + G - 1) / G;
  const int jr = (int)(blockIdx.x >> 3) / G, jc = (int)(blockIdx.x >> 3) % G;
  const int n_steps = by_xcd ? n_rb * n_cg : (n_tiles + (int)gridDim.x - 1) / (int)gridDim.x;
  // the first step >= k at which this workgroup has a tile (n_steps if none), and that tile
  auto next_step = [&](int k, int &tm_, int &tn_) {
    for (; k < n_steps; ++k) {
      if (by_xcd) {
        const int cg = k / n_rb, rb = k - cg * n_rb, lr = rb * Rb + jr, col = cg * G + jc;
        if (jr < Rb && lr < my_rows && col < nt_n) {
          tm_ = lr * kXcd + xcd;
          tn_ = col;
          break;
        }
      } else {
        const int v = (int)blockIdx.x + k * (int)gridDim.x;
        if (v < n_tiles) {
          tm_ = v / nt_n;
          tn_ = v % nt_n;
          break;
        }
      }
    }
    return k;
  };
  bool primed = false;   // the previous tile's epilogue has issued this tile's first stages
  int parity = 0;
  int tm = 0, tn = 0, tm2 = 0, tn2 = 0, k2 = 0;
  for (int k = next_step(0, tm, tn); k < n_steps; k = k2, tm = tm2, tn = tn2, parity ^= 1) {
  k2 = next_step(k + 1, tm2, tn2);
  // this tile's 256 bias values wait in LDS behind the ring (read in the epilogue, many barriers
  // later); two buffers in turn, so a wave still in the previous tile's epilogue reads its own
  float *bias_lds = (float *)(ring + (size_t)kStages * kStageU4) + parity * kTile;
  if (tid < kTile) bias_lds[tid] = bias ? bias[tn * kTile + tid] : 0.f;

  // fetch: this wave moves fragments f = 4*wave .. 4*wave+3 of a stage (f = op*16 + ks*8 + a)
  const int f_op = wave >> 2, f_ks = (wave >> 1) & 1, f_a0 = (wave & 1) * 4;
  int pf_g = 0, f_tm = tm, f_tn = tn;
  auto fetch = [&]() {
    const int s = pf_g < total ? pf_g : total - 1;   // past the end: the last stage again, into a free slot
    const u32x4 *src = (f_op ? ap + (size_t)(f_tm * 8 + f_a0) * KS * 64 : wp + (size_t)(f_tn * 8 + f_a0) * KS * 64) +
                       (size_t)(s * 2 + f_ks) * 64 + lane;
    u32x4 *dst = ring + (size_t)(pf_g & (kStages - 1)) * kStageU4 + (size_t)(wave * 4) * 64;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds(src + (size_t)i * KS * 64, dst + i * 64, 16, 0, 0);
    ++pf_g;
  };
  const uint32_t ring_lane = lds_addr(&ring[lane]);
  const uint32_t b_off = (uint32_t)((wn * 4) * 1024), a_off = (uint32_t)((16 + wd * 2) * 1024);
  u32x4 fb[2][4], fa[2][2];
  auto read_frags = [&](int g, int ks, u32x4(&b)[4], u32x4(&a)[2]) {
    const uint32_t base = ring_lane + (uint32_t)((g & (kStages - 1)) * kStageU4 * 16 + ks * 8 * 1024);
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
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
  auto mma = [&](const u32x4(&b)[4], const u32x4(&a)[2]) {
#pragma unroll
    for (int bi = 0; bi < 4; ++bi)
#pragma unroll
      for (int ai = 0; ai < 2; ++ai)
        acc[ai][bi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, b[bi]),
                                                             __builtin_bit_cast(bf16x8, a[ai]),
                                                             acc[ai][bi], 0, 0, 0);
  };

  if (primed) {
    pf_g = kStages;
    // the stages were issued ahead of the previous epilogue's stores: wait for everything
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  } else {
#pragma unroll
    for (int i = 0; i < kStages; ++i) fetch();               // stages 0..3
    asm volatile("s_waitcnt vmcnt(12)" ::: "memory");        // stage 0 has landed (this wave's part)
  }
  __builtin_amdgcn_s_barrier();
  if constexpr (!FP8) {
    read_frags(0, 0, fb[0], fa[0]);
    for (int g = 0; g < total; ++g) {
      __builtin_amdgcn_sched_barrier(0);
      wait_frags(fb[0], fa[0]);
      read_frags(g, 1, fb[1], fa[1]);
      __builtin_amdgcn_sched_barrier(0);
      mma(fb[0], fa[0]);
      __builtin_amdgcn_sched_barrier(0);
      wait_frags(fb[1], fa[1]);
      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");         // stage g+1 has landed; g+2, g+3 may be in flight
      __builtin_amdgcn_s_barrier();
      fetch();                                                 // stage g+4 -> slot of stage g
      read_frags(g + 1, 0, fb[0], fa[0]);                      // past the end: a stale slot, never used
      __builtin_amdgcn_sched_barrier(0);
      mma(fb[1], fa[1]);
    }
  } else {
    // fb[u][bi], fa[set][u][ai]: unit u of a fragment; an operand is (unit 0, unit 1)
    u32x4 fa2[2][2][2];
    read_frags(0, 0, fb[0], fa2[0][0]);
    read_frags(0, 1, fb[1], fa2[0][1]);
    auto stage = [&](int g, u32x4(&ac)[2][2], u32x4(&an)[2][2]) {
      __builtin_amdgcn_sched_barrier(0);
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(fb[0][0]), "+v"(fb[0][1]), "+v"(fb[0][2]), "+v"(fb[0][3]), "+v"(fb[1][0]),
                     "+v"(fb[1][1]), "+v"(fb[1][2]), "+v"(fb[1][3]), "+v"(ac[0][0]), "+v"(ac[0][1]),
                     "+v"(ac[1][0]), "+v"(ac[1][1])
                   :
                   : "memory");
      asm volatile("s_waitcnt vmcnt(8)" ::: "memory");       // stage g+1 has landed; g+2, g+3 may be in flight
      __builtin_amdgcn_s_barrier();                          // and nobody reads stage g from LDS any more
      fetch();                                               // stage g+4 -> slot of stage g
      // past the end these read a stale slot; the values are never used
      const uint32_t base = ring_lane + (uint32_t)(((g + 1) & (kStages - 1)) * kStageU4 * 16);
      lds_read2_async(an[0], base + a_off);
      lds_read2_async(an[1], base + 8 * 1024 + a_off);
#pragma unroll
      for (int bi = 0; bi < 4; ++bi) {
        __builtin_amdgcn_sched_barrier(0);
        const i32x8 b8 = cat8(fb[0][bi], fb[1][bi]);
#pragma unroll
        for (int ai = 0; ai < 2; ++ai)
          acc[ai][bi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b8, cat8(ac[0][ai], ac[1][ai]),
                                                                        acc[ai][bi], 0, 0, 0, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        lds_read1_async(fb[0][bi], base + b_off + bi * 1024);
        lds_read1_async(fb[1][bi], base + 8 * 1024 + b_off + bi * 1024);
      }
    };
    int g = 0;
    for (; g + 1 < total; g += 2) {
      stage(g, fa2[0], fa2[1]);
      stage(g + 1, fa2[1], fa2[0]);
    }
    if (g < total) stage(g, fa2[0], fa2[1]);
    // the reads issued by the last stage are waited for below, before their registers die
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(fb[0][0]), "+v"(fb[0][1]), "+v"(fb[0][2]), "+v"(fb[0][3]), "+v"(fb[1][0]),
                   "+v"(fb[1][1]), "+v"(fb[1][2]), "+v"(fb[1][3]), "+v"(fa2[0][0][0]), "+v"(fa2[0][0][1]),
                   "+v"(fa2[0][1][0]), "+v"(fa2[0][1][1]), "+v"(fa2[1][0][0]), "+v"(fa2[1][0][1]),
                   "+v"(fa2[1][1][0]), "+v"(fa2[1][1][1])
                 :
                 : "memory");
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");   // nothing may land in LDS any more
  __syncthreads();

  // Epilogue: bias, activation, bf16, straight from the accumulators to global memory; nothing
  // goes through LDS, so the next tile's first stages are issued first and land while the
  // arithmetic runs.  The weights are the first MFMA operand, so a lane holds one token (column)
  // and, per group of four accumulator registers, four consecutive output channels 8g + 4h .. + 3:
  // lanes l and l + 32 trade halves (one v_permlane32_swap per register pair: the first operand's
  // lanes 32-63 against the second operand's lanes 0-31), after which lane l has channels 0-7 and
  // lane l + 32 channels 8-15 of a run of 16, 16 bytes per lane.
  const float alpha = alpha_p ? *alpha_p : 1.0f;
  int anchor = 0;   // opaque zero: keeps the address arithmetic below inside this tile's epilogue
  asm volatile("" : "+v"(anchor));   // (hoisted out of the tile loop it would stay live through the main loop)
  if (k2 < n_steps) {
    f_tn = tn2;
    f_tm = tm2;
    pf_g = 0;
#pragma unroll
    for (int i = 0; i < kStages; ++i) fetch();
    primed = true;
  } else {
    primed = false;
  }
  if constexpr (PACKED) {
    // The output is the next linear layer's activation operand and is written in that kernel's
    // fragment order: out[(row / 32) * KSn + k-step][lane], where a k-step is 16 of this layer's
    // output channels and lane = row % 32 + 32 * (second 8 of the 16), which is exactly what the
    // lanes hold after the swap: a wave stores 1 KB in a row.
    if constexpr (FP8) {
      // E4M3 codes for an FP8 layer with K = Nout (units of 32 rows x 32 channels, lane h * 32 + r
      // holds the 16 codes of channels 32u + 16h .. + 15 of row r): every value is rounded to
      // bf16 as if it had been stored, then scaled by *out_inv; a lane has one dword of four codes
      // per register group g, lanes l and l + 32 trade groups 2, 3 against groups 0, 1.  The
      // largest |value| of the rows below M goes into *out_amax; rows beyond M are written as zeros.
      const float r = __uint_as_float(*out_inv);
      const int KSn = nt_n * (kTile / 32);
      u32x4 *op = (u32x4 *)out + ((size_t)(tm * 8 + wd * 2) * KSn + tn * (kTile / 32) + wn * 4) * 64 + lane + anchor;
      float m = 0.f;
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int a = 0; a < 2; ++a) {
          const bool live = (int64_t)tm * kTile + wd * 64 + 32 * a + (lane & 31) < M;
          uint32_t d[4];
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x4 bv = *(const f32x4 *)(bias_lds + wn * 128 + 32 * b + 8 * g + 4 * h);
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              v[i] = acc[a][b][4 * g + i] * alpha + bv[i];
              if (gelu) v[i] = gelu_erf(v[i]);
            }
            const uint32_t p0 = pack_bf16(v[0], v[1]), p1 = pack_bf16(v[2], v[3]);
            if (live) m = fmaxf(m, fmaxf(fmaxf(fabsf(bf16_lo(p0)), fabsf(bf16_hi(p0))), fmaxf(fabsf(bf16_lo(p1)), fabsf(bf16_hi(p1)))));
            d[g] = live ? cvt4_fp8(clamp448(bf16_lo(p0) * r), clamp448(bf16_hi(p0) * r), clamp448(bf16_lo(p1) * r),
                                   clamp448(bf16_hi(p1) * r))
                        : 0u;
          }
          const auto s0 = __builtin_amdgcn_permlane32_swap(d[0], d[2], false, false);
          const auto s1 = __builtin_amdgcn_permlane32_swap(d[1], d[3], false, false);
          op[((size_t)a * KSn + b) * 64] = u32x4{s0[0], s0[1], s1[0], s1[1]};
        }
      m = wave_max(m);
      if (lane == 0 && __float_as_uint(m) > __hip_atomic_load(out_amax, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomicMax(out_amax, __float_as_uint(m));
      continue;
    }
    const int KSn = nt_n * (kTile / 16);
    u32x4 *op = (u32x4 *)out + ((size_t)(tm * 8 + wd * 2) * KSn + tn * (kTile / 16) + wn * 8) * 64 + lane + anchor;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int gp = 0; gp < 2; ++gp) {
        const int ch0 = wn * 128 + 32 * b + 16 * gp + 4 * h;
        const f32x4 bv0 = *(const f32x4 *)(bias_lds + ch0), bv1 = *(const f32x4 *)(bias_lds + ch0 + 8);
#pragma unroll
        for (int a = 0; a < 2; ++a) {
          float v0[4], v1[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            v0[i] = acc[a][b][8 * gp + i] + bv0[i];
            v1[i] = acc[a][b][8 * gp + 4 + i] + bv1[i];
            if (gelu) {
              v0[i] = gelu_erf(v0[i]);
              v1[i] = gelu_erf(v1[i]);
            }
          }
          // first operand's lanes 32-63 <-> second operand's lanes 0-31
          const auto s0 = __builtin_amdgcn_permlane32_swap(pack_bf16(v0[0], v0[1]), pack_bf16(v1[0], v1[1]), false, false);
          const auto s1 = __builtin_amdgcn_permlane32_swap(pack_bf16(v0[2], v0[3]), pack_bf16(v1[2], v1[3]), false, false);
          op[((size_t)a * KSn + 2 * b + gp) * 64] = u32x4{s0[0], s1[0], s0[1], s1[1]};
        }
      }
    continue;
  }
  // row-major rows of `split` channels: per store instruction a wave writes 32 bytes of each of
  // 32 rows; the four stores that complete a 128-byte line follow each other
  const int blk = (tn * kTile) / split, col0 = (tn * kTile) % split;   // a tile never straddles two blocks
  uint16_t *ob = out + (size_t)blk * M * split + col0 + wn * 128 + 8 * h + anchor;
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int gp = 0; gp < 2; ++gp) {
      const int ch0 = wn * 128 + 32 * b + 16 * gp + 4 * h;
      const f32x4 bv0 = *(const f32x4 *)(bias_lds + ch0), bv1 = *(const f32x4 *)(bias_lds + ch0 + 8);
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        float v0[4], v1[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v0[i] = FP8 ? acc[a][b][8 * gp + i] * alpha + bv0[i] : acc[a][b][8 * gp + i] + bv0[i];
          v1[i] = FP8 ? acc[a][b][8 * gp + 4 + i] * alpha + bv1[i] : acc[a][b][8 * gp + 4 + i] + bv1[i];
          if (gelu) {
            v0[i] = gelu_erf(v0[i]);
            v1[i] = gelu_erf(v1[i]);
          }
        }
        const auto s0 = __builtin_amdgcn_permlane32_swap(pack_bf16(v0[0], v0[1]), pack_bf16(v1[0], v1[1]), false, false);
        const auto s1 = __builtin_amdgcn_permlane32_swap(pack_bf16(v0[2], v0[3]), pack_bf16(v1[2], v1[3]), false, false);
        u32x4 t = u32x4{s0[0], s1[0], s0[1], s1[1]};
        const int64_t m = (int64_t)tm * kTile + wd * 64 + 32 * a + (lane & 31);
        if (addend) {   // out = addend + (this layer's output, already rounded to bf16): one more rounding
          const u32x4 y = m < M ? *(const u32x4 *)(addend + (ob - out) + (size_t)m * split + 32 * b + 16 * gp)
                                : u32x4{0u, 0u, 0u, 0u};
          t.x = pack_bf16(bf16_lo(t.x) + bf16_lo(y.x), bf16_hi(t.x) + bf16_hi(y.x));
          t.y = pack_bf16(bf16_lo(t.y) + bf16_lo(y.y), bf16_hi(t.y) + bf16_hi(y.y));
          t.z = pack_bf16(bf16_lo(t.z) + bf16_lo(y.z), bf16_hi(t.z) + bf16_hi(y.z));
          t.w = pack_bf16(bf16_lo(t.w) + bf16_lo(y.w), bf16_hi(t.w) + bf16_hi(y.w));
        }
        if (m < M) *(u32x4 *)(ob + (size_t)m * split + 32 * b + 16 * gp) = t;
      }
    }
  }   // tiles
}

// ---------------------------------------------------------------------------------------
struct BlockWs {
  uint16_t *h, *qkv, *a, *u1, *h3;
  u32x4 *apack, *wpack;
  uint32_t *fp8sc;
  void *attn;
  size_t bytes;
  int64_t Mp;
};

// the four weight matrices in operand order, one after the other (qkv, output, MLP 1, MLP 2),
// then a 256-byte tail for their four amaxes (FP8 layers)
size_t block_wpack_bytes(int C) { return align_up((size_t)12 * C * C * 2, 256) + 256; }

static BlockWs carve_block(int64_t M, int C, int heads, int attn_dtype, char *base) {
  BlockWs w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    char *p = base ? base + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  w.Mp = (int64_t)align_up((size_t)M, kTile);
  w.h = (uint16_t *)take((size_t)M * C * 2);
  w.qkv = (uint16_t *)take((size_t)3 * M * C * 2);
  w.a = (uint16_t *)take((size_t)M * C * 2);
  w.u1 = (uint16_t *)take((size_t)M * C * 2);
  w.h3 = (uint16_t *)take((size_t)w.Mp * 4 * C * 2);   // row-major (FP8 layers) or in fragment order (bf16 layers)
  w.apack = (u32x4 *)take((size_t)w.Mp * 4 * C);       // a layer's activation operand: bf16 with K = C, FP8 with K <= 4C
  w.wpack = (u32x4 *)take(block_wpack_bytes(C));
  w.fp8sc = (uint32_t *)take(4 * kFp8Words * sizeof(uint32_t));   // one set per linear layer
  w.attn = take(attn_ws_bytes(heads, M, attn_dtype));
  w.bytes = off;
  return w;
}

size_t block_ws_bytes(int64_t M, int C, int heads, int attn_dtype) {
  return carve_block(M, C, heads, attn_dtype, nullptr).bytes;
}

// What a linear layer finds ready and what it leaves behind.
struct LinearOpts {
  bool fp8 = false;
  const u32x4 *a_packed = nullptr;     // the activation operand, already in operand order (then A is unused)
  bool pack_out = false;               // out receives the next layer's (K = Nout) operand, Mp rows, instead of row-major rows
  const uint16_t *addend = nullptr;    // row-major, same shape as out: out = addend + result
  u32x4 *w_packed = nullptr;           // where the weight operand lives (default: the workspace)
  bool pack_w = true;                  // false: w_packed already holds it
  // FP8 with this layer's scalars prepared by k_fp8_prepare (nothing is zeroed, derived or
  // recorded here): A, unless a_packed, is quantised with sc[2] and its amax reduced into sc[0];
  // W, if pack_w, is quantised with sc[3]
  uint32_t *sc = nullptr;
  const uint32_t *out_inv = nullptr;   // FP8 pack_out: the next layer's input scale ...
  uint32_t *out_amax = nullptr;        // ... and where the largest |output| is reduced into
};

// Y = A W^T + bias: brings both operands into operand order where they are not yet (FP8: after
// taking their amax and quantising them), then the tiled kernel.
static int launch_linear(const uint16_t *A, int64_t M, int K, const uint16_t *W, int Nout,
                         const float *bias, int gelu, uint16_t *out, int split, BlockWs &w,
                         hipStream_t st, const LinearOpts &o) {
  u32x4 *const w_packed = o.w_packed ? o.w_packed : w.wpack;
  if (o.fp8 && !o.sc && (!o.pack_w || o.a_packed || o.pack_out)) return LV_ERR_PARAM;
  if (o.pack_out && (o.addend || split != Nout || (o.fp8 && (!o.out_inv || !o.out_amax)))) return LV_ERR_PARAM;
  if (K % 64 != 0 || Nout % kTile != 0 || split % kTile != 0 || Nout % split != 0) return LV_ERR_SHAPE;
  int rc;
  const size_t lds = (size_t)kStages * kStageU4 * 16 + 2 * kTile * sizeof(float);   // + two tiles' bias values
  static std::atomic<uint64_t> lds_done[4];
  if ((rc = allow_dynamic_lds((const void *)k_gemm_bt<false, false>, lds, lds_done[0]))) return rc;
  if ((rc = allow_dynamic_lds((const void *)k_gemm_bt<true, false>, lds, lds_done[1]))) return rc;
  if ((rc = allow_dynamic_lds((const void *)k_gemm_bt<false, true>, lds, lds_done[2]))) return rc;
  if ((rc = allow_dynamic_lds((const void *)k_gemm_bt<true, true>, lds, lds_done[3]))) return rc;
  const int nt_n = Nout / kTile;
  const int64_t nt_m = w.Mp / kTile;
  if (nt_m * nt_n >= ((int64_t)1 << 31) || w.Mp >= ((int64_t)1 << 31)) return LV_ERR_SHAPE;
  const int n_tiles = (int)(nt_m * nt_n);
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
    return LV_ERR_HIP;
  const unsigned grid = (unsigned)(n_tiles < n_cu ? n_tiles : n_cu);
  const u32x4 *a_packed = o.a_packed;
  if (o.fp8) {
    auto amax = [&](const uint16_t *t, int64_t n16, uint32_t *dst) {
      const unsigned g = (unsigned)(((n16 + 255) / 256) < 4096 ? ((n16 + 255) / 256) : 4096);
      hipLaunchKernelGGL(k_amax_bf16, dim3(g), dim3(256), 0, st, (const u32x4 *)t, n16, dst);
    };
    auto quant = [&](const uint16_t *t, int64_t n, int64_t n_pad, const uint32_t *inv, u32x4 *dst, uint32_t *amax_out) {
      hipLaunchKernelGGL(k_quant_pack_fp8, dim3((unsigned)(n_pad / 32), (unsigned)((K / 32 + 15) / 16)), dim3(256), 0, st, t, (int)n,
                         K, inv, dst, amax_out);
    };
    uint32_t *sc = o.sc;
    if (!sc) {
      // current scaling: both amaxes first, then the scales, then the two quantisation passes
      sc = w.fp8sc;
      hipLaunchKernelGGL(k_fp8_zero, dim3(1), dim3(64), 0, st, sc);
      amax(A, M * (K / 8), sc);
      amax(W, (int64_t)Nout * (K / 8), sc + 1);
      hipLaunchKernelGGL(k_fp8_scales, dim3(1), dim3(64), 0, st, sc);
      quant(A, M, w.Mp, sc + 2, w.apack, (uint32_t *)nullptr);
      quant(W, Nout, Nout, sc + 3, w_packed, (uint32_t *)nullptr);
      a_packed = w.apack;
    } else {
      if (!a_packed) {
        quant(A, M, w.Mp, sc + 2, w.apack, sc);
        a_packed = w.apack;
      }
      if (o.pack_w) quant(W, Nout, Nout, sc + 3, w_packed, (uint32_t *)nullptr);
    }
    if (o.pack_out)
      hipLaunchKernelGGL((k_gemm_bt<true, true>), dim3(grid), dim3(512), lds, st, a_packed, w_packed, M, K / 32,
                         nt_n, bias, gelu, out, split, (const float *)(sc + 4), n_tiles, o.addend, o.out_inv,
                         o.out_amax);
    else
      hipLaunchKernelGGL((k_gemm_bt<true, false>), dim3(grid), dim3(512), lds, st, a_packed, w_packed, M, K / 32,
                         nt_n, bias, gelu, out, split, (const float *)(sc + 4), n_tiles, o.addend,
                         (const uint32_t *)nullptr, (uint32_t *)nullptr);
  } else {
    if (!a_packed) {
      if ((rc = launch_pack_rows(A, M, w.Mp, K, w.apack, st))) return rc;
      a_packed = w.apack;
    }
    if (o.pack_w && (rc = launch_pack_rows(W, Nout, Nout, K, w_packed, st))) return rc;
    if (o.pack_out)
      hipLaunchKernelGGL((k_gemm_bt<false, true>), dim3(grid), dim3(512), lds, st, a_packed, w_packed, M, K / 16,
                         nt_n, bias, gelu, out, split, (const float *)nullptr, n_tiles, o.addend,
                         (const uint32_t *)nullptr, (uint32_t *)nullptr);
    else
      hipLaunchKernelGGL((k_gemm_bt<false, false>), dim3(grid), dim3(512), lds, st, a_packed, w_packed, M, K / 16,
                         nt_n, bias, gelu, out, split, (const float *)nullptr, n_tiles, o.addend,
                         (const uint32_t *)nullptr, (uint32_t *)nullptr);
  }
  LV_HIP_CHECK_LAUNCH();
  return LV_OK;
}

// Delayed scaling with every layer's scalars prepared ahead of the kernels that produce the
// layers' inputs: block L of the grid fills the 8 words of layer L (input amax cleared, the
// weight's amax, 448 / the largest recorded input amax, 448 / the weight's amax, the product of
// the two inverse scales).  Same arithmetic as k_fp8_scales; a history with nothing recorded yet gives scale 1.
__global__ __launch_bounds__(64) void k_fp8_prepare(uint32_t *__restrict__ sc, const float *__restrict__ state,
                                                    const uint32_t *__restrict__ wamax) {
  const int lane = threadIdx.x, L = blockIdx.x;
  const float *hist = state + (size_t)L * (LV_FP8_HISTORY + 2);
  const float m = wave_max(fmaxf(hist[lane], lane + 64 < LV_FP8_HISTORY ? hist[lane + 64] : 0.f));
  if (lane == 0) {
    uint32_t *s = sc + L * kFp8Words;
    const float ia = fp8_scale_inv(__float_as_uint(m)), iw = fp8_scale_inv(wamax[L]);
    s[0] = 0u;
    s[1] = wamax[L];
    s[2] = __float_as_uint(ia);
    s[3] = __float_as_uint(iw);
    s[4] = __float_as_uint((1.0f / ia) * (1.0f / iw));
  }
}

// ... and, once the four layers have run, each layer's input amax goes into its history
__global__ void k_fp8_record_all(const uint32_t *__restrict__ sc, float *__restrict__ state) {
  if (threadIdx.x < 4) {
    float *hist = state + (size_t)threadIdx.x * (LV_FP8_HISTORY + 2);
    uint32_t *step = (uint32_t *)(hist + LV_FP8_HISTORY);
    hist[*step % LV_FP8_HISTORY] = __uint_as_float(sc[threadIdx.x * kFp8Words]);
    *step += 1;
  }
}

int launch_global_block(const uint16_t *z, int64_t M, int C, int heads, float scale, int attn_dtype,
                        int qk_norm, const litevggt_block_weights &bw, uint16_t *delta, void *ws,
                        hipStream_t st, hipEvent_t after_pack, hipEvent_t after_attn, void *wpack_keep,
                        bool wpack_ready) {
  if (C % kTile != 0) return LV_ERR_SHAPE;
  BlockWs w = carve_block(M, C, heads, attn_dtype, (char *)ws);
  int rc;
  const bool f8 = bw.linear_dtype == LV_LINEAR_FP8_E4M3;
  const bool delayed = f8 && bw.fp8_recipe == LV_FP8_DELAYED;
  // The weights in operand order: in the workspace, or in a buffer of the caller's that outlives
  // the call and may already hold them (bf16 layers, and FP8 layers under delayed scaling, where
  // a weight's scale depends on nothing but the weight; the four amaxes follow the matrices).
  const bool keep = wpack_keep && (!f8 || delayed);
  u32x4 *const wp = keep ? (u32x4 *)wpack_keep : w.wpack;
  const bool pack_w = !(keep && wpack_ready);
  const size_t cc16 = (size_t)C * C * 2 / 16;
  u32x4 *const wp_l[4] = {wp, wp + 3 * cc16, wp + 4 * cc16, wp + 8 * cc16};
  uint32_t *const wamax = (uint32_t *)(wp + 12 * cc16);
  const uint16_t *const W[4] = {(const uint16_t *)bw.w_qkv, (const uint16_t *)bw.w_o, (const uint16_t *)bw.w_1,
                                (const uint16_t *)bw.w_2};
  const int w_rows[4] = {3 * C, C, 4 * C, C}, w_k[4] = {C, C, C, 4 * C};
  const float *const bias[4] = {bw.b_qkv, bw.b_o, bw.b_1, bw.b_2};
  const uint16_t *q = w.qkv, *k = w.qkv + (size_t)M * C, *v = w.qkv + (size_t)2 * M * C;

  if (delayed) {
    // FP8 layers, delayed scaling: every input scale is known before its tensor exists, so the
    // LayerNorms and the first MLP layer quantise their results themselves (taking the amax for
    // the history on the way); only the attention output goes through k_quant_pack_fp8.
    uint32_t *const sc = w.fp8sc;
    if (pack_w) {
      hipLaunchKernelGGL(k_fp8_zero, dim3(1), dim3(64), 0, st, wamax);
      for (int l = 0; l < 4; ++l) {
        const int64_t n16 = (int64_t)w_rows[l] * (w_k[l] / 8);
        const unsigned g = (unsigned)(((n16 + 255) / 256) < 4096 ? ((n16 + 255) / 256) : 4096);
        hipLaunchKernelGGL(k_amax_bf16, dim3(g), dim3(256), 0, st, (const u32x4 *)W[l], n16, wamax + l);
      }
    }
    hipLaunchKernelGGL(k_fp8_prepare, dim3(4), dim3(64), 0, st, sc, (const float *)bw.fp8_state, (const uint32_t *)wamax);
    auto layer = [&](int l) {
      LinearOpts o;
      o.fp8 = true;
      o.sc = sc + l * kFp8Words;
      o.w_packed = wp_l[l];
      o.pack_w = pack_w;
      return o;
    };
    if ((rc = launch_layernorm(z, nullptr, bw.ln1_g, bw.ln1_b, M, C, nullptr, st, w.apack, w.Mp, sc + 2, sc))) return rc;
    LinearOpts o = layer(0);
    o.a_packed = w.apack;
    if ((rc = launch_linear(nullptr, M, C, W[0], 3 * C, bias[0], 0, w.qkv, C, w, st, o))) return rc;
    if ((rc = launch_attn(q, k, v, w.a, M, heads, scale, attn_dtype, qk_norm, w.attn, st, after_pack))) return rc;
    if (after_attn && hipEventRecord(after_attn, st) != hipSuccess) return LV_ERR_HIP;
    o = layer(1);
    if ((rc = launch_linear(w.a, M, C, W[1], C, bias[1], 0, w.u1, C, w, st, o))) return rc;
    if ((rc = launch_layernorm(z, w.u1, bw.ln2_g, bw.ln2_b, M, C, nullptr, st, w.apack, w.Mp,
                               sc + 2 * kFp8Words + 2, sc + 2 * kFp8Words)))
      return rc;
    o = layer(2);
    o.a_packed = w.apack;
    o.pack_out = true;
    o.out_inv = sc + 3 * kFp8Words + 2;
    o.out_amax = sc + 3 * kFp8Words;
    if ((rc = launch_linear(nullptr, M, C, W[2], 4 * C, bias[2], 1, w.h3, 4 * C, w, st, o))) return rc;
    o = layer(3);
    o.a_packed = (const u32x4 *)w.h3;
    o.addend = w.u1;
    if ((rc = launch_linear(nullptr, M, 4 * C, W[3], C, bias[3], 0, delta, C, w, st, o))) return rc;
    hipLaunchKernelGGL(k_fp8_record_all, dim3(1), dim3(64), 0, st, (const uint32_t *)sc, (float *)bw.fp8_state);
    LV_HIP_CHECK_LAUNCH();
    return LV_OK;
  }

  auto layer = [&](int l) {
    LinearOpts o;
    o.fp8 = f8;
    o.w_packed = wp_l[l];
    o.pack_w = f8 || pack_w;
    return o;
  };
  // bf16 layers: the LayerNorms write their result in the following layer's operand order
  u32x4 *const ln_packed = f8 ? nullptr : w.apack;
  if ((rc = launch_layernorm(z, nullptr, bw.ln1_g, bw.ln1_b, M, C, w.h, st, ln_packed, w.Mp))) return rc;
  LinearOpts o = layer(0);
  o.a_packed = ln_packed;
  if ((rc = launch_linear(w.h, M, C, W[0], 3 * C, bias[0], 0, w.qkv, C, w, st, o))) return rc;
  // bf16 layers: where the attention kernel can, it writes the output projection's operand itself
  bool a_is_packed = false;
  if ((rc = launch_attn(q, k, v, w.a, M, heads, scale, attn_dtype, qk_norm, w.attn, st, after_pack, 1, nullptr,
                        f8 ? nullptr : (void *)w.apack, &a_is_packed)))
    return rc;
  if (after_attn && hipEventRecord(after_attn, st) != hipSuccess) return LV_ERR_HIP;
  o = layer(1);
  o.a_packed = a_is_packed ? w.apack : nullptr;
  if ((rc = launch_linear(w.a, M, C, W[1], C, bias[1], 0, w.u1, C, w, st, o))) return rc;
  if ((rc = launch_layernorm(z, w.u1, bw.ln2_g, bw.ln2_b, M, C, w.h, st, ln_packed, w.Mp))) return rc;
  // bf16 layers: the first MLP layer writes its output in the second one's operand order.  All
  // layers: the second one's epilogue adds u1 (delta = u1 + u2, u2 rounded to bf16 first as if
  // it had been stored).
  o = layer(2);
  o.a_packed = ln_packed;
  o.pack_out = !f8;
  if ((rc = launch_linear(w.h, M, C, W[2], 4 * C, bias[2], 1, w.h3, 4 * C, w, st, o))) return rc;
  o = layer(3);
  o.a_packed = f8 ? nullptr : (const u32x4 *)w.h3;
  o.addend = w.u1;
  return launch_linear(w.h3, M, 4 * C, W[3], C, bias[3], 0, delta, C, w, st, o);
}

}  // namespace lv
