// Host-side launch functions of the kernel files; the C ABI in api.hip calls these
// after validating arguments.  All pointers are device pointers unless noted.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "../../include/litevggt.h"

namespace lv {

struct Dims {
  int F, H, W, S, C, heads, P, T;
  int64_t N;
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Raise a kernel's dynamic LDS limit on the current device.  The attribute is per device, so
// `done` (one per kernel, zero-initialised) remembers the devices that have it; setting it
// twice is harmless, which makes concurrent first calls safe.
inline int allow_dynamic_lds(const void *kernel, size_t bytes, std::atomic<uint64_t> &done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return LV_ERR_HIP;
  const uint64_t bit = dev >= 0 && dev < 64 ? (uint64_t)1 << dev : 0;
  if (bit && (done.load(std::memory_order_acquire) & bit)) return LV_OK;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
    return LV_ERR_HIP;
  done.fetch_or(bit, std::memory_order_release);
  return LV_OK;
}

// importance.hip
int launch_grad_map(const void *images, int img_dtype, const Dims &d, int patch, float *psi_g,
                    hipStream_t st);
int launch_naive_score(const Dims &d, int policy, uint32_t seed, float *score, hipStream_t st);
int launch_var_map(const uint16_t *x, const Dims &d, int pool, float *psi_v, hipStream_t st);
int launch_ga_fuse(const float *psi_g, const float *psi_v, const Dims &d, float alpha, float beta,
                   float *score, hipStream_t st);

// Capacity of the library-owned variance-map scratch of litevggt_importance_static, and the
// device address of that scratch on the current device (looked up once per device).
constexpr size_t kStaticScoreFloats = LV_STATIC_SCORE_MAX;
int static_importance_scratch(float **out);

// select.hip
int launch_select(const float *score, const Dims &d, const litevggt_plan_t &pl,
                  const litevggt_index &ix, hipStream_t st);

// match.hip
size_t match_ws_bytes(const Dims &d, const litevggt_plan_t &pl);
int launch_match(const uint16_t *x, const Dims &d, const litevggt_plan_t &pl,
                 const litevggt_index &ix, float *best_sim, void *ws, hipStream_t st);

// rows 0..n-1 of a row-major [n, C] bf16 matrix -> fragment-major (1 KB per 32 rows x 16
// channels), padded with zero rows to n_pad
int launch_pack_rows(const uint16_t *x, int64_t n, int64_t n_pad, int C, void *packed,
                     hipStream_t st);

// block.hip
size_t block_ws_bytes(int64_t M, int C, int heads, int attn_dtype);
size_t block_wpack_bytes(int C);
// delta = Block(z) - z for M tokens; the two events (optional) are recorded around the
// attention kernel inside the block.  wpack_keep (optional, block_wpack_bytes(C), bf16 layers
// only): receives the weights in the linear kernel's operand order, or, with wpack_ready,
// already holds them from an earlier call with the same weights.
int launch_global_block(const uint16_t *z, int64_t M, int C, int heads, float scale, int attn_dtype,
                        int qk_norm, const litevggt_block_weights &bw, uint16_t *delta, void *ws,
                        hipStream_t st, hipEvent_t after_pack = nullptr,
                        hipEvent_t after_attn = nullptr, void *wpack_keep = nullptr,
                        bool wpack_ready = false);

// merge.hip
int launch_merge(const uint16_t *x, const Dims &d, int64_t M, const litevggt_index &ix,
                 uint16_t *z, hipStream_t st);
int launch_unmerge(const uint16_t *y, const Dims &d, const litevggt_index &ix,
                   const uint16_t *residual, uint16_t *out, hipStream_t st);

// attn.hip
size_t attn_ws_bytes(int heads, int64_t n_tokens, int attn_dtype, int n_seq = 1);
// `after_pack`, when not NULL, is recorded between the K/V re-layout and the main kernel;
// n_seq sequences of n_tokens each; res: optional residual added to the output.  o_packed
// (optional, with wrote_packed): a linear layer's activation operand buffer for align_up(n_tokens,
// 256) rows; when the bf16 fixed-reference kernel runs it writes the output there in that
// layer's fragment order instead of to o, and *wrote_packed tells whether it did.
int launch_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v, uint16_t *o,
                int64_t n_tokens, int heads, float scale, int attn_dtype, int qk_norm, void *ws,
                hipStream_t st, hipEvent_t after_pack = nullptr, int n_seq = 1,
                const uint16_t *res = nullptr, void *o_packed = nullptr, bool *wrote_packed = nullptr);

}  // namespace lv
