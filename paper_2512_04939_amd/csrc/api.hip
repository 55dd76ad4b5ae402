// C ABI: argument validation, closed-form size planning, workspace carving and the
// cached-index layer loop.  Everything here is host code; kernels live in the other files.
#include <math.h>
#include <string.h>

#include "internal.h"

using namespace lv;

namespace {

int check_params(const litevggt_params *p, Dims *d) {
  if (!p) return LV_ERR_NULL;
  if (p->frames < 1 || p->grid_h < 1 || p->grid_w < 1 || p->n_special < 0) return LV_ERR_SHAPE;
  if (p->head_dim != 64 || p->heads < 1 || p->dim != p->heads * p->head_dim) return LV_ERR_SHAPE;
  if (p->dim > 2048) return LV_ERR_SHAPE;
  if (p->patch < 1) return LV_ERR_SHAPE;
  if (p->img_dtype != LV_IMG_F32 && p->img_dtype != LV_IMG_U8) return LV_ERR_DTYPE;
  if (p->attn_dtype != LV_ATTN_BF16 && p->attn_dtype != LV_ATTN_FP8_E4M3) return LV_ERR_DTYPE;
  if (p->var_pool != 1 && p->var_pool != 3 && p->var_pool != 5) return LV_ERR_PARAM;
  if (p->refresh_interval < 1) return LV_ERR_PARAM;
  if (p->anchor_policy < LV_POLICY_GA || p->anchor_policy > LV_POLICY_RANDOM) return LV_ERR_PARAM;
  if (!(p->merge_ratio < 1.0)) return LV_ERR_PARAM;            // also rejects NaN
  if (p->merge_ratio < 0 && !(p->ga_frac >= 0.0 && p->ga_frac <= 1.0)) return LV_ERR_PARAM;
  if (!isfinite(p->alpha) || !isfinite(p->beta) || !isfinite(p->softmax_scale)) return LV_ERR_PARAM;
  const int64_t P = (int64_t)p->grid_h * p->grid_w;
  const int64_t N = (int64_t)p->frames * (P + p->n_special);
  if (P > 6000 || N >= ((int64_t)1 << 31)) return LV_ERR_SHAPE;
  d->F = p->frames;
  d->H = p->grid_h;
  d->W = p->grid_w;
  d->S = p->n_special;
  d->C = p->dim;
  d->heads = p->heads;
  d->P = (int)P;
  d->T = (int)P + p->n_special;
  d->N = N;
  return LV_OK;
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

int make_plan(const litevggt_params *p, const Dims &d, litevggt_plan_t *pl) {
  const int P = d.P;
  int cell, n_dst, n_ga, n_src;
  if (p->merge_ratio < 0) {
    cell = 2;
    n_dst = ceil_div(d.H, cell) * ceil_div(d.W, cell);
    n_ga = (int)floor(p->ga_frac * P + 1e-9);
    if (n_ga > P - n_dst) n_ga = P - n_dst;
    n_src = P - n_dst - n_ga;
  } else {
    n_src = (int)floor(p->merge_ratio * P + 1e-9);
    const int K = P - n_src;
    if (n_src == 0) {
      cell = 1;
      n_dst = P;
      n_ga = 0;
    } else {
      if (K < 1) return LV_ERR_PARAM;
      cell = 2;
      while (ceil_div(d.H, cell) * ceil_div(d.W, cell) > K) ++cell;
      n_dst = ceil_div(d.H, cell) * ceil_div(d.W, cell);
      n_ga = K - n_dst;
    }
  }
  const int K = n_dst + n_ga;
  pl->N = d.N;
  pl->M = (int64_t)d.S * d.F + P + (int64_t)(d.F - 1) * K;
  pl->n_dst = (int64_t)P + (int64_t)(d.F - 1) * n_dst;
  pl->n_src = (int64_t)(d.F - 1) * n_src;
  pl->cell = cell;
  pl->n_dst_per_frame = n_dst;
  pl->n_ga_per_frame = n_ga;
  pl->n_src_per_frame = n_src;
  pl->ws_bytes = 0;
  return LV_OK;
}

size_t importance_ws_bytes(const Dims &d) { return align_up((size_t)d.F * d.P * sizeof(float), 256); }

// driver scratch: z and y [M,C] bf16, then the larger of the per-op scratches
size_t driver_ws_bytes(const litevggt_params *p, const Dims &d, const litevggt_plan_t &pl) {
  size_t zy = 2 * align_up((size_t)pl.M * d.C * 2, 256);
  if (p->block) zy += block_wpack_bytes(d.C);   // the block's weights in operand order, kept across the layers
  size_t op = importance_ws_bytes(d);
  size_t m = match_ws_bytes(d, pl);
  if (m > op) op = m;
  size_t a = attn_ws_bytes(d.heads, pl.M, p->attn_dtype);
  if (a > op) op = a;
  if (p->frame_attn) {
    a = attn_ws_bytes(d.heads, d.T, LV_ATTN_BF16, d.F);
    if (a > op) op = a;
  }
  if (p->block) {
    a = block_ws_bytes(pl.M, d.C, d.heads, p->attn_dtype);
    if (a > op) op = a;
  }
  return zy + op;
}

bool ws_ok(const void *ws, size_t have, size_t need) {
  if (need == 0) return true;
  return ws && have >= need && ((uintptr_t)ws & 255u) == 0;
}

bool index_ok(const litevggt_index *ix) {
  return ix && ix->role && ix->kept_idx && ix->dst_idx && ix->src_idx && ix->anchor_of &&
         ix->slot_of && ix->group_off && ix->group_mem;
}

float scale_of(const litevggt_params *p) {
  return p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->head_dim);
}

}  // namespace

extern "C" {

const char *litevggt_strerror(int code) {
  switch (code) {
    case LV_OK: return "ok";
    case LV_ERR_NULL: return "required pointer is NULL";
    case LV_ERR_SHAPE: return "inconsistent or unsupported shape";
    case LV_ERR_PARAM: return "hyper-parameter out of range";
    case LV_ERR_WORKSPACE: return "workspace too small or not 256-byte aligned";
    case LV_ERR_DTYPE: return "unsupported dtype";
    case LV_ERR_HIP: return "HIP runtime error";
    default: return "unknown error code";
  }
}

int litevggt_plan(const litevggt_params *p, litevggt_plan_t *out) {
  if (!out) return LV_ERR_NULL;
  Dims d;
  int rc = check_params(p, &d);
  if (rc) return rc;
  rc = make_plan(p, d, out);
  if (rc) return rc;
  out->ws_bytes = driver_ws_bytes(p, d, *out);
  return LV_OK;
}

size_t litevggt_attn_ws_bytes(const litevggt_params *p, int64_t n_tokens) {
  Dims d;
  if (check_params(p, &d) || n_tokens < 1) return 0;
  return attn_ws_bytes(d.heads, n_tokens, p->attn_dtype);
}

int litevggt_importance(const litevggt_params *p, const void *images, const void *x,
                        float *grad_cache, int recompute_grad, float *score, void *ws,
                        size_t ws_bytes, void *stream) {
  Dims d;
  int rc = check_params(p, &d);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  if (p->anchor_policy != LV_POLICY_GA) {
    if (!score) return LV_ERR_NULL;
    return launch_naive_score(d, p->anchor_policy, p->policy_seed, score, st);
  }
  if (!x || !grad_cache || !score || (recompute_grad && !images)) return LV_ERR_NULL;
  if (!ws_ok(ws, ws_bytes, importance_ws_bytes(d))) return LV_ERR_WORKSPACE;
  float *psi_v = (float *)ws;
  if (recompute_grad) {
    rc = launch_grad_map(images, p->img_dtype, d, p->patch, grad_cache, st);
    if (rc) return rc;
  }
  rc = launch_var_map((const uint16_t *)x, d, p->var_pool, psi_v, st);
  if (rc) return rc;
  return launch_ga_fuse(grad_cache, psi_v, d, p->alpha, p->beta, score, st);
}

int litevggt_importance_static(const litevggt_params *p, const void *images, const void *x,
                               float *grad_cache, int recompute_grad, float *score, void *stream) {
  Dims d;
  int rc = check_params(p, &d);
  if (rc) return rc;
  if (p->anchor_policy == LV_POLICY_GA) {
    if (!x || !grad_cache || !score || (recompute_grad && !images)) return LV_ERR_NULL;
    if ((size_t)d.F * d.P > kStaticScoreFloats) return LV_ERR_WORKSPACE;
  }
  float *psi_v = nullptr;
  if ((rc = static_importance_scratch(&psi_v))) return rc;
  return litevggt_importance(p, images, x, grad_cache, recompute_grad, score, psi_v,
                             kStaticScoreFloats * sizeof(float), stream);
}

int litevggt_select_anchors(const litevggt_params *p, const float *score, litevggt_index *index,
                            void *stream) {
  Dims d;
  litevggt_plan_t pl;
  int rc = check_params(p, &d);
  if (rc) return rc;
  rc = make_plan(p, d, &pl);
  if (rc) return rc;
  if (!score || !index_ok(index)) return LV_ERR_NULL;
  return launch_select(score, d, pl, *index, (hipStream_t)stream);
}

int litevggt_match(const litevggt_params *p, const void *x, litevggt_index *index, float *best_sim,
                   void *ws, size_t ws_bytes, void *stream) {
  Dims d;
  litevggt_plan_t pl;
  int rc = check_params(p, &d);
  if (rc) return rc;
  rc = make_plan(p, d, &pl);
  if (rc) return rc;
  if (!x || !index_ok(index)) return LV_ERR_NULL;
  if (d.C > 1024) return LV_ERR_SHAPE;
  if (!ws_ok(ws, ws_bytes, match_ws_bytes(d, pl))) return LV_ERR_WORKSPACE;
  return launch_match((const uint16_t *)x, d, pl, *index, best_sim, ws, (hipStream_t)stream);
}

int litevggt_merge(const litevggt_params *p, const void *x, const litevggt_index *index, void *z,
                   void *stream) {
  Dims d;
  litevggt_plan_t pl;
  int rc = check_params(p, &d);
  if (rc) return rc;
  rc = make_plan(p, d, &pl);
  if (rc) return rc;
  if (!x || !z || !index || !index->group_off || !index->group_mem) return LV_ERR_NULL;
  return launch_merge((const uint16_t *)x, d, pl.M, *index, (uint16_t *)z, (hipStream_t)stream);
}

int litevggt_global_attn(const litevggt_params *p, int64_t n_tokens, const void *q, const void *k,
                         const void *v, void *o, void *ws, size_t ws_bytes, void *stream) {
  Dims d;
  int rc = check_params(p, &d);
  if (rc) return rc;
  if (!q || !k || !v || !o) return LV_ERR_NULL;
  if (n_tokens < 1 || n_tokens >= ((int64_t)1 << 31)) return LV_ERR_SHAPE;
  if (!ws_ok(ws, ws_bytes, attn_ws_bytes(d.heads, n_tokens, p->attn_dtype))) return LV_ERR_WORKSPACE;
  return launch_attn((const uint16_t *)q, (const uint16_t *)k, (const uint16_t *)v, (uint16_t *)o,
                     n_tokens, d.heads, scale_of(p), p->attn_dtype, p->qk_norm, ws, (hipStream_t)stream);
}

static int check_block_weights(const litevggt_block_weights *w) {
  if (!(w && w->ln1_g && w->ln1_b && w->w_qkv && w->b_qkv && w->w_o && w->b_o && w->ln2_g &&
        w->ln2_b && w->w_1 && w->b_1 && w->w_2 && w->b_2))
    return LV_ERR_NULL;
  if (w->linear_dtype != LV_LINEAR_BF16 && w->linear_dtype != LV_LINEAR_FP8_E4M3) return LV_ERR_DTYPE;
  if (w->linear_dtype == LV_LINEAR_FP8_E4M3) {
    if (w->fp8_recipe != LV_FP8_CURRENT && w->fp8_recipe != LV_FP8_DELAYED) return LV_ERR_PARAM;
    if (w->fp8_recipe == LV_FP8_DELAYED && !w->fp8_state) return LV_ERR_NULL;
  }
  return LV_OK;
}

size_t litevggt_global_block_ws_bytes(const litevggt_params *p, int64_t n_tokens) {
  Dims d;
  if (check_params(p, &d) || n_tokens < 1) return 0;
  return block_ws_bytes(n_tokens, d.C, d.heads, p->attn_dtype);
}

int litevggt_global_block(const litevggt_params *p, int64_t n_tokens, const void *z,
                          const litevggt_block_weights *weights, void *delta, void *ws,
                          size_t ws_bytes, void *stream) {
  Dims d;
  int rc = check_params(p, &d);
  if (rc) return rc;
  if (!z || !delta) return LV_ERR_NULL;
  if ((rc = check_block_weights(weights))) return rc;
  if (n_tokens < 1 || n_tokens >= ((int64_t)1 << 31) || d.C % 256 != 0) return LV_ERR_SHAPE;
  if (!ws_ok(ws, ws_bytes, block_ws_bytes(n_tokens, d.C, d.heads, p->attn_dtype))) return LV_ERR_WORKSPACE;
  return launch_global_block((const uint16_t *)z, n_tokens, d.C, d.heads, scale_of(p), p->attn_dtype,
                             p->qk_norm, *weights, (uint16_t *)delta, ws, (hipStream_t)stream);
}

size_t litevggt_frame_attn_ws_bytes(const litevggt_params *p) {
  Dims d;
  if (check_params(p, &d)) return 0;
  return attn_ws_bytes(d.heads, d.T, LV_ATTN_BF16, d.F);
}

int litevggt_frame_attn(const litevggt_params *p, const void *q, const void *k, const void *v,
                        const void *residual, void *o, void *ws, size_t ws_bytes, void *stream) {
  Dims d;
  int rc = check_params(p, &d);
  if (rc) return rc;
  if (!q || !k || !v || !o) return LV_ERR_NULL;
  if (!ws_ok(ws, ws_bytes, attn_ws_bytes(d.heads, d.T, LV_ATTN_BF16, d.F))) return LV_ERR_WORKSPACE;
  return launch_attn((const uint16_t *)q, (const uint16_t *)k, (const uint16_t *)v, (uint16_t *)o,
                     d.T, d.heads, scale_of(p), LV_ATTN_BF16, p->qk_norm, ws, (hipStream_t)stream,
                     nullptr, d.F, (const uint16_t *)residual);
}

int litevggt_unmerge(const litevggt_params *p, const void *y, const litevggt_index *index,
                     const void *residual, void *out, void *stream) {
  Dims d;
  int rc = check_params(p, &d);
  if (rc) return rc;
  if (!y || !out || !index || !index->slot_of) return LV_ERR_NULL;
  return launch_unmerge((const uint16_t *)y, d, *index, (const uint16_t *)residual, (uint16_t *)out,
                        (hipStream_t)stream);
}

int litevggt_layers_run(const litevggt_params *p, int n_layers, const void *images, void *x,
                        litevggt_index *index, float *grad_cache, float *score,
                        int32_t *refresh_log, void **events, void *ws, size_t ws_bytes,
                        void *stream) {
  Dims d;
  litevggt_plan_t pl;
  int rc = check_params(p, &d);
  if (rc) return rc;
  rc = make_plan(p, d, &pl);
  if (rc) return rc;
  if (n_layers < 0) return LV_ERR_PARAM;
  const bool ga = p->anchor_policy == LV_POLICY_GA;   // the other policies read no image, cache no map
  if (!x || !score || !index_ok(index) || (ga && (!images || !grad_cache))) return LV_ERR_NULL;
  if (d.C > 1024) return LV_ERR_SHAPE;
  if (p->block) {
    if (d.C % 256 != 0) return LV_ERR_SHAPE;
    if ((rc = check_block_weights(p->block))) return rc;
  }
  if (!ws_ok(ws, ws_bytes, driver_ws_bytes(p, d, pl))) return LV_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const size_t zy = align_up((size_t)pl.M * d.C * 2, 256);
  uint16_t *z = (uint16_t *)ws;
  uint16_t *y = (uint16_t *)((char *)ws + zy);
  void *wpack = (char *)ws + 2 * zy;   // block only: the weights in operand order, written by the first layer
  void *op_ws = (char *)wpack + (p->block ? block_wpack_bytes(d.C) : 0);
  uint16_t *xx = (uint16_t *)x;
  for (int l = 0; l < n_layers; ++l) {
    const bool refresh = (l % p->refresh_interval) == 0;
    if (refresh_log) refresh_log[l] = refresh ? 1 : 0;
    hipEvent_t *ev = events ? (hipEvent_t *)events + (size_t)l * LV_EVENTS_PER_LAYER : nullptr;
    auto mark = [&](int which) -> int {
      if (ev && hipEventRecord(ev[which], st) != hipSuccess) return LV_ERR_HIP;
      return LV_OK;
    };
    if ((rc = mark(LV_EV_LAYER_BEGIN))) return rc;
    if (refresh && ga) {
      if (l == 0) {
        rc = launch_grad_map(images, p->img_dtype, d, p->patch, grad_cache, st);
        if (rc) return rc;
      }
      rc = launch_var_map(xx, d, p->var_pool, (float *)op_ws, st);
      if (rc) return rc;
      rc = launch_ga_fuse(grad_cache, (const float *)op_ws, d, p->alpha, p->beta, score, st);
      if (rc) return rc;
    } else if (refresh) {
      rc = launch_naive_score(d, p->anchor_policy, p->policy_seed, score, st);
      if (rc) return rc;
    }
    if ((rc = mark(LV_EV_IMPORTANCE_END))) return rc;
    if (refresh) {
      rc = launch_select(score, d, pl, *index, st);
      if (rc) return rc;
    }
    if ((rc = mark(LV_EV_SELECT_END))) return rc;
    if (refresh) {
      rc = launch_match(xx, d, pl, *index, nullptr, op_ws, st);
      if (rc) return rc;
    }
    if ((rc = mark(LV_EV_MATCH_END))) return rc;
    rc = launch_merge(xx, d, pl.M, *index, z, st);
    if (rc) return rc;
    if ((rc = mark(LV_EV_MERGE_END))) return rc;
    if (p->block) {
      rc = launch_global_block(z, pl.M, d.C, d.heads, scale_of(p), p->attn_dtype, p->qk_norm,
                               *p->block, y, op_ws, st, ev ? ev[LV_EV_ATTN_PACK_END] : nullptr,
                               ev ? ev[LV_EV_ATTN_END] : nullptr, wpack, l > 0);
      if (rc) return rc;
    } else {
      rc = launch_attn(z, z, z, y, pl.M, d.heads, scale_of(p), p->attn_dtype, p->qk_norm, op_ws, st,
                       ev ? ev[LV_EV_ATTN_PACK_END] : nullptr);
      if (rc) return rc;
      if ((rc = mark(LV_EV_ATTN_END))) return rc;
    }
    if ((rc = mark(LV_EV_BLOCK_END))) return rc;
    rc = launch_unmerge(y, d, *index, xx, xx, st);
    if (rc) return rc;
    if ((rc = mark(LV_EV_UNMERGE_END))) return rc;
    if (p->frame_attn) {
      rc = launch_attn(xx, xx, xx, xx, d.T, d.heads, scale_of(p), LV_ATTN_BF16, p->qk_norm, op_ws,
                       st, nullptr, d.F, xx);
      if (rc) return rc;
    }
    if ((rc = mark(LV_EV_FRAME_ATTN_END))) return rc;
  }
  return LV_OK;
}

}  // extern "C"
