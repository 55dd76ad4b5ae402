/*
 * litevggt.h -- C ABI of the MI355X (gfx950) implementation of LiteVGGT's hot path:
 * geometry-aware cached token merging wrapped around VGGT's frame-global
 * self-attention (LiteVGGT, arXiv 2512.04939, Sec. 3.4).
 *
 * Conventions (every entry point):
 *   - returns 0 (LV_OK) or a negative LV_ERR_* code; litevggt_strerror() names it.
 *     Arguments are validated on the host before anything is launched: on an argument
 *     error (every code but LV_ERR_HIP) nothing has been enqueued.  LV_ERR_HIP reports a
 *     failed launch or event record; work enqueued before it stays enqueued.
 *   - pointers marked [device] are device memory owned by the caller; the library
 *     never allocates, frees or keeps them.  Pointers marked [host] are host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls only
 *     enqueue work; they never synchronise.  Kernel faults surface at the caller's
 *     next synchronisation.
 *   - token order: frame-major; inside a frame the n_special camera/register tokens
 *     come first, then the grid_h*grid_w patch tokens row-major.  N = frames*(P+S).
 *   - features are bf16 (raw 16-bit patterns), row-major [tokens, dim], rows 16-byte
 *     aligned; indices are int32; scores are fp32.
 *   - inputs are never written; outputs must not overlap inputs unless stated.
 *   - `ws` is scratch device memory of at least the size the matching *_ws_bytes /
 *     litevggt_plan reports, 256-byte aligned; its contents are undefined afterwards.
 */
#ifndef LITEVGGT_H
#define LITEVGGT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  LV_OK = 0,
  LV_ERR_NULL = -1,       /* a required pointer is NULL                          */
  LV_ERR_SHAPE = -2,      /* sizes inconsistent or unsupported                    */
  LV_ERR_PARAM = -3,      /* hyper-parameter out of range                         */
  LV_ERR_WORKSPACE = -4,  /* ws too small or misaligned                           */
  LV_ERR_DTYPE = -5,      /* unsupported dtype selector                           */
  LV_ERR_HIP = -6         /* a HIP runtime call failed (launch error)             */
};

enum { LV_IMG_F32 = 0, LV_IMG_U8 = 1 };        /* image element type              */
enum { LV_ATTN_BF16 = 0, LV_ATTN_FP8_E4M3 = 1 }; /* attention MFMA operand type   */
enum { LV_ROLE_PROTECTED = 0, LV_ROLE_DST = 1, LV_ROLE_SRC = 2 };
enum { LV_POLICY_GA = 0, LV_POLICY_FIXED = 1, LV_POLICY_RANDOM = 2 }; /* what ranks the tokens */
enum { LV_LINEAR_BF16 = 0, LV_LINEAR_FP8_E4M3 = 1 }; /* MFMA operand type of the block's linear layers */
enum { LV_FP8_CURRENT = 0, LV_FP8_DELAYED = 1 };     /* where a quantised input's scale comes from */

/* Delayed scaling (supplementary "FP8 Quantization Details": E4M3, delayed scaling, amax
 * history of 80 steps reduced with max): per quantised input, the last 80 amaxes and a step
 * counter.  One state block covers the four linear layers of a transformer block. */
#define LV_FP8_HISTORY 80
#define LV_FP8_STATE_BYTES (4 * (LV_FP8_HISTORY + 2) * 4)

/* Weights of the transformer block around the global attention (litevggt_global_block):
 * device pointers, matrices bf16 row-major [out features, in features], vectors fp32. */
typedef struct {
  const float *ln1_g, *ln1_b;   /* [dim]  LayerNorm before the attention                  */
  const void  *w_qkv;           /* [3 dim, dim]: rows 0..dim-1 give q, then k, then v     */
  const float *b_qkv;           /* [3 dim]                                                */
  const void  *w_o;             /* [dim, dim]   output projection                         */
  const float *b_o;             /* [dim]                                                  */
  const float *ln2_g, *ln2_b;   /* [dim]  LayerNorm before the MLP                        */
  const void  *w_1;             /* [4 dim, dim] */
  const float *b_1;             /* [4 dim]      */
  const void  *w_2;             /* [dim, 4 dim] */
  const float *b_2;             /* [dim]        */
  int32_t linear_dtype;         /* LV_LINEAR_BF16, or LV_LINEAR_FP8_E4M3: the four linear layers
                                   quantise their input and their weight per tensor to E4M3
                                   (code = RNE(value * (448 / amax)), saturating, products
                                   accumulated in fp32 and rescaled); bias, activation and
                                   every stored intermediate stay as in the bf16 block        */
  int32_t fp8_recipe;           /* scale of a linear layer's input: LV_FP8_CURRENT takes amax
                                   from the tensor being quantised; LV_FP8_DELAYED from the
                                   largest amax of the previous (up to) 80 uses of that layer,
                                   scale 1 before the first use, and records the tensor's own
                                   amax afterwards.  Weights always use their own amax.      */
  void *fp8_state;              /* [device] LV_FP8_STATE_BYTES, read and written by every
                                   call with LV_FP8_DELAYED: per layer (qkv, out-proj, fc1,
                                   fc2) 80 fp32 amaxes, a uint32 step counter and a pad word.
                                   The caller zero-fills it once; may be NULL otherwise.      */
} litevggt_block_weights;

/* Shape and hyper-parameters (host memory). */
typedef struct {
  int32_t frames;          /* F                                                    */
  int32_t grid_h, grid_w;  /* patch grid; P = grid_h*grid_w                        */
  int32_t n_special;       /* camera + register tokens per frame (Sec. 3.1: 5)     */
  int32_t dim;             /* C = heads*head_dim, multiple of 64                   */
  int32_t heads;
  int32_t head_dim;        /* must be 64                                           */
  int32_t patch;           /* pixels per patch side (14); image = grid*patch       */
  int32_t img_dtype;       /* LV_IMG_F32 ([0,1]) or LV_IMG_U8 ([0,255])            */
  int32_t var_pool;        /* window of the local variance pooling (3), odd        */
  int32_t refresh_interval;/* layers between merge-index recomputations (6)        */
  int32_t attn_dtype;      /* LV_ATTN_BF16 or LV_ATTN_FP8_E4M3                     */
  int32_t qk_norm;         /* != 0: attention RMS-normalises q and k per head first:
                              q <- bf16(q / sqrt(mean(q^2) + 1e-6)), same for k      */
  float   alpha, beta;     /* weights of the gradient and variance maps            */
  float   softmax_scale;   /* <= 0 selects 1/sqrt(head_dim)                        */
  double  merge_ratio;     /* r in [0,1): fraction of patch tokens per non-first
                              frame that become src; < 0 selects the paper's fixed
                              rule (top ga_frac GA tokens, one dst per 2x2 cell)   */
  double  ga_frac;         /* 0.10; used only when merge_ratio < 0                 */
  int32_t anchor_policy;   /* LV_POLICY_GA, or one of the geometry-blind partitions
                              of Sec. 3.2 (see litevggt_importance)                  */
  uint32_t policy_seed;    /* seed of LV_POLICY_RANDOM                              */
  int32_t frame_attn;      /* != 0: the layer driver runs a frame attention after every
                              global layer (see litevggt_frame_attn)                */
  const litevggt_block_weights *block; /* [host] NULL: the layer driver's global layer is the
                              projection-free attention; else it is litevggt_global_block
                              with these weights (the same in every layer)          */
} litevggt_params;

/* Token counts that follow from the parameters (closed form, Sec. 3.4 partition). */
typedef struct {
  int64_t N;               /* tokens in the sequence                               */
  int64_t M;               /* tokens after merging                                 */
  int64_t n_dst, n_src;    /* totals over all frames                               */
  int32_t cell;            /* side of the grid cell that yields one dst token      */
  int32_t n_dst_per_frame, n_ga_per_frame, n_src_per_frame; /* frames 1..F-1       */
  size_t  ws_bytes;        /* scratch that covers every call below at these sizes
                              with n_tokens <= M for litevggt_global_attn          */
} litevggt_plan_t;

/* The cached merge index: caller-owned device buffers, filled by
 * litevggt_select_anchors (role, kept_idx, dst_idx, src_idx, and the entries of
 * anchor_of/slot_of that belong to kept tokens) and litevggt_match (the rest). */
typedef struct {
  uint8_t *role;           /* [N]   LV_ROLE_*                                      */
  int32_t *kept_idx;       /* [M]   token index of merged slot m, ascending        */
  int32_t *dst_idx;        /* [n_dst] ascending                                    */
  int32_t *src_idx;        /* [n_src] ascending                                    */
  int32_t *anchor_of;      /* [N]   token index of the token's anchor (self if kept)*/
  int32_t *slot_of;        /* [N]   merged slot of the token's anchor              */
  int32_t *group_off;      /* [M+1] CSR offsets into group_mem                     */
  int32_t *group_mem;      /* [N]   members of each slot, ascending inside a slot  */
} litevggt_index;

const char *litevggt_strerror(int code);

/* Host only.  Validates the parameters and fills the closed-form counts. */
int litevggt_plan(const litevggt_params *p, litevggt_plan_t *out /*[host]*/);

/* Scratch needed by litevggt_global_attn for a sequence of n_tokens (host only). */
size_t litevggt_attn_ws_bytes(const litevggt_params *p, int64_t n_tokens);

/* Step 1, Sec. 3.4 "Geometry-aware Feature Map": score = alpha*norm(Psi_g) +
 * beta*norm(Psi_v).  Psi_g = Sobel gradient magnitude of the luma image (3x3
 * kernels, replicated border) averaged over each patch; Psi_v = variance of the
 * patch tokens over a var_pool x var_pool grid neighbourhood (clipped at the grid
 * border), averaged over channels; norm = per-frame min-max (a flat map -> 0).
 * With anchor_policy != LV_POLICY_GA the score carries no geometry (Sec. 3.2 "Naive
 * Token Merging": dst/src sets from a fixed pattern or from random sampling) and images,
 * x, grad_cache are not read and may be NULL:
 *   LV_POLICY_FIXED   score[f][p] = ((p+1) * 2654435769 mod 2^32) >> 8, / 2^24: the same
 *                     low-discrepancy pattern in every frame
 *   LV_POLICY_RANDOM  score[f][p] = fmix32(policy_seed ^ f*0x9E3779B9 ^ p*0x85EBCA6B) >> 8,
 *                     / 2^24, fmix32 = the 32-bit finaliser of MurmurHash3
 * The partition rule of litevggt_select_anchors is the same for every policy.
 *   images     [device] [F,3,grid_h*patch,grid_w*patch] img_dtype; may be NULL when
 *              recompute_grad == 0
 *   x          [device] [N,dim] bf16 tokens entering the layer
 *   grad_cache [device] [F,P] fp32, written when recompute_grad != 0, else read
 *   score      [device] [F,P] fp32 out
 */
int litevggt_importance(const litevggt_params *p, const void *images, const void *x,
                        float *grad_cache, int recompute_grad, float *score,
                        void *ws, size_t ws_bytes, void *stream);

/* litevggt_importance for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels and the same results, but the variance map that litevggt_importance keeps in `ws` lives
 * in a device array inside the library (LV_STATIC_SCORE_MAX fp32 = 8 MiB, held on every GPU the
 * library runs on until the process ends).  The call allocates and frees nothing.
 *   frames * grid_h * grid_w > LV_STATIC_SCORE_MAX -> LV_ERR_WORKSPACE, nothing enqueued.
 *   All calls on one GPU share that array: calls that overlap on one GPU (different streams,
 *   or threads) race; calls on one stream are ordered.  Nothing in it has to start at zero
 *   (every element that is read was written earlier in the same call).
 * Other arguments as for litevggt_importance.
 */
#define LV_STATIC_SCORE_MAX (2u * 1024u * 1024u)
int litevggt_importance_static(const litevggt_params *p, const void *images, const void *x,
                               float *grad_cache, int recompute_grad, float *score, void *stream);

/* Step 2, Sec. 3.4 "GA Token Partitioning".  Special tokens: PROTECTED.  Frame 0:
 * every patch token DST.  Other frames: in every cell x cell block of the grid the
 * lowest-scoring token is DST (ties: lowest index); of the remaining patch tokens
 * the n_ga_per_frame highest-scoring are PROTECTED GA tokens (ties: lowest index);
 * the rest are SRC.  Scores are compared as fp32 (-0 == +0); NaN scores give an
 * unspecified but valid partition.  Writes role, kept_idx, dst_idx, src_idx and,
 * for kept tokens, anchor_of[i] = i and slot_of[i] = position in kept_idx.
 *   score [device] [F,P] fp32
 */
int litevggt_select_anchors(const litevggt_params *p, const float *score,
                            litevggt_index *index, void *stream);

/* Step 3, Sec. 3.4 "Cached Token Merging": every SRC token is assigned the DST token
 * (of any frame) with the largest cosine similarity of the full dim-vectors; the
 * decision is taken on fp32 similarities, ties go to the lowest token index.
 * Fills anchor_of/slot_of for SRC tokens and builds group_off/group_mem.
 * Requires the outputs of litevggt_select_anchors in `index`.
 *   best_sim [device] [n_src] fp32 similarity of each src (order of src_idx), or NULL
 */
int litevggt_match(const litevggt_params *p, const void *x, litevggt_index *index,
                   float *best_sim, void *ws, size_t ws_bytes, void *stream);

/* Step 4, Sec. 3.4 merge equation: z[m] = mean of x over the members of slot m
 * (fp32 sum in ascending token order, one rounding to bf16).
 *   x [device] [N,dim] bf16;  z [device] [M,dim] bf16 out
 */
int litevggt_merge(const litevggt_params *p, const void *x, const litevggt_index *index,
                   void *z, void *stream);

/* Step 5, Sec. 3.1 "Bottleneck Analysis": unmasked self-attention over the whole
 * sequence, per head: O = softmax(Q K^T * softmax_scale) V.
 *   q,k,v [device] [n_tokens, heads, 64] bf16 (row stride dim); o likewise, out.
 *   n_tokens = M for the merged path, N for the unmerged baseline.
 * With qk_norm the scores use the per-head RMS-normalised q and k (see litevggt_params);
 * v is used as given.  Normalised q and k whose scaled scores cannot leave the exponent range
 * need no softmax reference at all; otherwise (q and k as given, or a large softmax_scale) the
 * softmax is computed online: a running reference per wave of 64 queries, raised when a row sum
 * shows that a score went far above it, with a running maximum per query row for the query
 * blocks where rows lie more than 60 binades apart or scores exceed 256 in log2 units.
 * Exponents are always taken from the difference to the reference, so scores of any finite
 * size give finite weights.
 * attn_dtype LV_ATTN_FP8_E4M3 quantises q,k,v per tensor (scale = amax/448, amax taken in
 * this call) and the softmax weights to e4m3 for the MFMAs; accumulation and softmax stay
 * fp32.  Without qk_norm the weights are rounded relative to a running row maximum and
 * normalised by their fp32 sum.  With qk_norm they are rounded relative to the largest score
 * unit-RMS heads can reach and normalised by the sum of the e4m3 weights themselves (they
 * sum to one exactly), and q's scale may be up to 2x smaller than 448/amax; rows whose
 * scores all lie more than 8.75 binades below that bound are recomputed the first way.
 */
int litevggt_global_attn(const litevggt_params *p, int64_t n_tokens, const void *q,
                         const void *k, const void *v, void *o,
                         void *ws, size_t ws_bytes, void *stream);

/* Step 6, Sec. 3.4 "Token Unmerging": out[i] = y[slot_of[i]] (+ residual[i]).
 *   y [device] [M,dim] bf16; residual [device] [N,dim] bf16 or NULL;
 *   out [device] [N,dim] bf16, may be the same buffer as residual.
 */
int litevggt_unmerge(const litevggt_params *p, const void *y, const litevggt_index *index,
                     const void *residual, void *out, void *stream);

/* The transformer block around the global attention core, on a sequence of n_tokens
 * (Sec. 3.1: the aggregator's global layers are pre-norm attention + MLP blocks; the paper
 * does not restate them, so this is the plain block, with caller-supplied weights):
 *   h = LN(z; ln1)                q|k|v = h w_qkv^T + b_qkv       (LN eps 1e-6)
 *   a = attention(q, k, v)        as litevggt_global_attn (attn_dtype, qk_norm, softmax_scale)
 *   u1 = a w_o^T + b_o            h2 = LN(z + u1; ln2)
 *   u2 = GELU(h2 w_1^T + b_1) w_2^T + b_2     (GELU with erf)
 *   delta = u1 + u2               the block's output is z + delta
 * Every intermediate (h, q, k, v, a, u1, h2, the MLP hidden layer, u2) is stored as bf16;
 * accumulation is fp32.  dim must be a multiple of 256.  weights->linear_dtype selects FP8
 * E4M3 operands for the four linear layers (see litevggt_block_weights).
 *   z      [device] [n_tokens, dim] bf16
 *   delta  [device] [n_tokens, dim] bf16 out
 *   ws     litevggt_global_block_ws_bytes(p, n_tokens) bytes
 */
size_t litevggt_global_block_ws_bytes(const litevggt_params *p, int64_t n_tokens);
int litevggt_global_block(const litevggt_params *p, int64_t n_tokens, const void *z,
                          const litevggt_block_weights *weights /*[host]*/, void *delta, void *ws,
                          size_t ws_bytes, void *stream);

/* Frame attention, Sec. 3.1 (VGGT alternates frame-wise and global self-attention; Sec. 3.4
 * "Token Unmerging": the unmerged tokens go to the next frame attention): for every frame f
 * separately, O_f = softmax(Q_f K_f^T * softmax_scale) V_f over that frame's own P + n_special
 * tokens, all heads; q and k RMS-normalised per head first when qk_norm is set.  Always
 * computed with bf16 MFMAs (attn_dtype is ignored).
 *   q, k, v   [device] [N,dim] bf16
 *   residual  [device] [N,dim] bf16 or NULL; when given, o = residual + O with one rounding.
 *             residual may be the same buffer as o (and as q, k, v): K and V are re-laid out
 *             into ws before any output is written and every query row is read by the
 *             workgroup that writes it.
 *   o         [device] [N,dim] bf16 out
 *   ws        litevggt_frame_attn_ws_bytes(p) bytes
 */
size_t litevggt_frame_attn_ws_bytes(const litevggt_params *p);
int litevggt_frame_attn(const litevggt_params *p, const void *q, const void *k, const void *v,
                        const void *residual, void *o, void *ws, size_t ws_bytes, void *stream);

/* Cached-index layer driver, Sec. 3.4: for layer l = 0..n_layers-1, recompute the
 * merge index (steps 1-3; the gradient map only at l = 0) when
 * l % refresh_interval == 0, then x <- x + unmerge(attn(merge(x))) with
 * Q = K = V = the merged tokens viewed as [M, heads, 64] (q, k normalised when qk_norm),
 * or, when p->block is set, x <- x + unmerge(delta of litevggt_global_block(merge(x))),
 * which at merge ratio 0 is the block applied to the unmerged sequence,
 * then, when frame_attn is set, x <- x + frame_attn(x) with Q = K = V = x.
 *   x           [device] [N,dim] bf16, in/out
 *   images      [device] as for litevggt_importance; with anchor_policy != LV_POLICY_GA
 *               images and grad_cache are not read and may be NULL
 *   grad_cache, score [device] [F,P] fp32 scratch/outputs of the last refresh
 *   refresh_log [host] [n_layers] set to 1 where the index was recomputed, or NULL
 *   events      [host] NULL, or LV_EVENTS_PER_LAYER*n_layers hipEvent_t handles (as
 *               void*) created by the caller; the driver records them on `stream` at the
 *               step boundaries of every layer (LV_EV_* below) so the caller can time each
 *               step inside a run.  On layers without a refresh the first four boundaries
 *               are recorded back to back.
 */
enum {
  LV_EV_LAYER_BEGIN = 0,   /* before importance                                    */
  LV_EV_IMPORTANCE_END,    /* after the GA map, before the partition               */
  LV_EV_SELECT_END,        /* after the partition, before matching                 */
  LV_EV_MATCH_END,         /* after matching + CSR, before merge                   */
  LV_EV_MERGE_END,         /* after merge, before the K/V re-layout of attention   */
  LV_EV_ATTN_PACK_END,     /* after the re-layout, before the attention kernel     */
  LV_EV_ATTN_END,          /* after the attention kernel                           */
  LV_EV_BLOCK_END,         /* after the rest of the block (if any), before unmerge */
  LV_EV_UNMERGE_END,       /* after unmerge, before the frame attention (if any)   */
  LV_EV_FRAME_ATTN_END,    /* after the frame attention                            */
  LV_EVENTS_PER_LAYER
};
int litevggt_layers_run(const litevggt_params *p, int n_layers, const void *images,
                        void *x, litevggt_index *index, float *grad_cache, float *score,
                        int32_t *refresh_log, void **events, void *ws, size_t ws_bytes,
                        void *stream);

/* ---------------------------------------------------------------------------------------
 * Measurement aids (no part of the method): what this GPU sustains on the two resources the
 * kernels' rooflines are quoted against, with nothing else in the way.  A benchmark runs them
 * next to the hot path and times them with events on `stream`.
 *
 * litevggt_probe_mfma: 2048 workgroups of 8 waves, each wave `iters` times 8 independent
 *   32x32 MFMAs (dtype LV_ATTN_BF16: 32x32x16 bf16; LV_ATTN_FP8_E4M3: 32x32x64 E4M3) on operands
 *   it loads once.  litevggt_probe_mfma_flop returns the flop of one such call (0 for bad
 *   arguments).
 *     operands [device] 128 KiB of operand bits (any finite bf16 / E4M3 values), read only
 *     out      [device] 2048*512 fp32, written (keeps the result alive; no meaning)
 *   errors: NULL -> LV_ERR_NULL, iters outside 1 .. 2^20 -> LV_ERR_SHAPE, other dtype ->
 *   LV_ERR_DTYPE.
 * litevggt_probe_stream: dst != NULL: copies `bytes` from src to dst (bytes read + bytes
 *   written = 2*bytes of HBM traffic); dst == NULL: reads src only.  16 B per lane and access.
 *     src, dst [device] 16-byte aligned, bytes a positive multiple of 16; sink [device] 4 bytes
 * litevggt_probe_gather: reads n_rows whole rows of row_bytes each, row order[i] of src at step i,
 *   one row per wave, eight in flight: what HBM gives the merge step's access pattern (token rows
 *   gathered through an index), with nothing written.
 *     src [device] 16-byte aligned; row_bytes a multiple of 16, at most 2^20; order [device]
 *     n_rows int32 row numbers, every one inside src (the caller's responsibility); sink as above
 */
double litevggt_probe_mfma_flop(int dtype, int iters);
int litevggt_probe_mfma(int dtype, const void *operands, int iters, float *out, void *stream);
int litevggt_probe_stream(const void *src, void *dst, size_t bytes, void *sink, void *stream);
int litevggt_probe_gather(const void *src, size_t row_bytes, const int32_t *order, int64_t n_rows,
                          void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LITEVGGT_H */
