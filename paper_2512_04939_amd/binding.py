"""ctypes binding of liblitevggt.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/litevggt.h) and passes
torch tensors' device pointers and the current HIP stream.  There is no CPU fallback: a
missing library raises at import of the symbols, a failing call raises ``LiteVGGTError``.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liblitevggt.so")

IMG_F32, IMG_U8 = 0, 1
ATTN_BF16, ATTN_FP8_E4M3 = 0, 1
POLICY_GA, POLICY_FIXED, POLICY_RANDOM = 0, 1, 2
LINEAR_BF16, LINEAR_FP8_E4M3 = 0, 1
FP8_CURRENT, FP8_DELAYED = 0, 1
FP8_HISTORY = 80
FP8_STATE_BYTES = 4 * (FP8_HISTORY + 2) * 4
ROLE_PROTECTED, ROLE_DST, ROLE_SRC = 0, 1, 2

STATIC_SCORE_MAX = 2 * 1024 * 1024
EXPORTS = ["litevggt_strerror", "litevggt_plan", "litevggt_attn_ws_bytes", "litevggt_importance",
           "litevggt_importance_static",
           "litevggt_select_anchors", "litevggt_match", "litevggt_merge", "litevggt_global_attn",
           "litevggt_unmerge", "litevggt_frame_attn_ws_bytes", "litevggt_frame_attn",
           "litevggt_global_block_ws_bytes", "litevggt_global_block",
           "litevggt_layers_run", "litevggt_probe_mfma", "litevggt_probe_stream",
           "litevggt_probe_mfma_flop", "litevggt_probe_gather"]


class LiteVGGTError(RuntimeError):
    pass


class BlockWeights(C.Structure):
    """Mirror of ``litevggt_block_weights`` (device pointers)."""
    _fields_ = [(n, C.c_void_p) for n in ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g",
                                          "ln2_b", "w_1", "b_1", "w_2", "b_2")] + [
        ("linear_dtype", C.c_int32), ("fp8_recipe", C.c_int32), ("fp8_state", C.c_void_p)]


class Params(C.Structure):
    """Mirror of ``litevggt_params``."""
    _fields_ = [("frames", C.c_int32), ("grid_h", C.c_int32), ("grid_w", C.c_int32),
                ("n_special", C.c_int32), ("dim", C.c_int32), ("heads", C.c_int32),
                ("head_dim", C.c_int32), ("patch", C.c_int32), ("img_dtype", C.c_int32),
                ("var_pool", C.c_int32), ("refresh_interval", C.c_int32),
                ("attn_dtype", C.c_int32), ("qk_norm", C.c_int32), ("alpha", C.c_float), ("beta", C.c_float),
                ("softmax_scale", C.c_float), ("merge_ratio", C.c_double),
                ("ga_frac", C.c_double), ("anchor_policy", C.c_int32), ("policy_seed", C.c_uint32),
                ("frame_attn", C.c_int32), ("block", C.POINTER(BlockWeights))]


class Plan(C.Structure):
    """Mirror of ``litevggt_plan_t``."""
    _fields_ = [("N", C.c_int64), ("M", C.c_int64), ("n_dst", C.c_int64), ("n_src", C.c_int64),
                ("cell", C.c_int32), ("n_dst_per_frame", C.c_int32),
                ("n_ga_per_frame", C.c_int32), ("n_src_per_frame", C.c_int32),
                ("ws_bytes", C.c_size_t)]


class Index(C.Structure):
    """Mirror of ``litevggt_index`` (device pointers)."""
    _fields_ = [("role", C.c_void_p), ("kept_idx", C.c_void_p), ("dst_idx", C.c_void_p),
                ("src_idx", C.c_void_p), ("anchor_of", C.c_void_p), ("slot_of", C.c_void_p),
                ("group_off", C.c_void_p), ("group_mem", C.c_void_p)]


def make_params(frames, grid_h, grid_w, dim, heads, *, head_dim=64, n_special=5, patch=14,
                img_dtype=IMG_F32, var_pool=3, refresh_interval=6, attn_dtype=ATTN_BF16,
                qk_norm=0, alpha=0.5, beta=0.5, softmax_scale=0.0, merge_ratio=0.9, ga_frac=0.10,
                anchor_policy=POLICY_GA, policy_seed=0, frame_attn=0, block=None) -> Params:
    """``block``: a BlockWeights the caller keeps alive, or None."""
    return Params(frames, grid_h, grid_w, n_special, dim, heads, head_dim, patch, img_dtype,
                  var_pool, refresh_interval, attn_dtype, qk_norm, alpha, beta, softmax_scale,
                  merge_ratio, ga_frac, anchor_policy, policy_seed, frame_attn,
                  C.pointer(block) if block is not None else None)


_lib = None


def lib() -> C.CDLL:
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise LiteVGGTError(f"{LIB_PATH} not found: run paper_2512_04939_amd/build.py "
                                "(or __graft_entry__.build()) first; there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, sz, i32, i64 = C.c_void_p, C.c_size_t, C.c_int, C.c_int64
        PP = C.POINTER(Params)
        L.litevggt_strerror.restype = C.c_char_p
        L.litevggt_strerror.argtypes = [i32]
        L.litevggt_plan.argtypes = [PP, C.POINTER(Plan)]
        L.litevggt_attn_ws_bytes.restype = sz
        L.litevggt_attn_ws_bytes.argtypes = [PP, i64]
        L.litevggt_importance.argtypes = [PP, vp, vp, vp, i32, vp, vp, sz, vp]
        L.litevggt_importance_static.argtypes = [PP, vp, vp, vp, i32, vp, vp]
        L.litevggt_select_anchors.argtypes = [PP, vp, C.POINTER(Index), vp]
        L.litevggt_match.argtypes = [PP, vp, C.POINTER(Index), vp, vp, sz, vp]
        L.litevggt_merge.argtypes = [PP, vp, C.POINTER(Index), vp, vp]
        L.litevggt_global_attn.argtypes = [PP, i64, vp, vp, vp, vp, vp, sz, vp]
        L.litevggt_unmerge.argtypes = [PP, vp, C.POINTER(Index), vp, vp, vp]
        L.litevggt_global_block_ws_bytes.restype = sz
        L.litevggt_global_block_ws_bytes.argtypes = [PP, i64]
        L.litevggt_global_block.argtypes = [PP, i64, vp, C.POINTER(BlockWeights), vp, vp, sz, vp]
        L.litevggt_frame_attn_ws_bytes.restype = sz
        L.litevggt_frame_attn_ws_bytes.argtypes = [PP]
        L.litevggt_frame_attn.argtypes = [PP, vp, vp, vp, vp, vp, vp, sz, vp]
        L.litevggt_layers_run.argtypes = [PP, i32, vp, vp, C.POINTER(Index), vp, vp,
                                          C.POINTER(C.c_int32), C.POINTER(C.c_void_p), vp, sz, vp]
        L.litevggt_probe_mfma.argtypes = [i32, vp, i32, vp, vp]
        L.litevggt_probe_stream.argtypes = [vp, vp, sz, vp, vp]
        L.litevggt_probe_mfma_flop.argtypes = [i32, i32]
        L.litevggt_probe_gather.argtypes = [vp, sz, vp, i64, vp, vp]
        for name in EXPORTS[1:]:
            if not name.endswith("_ws_bytes"):
                getattr(L, name).restype = i32
        L.litevggt_probe_mfma_flop.restype = C.c_double
        _lib = L
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise LiteVGGTError(f"{what} failed: {lib().litevggt_strerror(rc).decode()} ({rc})")


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def litevggt_strerror(code: int) -> str:
    return lib().litevggt_strerror(code).decode()


def litevggt_plan(p: Params) -> Plan:
    out = Plan()
    _check(lib().litevggt_plan(C.byref(p), C.byref(out)), "litevggt_plan")
    return out


def litevggt_attn_ws_bytes(p: Params, n_tokens: int) -> int:
    return int(lib().litevggt_attn_ws_bytes(C.byref(p), n_tokens))


@dataclass
class IndexBuffers:
    """Device tensors backing a ``litevggt_index`` (allocated by torch, owned by the caller)."""
    role: "object"
    kept_idx: "object"
    dst_idx: "object"
    src_idx: "object"
    anchor_of: "object"
    slot_of: "object"
    group_off: "object"
    group_mem: "object"

    def struct(self) -> Index:
        return Index(*(t.data_ptr() for t in (self.role, self.kept_idx, self.dst_idx, self.src_idx,
                                              self.anchor_of, self.slot_of, self.group_off,
                                              self.group_mem)))


def alloc_index(pl: Plan, device="cuda") -> IndexBuffers:
    import torch
    i32 = dict(dtype=torch.int32, device=device)
    return IndexBuffers(
        role=torch.empty(pl.N, dtype=torch.uint8, device=device),
        kept_idx=torch.empty(pl.M, **i32), dst_idx=torch.empty(max(pl.n_dst, 1), **i32),
        src_idx=torch.empty(max(pl.n_src, 1), **i32), anchor_of=torch.empty(pl.N, **i32),
        slot_of=torch.empty(pl.N, **i32), group_off=torch.empty(pl.M + 1, **i32),
        group_mem=torch.empty(pl.N, **i32))


def alloc_ws(nbytes: int, device="cuda"):
    import torch
    return torch.empty(max(int(nbytes), 256) + 256, dtype=torch.uint8, device=device)


def _ws_args(ws):
    """256-byte aligned pointer and usable size of a uint8 workspace tensor."""
    if ws is None:
        return None, 0
    base = ws.data_ptr()
    aligned = (base + 255) // 256 * 256
    return aligned, ws.numel() - (aligned - base)


def litevggt_importance(p: Params, images, x, grad_cache, recompute_grad: bool, score, ws) -> None:
    wp, wn = _ws_args(ws)
    _check(lib().litevggt_importance(C.byref(p), _ptr(images), _ptr(x), _ptr(grad_cache),
                                     1 if recompute_grad else 0, _ptr(score), wp, wn, _stream()),
           "litevggt_importance")


def litevggt_importance_static(p: Params, images, x, grad_cache, recompute_grad: bool, score) -> None:
    _check(lib().litevggt_importance_static(C.byref(p), _ptr(images), _ptr(x), _ptr(grad_cache),
                                            1 if recompute_grad else 0, _ptr(score), _stream()),
           "litevggt_importance_static")


def litevggt_select_anchors(p: Params, score, index: IndexBuffers) -> None:
    ix = index.struct()
    _check(lib().litevggt_select_anchors(C.byref(p), _ptr(score), C.byref(ix), _stream()),
           "litevggt_select_anchors")


def litevggt_match(p: Params, x, index: IndexBuffers, best_sim, ws) -> None:
    ix = index.struct()
    wp, wn = _ws_args(ws)
    _check(lib().litevggt_match(C.byref(p), _ptr(x), C.byref(ix), _ptr(best_sim), wp, wn, _stream()),
           "litevggt_match")


def litevggt_merge(p: Params, x, index: IndexBuffers, z) -> None:
    ix = index.struct()
    _check(lib().litevggt_merge(C.byref(p), _ptr(x), C.byref(ix), _ptr(z), _stream()),
           "litevggt_merge")


def litevggt_global_attn(p: Params, n_tokens: int, q, k, v, o, ws) -> None:
    wp, wn = _ws_args(ws)
    _check(lib().litevggt_global_attn(C.byref(p), n_tokens, _ptr(q), _ptr(k), _ptr(v), _ptr(o),
                                      wp, wn, _stream()), "litevggt_global_attn")


def litevggt_unmerge(p: Params, y, index: IndexBuffers, residual, out) -> None:
    ix = index.struct()
    _check(lib().litevggt_unmerge(C.byref(p), _ptr(y), C.byref(ix), _ptr(residual), _ptr(out),
                                  _stream()), "litevggt_unmerge")


def litevggt_frame_attn_ws_bytes(p: Params) -> int:
    return int(lib().litevggt_frame_attn_ws_bytes(C.byref(p)))


def litevggt_frame_attn(p: Params, q, k, v, residual, o, ws) -> None:
    wp, wn = _ws_args(ws)
    _check(lib().litevggt_frame_attn(C.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(residual), _ptr(o),
                                     wp, wn, _stream()), "litevggt_frame_attn")


def block_weights(tensors: dict, linear_dtype: int = LINEAR_BF16, fp8_recipe: int = FP8_CURRENT,
                  fp8_state=None) -> BlockWeights:
    """BlockWeights from a dict of device tensors (keys = the pointer fields' names); keep the
    dict alive.  ``fp8_state``: a zero-filled uint8 device tensor of FP8_STATE_BYTES for
    FP8_DELAYED, kept alive and passed again on later calls."""
    ptrs = {k: tensors[k].data_ptr() for k, t in BlockWeights._fields_ if t is C.c_void_p and k != "fp8_state"}
    return BlockWeights(linear_dtype=linear_dtype, fp8_recipe=fp8_recipe,
                        fp8_state=_ptr(fp8_state) if fp8_state is not None else None, **ptrs)


def litevggt_global_block_ws_bytes(p: Params, n_tokens: int) -> int:
    return int(lib().litevggt_global_block_ws_bytes(C.byref(p), n_tokens))


def litevggt_global_block(p: Params, n_tokens: int, z, weights: BlockWeights, delta, ws) -> None:
    wp, wn = _ws_args(ws)
    _check(lib().litevggt_global_block(C.byref(p), n_tokens, _ptr(z), C.byref(weights), _ptr(delta),
                                       wp, wn, _stream()), "litevggt_global_block")


EVENTS_PER_LAYER = 10
(EV_LAYER_BEGIN, EV_IMPORTANCE_END, EV_SELECT_END, EV_MATCH_END, EV_MERGE_END, EV_ATTN_PACK_END,
 EV_ATTN_END, EV_BLOCK_END, EV_UNMERGE_END, EV_FRAME_ATTN_END) = range(EVENTS_PER_LAYER)


def litevggt_layers_run(p: Params, n_layers: int, images, x, index: IndexBuffers, grad_cache,
                        score, ws, events=None):
    """``events``: optional ctypes array of EVENTS_PER_LAYER*n_layers hipEvent_t handles."""
    ix = index.struct()
    wp, wn = _ws_args(ws)
    log = (C.c_int32 * max(n_layers, 1))()
    _check(lib().litevggt_layers_run(C.byref(p), n_layers, _ptr(images), _ptr(x), C.byref(ix),
                                     _ptr(grad_cache), _ptr(score), log, events, wp, wn,
                                     _stream()),
           "litevggt_layers_run")
    return list(log)[:n_layers]


# ------------------------------------------------------------------ measurement aids
def litevggt_probe_mfma_flop(dtype: int, iters: int) -> float:
    return float(lib().litevggt_probe_mfma_flop(dtype, iters))


def litevggt_probe_mfma(dtype: int, operands, iters: int, out) -> None:
    _check(lib().litevggt_probe_mfma(dtype, _ptr(operands), iters, _ptr(out), _stream()), "litevggt_probe_mfma")


def litevggt_probe_stream(src, dst, nbytes: int, sink) -> None:
    _check(lib().litevggt_probe_stream(_ptr(src), _ptr(dst), nbytes, _ptr(sink), _stream()),
           "litevggt_probe_stream")


def litevggt_probe_gather(src, row_bytes: int, order, n_rows: int, sink) -> None:
    _check(lib().litevggt_probe_gather(_ptr(src), row_bytes, _ptr(order), n_rows, _ptr(sink), _stream()),
           "litevggt_probe_gather")
