"""Seeded synthetic inputs with the shapes of VGGT token sequences.

This module produces *data only*: patch/special token features and RGB frames
that stand in for the image sequences and backbone features the paper evaluates
on (its datasets and trained weights are not available).  It contains none of
the method's arithmetic (no Sobel, variance, similarity, merge or attention) and
is the only module that both the CPU oracle's tests and the HIP path's tests
import.

Recipe (all randomness from numpy ``PCG64`` streams derived from ``seed``):

* a feature canvas ``[Hc, Wc, C]`` = sum of 3 independent N(0,1) fields, each
  Gaussian-smoothed over the two spatial axes (sigma = 2 patches, periodic
  border so that crops may wrap around);
* frame ``f`` reads the canvas at an integer patch offset ``(oy_f, ox_f)`` and
  adds fresh N(0, 0.1^2) noise; camera/register tokens are N(0,1);
* an RGB canvas of ``Hc*patch x Wc*patch`` pixels = smooth two-axis gradient
  plus random axis-aligned rectangles of random colour (sharp edges); frame
  ``f`` is the crop at ``(oy_f*patch, ox_f*patch)``, so pixels and tokens move
  together.

Frames can be generated independently of each other (per-frame noise streams),
so a caller can build any subset of a 1000-frame workload.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Iterable, Optional, Sequence

import numpy as np
from scipy.ndimage import gaussian_filter1d


@dataclass(frozen=True)
class Workload:
    """Shape and generator settings of one synthetic sequence."""
    name: str
    frames: int
    grid_h: int
    grid_w: int
    dim: int
    heads: int
    head_dim: int = 64
    n_special: int = 5          # 1 camera + 4 register tokens per frame
    patch: int = 14
    merge_ratio: float = 0.9
    layers: int = 24
    refresh_interval: int = 6
    seed: int = 0
    motion: str = "uniform"     # "fixed3" | "uniform" | "walk"
    store: str = "bf16"         # "f32" | "bf16": how features are stored
    canvas: int = 64            # canvas side, in patches

    @property
    def patches(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def tokens_per_frame(self) -> int:
        return self.patches + self.n_special

    @property
    def n_tokens(self) -> int:
        return self.frames * self.tokens_per_frame

    @property
    def img_h(self) -> int:
        return self.grid_h * self.patch

    @property
    def img_w(self) -> int:
        return self.grid_w * self.patch


# The five configurations the benchmark definition names, plus small extras the
# parity tests use.  "fixed3": frame f is frame 0 shifted by 3*f patches.
WORKLOADS = {
    "tiny2": Workload("tiny2", frames=2, grid_h=16, grid_w=16, dim=256, heads=4,
                      merge_ratio=0.5, layers=2, seed=0, motion="fixed3",
                      store="f32", canvas=32),
    "f32": Workload("f32", frames=32, grid_h=37, grid_w=37, dim=1024, heads=16,
                    merge_ratio=0.9, seed=2, motion="uniform"),
    "f100": Workload("f100", frames=100, grid_h=37, grid_w=37, dim=1024, heads=16,
                     merge_ratio=0.9, seed=3, motion="uniform"),
    "f500": Workload("f500", frames=500, grid_h=37, grid_w=37, dim=1024, heads=16,
                     merge_ratio=0.9, seed=4, motion="walk"),
    "f1000": Workload("f1000", frames=1000, grid_h=37, grid_w=37, dim=1024, heads=16,
                      merge_ratio=0.9, seed=5, motion="walk"),
    # the paper's own shape: 392 x 518 images (28 x 37 patches), its fixed partition rule
    # (merge_ratio < 0: top 10 % GA tokens, one dst per 2 x 2 cell)
    "paper1000": Workload("paper1000", frames=1000, grid_h=28, grid_w=37, dim=1024, heads=16,
                          merge_ratio=-1.0, seed=6, motion="walk"),
}


def workload(name: str, **overrides) -> Workload:
    return replace(WORKLOADS[name], **overrides)


# ----------------------------------------------------------------------------
# bf16 storage helpers (a storage format, not method arithmetic)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (uint16)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    out = ((u + rounding) >> 16).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------
# generators
# ----------------------------------------------------------------------------
def _stream(seed: int, *path: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, *path])))


def frame_offsets(wl: Workload) -> np.ndarray:
    """Integer patch offsets ``[F, 2]`` (row, col) of each frame on the canvas."""
    rng = _stream(wl.seed, 10)
    off = np.zeros((wl.frames, 2), dtype=np.int64)
    if wl.motion == "fixed3":
        off[:, 1] = 3 * np.arange(wl.frames)
    elif wl.motion == "uniform":
        off[1:] = rng.integers(0, 6, size=(wl.frames - 1, 2))
    elif wl.motion == "walk":
        # a panning camera: 1-3 patches per frame along the row, small vertical jitter
        dx = rng.integers(1, 4, size=wl.frames - 1)
        dy = rng.integers(-1, 2, size=wl.frames - 1)
        off[1:, 1] = np.cumsum(dx)
        off[1:, 0] = np.cumsum(dy)
    else:
        raise ValueError(f"unknown motion {wl.motion!r}")
    return off


def feature_canvas(wl: Workload) -> np.ndarray:
    """``[Hc, Wc, C]`` float32 smooth field (sum of 3 smoothed N(0,1) fields)."""
    rng = _stream(wl.seed, 20)
    hc = wc = wl.canvas
    acc = np.zeros((hc, wc, wl.dim), dtype=np.float32)
    for _ in range(3):
        fld = rng.standard_normal((hc, wc, wl.dim), dtype=np.float32)
        fld = gaussian_filter1d(fld, sigma=2.0, axis=0, mode="wrap")
        fld = gaussian_filter1d(fld, sigma=2.0, axis=1, mode="wrap")
        acc += fld
    return acc


def image_canvas(wl: Workload) -> np.ndarray:
    """``[3, Hc*patch, Wc*patch]`` float32 in [0,1]: gradient + sharp rectangles."""
    rng = _stream(wl.seed, 30)
    hp = wp = wl.canvas * wl.patch
    yy = np.linspace(0.0, 1.0, hp, dtype=np.float32)[:, None]
    xx = np.linspace(0.0, 1.0, wp, dtype=np.float32)[None, :]
    img = np.empty((3, hp, wp), dtype=np.float32)
    img[0] = 0.15 + 0.5 * xx + 0.0 * yy
    img[1] = 0.15 + 0.5 * yy + 0.0 * xx
    img[2] = 0.15 + 0.25 * (xx + yy)
    # about 5 rectangles per frame-sized window of the canvas
    n_rect = max(5, int(round(5.0 * (hp * wp) / float(wl.img_h * wl.img_w))))
    for _ in range(n_rect):
        h = int(rng.integers(wl.patch, max(wl.patch + 1, wl.img_h // 2)))
        w = int(rng.integers(wl.patch, max(wl.patch + 1, wl.img_w // 2)))
        y0 = int(rng.integers(0, hp - h))
        x0 = int(rng.integers(0, wp - w))
        img[:, y0:y0 + h, x0:x0 + w] = rng.random(3, dtype=np.float32)[:, None, None]
    return img


def _crop_wrap(canvas: np.ndarray, oy: int, ox: int, h: int, w: int, ax: int) -> np.ndarray:
    ys = (oy + np.arange(h)) % canvas.shape[ax]
    xs = (ox + np.arange(w)) % canvas.shape[ax + 1]
    if ax == 0:
        return canvas[np.ix_(ys, xs)]
    return canvas[:, ys][:, :, xs]


@dataclass
class Generator:
    """Holds the canvases of one workload and produces frames on demand."""
    wl: Workload
    noise_std: float = 0.1
    _fcanvas: Optional[np.ndarray] = field(default=None, repr=False)
    _icanvas: Optional[np.ndarray] = field(default=None, repr=False)
    _offsets: Optional[np.ndarray] = field(default=None, repr=False)

    @property
    def offsets(self) -> np.ndarray:
        if self._offsets is None:
            self._offsets = frame_offsets(self.wl)
        return self._offsets

    def frame_tokens(self, f: int) -> np.ndarray:
        """``[T, C]`` float32 tokens of frame ``f`` (specials first, patches row-major)."""
        wl = self.wl
        if self._fcanvas is None:
            self._fcanvas = feature_canvas(wl)
        oy, ox = (int(v) for v in self.offsets[f])
        rng = _stream(wl.seed, 40, f)
        out = np.empty((wl.tokens_per_frame, wl.dim), dtype=np.float32)
        out[:wl.n_special] = rng.standard_normal((wl.n_special, wl.dim), dtype=np.float32)
        patch = _crop_wrap(self._fcanvas, oy, ox, wl.grid_h, wl.grid_w, 0)
        noise = rng.standard_normal((wl.patches, wl.dim), dtype=np.float32)
        out[wl.n_special:] = patch.reshape(wl.patches, wl.dim) + np.float32(self.noise_std) * noise
        return out

    def frame_image(self, f: int) -> np.ndarray:
        """``[3, img_h, img_w]`` float32 image of frame ``f``."""
        wl = self.wl
        if self._icanvas is None:
            self._icanvas = image_canvas(wl)
        oy, ox = (int(v) for v in self.offsets[f])
        return np.ascontiguousarray(
            _crop_wrap(self._icanvas, oy * wl.patch, ox * wl.patch, wl.img_h, wl.img_w, 1))

    # -- whole-sequence helpers -------------------------------------------------
    def tokens(self, frames: Optional[Iterable[int]] = None, threads: int = 8) -> np.ndarray:
        """Features of ``frames`` (default all) as stored: float32 values for
        ``store="f32"``, bf16 bit patterns (uint16) for ``store="bf16"``;
        shape ``[len(frames)*T, C]``."""
        wl = self.wl
        fl = list(range(wl.frames)) if frames is None else list(frames)
        t = wl.tokens_per_frame
        dt = np.float32 if wl.store == "f32" else np.uint16
        out = np.empty((len(fl) * t, wl.dim), dtype=dt)
        if self._fcanvas is None:
            self._fcanvas = feature_canvas(wl)
        _ = self.offsets

        def one(j: int) -> None:
            x = self.frame_tokens(fl[j])
            out[j * t:(j + 1) * t] = x if wl.store == "f32" else f32_to_bf16_bits(x)

        if threads > 1 and len(fl) > 1:
            with ThreadPoolExecutor(max_workers=threads) as ex:
                list(ex.map(one, range(len(fl))))
        else:
            for j in range(len(fl)):
                one(j)
        return out

    def images(self, frames: Optional[Iterable[int]] = None) -> np.ndarray:
        """``[len(frames), 3, img_h, img_w]`` float32 images."""
        wl = self.wl
        fl = list(range(wl.frames)) if frames is None else list(frames)
        out = np.empty((len(fl), 3, wl.img_h, wl.img_w), dtype=np.float32)
        for j, f in enumerate(fl):
            out[j] = self.frame_image(f)
        return out


def stored_to_f32(x: np.ndarray) -> np.ndarray:
    """Widen stored features (float32 or bf16 bits) to float32 values."""
    return bf16_bits_to_f32(x) if x.dtype == np.uint16 else np.asarray(x, dtype=np.float32)


def random_qkv(n_tokens: int, heads: int, head_dim: int, seed: int, scale: float = 1.0,
               ) -> Sequence[np.ndarray]:
    """Three ``[n_tokens, heads, head_dim]`` float32 N(0, scale^2) tensors for
    attention-only tests (queries, keys, values)."""
    rng = _stream(seed, 50)
    return tuple((scale * rng.standard_normal((n_tokens, heads, head_dim), dtype=np.float32))
                 for _ in range(3))


# ----------------------------------------------------------------------------
# synthetic weights of the transformer block around the global attention
# ----------------------------------------------------------------------------
def block_weights(dim: int, seed: int = 0) -> dict:
    """Seeded random weights of one pre-norm block (no trained weights exist here): matrices
    [out, in] ~ N(0, 1/in) rounded to bf16 (returned as float32 holding bf16 values), the two
    residual-branch outputs (w_o, w_2) scaled by 0.5 so a stack of blocks grows slowly; biases
    and LayerNorm offsets ~ N(0, 0.02^2), LayerNorm gains 1 + N(0, 0.1^2); vectors float32."""
    rng = np.random.Generator(np.random.PCG64([seed, 0xB10C]))

    def mat(o, i, gain=1.0):
        w = (rng.standard_normal((o, i)) * (gain / np.sqrt(i))).astype(np.float32)
        return bf16_bits_to_f32(f32_to_bf16_bits(w))

    def vec(n, std, mean=0.0):
        return (mean + std * rng.standard_normal(n)).astype(np.float32)

    return dict(ln1_g=vec(dim, 0.1, 1.0), ln1_b=vec(dim, 0.02),
                w_qkv=mat(3 * dim, dim), b_qkv=vec(3 * dim, 0.02),
                w_o=mat(dim, dim, 0.5), b_o=vec(dim, 0.02),
                ln2_g=vec(dim, 0.1, 1.0), ln2_b=vec(dim, 0.02),
                w_1=mat(4 * dim, dim), b_1=vec(4 * dim, 0.02),
                w_2=mat(dim, 4 * dim, 0.5), b_2=vec(dim, 0.02))
