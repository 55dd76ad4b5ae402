"""Shared helpers of the parity tests: build the same seeded inputs for both sides."""
from __future__ import annotations

import numpy as np

from oracle import litevggt_oracle as O
from paper_2512_04939_amd import synth


def oracle_params(wl: synth.Workload, **kw) -> O.Params:
    base = dict(frames=wl.frames, grid_h=wl.grid_h, grid_w=wl.grid_w, n_special=wl.n_special,
                dim=wl.dim, heads=wl.heads, head_dim=wl.head_dim, patch=wl.patch,
                merge_ratio=wl.merge_ratio, refresh_interval=wl.refresh_interval, qk_norm=True)
    base.update(kw)
    return O.Params(**base)


def hip_params(wl: synth.Workload, **kw):
    from paper_2512_04939_amd import binding as B
    base = dict(n_special=wl.n_special, patch=wl.patch, merge_ratio=wl.merge_ratio,
                refresh_interval=wl.refresh_interval, qk_norm=1)
    base.update(kw)
    return B.make_params(wl.frames, wl.grid_h, wl.grid_w, wl.dim, wl.heads, **base)


def stored_inputs(wl: synth.Workload):
    """(bf16 bit patterns [N,C] uint16, the same values as float32, images float32)."""
    gen = synth.Generator(wl)
    x = gen.tokens()
    if x.dtype != np.uint16:                    # the HIP path stores features as bf16
        x = synth.f32_to_bf16_bits(x)
    return x, synth.bf16_bits_to_f32(x), gen.images()


def to_dev_bf16(bits: np.ndarray):
    import torch
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def f32_to_dev_bf16(a: np.ndarray):
    return to_dev_bf16(synth.f32_to_bf16_bits(a))


def dev_bf16_to_f64(t) -> np.ndarray:
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def max_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref| over the whole tensor."""
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def small_workload(frames=3, grid=37, dim=256, heads=4, r=0.9, seed=7, motion="uniform", **kw):
    return synth.Workload("small", frames=frames, grid_h=grid, grid_w=grid, dim=dim, heads=heads,
                          merge_ratio=r, seed=seed, motion=motion, canvas=max(48, grid + 8), **kw)
