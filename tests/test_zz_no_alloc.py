"""The entry point that allocates nothing (litevggt_importance_static: the variance map lives in
a device array inside the library) against litevggt_importance with a caller workspace, through
the C ABI: bit-identical scores and cached gradient maps, on two calls in a row, the second on a
smaller input (the array keeps the first call's contents), then the cached-gradient form."""
import numpy as np
import pytest

from paper_2512_04939_amd import synth

from helpers import hip_params, small_workload, stored_inputs, to_dev_bf16

pytestmark = pytest.mark.gpu


def _both(B, wl, recompute=True, grads=None):
    import torch
    bits, _, im = stored_inputs(wl)
    ph = hip_params(wl)
    F, P = wl.frames, wl.patches
    x, imd = to_dev_bf16(bits), torch.from_numpy(im).cuda()
    out = []
    for k, static in enumerate((False, True)):
        grad = grads[k] if grads is not None else torch.full((F, P), -3.0, device="cuda")
        score = torch.full((F, P), -5.0, device="cuda")
        if static:
            before = torch.cuda.memory_allocated()
            B.litevggt_importance_static(ph, imd if recompute else None, x, grad, recompute, score)
            assert torch.cuda.memory_allocated() == before
        else:
            B.litevggt_importance(ph, imd if recompute else None, x, grad, recompute, score,
                                  B.alloc_ws(F * P * 4))
        torch.cuda.synchronize()
        out.append((grad, score))
    return out


def test_importance_static_matches_importance_twice_then_cached():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2512_04939_amd import binding as B
    B.lib()
    big = small_workload(frames=5, grid=37, dim=256, heads=4, r=0.9, seed=21)
    small = small_workload(frames=2, grid=12, dim=128, heads=2, r=0.5, seed=22)
    for wl in (big, small):                       # second call: smaller input, stale scratch
        (g0, s0), (g1, s1) = _both(B, wl)
        assert torch.equal(g0, g1) and torch.equal(s0, s1)
        assert float(s0.min()) >= 0.0 and float(s0.max()) <= 1.0 + 1e-6
        # cached gradient map, images not passed
        (_, c0), (_, c1) = _both(B, wl, recompute=False, grads=(g0, g1))
        assert torch.equal(c0, c1) and torch.equal(c0, s0)
    # sizes beyond the array are refused before anything is launched
    huge = B.make_params(2000, 37, 37, 1024, 16)
    fake = torch.empty(16, device="cuda")
    with pytest.raises(B.LiteVGGTError, match="workspace"):
        B.litevggt_importance_static(huge, fake, fake, fake, True, fake)
