"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, the
closed-form plan agrees with the oracle's, and argument validation rejects bad calls before
anything is launched (no GPU needed: validation is host code)."""
import ctypes as C
import os
import re

import pytest

from oracle import litevggt_oracle as O
from paper_2512_04939_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "litevggt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(litevggt_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = _declared_symbols()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_strerror_codes():
    assert B.litevggt_strerror(0) == "ok"
    seen = {B.litevggt_strerror(c) for c in range(-6, 1)}
    assert len(seen) == 7
    assert "unknown" in B.litevggt_strerror(-99)


@pytest.mark.parametrize("F,G,r", [(2, 16, 0.5), (32, 37, 0.9), (100, 37, 0.5), (100, 37, 0.75),
                                   (1000, 37, 0.9), (1000, 37, -1.0), (5, 9, 0.0)])
def test_plan_matches_oracle(F, G, r):
    dim, heads = (256, 4) if G == 16 else (1024, 16)
    pl = B.litevggt_plan(B.make_params(F, G, G, dim, heads, merge_ratio=r))
    ref = O.plan(O.Params(frames=F, grid_h=G, grid_w=G, dim=dim, heads=heads, merge_ratio=r))
    for k in ("N", "M", "n_dst", "n_src", "cell", "n_dst_per_frame", "n_ga_per_frame",
              "n_src_per_frame"):
        assert getattr(pl, k) == ref[k], k
    assert pl.ws_bytes > 0


def test_plan_rejects_bad_parameters():
    lib = B.lib()
    out = B.Plan()
    good = dict(frames=4, grid_h=8, grid_w=8, dim=256, heads=4)

    def rc(**kw):
        args = {**good, **kw}
        p = B.make_params(args.pop("frames"), args.pop("grid_h"), args.pop("grid_w"),
                          args.pop("dim"), args.pop("heads"), **args)
        return lib.litevggt_plan(C.byref(p), C.byref(out))

    assert rc() == 0
    assert rc(frames=0) == -2
    assert rc(dim=250) == -2
    assert rc(head_dim=32) == -2
    assert rc(merge_ratio=1.0) == -3
    assert rc(merge_ratio=float("nan")) == -3
    assert rc(merge_ratio=0.995) == 0             # one anchor per frame is still valid
    assert rc(var_pool=4) == -3
    assert rc(refresh_interval=0) == -3
    assert rc(img_dtype=7) == -5
    assert rc(attn_dtype=9) == -5
    assert lib.litevggt_plan(None, C.byref(out)) == -1
    p = B.make_params(4, 8, 8, 256, 4)
    assert lib.litevggt_plan(C.byref(p), None) == -1


def test_entry_points_validate_before_launch():
    """NULL pointers, short or misaligned workspaces come back as error codes (host checks)."""
    lib = B.lib()
    p = B.make_params(4, 8, 8, 256, 4)
    ix = B.Index()                                   # all NULL
    fake = C.c_void_p(0x1000)
    assert lib.litevggt_importance(C.byref(p), None, None, None, 1, None, None, 0, None) == -1
    assert lib.litevggt_importance(C.byref(p), fake, fake, fake, 1, fake, None, 0, None) == -4
    assert lib.litevggt_importance(C.byref(p), fake, fake, fake, 1, fake, C.c_void_p(0x1001),
                                   1 << 30, None) == -4
    # the variant with library-owned scratch: NULL and over-size checks come before any HIP call
    assert lib.litevggt_importance_static(C.byref(p), None, None, None, 1, None, None) == -1
    big = B.make_params(2000, 37, 37, 1024, 16)
    assert 2000 * 37 * 37 > B.STATIC_SCORE_MAX
    assert lib.litevggt_importance_static(C.byref(big), fake, fake, fake, 1, fake, None) == -4
    assert lib.litevggt_select_anchors(C.byref(p), fake, C.byref(ix), None) == -1
    assert lib.litevggt_match(C.byref(p), fake, C.byref(ix), None, fake, 1 << 30, None) == -1
    assert lib.litevggt_merge(C.byref(p), fake, C.byref(ix), fake, None) == -1
    assert lib.litevggt_global_attn(C.byref(p), 0, fake, fake, fake, fake, fake, 1 << 30, None) == -2
    assert lib.litevggt_global_attn(C.byref(p), 100, fake, fake, fake, fake, fake, 16, None) == -4
    assert lib.litevggt_unmerge(C.byref(p), None, C.byref(ix), None, fake, None) == -1
    assert lib.litevggt_layers_run(C.byref(p), 2, fake, fake, C.byref(ix), fake, fake, None, None,
                                   fake, 1 << 30, None) == -1
    assert B.litevggt_attn_ws_bytes(p, 1000) > 0
    # the block: weights struct is checked before anything is launched
    bw = B.BlockWeights()                            # all NULL
    assert lib.litevggt_global_block(C.byref(p), 100, fake, C.byref(bw), fake, fake, 1 << 30, None) == -1
    for k, t in B.BlockWeights._fields_:
        if t is C.c_void_p and k != "fp8_state":
            setattr(bw, k, 0x1000)
    bw.linear_dtype = 7
    assert lib.litevggt_global_block(C.byref(p), 100, fake, C.byref(bw), fake, fake, 1 << 30, None) == -5
    bw.linear_dtype, bw.fp8_recipe = B.LINEAR_FP8_E4M3, 5
    assert lib.litevggt_global_block(C.byref(p), 100, fake, C.byref(bw), fake, fake, 1 << 30, None) == -3
    bw.fp8_recipe = B.FP8_DELAYED                    # needs a state block
    assert lib.litevggt_global_block(C.byref(p), 100, fake, C.byref(bw), fake, fake, 1 << 30, None) == -1
    bw.fp8_state = 0x1000                            # now only the workspace is wrong
    assert lib.litevggt_global_block(C.byref(p), 100, fake, C.byref(bw), fake, fake, 16, None) == -4
    assert C.sizeof(B.BlockWeights) == 12 * 8 + 2 * 4 + 8 and B.FP8_STATE_BYTES == 1312
