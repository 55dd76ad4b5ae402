"""Parity at the benchmark configurations' full sizes (32, 100, 500 and 1000 frames of 37 x 37
patches, dim 1024; 100 frames at merge ratios 0.5, 0.75, 0.9; the paper's own shape, 1000 frames
of 28 x 37 patches under its partition rule), in the launch configuration
bench.py times: every step runs on the whole sequence, the oracle checks sampled outputs it can
compute one by one, plus structural properties that hold at any size.  At 100 frames the
unmerged attention (the speedup baseline) is sampled as well."""
from __future__ import annotations

import numpy as np
import pytest

from helpers import hip_params, max_rel_err, oracle_params
from oracle import litevggt_oracle as O
from paper_2512_04939_amd import synth

pytestmark = pytest.mark.gpu

BF16_TOL = 2e-2


def _f64(bits_rows: np.ndarray) -> np.ndarray:
    return synth.bf16_bits_to_f32(bits_rows).astype(np.float64)


def _host_bits(t) -> np.ndarray:
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


CASES = [("f32", {}), ("f100", {"merge_ratio": 0.5}), ("f100", {"merge_ratio": 0.75}), ("f100", {}),
         ("f500", {}), ("f1000", {}), ("paper1000", {})]


@pytest.mark.parametrize("name,over", CASES, ids=[n + "".join(f"-r{v}" for v in o.values()) for n, o in CASES])
def test_full_size_steps_against_sampled_oracle(name, over):
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2512_04939_amd import binding as B
    wl = synth.workload(name, **over)
    po, ph = oracle_params(wl), hip_params(wl)
    pl = B.litevggt_plan(ph)
    F, T, P, S, C, heads = wl.frames, wl.tokens_per_frame, wl.patches, wl.n_special, wl.dim, wl.heads
    N, M = pl.N, pl.M
    if name == "f1000":
        assert (N, M, pl.n_dst, pl.n_src) == (1374000, 143232, 101269, 1230768)
    print(f"{name} {over}: N={N} M={M} n_dst={pl.n_dst} n_src={pl.n_src}", flush=True)
    gen = synth.Generator(wl)
    bits = gen.tokens(threads=16)                        # [N, C] bf16 bit patterns
    x = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    im = torch.empty(F, 3, wl.img_h, wl.img_w, dtype=torch.float32, device="cuda")
    for f0 in range(0, F, 50):
        fr = range(f0, min(F, f0 + 50))
        im[f0:f0 + len(fr)].copy_(torch.from_numpy(gen.images(fr)))
    rng = np.random.default_rng(2024)

    # ---- every step of one layer with a refresh, whole sequence
    ib = B.alloc_index(pl)
    ws = B.alloc_ws(pl.ws_bytes)
    grad = torch.zeros(F, P, device="cuda")
    score = torch.zeros(F, P, device="cuda")
    z = torch.empty(M, C, dtype=torch.bfloat16, device="cuda")
    y = torch.empty_like(z)
    out = torch.empty_like(x)
    B.litevggt_importance(ph, im, x, grad, True, score, ws)
    B.litevggt_select_anchors(ph, score, ib)
    B.litevggt_match(ph, x, ib, None, ws)
    B.litevggt_merge(ph, x, ib, z)
    B.litevggt_global_attn(ph, M, z, z, z, y, ws)
    B.litevggt_unmerge(ph, y, ib, x, out)
    torch.cuda.synchronize()

    # ---- importance: sampled frames (the map of a frame depends on that frame only)
    frames = np.array([0, 1, F // 2, F - 2, F - 1])
    rows = np.concatenate([np.arange(f * T, (f + 1) * T) for f in frames])
    psub = oracle_params(synth.Workload(**{**wl.__dict__, "frames": len(frames)}))
    want, _ = O.importance(gen.images(frames), _f64(bits[rows]), psub)
    got = score[torch.from_numpy(frames).cuda()].cpu().numpy().astype(np.float64)
    assert np.abs(got - want).max() <= 2e-5

    # ---- partition: the oracle's rule on the GPU's own scores, frame 0 plus sampled frames
    sel = O.select_anchors(score[torch.from_numpy(frames).cuda()].cpu().numpy(), psub)
    role = ib.role.cpu().numpy().reshape(F, T)
    assert np.array_equal(role[frames].ravel(), sel["role"])
    src_idx = ib.src_idx.cpu().numpy()[:pl.n_src].astype(np.int64)
    dst_idx = ib.dst_idx.cpu().numpy()[:pl.n_dst].astype(np.int64)
    kept_idx = ib.kept_idx.cpu().numpy().astype(np.int64)
    flat = role.ravel()
    assert np.array_equal(np.flatnonzero(flat == O.ROLE_SRC), src_idx)
    assert np.array_equal(np.flatnonzero(flat == O.ROLE_DST), dst_idx)
    assert np.array_equal(np.flatnonzero(flat != O.ROLE_SRC), kept_idx)

    # ---- match: sampled src tokens against all dst tokens
    pick = np.sort(rng.choice(pl.n_src, size=96, replace=False))
    small = _f64(bits[np.concatenate([dst_idx, src_idx[pick]])])
    mt = O.match(small, np.arange(pl.n_dst), pl.n_dst + np.arange(len(pick)))
    want_anchor = dst_idx[mt["anchor"]]
    anchor_of = ib.anchor_of.cpu().numpy().astype(np.int64)
    got_anchor = anchor_of[src_idx[pick]]
    differ = got_anchor != want_anchor
    assert np.all((mt["best"] - mt["second"])[differ] < 1e-6), "disagreement outside near-ties"
    assert differ.sum() <= 2
    assert np.array_equal(anchor_of[kept_idx], kept_idx)

    # ---- index structure at full size
    slot_of = ib.slot_of.cpu().numpy().astype(np.int64)
    goff = ib.group_off.cpu().numpy().astype(np.int64)
    gmem = ib.group_mem.cpu().numpy().astype(np.int64)
    assert goff[0] == 0 and goff[-1] == N and np.all(np.diff(goff) >= 1)
    assert np.array_equal(np.sort(gmem), np.arange(N))                 # every token in one group
    assert np.array_equal(slot_of[gmem], np.repeat(np.arange(M), np.diff(goff)))
    assert np.array_equal(slot_of[kept_idx], np.arange(M))
    assert np.array_equal(slot_of, slot_of[anchor_of])
    inside = np.ones(N, dtype=bool)
    inside[goff[1:-1]] = False                                          # group starts
    assert np.all(np.diff(gmem)[inside[1:]] > 0)                        # ascending inside a group

    # ---- merge: the largest group and random slots
    sizes = np.diff(goff)
    slots = np.unique(np.concatenate([[int(np.argmax(sizes)), 0, M - 1], rng.choice(M, size=40, replace=False)]))
    zb = _host_bits(z)
    want_z = np.stack([_f64(bits[gmem[goff[m]:goff[m + 1]]]).mean(axis=0) for m in slots])
    assert max_rel_err(_f64(zb[slots]), want_z) <= BF16_TOL

    # ---- attention: sampled query rows of two heads over all M keys (inputs: the GPU's z)
    qrows = np.sort(rng.choice(M, size=12, replace=False))
    yb = _host_bits(y)
    for head in (3, 12):
        cols = slice(head * 64, (head + 1) * 64)
        zh = _f64(zb[:, cols]).reshape(M, 1, 64)
        qk = O.round_bf16(O.qk_normalize(zh))
        want_y = O.attention(qk, qk, zh, rows=qrows).reshape(len(qrows), 64)
        assert max_rel_err(_f64(yb[qrows][:, cols]), want_y) <= BF16_TOL

    # ---- FP8 attention at the largest size: the same sampled rows against exact attention
    if name == "f1000":
        p8 = hip_params(wl, attn_dtype=B.ATTN_FP8_E4M3)
        y8 = torch.empty_like(z)
        ws8 = B.alloc_ws(B.litevggt_attn_ws_bytes(p8, M))
        B.litevggt_global_attn(p8, M, z, z, z, y8, ws8)
        torch.cuda.synchronize()
        y8b = _host_bits(y8)
        for head in (3, 12):
            cols = slice(head * 64, (head + 1) * 64)
            zh = _f64(zb[:, cols]).reshape(M, 1, 64)
            qk = O.round_bf16(O.qk_normalize(zh))
            want_y = O.attention(qk, qk, zh, rows=qrows).reshape(len(qrows), 64)
            assert max_rel_err(_f64(y8b[qrows][:, cols]), want_y) <= 6e-2
        del y8, ws8

    # ---- q, k as given (no qk_norm; per-wave score bound, second pass where it is loose), with a
    # softmax scale small enough that rows mix many keys: the same sampled rows (500 frames)
    if name == "f500":
        pn = hip_params(wl, qk_norm=0, softmax_scale=0.02)
        yn = torch.empty_like(z)
        B.litevggt_global_attn(pn, M, z, z, z, yn, B.alloc_ws(B.litevggt_attn_ws_bytes(pn, M)))
        torch.cuda.synchronize()
        ynb = _host_bits(yn)
        for head in (0, 9):
            cols = slice(head * 64, (head + 1) * 64)
            zh = _f64(zb[:, cols]).reshape(M, 1, 64)
            want_y = O.attention(zh, zh, zh, rows=qrows, scale=0.02).reshape(len(qrows), 64)
            assert max_rel_err(_f64(ynb[qrows][:, cols]), want_y) <= BF16_TOL
        del yn

    # ---- unmerge with the fused residual: bit-exact on sampled tokens
    toks = np.sort(rng.choice(N, size=4096, replace=False))
    s = synth.bf16_bits_to_f32(bits[toks]) + synth.bf16_bits_to_f32(yb[slot_of[toks]])
    assert np.array_equal(_host_bits(out[torch.from_numpy(toks).cuda()]), synth.f32_to_bf16_bits(s))

    # ---- the speedup baseline: unmerged attention over all N tokens, sampled rows (100 frames)
    if name == "f100" and not over:
        ws_u = B.alloc_ws(B.litevggt_attn_ws_bytes(ph, N))
        yu = torch.empty_like(x)
        B.litevggt_global_attn(ph, N, x, x, x, yu, ws_u)
        torch.cuda.synchronize()
        yub = _host_bits(yu)
        qrows = np.sort(rng.choice(N, size=8, replace=False))
        cols = slice(5 * 64, 6 * 64)
        xh = _f64(bits[:, cols]).reshape(N, 1, 64)
        qk = O.round_bf16(O.qk_normalize(xh))
        want_u = O.attention(qk, qk, xh, rows=qrows).reshape(len(qrows), 64)
        assert max_rel_err(_f64(yub[qrows][:, cols]), want_u) <= BF16_TOL


def test_full_size_block_against_sampled_oracle():
    """The transformer block around the attention core at the benchmark's merged length
    (M = 143,232 rows, dim 1024, 16 heads): the whole block runs on the GPU, the oracle follows
    the same sequence of stored intermediates for a sample of rows (LayerNorm and the k, v
    projections for every row, since sampled queries attend over all of them; everything after
    the attention for the sampled rows only)."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from helpers import f32_to_dev_bf16
    from paper_2512_04939_amd import binding as B
    wl = synth.workload("f1000")
    po, ph = oracle_params(wl), hip_params(wl)
    pl = B.litevggt_plan(ph)
    M, C, heads = pl.M, wl.dim, wl.heads
    print(f"block at M={M}", flush=True)
    gen = synth.Generator(wl)
    zb = gen.tokens(range((M + wl.tokens_per_frame - 1) // wl.tokens_per_frame), threads=16)[:M]   # bf16 bit patterns
    z = _f64(zb)
    w = synth.block_weights(C, seed=wl.seed)
    tens = {k: (f32_to_dev_bf16(v) if v.ndim == 2 else torch.from_numpy(v).cuda()) for k, v in w.items()}
    bw = B.block_weights(tens)
    delta = torch.empty(M, C, dtype=torch.bfloat16, device="cuda")
    ws = B.alloc_ws(B.litevggt_global_block_ws_bytes(ph, M))
    B.litevggt_global_block(ph, M, torch.from_numpy(zb.view(np.int16)).cuda().view(torch.bfloat16), bw, delta, ws)
    torch.cuda.synchronize()
    got = _f64(_host_bits(delta))
    assert np.all(np.isfinite(got))

    st = lambda a: O.round_bf16(a)
    w64 = {k: v.astype(np.float64) for k, v in w.items()}
    rows = np.sort(np.random.default_rng(77).choice(M, size=8, replace=False))
    h = st(O.layer_norm(z, w64["ln1_g"], w64["ln1_b"]))
    wq, wk, wv = (w64["w_qkv"][i * C:(i + 1) * C] for i in range(3))
    bq, bk, bv = (w64["b_qkv"][i * C:(i + 1) * C] for i in range(3))
    k = st(O.linear(h, wk, bk)).reshape(M, heads, 64)
    v = st(O.linear(h, wv, bv)).reshape(M, heads, 64)
    q = np.zeros((M, heads, 64))
    q[rows] = st(O.linear(h[rows], wq, bq)).reshape(len(rows), heads, 64)
    qn, kn = st(O.qk_normalize(q)), st(O.qk_normalize(k))
    a = st(O.attention(qn, kn, v, rows=rows).reshape(len(rows), C))
    u1 = st(O.linear(a, w64["w_o"], w64["b_o"]))
    h2 = st(O.layer_norm(z[rows] + u1, w64["ln2_g"], w64["ln2_b"]))
    h3 = st(O.gelu(O.linear(h2, w64["w_1"], w64["b_1"])))
    u2 = st(O.linear(h3, w64["w_2"], w64["b_2"]))
    want = st(u1 + u2)
    assert max_rel_err(got[rows], want) <= BF16_TOL


def test_full_size_frame_attention_against_oracle_on_sampled_frames():
    """Frame attention over all 1000 frames (16000 independent (frame, head) sequences of 1374
    tokens) with the residual fused; the oracle recomputes three whole frames."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2512_04939_amd import binding as B
    wl = synth.workload("f1000")
    po, ph = oracle_params(wl, frame_attn=True), hip_params(wl, frame_attn=1)
    T, C, heads, N = wl.tokens_per_frame, wl.dim, wl.heads, wl.n_tokens
    gen = synth.Generator(wl)
    bits = gen.tokens(threads=16)
    x = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    out = torch.empty_like(x)
    ws = B.alloc_ws(B.litevggt_frame_attn_ws_bytes(ph))
    B.litevggt_frame_attn(ph, x, x, x, x, out, ws)
    torch.cuda.synchronize()
    for f in (0, 517, wl.frames - 1):
        rows = slice(f * T, (f + 1) * T)
        xf = _f64(bits[rows]).reshape(T, heads, 64)
        qk = O.round_bf16(O.qk_normalize(xf))
        want = xf.reshape(T, C) + O.attention(qk, qk, xf).reshape(T, C)
        got = _f64(_host_bits(out[rows]))
        assert max_rel_err(got, want) <= BF16_TOL, f"frame {f}"
