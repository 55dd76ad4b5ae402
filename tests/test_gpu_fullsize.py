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


def _check_sampled_match(bits, dst_idx, src_idx, anchor_of, pick, label=""):
    """Sampled src rows (positions `pick` in src_idx) against ALL dst rows with the oracle: the
    anchors agree, except on near-ties: the oracle's best similarity and the float64 similarity
    of the GPU's choice are closer than 1e-6.  Those are counted and returned."""
    small = _f64(bits[np.concatenate([dst_idx, src_idx[pick]])])
    n_dst = len(dst_idx)
    mt = O.match(small, np.arange(n_dst), n_dst + np.arange(len(pick)))
    want_anchor = dst_idx[mt["anchor"]]
    got_anchor = anchor_of[src_idx[pick]]
    differ = np.flatnonzero(got_anchor != want_anchor)
    gap = mt["best"] - mt["second"]
    inv = O.inv_norms(small)
    lost = np.zeros(len(differ))
    for n, i in enumerate(differ):
        d = int(np.searchsorted(dst_idx, got_anchor[i]))
        assert d < n_dst and dst_idx[d] == got_anchor[i], "anchor is not a dst token"
        lost[n] = mt["best"][i] - float(small[n_dst + i] @ small[d]) * inv[n_dst + i] * inv[d]
    print(f"match {label}: {len(pick)} src rows, oracle top-2 gap < 1e-6 on {int((gap < 1e-6).sum())}, < 1e-5 on "
          f"{int((gap < 1e-5).sum())}, < 1e-4 on {int((gap < 1e-4).sum())}; {len(differ)} anchors differ, "
          f"largest similarity lost {np.abs(lost).max() if len(lost) else 0.0:.2e}, "
          f"{int((gap[differ] >= 1e-6).sum())} of them with an oracle top-2 gap >= 1e-6", flush=True)
    assert np.all(gap[differ] < 1e-6) and np.all(np.abs(lost) < 1e-6), f"disagreement outside near-ties: {lost[:8]}"
    return len(differ)


def _check_sampled_merge(bits, zb, goff, gmem, rng, n_random=512, n_largest=20):
    M = len(goff) - 1
    sizes = np.diff(goff)
    largest = np.argsort(-sizes, kind="stable")[:n_largest]
    slots = np.unique(np.concatenate([largest, [0, M - 1], rng.choice(M, size=min(n_random, M), replace=False)]))
    want_z = np.stack([_f64(bits[gmem[goff[m]:goff[m + 1]]]).mean(axis=0) for m in slots])
    got_z = _f64(zb[slots])
    assert max_rel_err(got_z, want_z) <= BF16_TOL
    # one rounding of an fp32 sum: half a bf16 step of the row's own scale, and some
    assert np.all(np.abs(got_z - want_z) <= 2.0 ** -8 * np.abs(want_z).max(axis=1, keepdims=True) + 1e-30)
    return slots


def _query_rows(M, rng, n_random=128):
    blocks = (M + 255) // 256
    whole = int(rng.integers(1, max(2, blocks - 1))) if blocks > 2 else 0
    rows = np.concatenate([np.arange(whole * 256, min(M, whole * 256 + 256)),
                           np.arange((blocks - 1) * 256, M),
                           rng.choice(M, size=min(n_random, M), replace=False)])
    return np.unique(rows)


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
    anchor_of = ib.anchor_of.cpu().numpy().astype(np.int64)
    n_near = _check_sampled_match(bits, dst_idx, src_idx, anchor_of,
                                  np.sort(rng.choice(pl.n_src, size=min(2048, pl.n_src), replace=False)))
    print(f"match: {n_near} near-tie differences on the sampled src rows", flush=True)
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

    # ---- merge: the largest groups and random slots
    sizes = np.diff(goff)
    zb = _host_bits(z)
    _check_sampled_merge(bits, zb, goff, gmem, rng)

    # ---- attention, all heads over all M keys (inputs: the GPU's z): one whole 256-query block
    # (every wave slot and lane half of a workgroup), the ragged last block, and random rows
    qrows = _query_rows(M, rng)
    yb = _host_bits(y)
    zf = _f64(zb).reshape(M, heads, 64)
    qk = O.round_bf16(O.qk_normalize(zf))
    want_y = O.attention(qk, qk, zf, rows=qrows).reshape(len(qrows), C)
    err = max_rel_err(_f64(yb[qrows]), want_y)
    print(f"attention bf16: {len(qrows)} rows x {heads} heads, max rel err {err:.3e}", flush=True)
    assert err <= BF16_TOL

    # ---- FP8 attention at the largest size: the same rows against exact attention
    if name == "f1000":
        p8 = hip_params(wl, attn_dtype=B.ATTN_FP8_E4M3)
        y8 = torch.empty_like(z)
        ws8 = B.alloc_ws(B.litevggt_attn_ws_bytes(p8, M))
        B.litevggt_global_attn(p8, M, z, z, z, y8, ws8)
        torch.cuda.synchronize()
        err8 = max_rel_err(_f64(_host_bits(y8)[qrows]), want_y)
        print(f"attention fp8: max rel err {err8:.3e}", flush=True)
        assert err8 <= 6e-2
        del y8, ws8
    del qk, want_y

    # ---- q, k as given (no qk_norm; per-wave score bound, second pass where it is loose), with a
    # softmax scale small enough that rows mix many keys: the same sampled rows (500 frames)
    if name == "f500":
        pn = hip_params(wl, qk_norm=0, softmax_scale=0.02)
        yn = torch.empty_like(z)
        B.litevggt_global_attn(pn, M, z, z, z, yn, B.alloc_ws(B.litevggt_attn_ws_bytes(pn, M)))
        torch.cuda.synchronize()
        ynb = _host_bits(yn)
        rows_n = qrows[::4]
        want_n = O.attention(zf, zf, zf, rows=rows_n, scale=0.02).reshape(len(rows_n), C)
        assert max_rel_err(_f64(ynb[rows_n]), want_n) <= BF16_TOL
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


@pytest.mark.parametrize("name", ["f100", "f1000"])
def test_full_size_later_refreshes_against_sampled_oracle(name, capsys):
    """The refreshes after layer 0 (Sec. 3.4 "Cached Token Merging": layers 6, 12, 18 of 24) see
    features the stack itself produced: heavy-tailed merge groups, near-duplicate rows.  The
    driver runs 6 and then 12 more layers on the whole sequence; the features entering layers 6
    and 18 are downloaded and one refresh + merge + attention on exactly those features is
    checked against the oracle (every sampled output depends on its own rows only, so the check
    is exact): score map and roles of sampled frames, 2048+ src rows against all dst rows
    (random rows, members of the largest groups, the rows most similar to their anchor), the
    merged rows of the 20 largest groups and 512 random slots, a whole query block of the
    attention."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2512_04939_amd import binding as B
    wl = synth.workload(name)
    po, ph = oracle_params(wl), hip_params(wl)
    pl = B.litevggt_plan(ph)
    F, T, P, C, heads = wl.frames, wl.tokens_per_frame, wl.patches, wl.dim, wl.heads
    N, M = pl.N, pl.M
    gen = synth.Generator(wl)
    x = torch.from_numpy(gen.tokens(threads=16).view(np.int16)).cuda().view(torch.bfloat16)
    im = torch.empty(F, 3, wl.img_h, wl.img_w, dtype=torch.float32, device="cuda")
    for f0 in range(0, F, 50):
        fr = range(f0, min(F, f0 + 50))
        im[f0:f0 + len(fr)].copy_(torch.from_numpy(gen.images(fr)))
    ib = B.alloc_index(pl)
    ws = B.alloc_ws(pl.ws_bytes)
    grad = torch.zeros(F, P, device="cuda")
    score = torch.zeros(F, P, device="cuda")
    best = torch.zeros(pl.n_src, device="cuda")
    z = torch.empty(M, C, dtype=torch.bfloat16, device="cuda")
    y = torch.empty_like(z)
    rng = np.random.default_rng(606)
    frames = np.array([0, 1, F // 3, F - 1])
    frame_rows = np.concatenate([np.arange(f * T, (f + 1) * T) for f in frames])
    psub = oracle_params(synth.Workload(**{**wl.__dict__, "frames": len(frames)}))
    images_sub = gen.images(frames)
    done = 0
    for more in (6, 12):
        log = B.litevggt_layers_run(ph, more, im, x, ib, grad, score, ws)
        assert log == O.refresh_schedule(more, 6)
        done += more
        # one refresh on the features entering layer `done`, by hand, gradient map cached
        B.litevggt_importance(ph, None, x, grad, False, score, ws)
        B.litevggt_select_anchors(ph, score, ib)
        B.litevggt_match(ph, x, ib, best, ws)
        B.litevggt_merge(ph, x, ib, z)
        B.litevggt_global_attn(ph, M, z, z, z, y, ws)
        torch.cuda.synchronize()
        bits = _host_bits(x)
        assert np.all(np.isfinite(synth.bf16_bits_to_f32(bits[frame_rows])))

        want, _ = O.importance(images_sub, _f64(bits[frame_rows]), psub)
        got = score[torch.from_numpy(frames).cuda()].cpu().numpy()
        assert np.abs(got.astype(np.float64) - want).max() <= 2e-5
        sel = O.select_anchors(got, psub)
        role = ib.role.cpu().numpy().reshape(F, T)
        assert np.array_equal(role[frames].ravel(), sel["role"])
        src_idx = ib.src_idx.cpu().numpy()[:pl.n_src].astype(np.int64)
        dst_idx = ib.dst_idx.cpu().numpy()[:pl.n_dst].astype(np.int64)
        assert np.array_equal(np.flatnonzero(role.ravel() == O.ROLE_SRC), src_idx)
        assert np.array_equal(np.flatnonzero(role.ravel() == O.ROLE_DST), dst_idx)

        anchor_of = ib.anchor_of.cpu().numpy().astype(np.int64)
        slot_of = ib.slot_of.cpu().numpy().astype(np.int64)
        goff = ib.group_off.cpu().numpy().astype(np.int64)
        gmem = ib.group_mem.cpu().numpy().astype(np.int64)
        sizes = np.diff(goff)
        assert goff[0] == 0 and goff[-1] == N and sizes.min() >= 1
        assert np.array_equal(slot_of[gmem], np.repeat(np.arange(M), sizes))
        assert np.array_equal(slot_of, slot_of[anchor_of])
        # src rows: random, members of the 20 largest groups, the most anchor-like rows
        src_pos = np.full(N, -1, dtype=np.int64)
        src_pos[src_idx] = np.arange(pl.n_src)
        largest = np.argsort(-sizes, kind="stable")[:20]
        members = np.concatenate([gmem[goff[m] + 1:goff[m + 1]] for m in largest])   # a group's first member is its anchor
        members = src_pos[members[src_pos[members] >= 0]]
        top = np.argsort(-best.cpu().numpy(), kind="stable")[:384]
        pick = np.unique(np.concatenate([rng.choice(pl.n_src, size=1024, replace=False),
                                         rng.choice(members, size=min(768, len(members)), replace=False), top]))
        with capsys.disabled():
            n_near = _check_sampled_match(bits, dst_idx, src_idx, anchor_of, pick, f"[{name}] layer {done}")
        zb = _host_bits(z)
        _check_sampled_merge(bits, zb, goff, gmem, rng)
        qrows = _query_rows(M, rng, n_random=32)
        zf = _f64(zb).reshape(M, heads, 64)
        qk = O.round_bf16(O.qk_normalize(zf))
        want_y = O.attention(qk, qk, zf, rows=qrows).reshape(len(qrows), C)
        err = max_rel_err(_f64(_host_bits(y)[qrows]), want_y)
        assert err <= BF16_TOL
        with capsys.disabled():
            print(f"\n[{name}] refresh on the features entering layer {done}: {len(pick)} src rows, {n_near} near-tie "
                  f"differences; largest group {sizes.max()}, {int((sizes > 64).sum())} groups > 64 hold "
                  f"{sizes[sizes > 64].sum() / N:.1%} of the tokens; attention max rel err {err:.2e}", flush=True)
        del zf, qk, want_y


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
