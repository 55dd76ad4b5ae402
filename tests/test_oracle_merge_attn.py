"""Pins for the oracle's merge, attention core, unmerge, storage rounding and the
cached-index layer loop (Sec. 3.4 merge equation, "Token Unmerging", "Cached Token
Merging"; Sec. 3.1 for the full-sequence attention)."""
import os

import numpy as np
import pytest
import scipy.sparse as sp
import torch

from oracle import litevggt_oracle as O
from paper_2512_04939_amd import synth


def _small_index(seed=31, F=3, G=6, C=8, r=0.6):
    rng = np.random.default_rng(seed)
    p = O.Params(frames=F, grid_h=G, grid_w=G, dim=C, heads=2, head_dim=C // 2, merge_ratio=r)
    score = rng.random((F, G * G)).astype(np.float32)
    sel = O.select_anchors(score, p)
    x = rng.standard_normal((p.n_tokens, C)).astype(np.float32)
    m = O.match(x, sel["dst_idx"], sel["src_idx"])
    idx = O.build_index(sel["role"], sel["src_idx"], m["anchor"])
    idx.update(role=sel["role"])
    return p, x, idx


def test_merge_equation_by_hand():
    # anchor 0 with sources 2 and 3; token 1 kept alone
    x = np.array([[1.0, 10.0], [5.0, 5.0], [2.0, 20.0], [6.0, 0.0]])
    off = np.array([0, 3, 4])
    mem = np.array([0, 2, 3, 1])
    z = O.merge(x, off, mem)
    assert np.allclose(z[0], [(1 + 2 + 6) / 3, (10 + 20 + 0) / 3])
    assert np.array_equal(z[1], x[1])


def test_merge_conservation_and_sparse_matrix():
    p, x, idx = _small_index()
    z = O.merge(x, idx["group_off"], idx["group_mem"])
    sizes = np.diff(idx["group_off"])
    assert np.allclose((sizes[:, None] * z).sum(axis=0), x.astype(np.float64).sum(axis=0))
    # independent formulation: averaging matrix A[m, i] = 1/size_m if slot_of[i] == m
    N, M = len(idx["slot_of"]), len(sizes)
    A = sp.csr_matrix((1.0 / sizes[idx["slot_of"]], (idx["slot_of"], np.arange(N))), shape=(M, N))
    assert np.allclose(z, A @ x.astype(np.float64), atol=1e-13)
    # groups of one copy the row exactly
    single = np.flatnonzero(sizes == 1)
    assert np.array_equal(z[single], x[idx["kept_idx"][single]].astype(np.float64))


def test_merge_unmerge_identity_without_merging():
    p, x, idx = _small_index(r=0.0)
    assert len(idx["kept_idx"]) == p.n_tokens
    z = O.merge(x, idx["group_off"], idx["group_mem"])
    assert np.array_equal(z, x.astype(np.float64))
    assert np.array_equal(O.unmerge(z, idx["slot_of"]), x.astype(np.float64))


def test_unmerge_replicates_anchor_rows():
    p, x, idx = _small_index()
    M = len(idx["kept_idx"])
    y = np.random.default_rng(32).standard_normal((M, 8))
    u = O.unmerge(y, idx["slot_of"])
    assert np.array_equal(u[idx["kept_idx"]], y)                 # anchors get their own row
    for i in np.flatnonzero(idx["role"] == O.ROLE_SRC):
        assert np.array_equal(u[i], u[idx["anchor_of"][i]])
    res = np.ones((p.n_tokens, 8))
    assert np.array_equal(O.unmerge(y, idx["slot_of"], res), u + 1.0)


# ------------------------------------------------------------------------------ attention
def _naive_attention(q, k, v):
    M, h, d = q.shape
    out = np.zeros((M, h, d))
    for hh in range(h):
        for i in range(M):
            w = [np.exp(sum(q[i, hh, c] * k[j, hh, c] for c in range(d)) / np.sqrt(d))
                 for j in range(M)]
            tot = sum(w)
            for j in range(M):
                out[i, hh] += (w[j] / tot) * v[j, hh]
    return out


def test_attention_naive_loops():
    q, k, v = (a.astype(np.float64) for a in synth.random_qkv(7, 2, 4, seed=41))
    assert np.allclose(O.attention(q, k, v), _naive_attention(q, k, v), atol=1e-12)


def test_attention_against_torch_sdpa():
    q, k, v = synth.random_qkv(150, 3, 16, seed=42, scale=1.5)
    o = O.attention(q, k, v)
    tq, tk, tv = (torch.from_numpy(a.astype(np.float64)).permute(1, 0, 2)[None] for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0].permute(1, 0, 2).numpy()
    assert np.allclose(o, ref, atol=1e-12)
    rows = np.array([3, 77, 149])
    assert np.allclose(O.attention(q, k, v, rows=rows), ref[rows], atol=1e-12)


def test_attention_special_cases():
    q, k, v = synth.random_qkv(33, 2, 8, seed=43)
    ones = np.ones_like(v)
    assert np.allclose(O.attention(q, k, ones), 1.0, atol=1e-14)       # weights sum to one
    const = np.broadcast_to(np.arange(8.0), v.shape)
    assert np.allclose(O.attention(q, k, const), const, atol=1e-13)
    vmean = v.astype(np.float64).mean(axis=0, keepdims=True).repeat(33, axis=0)
    assert np.allclose(O.attention(np.zeros_like(q), k, v), vmean, atol=1e-13)   # uniform weights
    assert np.allclose(O.attention(q[:1], k[:1], v[:1]), v[:1])        # one token attends to itself
    # huge logits do not overflow (max subtraction)
    assert np.all(np.isfinite(O.attention(300 * q, k, v)))


def test_qk_normalize_against_torch_rms_norm():
    q, _, _ = synth.random_qkv(50, 3, 64, seed=44, scale=3.0)
    n = O.qk_normalize(q)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(q.astype(np.float64)), (64,), eps=1e-6).numpy()
    assert np.allclose(n, ref, atol=1e-13)
    assert np.allclose((n * n).mean(axis=-1), 1.0, atol=1e-5)          # unit RMS per head
    assert np.allclose(O.qk_normalize(1000.0 * q), n, atol=1e-6)       # scale invariant
    assert np.all(O.qk_normalize(np.zeros((2, 1, 64))) == 0.0)


def test_layer_with_qk_norm_stays_bounded_over_depth():
    p, x, im = _tiny_problem(0.5, interval=6, layers=12)
    pq = p.__class__(**{**p.__dict__, "qk_norm": True})
    out, _ = O.layers_run(im, x, pq, 12, store=O.round_bf16)
    assert np.all(np.isfinite(out))
    # every layer adds a convex combination of merged rows: at most a doubling per layer
    assert np.abs(out).max() <= 2.0 ** 12 * np.abs(x).max()


def test_attention_fp8_emulation_properties():
    # inputs that E4M3 holds exactly (small integers, amax 448 * 2^-5 = 14) and unquantised
    # weights: the emulation must reproduce exact attention
    rng = np.random.default_rng(45)
    q = rng.integers(-3, 4, size=(40, 2, 16)).astype(np.float64)
    k = rng.integers(-3, 4, size=(40, 2, 16)).astype(np.float64)
    v = rng.integers(-7, 8, size=(40, 2, 16)).astype(np.float64)
    for a in (q, k, v):
        a[0, 0, 0] = 14.0
    assert np.allclose(O.attention_fp8(q, k, v, quantize_p=False), O.attention(q, k, v), atol=1e-12)
    codes, sc = O.quantize_e4m3(v)
    assert sc == 14.0 / 448.0 and np.array_equal(codes * sc, v)
    # with everything quantised the result stays within the FP8 budget of the exact one and
    # the weights still form a convex combination (constant V is reproduced up to its own rounding)
    q, k, v = synth.random_qkv(200, 2, 64, seed=46)
    exact = O.attention(q, k, v)
    emu = O.attention_fp8(q, k, v)
    assert np.abs(emu - exact).max() / np.abs(exact).max() < 6e-2
    const = np.full_like(v, 1.75)
    assert np.abs(O.attention_fp8(q, k, const) - 1.75).max() < 0.05


# -------------------------------------------------------------------------------- rounding
def test_round_bf16_matches_torch():
    rng = np.random.default_rng(51)
    a = np.concatenate([rng.standard_normal(5000) * 10 ** rng.uniform(-6, 6, 5000),
                        [0.0, 1.0, 1.00390625, 1.01171875, -3.0e38]]).astype(np.float32)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.round_bf16(a), ref)
    bits = synth.f32_to_bf16_bits(a)
    assert np.array_equal(synth.bf16_bits_to_f32(bits).astype(np.float64), ref)


def test_attention_fp8_bounded_emulation_properties():
    """Fixed-reference FP8 emulation: weights sum to one exactly (constant V comes back up to its
    own quantisation, whatever the scores), close to exact attention on peaked rows, and rows
    whose scores all sit far below the bound fall back to the running-maximum emulation."""
    rng = np.random.default_rng(61)
    n, h = 300, 2
    q = O.round_bf16(O.qk_normalize(rng.standard_normal((n, h, 64))))
    k = O.round_bf16(O.qk_normalize(q + 0.3 * rng.standard_normal((n, h, 64))))
    v = rng.standard_normal((n, h, 64))
    const = np.broadcast_to(rng.standard_normal((1, h, 64)), (n, h, 64))
    c8, sc = O.quantize_e4m3(const)
    assert np.allclose(O.attention_fp8_bounded(q, k, const), c8 * sc, rtol=1e-12, atol=1e-12)
    got, exact = O.attention_fp8_bounded(q, k, v), O.attention(q, k, v)
    assert 1e-4 < np.abs(got - exact).max() / np.abs(exact).max() < 6e-2
    # every key near one direction and the queries opposite to it: every score near -64 * scale,
    # 2^-24 of the reference: nothing is representable and all rows take the other emulation
    u = rng.standard_normal((1, h, 64))
    kk = O.round_bf16(O.qk_normalize(u + 0.1 * rng.standard_normal((n, h, 64))))
    qq = O.round_bf16(O.qk_normalize(-u + 0.1 * rng.standard_normal((n, h, 64))))
    assert np.array_equal(O.attention_fp8_bounded(qq, kk, v), O.attention_fp8(qq, kk, v))
    assert not np.array_equal(O.attention_fp8_bounded(q, k, v), O.attention_fp8(q, k, v))
    # the bound itself: unit-RMS rows rounded to bf16 and then to E4M3 cannot exceed it
    worst = 64.0 * (1 + 2.0 ** -8) ** 2 * (1 + 2.0 ** -4) ** 2
    assert worst < O.FP8_SCORE_BOUND and 2.0 ** O.FP8_WEIGHT_TOP < 448.0


def test_round_e4m3_matches_torch():
    rng = np.random.default_rng(52)
    a = np.concatenate([rng.standard_normal(5000) * 10 ** rng.uniform(-4, 2.5, 5000),
                        [0.0, 448.0, 464.0, 1000.0, -1000.0, 2.0 ** -9, 2.0 ** -10, 1.5 * 2.0 ** -9,
                         0.0625, 17.0, 18.0, 19.0]]).astype(np.float32)
    clipped = np.clip(a, -448.0, 448.0)
    ref = torch.from_numpy(clipped).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(O.round_e4m3(a), ref)


# ---------------------------------------------------------------------------- FP8 linear layers
def test_linear_fp8_matches_torch_float8_casts():
    """Independent rounding (torch's float8_e4m3fn cast) and an independent product."""
    rng = np.random.default_rng(53)
    x = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(rng.standard_normal((37, 96)).astype(np.float32) * 3))
    w = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(rng.standard_normal((24, 96)).astype(np.float32) * 0.1))
    b = rng.standard_normal(24)
    ix = np.float32(448.0) / np.abs(x).max()
    iw = np.float32(448.0) / np.abs(w).max()
    x8 = (torch.from_numpy(x) * float(ix)).to(torch.float8_e4m3fn).to(torch.float64)
    w8 = (torch.from_numpy(w) * float(iw)).to(torch.float8_e4m3fn).to(torch.float64)
    ref = (torch.einsum("nk,ok->no", x8, w8) / float(ix) / float(iw)).numpy() + b
    got = O.linear_fp8(x, w, b)
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)
    # and it is a small perturbation of the exact layer (3 mantissa bits on both operands)
    exact = O.linear(x, w, b)
    assert 1e-4 < np.abs(got - exact).max() / np.abs(exact).max() < 4e-2


def test_linear_fp8_is_exact_on_representable_operands():
    """Operands on the E4M3 grid with amax 448 (scale 1) lose nothing."""
    rng = np.random.default_rng(54)
    grid = np.array([0, 0.25, 1, 1.5, 3, 10, 14, 28, 120, 208, 448], dtype=np.float64)
    x = rng.choice(grid, size=(9, 32)) * rng.choice([-1, 1], size=(9, 32))
    w = rng.choice(grid, size=(5, 32)) * rng.choice([-1, 1], size=(5, 32))
    x[0, 0], w[0, 0] = 448.0, -448.0
    b = rng.standard_normal(5)
    assert np.array_equal(O.linear_fp8(x, w, b), O.linear(x, w, b))
    # a transposed weight or a dropped bias would show
    assert O.linear_fp8(x, w, b).shape == (9, 5)


def test_fp8_delayed_scaling_history():
    """Scale from the largest amax of the previous <= 80 steps; 1 before anything is recorded."""
    w = np.array([[448.0]])
    b = np.zeros(1)
    h = O.Fp8History()
    # step 0: empty history -> scale 1: 1000 saturates at 448, 3.2 rounds to 3.25 (step 0.25 in [2, 4))
    y = O.linear_fp8(np.array([[1000.0], [3.2]]), w, b, h)
    assert np.array_equal(y.ravel(), [448.0 * 448.0, 3.25 * 448.0])
    assert h.step == 1 and h.hist[0] == 1000.0
    # step 1: scale from amax 1000: 1000 would be exact, 500 -> code 224 exactly
    y = O.linear_fp8(np.array([[500.0]]), w, b, h)
    inv = np.float32(448.0) / np.float32(1000.0)
    assert np.isclose(y[0, 0], 224.0 / float(inv) * 448.0, rtol=1e-12)
    # the window: amax t+1 at steps 1 + t; at step 100 the last 80 recorded amaxes are 20 .. 99
    h = O.Fp8History()
    for t in range(100):
        assert h.amax() == (0 if t == 0 else max(range(max(0, t - 80), t)) + 1)
        O.linear_fp8(np.array([[float(t + 1)]]), w, b, h)
    # a large amax is forgotten after 80 further steps, not earlier
    h = O.Fp8History()
    O.linear_fp8(np.array([[4480.0]]), w, b, h)
    for t in range(80):
        assert h.amax() == 4480.0
        O.linear_fp8(np.array([[1.0]]), w, b, h)
    assert h.amax() == 1.0
    # current scaling ignores all of it
    assert np.isclose(O.linear_fp8(np.array([[1000.0]]), w, b)[0, 0], 1000.0 * 448.0, rtol=1e-6)


def test_global_block_fp8_linear_is_close_to_exact_block():
    wl = synth.Workload("b8", frames=2, grid_h=4, grid_w=4, dim=256, heads=4, merge_ratio=0.0, seed=71)
    from helpers import oracle_params
    wts = {k: (synth.bf16_bits_to_f32(v).astype(np.float64) if v.dtype == np.uint16 else v.astype(np.float64))
           for k, v in synth.block_weights(wl.dim, seed=3).items()}
    z = synth.bf16_bits_to_f32(synth.Generator(wl).tokens()).astype(np.float64)
    exact = O.global_block(z, wts, oracle_params(wl, qk_norm=True))
    cur = O.global_block(z, wts, oracle_params(wl, qk_norm=True, linear_fp8=True))
    err = np.abs(cur - exact).max() / np.abs(exact).max()
    assert 1e-4 < err < 6e-2
    # delayed scaling: the first step runs at scale 1 everywhere (coarse or saturated where
    # the tensor's range is far from 448); later steps use the recorded amaxes and are close again
    p8 = oracle_params(wl, qk_norm=True, linear_fp8=True, fp8_history=[O.Fp8History() for _ in range(4)])
    first = O.global_block(z, wts, p8)
    assert not np.array_equal(first, cur)
    for _ in range(2):
        later = O.global_block(z, wts, p8)
    assert np.abs(later - exact).max() / np.abs(exact).max() < 6e-2
    assert [h.step for h in p8.fp8_history] == [3, 3, 3, 3]
    # the first layer's input does not depend on earlier quantisation: its recorded amax is the tensor's
    h1 = O.layer_norm(z, wts["ln1_g"], wts["ln1_b"])
    assert np.all(p8.fp8_history[0].hist[:3] == np.float32(np.abs(h1.astype(np.float32)).max()))

# ---------------------------------------------------------------------------- layer driver
def test_refresh_schedule_matches_paper_table(golden_dir):
    rows = [tuple(int(v) for v in ln.split()) for ln in open(os.path.join(golden_dir, "recompute_counts.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert (6, 4) in rows
    for interval, total in rows:
        log = O.refresh_schedule(24, interval)
        assert sum(log) == total and log[0] == 1
    assert O.refresh_schedule(24, 6) == [1, 0, 0, 0, 0, 0] * 4


def _tiny_problem(r, interval=6, layers=2):
    wl = synth.workload("tiny2", merge_ratio=r, refresh_interval=interval, layers=layers)
    gen = synth.Generator(wl)
    x = synth.stored_to_f32(gen.tokens())
    im = gen.images()
    p = O.Params(frames=wl.frames, grid_h=wl.grid_h, grid_w=wl.grid_w, dim=wl.dim, heads=wl.heads,
                 head_dim=wl.head_dim, merge_ratio=r, refresh_interval=interval)
    return p, x, im


def test_layer_with_ratio_zero_is_plain_attention():
    p, x, im = _tiny_problem(0.0)
    idx, *_ = O.compute_index(im, x, p)
    out = O.global_layer(x, idx, p)
    xx = x.astype(np.float64).reshape(-1, p.heads, p.head_dim)
    assert np.allclose(out, x + O.attention(xx, xx, xx).reshape(x.shape), atol=1e-12)


def test_layers_run_schedule_and_cache_reuse():
    p, x, im = _tiny_problem(0.5, interval=2, layers=4)
    trace = []
    out, log = O.layers_run(im, x, p, 4, trace=trace)
    assert log == [1, 0, 1, 0]
    assert trace[1]["index"] is trace[0]["index"] and trace[3]["index"] is trace[2]["index"]
    assert trace[2]["index"] is not trace[0]["index"]
    # interval 1 recomputes every layer; an interval beyond the depth computes once
    assert O.layers_run(im, x, p.__class__(**{**p.__dict__, "refresh_interval": 1}), 3)[1] == [1, 1, 1]
    assert O.layers_run(im, x, p.__class__(**{**p.__dict__, "refresh_interval": 99}), 3)[1] == [1, 0, 0]
    # group sizes always cover every token
    for t in trace:
        assert np.diff(t["index"]["group_off"]).sum() == p.n_tokens


def test_refresh_on_unchanged_features_reproduces_index():
    p, x, im = _tiny_problem(0.5)
    a, pg, *_ = O.compute_index(im, x, p)
    b, *_ = O.compute_index(None, x, p, psi_g=pg)
    for k in ("role", "anchor_of", "slot_of", "group_off", "group_mem", "kept_idx"):
        assert np.array_equal(a[k], b[k])
    # the plan's counts are what the partition produces on real scores
    pl = O.plan(p)
    assert len(a["kept_idx"]) == pl["M"] and len(a["src_idx"]) == pl["n_src"]
    assert len(a["dst_idx"]) == pl["n_dst"]


# ---------------------------------------------------------------------------
# frame attention (Sec. 3.1)
# ---------------------------------------------------------------------------
def test_frame_attention_is_block_diagonal_attention():
    rng = np.random.default_rng(3)
    p = O.Params(frames=3, grid_h=2, grid_w=3, n_special=1, dim=128, heads=2)
    T, N = p.tokens_per_frame, p.n_tokens
    q, k, v = (rng.standard_normal((N, 2, 64)) for _ in range(3))
    got = O.frame_attention(q, k, v, p)
    # the same thing written as one masked softmax over the whole sequence
    frame = np.arange(N) // T
    for h in range(2):
        s = (q[:, h] @ k[:, h].T) / 8.0
        s[frame[:, None] != frame[None, :]] = -np.inf
        w = np.exp(s - s.max(axis=1, keepdims=True))
        w /= w.sum(axis=1, keepdims=True)
        assert np.abs(got[:, h] - w @ v[:, h]).max() < 1e-12
    # one frame: the plain attention; other frames' tokens do not matter
    p1 = O.Params(frames=1, grid_h=2, grid_w=3, n_special=1, dim=128, heads=2)
    assert np.array_equal(O.frame_attention(q[:T], k[:T], v[:T], p1), O.attention(q[:T], k[:T], v[:T]))
    k2, v2 = k.copy(), v.copy()
    k2[T:], v2[T:] = rng.standard_normal(k[T:].shape), rng.standard_normal(v[T:].shape)
    assert np.array_equal(O.frame_attention(q, k2, v2, p)[:T], got[:T])


def test_frame_attention_against_torch_sdpa_per_frame():
    import torch
    rng = np.random.default_rng(4)
    p = O.Params(frames=2, grid_h=3, grid_w=3, n_special=5, dim=128, heads=2)
    T = p.tokens_per_frame
    q, k, v = (rng.standard_normal((2 * T, 2, 64)) for _ in range(3))
    got = O.frame_attention(q, k, v, p)
    for f in range(2):
        tq, tk, tv = (torch.from_numpy(a[f * T:(f + 1) * T]).permute(1, 0, 2) for a in (q, k, v))
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).permute(1, 0, 2).numpy()
        assert np.abs(got[f * T:(f + 1) * T] - ref).max() < 1e-12


def test_frame_layer_is_residual_plus_frame_attention():
    rng = np.random.default_rng(5)
    p = O.Params(frames=2, grid_h=2, grid_w=2, n_special=1, dim=64, heads=1, qk_norm=True)
    x = rng.standard_normal((p.n_tokens, 64))
    xx = x.reshape(-1, 1, 64)
    qk = O.qk_normalize(xx)
    want = x + O.frame_attention(qk, qk, xx, p).reshape(x.shape)
    assert np.array_equal(O.frame_layer(x, p), want)
    # constant value rows inside a frame: attention returns them, the layer doubles them
    xc = np.repeat(rng.standard_normal((2, 1, 64)), p.tokens_per_frame, axis=0).reshape(-1, 64)
    assert np.abs(O.frame_layer(xc, p) - 2 * xc).max() < 1e-12


# ---------------------------------------------------------------------------
# the transformer block around the global attention
# ---------------------------------------------------------------------------
def test_layer_norm_gelu_linear_against_torch():
    import torch
    rng = np.random.default_rng(6)
    x = rng.standard_normal((7, 96)) * 3 + 1
    g, b = rng.standard_normal(96), rng.standard_normal(96)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (96,), torch.from_numpy(g),
                                         torch.from_numpy(b), eps=O.LN_EPS).numpy()
    assert np.abs(O.layer_norm(x, g, b) - ref).max() < 1e-12
    y = O.layer_norm(x, np.ones(96), np.zeros(96))
    assert np.abs(y.mean(axis=1)).max() < 1e-12 and np.abs(y.var(axis=1) - 1).max() < 1e-5
    assert np.abs(O.gelu(x) - torch.nn.functional.gelu(torch.from_numpy(x)).numpy()).max() < 1e-12
    assert O.gelu(np.array([0.0]))[0] == 0 and abs(O.gelu(np.array([10.0]))[0] - 10) < 1e-12
    w, bias = rng.standard_normal((5, 96)), rng.standard_normal(5)
    ref = torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(bias)).numpy()
    assert np.abs(O.linear(x, w, bias) - ref).max() < 1e-12


def test_global_block_against_a_torch_block():
    """The block assembled from torch modules with the same weights (float64)."""
    import torch
    C, heads, n = 128, 2, 37
    w = {k: v.astype(np.float64) for k, v in synth.block_weights(C, seed=3).items()}
    rng = np.random.default_rng(7)
    z = rng.standard_normal((n, C))
    p = O.Params(frames=1, grid_h=1, grid_w=1, dim=C, heads=heads)
    t = {k: torch.from_numpy(v) for k, v in w.items()}
    zt = torch.from_numpy(z)
    h = torch.nn.functional.layer_norm(zt, (C,), t["ln1_g"], t["ln1_b"], eps=O.LN_EPS)
    q, k, v = torch.nn.functional.linear(h, t["w_qkv"], t["b_qkv"]).chunk(3, dim=1)
    sp = lambda a: a.reshape(n, heads, 64).permute(1, 0, 2)
    a = torch.nn.functional.scaled_dot_product_attention(sp(q), sp(k), sp(v)).permute(1, 0, 2).reshape(n, C)
    u1 = torch.nn.functional.linear(a, t["w_o"], t["b_o"])
    h2 = torch.nn.functional.layer_norm(zt + u1, (C,), t["ln2_g"], t["ln2_b"], eps=O.LN_EPS)
    u2 = torch.nn.functional.linear(torch.nn.functional.gelu(torch.nn.functional.linear(h2, t["w_1"], t["b_1"])),
                                    t["w_2"], t["b_2"])
    assert np.abs(O.global_block(z, w, p) - (u1 + u2).numpy()).max() < 1e-11
    # q, k normalisation enters only through the attention inputs
    pn = O.Params(frames=1, grid_h=1, grid_w=1, dim=C, heads=heads, qk_norm=True)
    assert np.abs(O.global_block(z, w, pn) - O.global_block(z, w, p)).max() > 1e-6


def test_block_layer_at_ratio_zero_is_the_block_on_the_unmerged_sequence():
    wl = synth.workload("tiny2", merge_ratio=0.0)
    p = O.Params(frames=wl.frames, grid_h=16, grid_w=16, dim=256, heads=4, merge_ratio=0.0,
                 block={k: v.astype(np.float64) for k, v in synth.block_weights(256, 1).items()})
    gen = synth.Generator(wl)
    x, im = synth.stored_to_f32(gen.tokens()).astype(np.float64), gen.images()
    idx = O.compute_index(im, x, p)[0]
    assert np.abs(O.global_layer(x, idx, p) - (x + O.global_block(x, p.block, p))).max() < 1e-12
