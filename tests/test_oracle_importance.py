"""Pins for the oracle's geometry-aware map (Sec. 3.4 "Geometry-aware Feature Map").

Each test checks the oracle against something fixed by mathematics or by an
independent library routine, never against the oracle's own formula.
"""
import numpy as np
import pytest
from scipy import ndimage

from oracle import litevggt_oracle as O


def _gray_to_rgb(g):
    return np.repeat(g[:, None], 3, axis=1)


def test_luma_weights_and_white():
    im = np.zeros((4, 3, 2, 2))
    im[0, 0] = 1.0
    im[1, 1] = 1.0
    im[2, 2] = 1.0
    im[3] = 1.0
    y = O.luma(im)
    assert np.allclose(y[0], 0.299) and np.allclose(y[1], 0.587) and np.allclose(y[2], 0.114)
    assert np.allclose(y[3], 1.0)      # the three weights sum to one


def test_sobel_constant_is_zero():
    g = np.full((2, 9, 11), 0.37)
    assert np.all(O.sobel_magnitude(g) < 1e-15)


@pytest.mark.parametrize("a", [0.01, -0.03])
def test_sobel_ramp_closed_form(a):
    # I = a*col: horizontal derivative kernel sums to (1+2+1)*2a = 8a, vertical response 0
    g = (a * np.arange(12, dtype=np.float64))[None, None, :].repeat(10, axis=1)
    m = O.sobel_magnitude(g)
    assert np.allclose(m[:, :, 1:-1], 8 * abs(a), rtol=0, atol=1e-15)
    # replicated border halves the horizontal difference there
    assert np.allclose(m[:, :, 0], 4 * abs(a)) and np.allclose(m[:, :, -1], 4 * abs(a))
    # transposed ramp exercises the vertical kernel
    mt = O.sobel_magnitude(np.swapaxes(g, 1, 2))
    assert np.allclose(mt[:, 1:-1, :], 8 * abs(a))


def test_sobel_step_edge():
    delta = 0.25
    g = np.zeros((1, 8, 10))
    g[:, :, 5:] = delta
    m = O.sobel_magnitude(g)
    expect = np.zeros(10)
    expect[4] = expect[5] = 4 * delta
    assert np.allclose(m[0], expect[None, :])


def test_sobel_rotation_equivariance():
    rng = np.random.default_rng(1)
    g = rng.random((1, 12, 12))
    m = O.sobel_magnitude(g)
    mr = O.sobel_magnitude(np.rot90(g, 1, axes=(1, 2)).copy())
    assert np.allclose(np.rot90(m, 1, axes=(1, 2)), mr, atol=1e-14)


def test_sobel_against_scipy():
    rng = np.random.default_rng(2)
    g = rng.random((3, 17, 23))
    m = O.sobel_magnitude(g)
    for f in range(3):
        gx = ndimage.sobel(g[f], axis=1, mode="nearest")
        gy = ndimage.sobel(g[f], axis=0, mode="nearest")
        assert np.allclose(m[f], np.hypot(gx, gy), atol=1e-13)


def test_grad_map_is_patch_mean():
    rng = np.random.default_rng(3)
    im = rng.random((2, 3, 28, 42))
    pg = O.grad_map(im, 14)
    assert pg.shape == (2, 2, 3)
    mag = O.sobel_magnitude(O.luma(im))
    assert np.allclose(pg.sum(axis=(1, 2)) * 196, mag.sum(axis=(1, 2)))
    assert np.allclose(pg[1, 1, 2], mag[1, 14:28, 28:42].mean())
    with pytest.raises(ValueError):
        O.grad_map(im[:, :, :27], 14)


def _params(F, H, W, C, **kw):
    return O.Params(frames=F, grid_h=H, grid_w=W, dim=C, heads=1, head_dim=C, **kw)


def _tokens_from_grid(grid, S):
    """[F,H,W,C] grid -> [N,C] with S random special tokens per frame in front."""
    F, H, W, C = grid.shape
    rng = np.random.default_rng(9)
    sp = 100.0 * rng.standard_normal((F, S, C))     # loud: must not leak into the map
    return np.concatenate([sp, grid.reshape(F, H * W, C)], axis=1).reshape(-1, C)


def test_var_map_constant_zero():
    p = _params(2, 5, 6, 8)
    x = _tokens_from_grid(np.full((2, 5, 6, 8), 1.7), p.n_special)
    assert np.allclose(O.var_map(x, p), 0.0, atol=1e-15)


def test_var_map_checkerboard_closed_form():
    H, W, C = 7, 8, 3
    i, j = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    cb = np.where((i + j) % 2 == 0, 1.0, -1.0)
    grid = np.repeat(cb[None, :, :, None], C, axis=3)
    p = _params(1, H, W, C)
    v = O.var_map(_tokens_from_grid(grid, p.n_special), p)[0]
    # interior 3x3 window: five of one sign, four of the other -> mean +-1/9, E[x^2] = 1
    assert np.allclose(v[1:-1, 1:-1], 1 - (1 / 9) ** 2)
    # 2x2 corner and 2x3 edge windows are balanced -> variance 1
    assert np.allclose(v[0, 0], 1.0) and np.allclose(v[0, 3], 1.0) and np.allclose(v[3, 0], 1.0)


def test_var_map_against_uniform_filter():
    rng = np.random.default_rng(4)
    F, H, W, C = 2, 6, 9, 5
    grid = rng.standard_normal((F, H, W, C))
    p = _params(F, H, W, C)
    v = O.var_map(_tokens_from_grid(grid, p.n_special), p)
    ones = ndimage.uniform_filter(np.ones((H, W)), size=3, mode="constant")
    for f in range(F):
        acc = np.zeros((H, W))
        for c in range(C):
            mu = ndimage.uniform_filter(grid[f, :, :, c], size=3, mode="constant") / ones
            nu = ndimage.uniform_filter(grid[f, :, :, c] ** 2, size=3, mode="constant") / ones
            acc += np.maximum(nu - mu * mu, 0)
        assert np.allclose(v[f], acc / C, atol=1e-12)


def test_var_map_bruteforce_neighbours():
    rng = np.random.default_rng(5)
    H, W, C = 4, 5, 2
    grid = rng.standard_normal((1, H, W, C))
    p = _params(1, H, W, C)
    v = O.var_map(_tokens_from_grid(grid, p.n_special), p)[0]
    for i in range(H):
        for j in range(W):
            tot = 0.0
            for c in range(C):
                vals = [grid[0, a, b, c] for a in range(i - 1, i + 2) for b in range(j - 1, j + 2)
                        if 0 <= a < H and 0 <= b < W]
                tot += np.var(vals)                     # population variance
            assert abs(v[i, j] - tot / C) < 1e-12


def test_var_map_shift_equivariant_interior():
    rng = np.random.default_rng(6)
    H, W, C = 8, 10, 3
    big = rng.standard_normal((1, H, W + 2, C))
    p = _params(1, H, W, C)
    va = O.var_map(_tokens_from_grid(big[:, :, :W], p.n_special), p)[0]
    vb = O.var_map(_tokens_from_grid(big[:, :, 2:], p.n_special), p)[0]
    assert np.allclose(va[:, 3:-1], vb[:, 1:-3])


def test_minmax_norm_and_fusion_range():
    rng = np.random.default_rng(7)
    m = rng.random((3, 4, 5)) * 10 - 3
    m[2] = 4.0                                           # flat frame
    n = O.minmax_norm(m)
    assert np.all(n[:2].reshape(2, -1).min(axis=1) == 0.0)
    assert np.all(n[:2].reshape(2, -1).max(axis=1) == 1.0)
    assert np.all(n[2] == 0.0)
    # order preserving inside a frame
    assert np.array_equal(np.argsort(m[0].ravel(), kind="stable"),
                          np.argsort(n[0].ravel(), kind="stable"))
    p = _params(3, 4, 5, 1, alpha=0.3, beta=0.6)
    s = O.ga_map(m, m[::-1].copy(), p)
    assert s.min() >= 0.0 and s.max() <= 0.9 + 1e-15
    # pure gradient weighting reproduces the normalised gradient map
    p1 = _params(3, 4, 5, 1, alpha=1.0, beta=0.0)
    assert np.allclose(O.ga_map(m, rng.random((3, 4, 5)), p1), n)


def test_importance_caches_gradient_and_ignores_specials():
    rng = np.random.default_rng(8)
    F, H, W, C = 2, 3, 4, 6
    p = _params(F, H, W, C, patch=2)
    im = rng.random((F, 3, H * 2, W * 2))
    grid = rng.standard_normal((F, H, W, C))
    x = _tokens_from_grid(grid, p.n_special)
    s1, pg = O.importance(im, x, p)
    s2, _ = O.importance(None, x, p, psi_g=pg)
    assert np.array_equal(s1, s2) and s1.shape == (F, H * W)
    x2 = x.copy().reshape(F, -1, C)
    x2[:, :p.n_special] = 0.0
    s3, _ = O.importance(im, x2.reshape(-1, C), p)
    assert np.array_equal(s1, s3)
