"""Pins for the fp64 oracle: each check ties an oracle function to something
other than itself (a library routine, a brute-force construction written
independently here, a closed form, an invariant, finite differences)."""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import oracle
import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))


def rng(seed=0):
    return np.random.default_rng(seed)


# ----------------------------------------------------------------- geometry
def test_geometry_from_paper_fixture():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "geometry.txt")) if l.strip() and l[0] != "#"]
    for H, R, S, side, locs, K, outs in [[int(v) for v in r] for r in rows]:
        g = wl.LCGeom(B=1, H=H, W=H, C=3, R=R, S=S, F=outs)
        assert oracle.n_loc(H, R, S) == side == g.LH
        assert g.L == locs and g.K == K
        assert g.params == 5184 * 768 * 384 == 1_528_823_808


def test_benchmark_param_counts():
    assert wl.CONFIG_GEOM["cfg3"].params == 81_254_400
    assert wl.CONFIG_GEOM["cfg4"].params == 220_463_104
    assert wl.CONFIG_GEOM["cfg3"].L == 2116 and wl.CONFIG_GEOM["cfg4"].L == 841
    # stage chaining of the three-stage workload: LC valid -> pool valid -> LCN same
    s1, s2, s3 = (wl.CONFIG_GEOM[k] for k in ("cfg5_s1", "cfg5_s2", "cfg5_s3"))
    assert (s1.LH - 2, s1.F) == (s2.H, s2.C) and (s2.LH - 2, s2.F) == (s3.H, s3.C)


# ------------------------------------------------- brute-force dense operator
def dense_operator(H, W, C, R, S, F, w):
    """M[(i,j,f),(row,col,c)] of the layer, built entry by entry."""
    LH, LW = (H - R) // S + 1, (W - R) // S + 1
    M = np.zeros((LH * LW * F, H * W * C))
    for i in range(LH):
        for j in range(LW):
            for f in range(F):
                for kh in range(R):
                    for kw in range(R):
                        for c in range(C):
                            k = (kh * R + kw) * C + c
                            M[(i * LW + j) * F + f, ((i * S + kh) * W + j * S + kw) * C + c] = w[i, j, k, f]
    return M


TINY = [
    (3, 7, 7, 2, 3, 2, 3),    # exact cover
    (2, 8, 9, 3, 3, 2, 4),    # floor geometry: trailing row/col covered by no field
    (2, 6, 5, 1, 2, 3, 2),    # stride larger than field: gaps between fields
]


@pytest.mark.parametrize("g", TINY)
def test_forward_and_backward_data_match_dense_operator(g):
    B, H, W, C, R, S, F = g
    LH, LW = (H - R) // S + 1, (W - R) // S + 1
    r = rng(1)
    x = r.standard_normal((B, H, W, C))
    w = r.standard_normal((LH, LW, R * R * C, F))
    dy = r.standard_normal((B, LH, LW, F))
    bias = r.standard_normal((LH, LW, F))
    M = dense_operator(H, W, C, R, S, F, w)
    y = oracle.lc_forward(g, x, w, bias, alpha=0.7)
    ref = 0.7 * (x.reshape(B, -1) @ M.T) + bias.reshape(1, -1)
    np.testing.assert_allclose(y.reshape(B, -1), ref, rtol=1e-12, atol=1e-12)
    dx = oracle.lc_backward_data(g, dy, w)
    np.testing.assert_allclose(dx.reshape(B, -1), dy.reshape(B, -1) @ M, rtol=1e-12, atol=1e-12)
    # uncovered pixels receive exactly zero
    cover = (np.abs(M).sum(axis=0) > 0).reshape(H, W, C)
    assert np.all(dx[:, ~cover] == 0.0)


@pytest.mark.parametrize("g", TINY)
def test_backward_weights_matches_dense_outer_products(g):
    B, H, W, C, R, S, F = g
    LH, LW = (H - R) // S + 1, (W - R) // S + 1
    r = rng(2)
    x = r.standard_normal((B, H, W, C))
    dy = r.standard_normal((B, LH, LW, F))
    dw = oracle.lc_backward_weights(g, x, dy)
    ref = np.zeros_like(dw)
    for i in range(LH):
        for j in range(LW):
            patch = x[:, i * S:i * S + R, j * S:j * S + R, :].reshape(B, -1)     # (kh,kw,c) order
            ref[i, j] = patch.T @ dy[:, i, j, :]
    np.testing.assert_allclose(dw, ref, rtol=1e-12, atol=1e-12)
    prev = r.standard_normal(dw.shape)
    acc = oracle.lc_backward_weights(g, x, dy, beta=1.0, dw=prev)
    np.testing.assert_allclose(acc, prev + ref, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------- library special cases
def test_forward_with_shared_weights_is_cross_correlation():
    """Untied weights set identical at every location = a direct convolution
    (cross-correlation, no flip) with the same stride."""
    B, H, W, C, R, S, F = g = (3, 17, 21, 3, 5, 2, 4)
    LH, LW = (H - R) // S + 1, (W - R) // S + 1
    r = rng(3)
    x = r.standard_normal((B, H, W, C))
    w1 = r.standard_normal((R, R, C, F))
    w = np.broadcast_to(w1.reshape(1, 1, R * R * C, F), (LH, LW, R * R * C, F)).copy()
    y = oracle.lc_forward(g, x, w)
    ref = TF.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2),
                    torch.from_numpy(w1).permute(3, 2, 0, 1).contiguous(), stride=S)
    np.testing.assert_allclose(y, ref.permute(0, 2, 3, 1).numpy(), rtol=1e-11, atol=1e-11)
    # and its adjoint is the transposed convolution
    dy = r.standard_normal(y.shape)
    dx = oracle.lc_backward_data(g, dy, w)
    ref_dx = TF.conv_transpose2d(torch.from_numpy(dy).permute(0, 3, 1, 2),
                                 torch.from_numpy(w1).permute(3, 2, 0, 1).contiguous(), stride=S)
    full = np.zeros_like(dx)
    hh, ww = ref_dx.shape[2], ref_dx.shape[3]
    full[:, :hh, :ww, :] = ref_dx.permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(dx, full, rtol=1e-11, atol=1e-11)


def test_single_location_is_a_matmul():
    B, H, C, F = 5, 4, 3, 6
    g = (B, H, H, C, H, 1, F)
    r = rng(4)
    x = r.standard_normal((B, H, H, C))
    w = r.standard_normal((1, 1, H * H * C, F))
    dy = r.standard_normal((B, 1, 1, F))
    X = x.reshape(B, -1)
    np.testing.assert_allclose(oracle.lc_forward(g, x, w).reshape(B, F), X @ w[0, 0], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.lc_backward_data(g, dy, w).reshape(B, -1), dy.reshape(B, F) @ w[0, 0].T,
                               rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.lc_backward_weights(g, x, dy)[0, 0], X.T @ dy.reshape(B, F),
                               rtol=1e-12, atol=1e-12)


def test_adjoint_identity():
    g = wl.LCGeom(B=4, H=22, W=19, C=3, R=6, S=3, F=5)
    r = rng(5)
    x = r.standard_normal((g.B, g.H, g.W, g.C))
    w = r.standard_normal((g.LH, g.LW, g.K, g.F))
    y = r.standard_normal((g.B, g.LH, g.LW, g.F))
    lhs = np.vdot(oracle.lc_forward(g.as_tuple(), x, w), y)
    rhs = np.vdot(x, oracle.lc_backward_data(g.as_tuple(), y, w))
    assert abs(lhs - rhs) <= 1e-12 * max(abs(lhs), 1.0)


def test_orthogonal_nonoverlapping_reconstruction_is_identity():
    """S=R, F=K and every W_l orthogonal: W^T (W x) = x on covered pixels."""
    B, H, W, C, R = 2, 9, 6, 2, 3
    K = R * R * C
    g = (B, H, W, C, R, R, K)
    r = rng(6)
    LH, LW = H // R, W // R
    w = np.stack([np.linalg.qr(r.standard_normal((K, K)))[0] for _ in range(LH * LW)]).reshape(LH, LW, K, K)
    x = r.standard_normal((B, H, W, C))
    xr = oracle.lc_backward_data(g, oracle.lc_forward(g, x, w), w)
    np.testing.assert_allclose(xr, x, rtol=1e-12, atol=1e-12)


def test_backward_weights_by_finite_differences():
    g = wl.LCGeom(B=3, H=9, W=8, C=2, R=4, S=2, F=3)
    r = rng(7)
    x = r.standard_normal((g.B, g.H, g.W, g.C))
    w = r.standard_normal((g.LH, g.LW, g.K, g.F))
    dy = r.standard_normal((g.B, g.LH, g.LW, g.F))
    dw = oracle.lc_backward_weights(g.as_tuple(), x, dy)
    phi = lambda ww: np.vdot(oracle.lc_forward(g.as_tuple(), x, ww), dy)
    for _ in range(6):
        d = r.standard_normal(w.shape)
        eps = 1e-4
        fd = (phi(w + eps * d) - phi(w - eps * d)) / (2 * eps)
        assert abs(fd - np.vdot(dw, d)) <= 1e-8 * max(1.0, abs(fd))
    # single entries too, so an index mix-up inside one location cannot hide
    for idx in [(0, 0, 0, 0), (1, 2, 5, 1), (g.LH - 1, g.LW - 1, g.K - 1, g.F - 1), (2, 1, 17, 2)]:
        d = np.zeros_like(w)
        d[idx] = 1.0
        fd = (phi(w + d) - phi(w - d)) / 2
        assert abs(fd - dw[idx]) <= 1e-10 * max(1.0, abs(fd))


def test_point_evaluators_agree_with_full_oracle():
    g = wl.LCGeom(B=3, H=13, W=11, C=3, R=5, S=2, F=4)
    x, w, dy, bias = wl.lc_inputs(g, "gaussian", seed=3, with_bias=True)
    t = g.as_tuple()
    y = oracle.lc_forward(t, x, w, bias, 0.5)
    dx = oracle.lc_backward_data(t, dy, w)
    dw = oracle.lc_backward_weights(t, x, dy)
    r = rng(8)
    for _ in range(20):
        b, i, j, f = r.integers(g.B), r.integers(g.LH), r.integers(g.LW), r.integers(g.F)
        assert abs(oracle.lc_forward_at(t, x, w, bias, 0.5, b, i, j, f) - y[b, i, j, f]) < 1e-12
        row, col, c = r.integers(g.H), r.integers(g.W), r.integers(g.C)
        assert abs(oracle.lc_backward_data_at(t, dy, w, b, row, col, c) - dx[b, row, col, c]) < 1e-12
        k = r.integers(g.K)
        assert abs(oracle.lc_backward_weights_at(t, x, dy, i, j, k, f) - dw[i, j, k, f]) < 1e-12


# -------------------------------------------------------------------- pooling
def test_l2pool_matches_library_lp_pool():
    r = rng(9)
    x = r.standard_normal((2, 9, 11, 5))
    for ks, st in [(3, 1), (2, 2), (3, 2)]:
        y = oracle.l2pool_fwd(x, ks, st, eps=0.0)
        ref = TF.lp_pool2d(torch.from_numpy(x).permute(0, 3, 1, 2), 2.0, ks, st).permute(0, 2, 3, 1).numpy()
        np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)
        ref2 = torch.sqrt(ks * ks * TF.avg_pool2d(torch.from_numpy(x * x).permute(0, 3, 1, 2), ks, st))
        np.testing.assert_allclose(y, ref2.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)


def test_l2pool_closed_forms_and_invariants():
    r = rng(10)
    c, eps = 0.37, 1e-6
    y = oracle.l2pool_fwd(np.full((1, 6, 7, 2), c), 3, 1, eps)
    np.testing.assert_allclose(y, np.sqrt(9 * c * c + eps), rtol=1e-14)
    assert y.shape == (1, 4, 5, 2)
    x = r.standard_normal((2, 8, 8, 3))
    y1 = oracle.l2pool_fwd(x, 3, 1, 0.0)
    np.testing.assert_allclose(oracle.l2pool_fwd(-2.5 * x, 3, 1, 0.0), 2.5 * y1, rtol=1e-13)
    xm = torch.from_numpy(np.abs(x)).permute(0, 3, 1, 2)
    mx = TF.max_pool2d(xm, 3, 1).permute(0, 2, 3, 1).numpy()
    assert np.all(y1 >= mx - 1e-14) and np.all(y1 <= 3 * mx + 1e-14)


def _fd_dir(fun, x, d, eps):
    return (fun(x + eps * d) - fun(x - eps * d)) / (2 * eps)


def test_l2pool_bwd_by_finite_differences():
    r = rng(11)
    x = r.standard_normal((2, 7, 6, 3))
    for ks, st in [(3, 1), (2, 2)]:
        y = oracle.l2pool_fwd(x, ks, st, 1e-6)
        dy = r.standard_normal(y.shape)
        dx = oracle.l2pool_bwd(x, y, dy, ks, st)
        f = lambda xx: np.vdot(oracle.l2pool_fwd(xx, ks, st, 1e-6), dy)
        for _ in range(4):
            d = r.standard_normal(x.shape)
            fd = _fd_dir(f, x, d, 1e-6)
            assert abs(fd - np.vdot(dx, d)) <= 1e-7 * max(1.0, abs(fd))
        d = np.zeros_like(x); d[1, 3, 2, 1] = 1.0
        assert abs(_fd_dir(f, x, d, 1e-6) - dx[1, 3, 2, 1]) <= 1e-7


# ------------------------------------------------------------------------ LCN
def _gauss2d(ks, sigma):
    p = np.arange(ks) - (ks - 1) // 2
    g = np.exp(-p ** 2 / (2 * sigma ** 2))
    g /= g.sum()
    return np.outer(g, g)


def test_lcn_interior_statistics_match_library_convolution():
    r = rng(12)
    B, H, W, C, ks, sigma = 2, 12, 13, 4, 5, 1.0
    x = r.standard_normal((B, H, W, C))
    y, mu, rstd = oracle.lcn_fwd(x, ks, sigma, eps=1e-4)
    k = torch.from_numpy(_gauss2d(ks, sigma))[None, None]
    m1 = TF.conv2d(torch.from_numpy(x.mean(axis=3))[:, None], k)[:, 0].numpy()
    m2 = TF.conv2d(torch.from_numpy((x * x).mean(axis=3))[:, None], k)[:, 0].numpy()
    np.testing.assert_allclose(mu[:, 2:-2, 2:-2], m1, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(rstd[:, 2:-2, 2:-2], 1 / np.sqrt(m2 - m1 ** 2 + 1e-4), rtol=1e-11)
    np.testing.assert_allclose(y, (x - mu[..., None]) * rstd[..., None], rtol=1e-13, atol=1e-13)


def test_lcn_zero_local_mean_unit_local_norm():
    """With eps=0, re-standardising each pixel's window with that pixel's own
    mu and rstd gives weighted mean 0 and weighted second moment 1, borders
    included (truncated window, renormalised weights)."""
    r = rng(13)
    B, H, W, C, ks, sigma = 2, 9, 10, 3, 5, 1.0
    x = r.standard_normal((B, H, W, C)) + 0.5
    _, mu, rstd = oracle.lcn_fwd(x, ks, sigma, eps=0.0)
    g2 = _gauss2d(ks, sigma)
    rad = (ks - 1) // 2
    for b in range(B):
        for i in range(H):
            for j in range(W):
                wsum = m1 = m2 = 0.0
                for p in range(-rad, rad + 1):
                    for q in range(-rad, rad + 1):
                        ii, jj = i + p, j + q
                        if 0 <= ii < H and 0 <= jj < W:
                            z = (x[b, ii, jj] - mu[b, i, j]) * rstd[b, i, j]
                            wsum += g2[p + rad, q + rad] * C
                            m1 += g2[p + rad, q + rad] * z.sum()
                            m2 += g2[p + rad, q + rad] * (z * z).sum()
                assert abs(m1 / wsum) < 1e-10
                assert abs(m2 / wsum - 1.0) < 1e-9


def test_lcn_shift_scale_and_constant():
    r = rng(14)
    x = r.standard_normal((2, 8, 9, 3))
    y0, _, _ = oracle.lcn_fwd(x, 5, 1.0, eps=0.0)
    y1, _, _ = oracle.lcn_fwd(x + 3.25, 5, 1.0, eps=0.0)
    y2, _, _ = oracle.lcn_fwd(4.0 * x, 5, 1.0, eps=0.0)
    np.testing.assert_allclose(y1, y0, rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(y2, y0, rtol=1e-11, atol=1e-11)
    yc, muc, rc = oracle.lcn_fwd(np.full((1, 6, 6, 2), 1.5), 5, 1.0, eps=1e-4)
    assert np.all(np.abs(yc) < 1e-6) and np.allclose(muc, 1.5) and np.allclose(rc, 100.0, rtol=1e-6)


def test_lcn_bwd_by_finite_differences():
    r = rng(15)
    for shape, ks in [((2, 7, 8, 3), 5), ((1, 4, 3, 2), 5), ((1, 6, 6, 1), 3)]:
        x = r.standard_normal(shape)
        y, mu, rstd = oracle.lcn_fwd(x, ks, 1.0, 1e-2)
        dy = r.standard_normal(shape)
        dx = oracle.lcn_bwd(x, mu, rstd, dy, ks, 1.0)
        f = lambda xx: np.vdot(oracle.lcn_fwd(xx, ks, 1.0, 1e-2)[0], dy)
        for _ in range(4):
            d = r.standard_normal(shape)
            fd = _fd_dir(f, x, d, 1e-6)
            assert abs(fd - np.vdot(dx, d)) <= 2e-7 * max(1.0, abs(fd))
        for idx in [(0, 0, 0, 0), tuple(s - 1 for s in shape), (0, shape[1] // 2, shape[2] // 2, 0)]:
            d = np.zeros(shape); d[idx] = 1.0
            assert abs(_fd_dir(f, x, d, 1e-6) - dx[idx]) <= 2e-7


# ----------------------------------------------------------------- LCN variants
def _lcn_var_by_library(x, ks, sigma, eps, flags):
    """The variant's definition with scipy's zero-padded correlation as the window operator."""
    from scipy import ndimage
    k = _gauss2d(ks, sigma)[None, :, :, None]
    corr = lambda f: ndimage.correlate(f, k, mode="constant", cval=0.0)
    norm = 1.0 if flags & 2 else corr(np.ones_like(x))
    pool = (lambda f: f) if flags & 1 else (lambda f: f.mean(axis=3, keepdims=True))
    mean = lambda f: pool(corr(f) / norm)
    m = mean(x)
    var = mean((x - m) ** 2) if flags & 4 else np.maximum(mean(x * x) - m * m, 0.0)
    rs = 1.0 / np.sqrt(var + eps)
    sq = (lambda a: a) if flags & 1 else (lambda a: a[..., 0])
    return (x - m) * rs, sq(m), sq(rs)


@pytest.mark.parametrize("flags", range(8))
def test_lcn_variants_match_library_correlation(flags):
    r = rng(40 + flags)
    for shape, ks, sigma in [((2, 9, 11, 3), 5, 1.0), ((1, 4, 3, 2), 7, 2.0), ((1, 6, 7, 1), 3, 0.7)]:
        x = r.standard_normal(shape) + 0.3
        y, mu, rstd = oracle.lcn_var_fwd(x, ks, sigma, 1e-3, flags)
        ry, rmu, rrs = _lcn_var_by_library(x, ks, sigma, 1e-3, flags)
        np.testing.assert_allclose(mu, rmu, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(rstd, rrs, rtol=1e-11)
        np.testing.assert_allclose(y, ry, rtol=1e-11, atol=1e-12)


def test_lcn_variant_without_flags_is_the_pooled_one_stage_form():
    r = rng(48)
    x, dy = r.standard_normal((2, 8, 7, 3)), r.standard_normal((2, 8, 7, 3))
    y0, mu0, rs0 = oracle.lcn_fwd(x, 5, 1.0, 1e-3)
    y1, mu1, rs1 = oracle.lcn_var_fwd(x, 5, 1.0, 1e-3, 0)
    for a, b in [(y0, y1), (mu0, mu1), (rs0, rs1)]:
        np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(oracle.lcn_var_bwd(x, mu0, rs0, dy, 5, 1.0, 0), oracle.lcn_bwd(x, mu0, rs0, dy, 5, 1.0),
                               rtol=1e-12, atol=1e-13)


def test_lcn_variants_closed_forms():
    ks, sigma = 5, 1.0
    g = _gauss2d(ks, sigma)
    # constant image: renormalised borders see the constant everywhere, zero padding sees less of it at the rim
    xc = np.full((1, 7, 8, 2), 2.5)
    for flags in range(8):
        y, mu, rstd = oracle.lcn_var_fwd(xc, ks, sigma, 1e-2, flags)
        if not flags & 2:
            assert np.allclose(mu, 2.5, rtol=1e-13) and np.all(np.abs(y) < 1e-12)
            assert np.allclose(rstd, 10.0, rtol=1e-9)
        else:
            assert np.isclose(mu.reshape(7, 8, -1)[0, 0, 0], 2.5 * g[2:, 2:].sum(), rtol=1e-13)
            assert np.isclose(mu.reshape(7, 8, -1)[3, 0, 0], 2.5 * g[:, 2:].sum(), rtol=1e-13)
            assert np.isclose(mu.reshape(7, 8, -1)[3, 4, 0], 2.5, rtol=1e-13)
    r = rng(49)
    x = r.standard_normal((2, 8, 9, 3))
    for flags in range(8):
        y0 = oracle.lcn_var_fwd(x, ks, sigma, 0.0, flags)[0]
        np.testing.assert_allclose(oracle.lcn_var_fwd(3.0 * x, ks, sigma, 0.0, flags)[0], y0, rtol=1e-10, atol=1e-11)
        if not flags & 2:   # a shift is removed by the mean only when the window weights sum to one
            np.testing.assert_allclose(oracle.lcn_var_fwd(x + 1.75, ks, sigma, 0.0, flags)[0], y0, rtol=1e-8, atol=1e-9)
    # one channel: per-channel and pooled statistics are the same thing
    x1 = r.standard_normal((2, 8, 9, 1))
    for base in (0, 2, 4, 6):
        a, b = oracle.lcn_var_fwd(x1, ks, sigma, 1e-3, base), oracle.lcn_var_fwd(x1, ks, sigma, 1e-3, base | 1)
        np.testing.assert_allclose(a[0], b[0], rtol=1e-13, atol=1e-14)
        np.testing.assert_allclose(a[1], b[1][..., 0], rtol=1e-13, atol=1e-14)
    # identical channels: pooling over them changes nothing
    xr = np.repeat(x1, 3, axis=3)
    for base in (0, 2, 4, 6):
        a, b = oracle.lcn_var_fwd(xr, ks, sigma, 1e-3, base), oracle.lcn_var_fwd(xr, ks, sigma, 1e-3, base | 1)
        np.testing.assert_allclose(a[0], b[0], rtol=1e-12, atol=1e-13)


def test_lcn_two_stage_unit_local_energy():
    """Two stages, eps=0: around every pixel the window-weighted mean of (v * rstd_pixel)^2 over the neighbours'
    own v is one, and v itself has zero window mean of x - mu only at the centre's statistics."""
    r = rng(50)
    B, H, W, C, ks = 1, 7, 8, 2, 5
    x = r.standard_normal((B, H, W, C)) + 0.4
    g2, rad = _gauss2d(ks, 1.0), 2
    for flags in (4, 5):
        _, mu, rstd = oracle.lcn_var_fwd(x, ks, 1.0, 0.0, flags)
        v = x - (mu if flags & 1 else mu[..., None])
        rs = rstd if flags & 1 else rstd[..., None]
        for i in range(H):
            for j in range(W):
                acc, z = np.zeros(C if flags & 1 else 1), 0.0
                for p in range(-rad, rad + 1):
                    for q in range(-rad, rad + 1):
                        if 0 <= i + p < H and 0 <= j + q < W:
                            z += g2[p + rad, q + rad]
                            e = v[0, i + p, j + q] ** 2
                            acc += g2[p + rad, q + rad] * (e if flags & 1 else e.mean())
                np.testing.assert_allclose(acc / z * rs[0, i, j] ** 2, 1.0, rtol=1e-10)


@pytest.mark.parametrize("flags", range(8))
def test_lcn_variant_bwd_by_finite_differences(flags):
    r = rng(60 + flags)
    for shape, ks in [((2, 7, 8, 3), 5), ((1, 4, 3, 2), 5), ((1, 6, 6, 1), 3)]:
        x = r.standard_normal(shape)
        y, mu, rstd = oracle.lcn_var_fwd(x, ks, 1.0, 1e-2, flags)
        dy = r.standard_normal(shape)
        dx = oracle.lcn_var_bwd(x, mu, rstd, dy, ks, 1.0, flags)
        f = lambda xx: np.vdot(oracle.lcn_var_fwd(xx, ks, 1.0, 1e-2, flags)[0], dy)
        for _ in range(4):
            d = r.standard_normal(shape)
            fd = _fd_dir(f, x, d, 1e-6)
            assert abs(fd - np.vdot(dx, d)) <= 5e-7 * max(1.0, abs(fd))
        for idx in [(0, 0, 0, 0), tuple(s - 1 for s in shape), (0, shape[1] // 2, shape[2] // 2, 0)]:
            d = np.zeros(shape); d[idx] = 1.0
            assert abs(_fd_dir(f, x, d, 1e-6) - dx[idx]) <= 5e-7


# ------------------------------------------------------------ RICA cost / step
SAE_G = wl.LCGeom(B=3, H=9, W=8, C=2, R=4, S=2, F=3)    # floor geometry: last column uncovered


def _sae_inputs(seed=16, g=SAE_G):
    r = rng(seed)
    x = r.standard_normal((g.B, g.H, g.W, g.C))
    w = r.standard_normal((g.LH, g.LW, g.K, g.F)) / np.sqrt(g.K)
    b = 0.1 * r.standard_normal((g.H, g.W, g.C))
    return r, x, w, b


def test_sae_cost_is_eq1_written_with_the_dense_operator():
    g = SAE_G
    r, x, w, b = _sae_inputs()
    alpha, lam, eps_s = 0.8, 0.1, 1e-3
    M = dense_operator(g.H, g.W, g.C, g.R, g.S, g.F, w)
    X = x.reshape(g.B, -1)
    Hh = alpha * X @ M.T
    rec = Hh @ M + b.reshape(1, -1) - X
    J_ref = ((rec ** 2).sum() + lam * np.sqrt(Hh ** 2 + eps_s).sum()) / g.B
    J, h, res = oracle.sae_cost(g.as_tuple(), x, w, b, alpha, lam, eps_s)
    assert abs(J - J_ref) <= 1e-12 * abs(J_ref)
    np.testing.assert_allclose(h.reshape(g.B, -1), Hh, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(res.reshape(g.B, -1), rec, rtol=1e-12, atol=1e-12)


def test_sae_gradient_by_finite_differences():
    g = SAE_G
    r, x, w, b = _sae_inputs()
    alpha, lam, eps_s = 0.8, 0.1, 1e-2
    t = g.as_tuple()
    J, dw, db, da, h = oracle.sae_grad(t, x, w, b, alpha, lam, eps_s)
    assert abs(J - oracle.sae_cost(t, x, w, b, alpha, lam, eps_s)[0]) < 1e-14
    e = 1e-6
    for _ in range(4):
        d = r.standard_normal(w.shape)
        fd = (oracle.sae_cost(t, x, w + e * d, b, alpha, lam, eps_s)[0] -
              oracle.sae_cost(t, x, w - e * d, b, alpha, lam, eps_s)[0]) / (2 * e)
        assert abs(fd - np.vdot(dw, d)) <= 1e-7 * max(1.0, abs(fd))
        d = r.standard_normal(b.shape)
        fd = (oracle.sae_cost(t, x, w, b + e * d, alpha, lam, eps_s)[0] -
              oracle.sae_cost(t, x, w, b - e * d, alpha, lam, eps_s)[0]) / (2 * e)
        assert abs(fd - np.vdot(db, d)) <= 1e-7 * max(1.0, abs(fd))
    fd = (oracle.sae_cost(t, x, w, b, alpha + e, lam, eps_s)[0] -
          oracle.sae_cost(t, x, w, b, alpha - e, lam, eps_s)[0]) / (2 * e)
    assert abs(fd - da) <= 1e-7 * max(1.0, abs(fd))
    # one weight at a time, so that the two tied paths are both needed
    for idx in [(0, 0, 0, 0), (1, 2, 7, 1), (g.LH - 1, g.LW - 1, g.K - 1, g.F - 1)]:
        d = np.zeros_like(w); d[idx] = 1.0
        fd = (oracle.sae_cost(t, x, w + e * d, b, alpha, lam, eps_s)[0] -
              oracle.sae_cost(t, x, w - e * d, b, alpha, lam, eps_s)[0]) / (2 * e)
        assert abs(fd - dw[idx]) <= 1e-7 * max(1.0, abs(fd))


def test_sae_orthogonal_case_has_zero_cost_and_gradient():
    B, H, W, C, R = 2, 6, 6, 2, 3
    K = R * R * C
    g = (B, H, W, C, R, R, K)
    r = rng(17)
    w = np.stack([np.linalg.qr(r.standard_normal((K, K)))[0] for _ in range(4)]).reshape(2, 2, K, K)
    x = r.standard_normal((B, H, W, C))
    J, dw, db, da, _ = oracle.sae_grad(g, x, w, np.zeros((H, W, C)), 1.0, 0.0, 1e-6)
    assert abs(J) < 1e-24 and np.abs(dw).max() < 1e-12 and np.abs(db).max() < 1e-12


def test_sae_newton_step_on_offset_and_descent():
    g = SAE_G
    t = g.as_tuple()
    r, x, w, b = _sae_inputs(18)
    # lambda=0: J is quadratic in b with Hessian 2I, so b - mean_b(r) has db = 0
    _, _, res = oracle.sae_cost(t, x, w, b, 1.0, 0.0, 1e-6)
    b2 = b - res.mean(axis=0)
    _, _, db, _, _ = oracle.sae_grad(t, x, w, b2, 1.0, 0.0, 1e-6)
    assert np.abs(db).max() < 1e-12
    # small SGD steps do not increase the cost, with and without the projection / learned alpha
    for flags in (0, 1, 2, 3):
        ww, bb, aa = w.copy(), b.copy(), 1.0
        if flags & 1:
            ww /= np.linalg.norm(ww, axis=2, keepdims=True)
        costs = []
        for _ in range(10):
            J, ww, bb, aa, _ = oracle.sae_step(t, x, ww, bb, aa, 0.1, 1e-6, 1e-2, flags)
            costs.append(J)
        assert all(c1 <= c0 + 1e-12 for c0, c1 in zip(costs, costs[1:])), (flags, costs)
        if flags & 1:
            np.testing.assert_allclose(np.linalg.norm(ww, axis=2), 1.0, rtol=1e-12)


def test_sae_step_is_grad_plus_sgd_update():
    g = SAE_G
    t = g.as_tuple()
    r, x, w, b = _sae_inputs(19)
    J, dw, db, da, h = oracle.sae_grad(t, x, w, b, 0.9, 0.1, 1e-6)
    J2, w2, b2, a2, h2 = oracle.sae_step(t, x, w, b, 0.9, 0.1, 1e-6, 0.05, flags=2)
    assert J == J2
    np.testing.assert_allclose(w2, w - 0.05 * dw, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(b2, b - 0.05 * db, rtol=1e-14, atol=1e-15)
    assert abs(a2 - (0.9 - 0.05 * da)) < 1e-14
    np.testing.assert_array_equal(h, h2)


def test_sae_projection_leaves_a_zero_filter_alone():
    """Eq. 1's constraint ||W^(k)||_2 = 1 cannot be met by a filter that is all zeros: such a filter has zero
    response, zero gradient through both tied paths, and nothing to normalise.  It stays zero (no NaN), and every
    other filter comes out with unit norm."""
    g = SAE_G
    t = g.as_tuple()
    r, x, w, b = _sae_inputs(23)
    w = w.copy()
    w[1, 0, :, 2] = 0.0
    _, dw, _, _, _ = oracle.sae_grad(t, x, w, b, 0.9, 0.1, 1e-6)
    assert np.all(dw[1, 0, :, 2] == 0.0)
    _, w2, _, _, _ = oracle.sae_step(t, x, w, b, 0.9, 0.1, 1e-6, 0.05, flags=1)
    assert np.all(np.isfinite(w2)) and np.all(w2[1, 0, :, 2] == 0.0)
    norms = np.linalg.norm(w2, axis=2)
    norms[1, 0, 2] = 1.0
    np.testing.assert_allclose(norms, 1.0, rtol=1e-12)


def test_one_field_step_written_with_matmuls_equals_the_loop_oracle():
    """The dense last layer (Sec. 3.1) is the one-field case; its matmul form must be the loop oracle's step."""
    g = wl.LCGeom(B=6, H=5, W=5, C=3, R=5, S=1, F=7)
    t = g.as_tuple()
    r = np.random.default_rng(31)
    x = r.standard_normal((g.B, g.H, g.W, g.C))
    w = r.standard_normal((1, 1, g.K, g.F)) / np.sqrt(g.K)
    b = 0.1 * r.standard_normal((g.H, g.W, g.C))
    for flags in range(4):
        ref = oracle.sae_step(t, x, w, b, 0.8, 0.01, 1e-6, 0.05, flags)
        got = oracle.sae_step_one_field(t, x, w, b, 0.8, 0.01, 1e-6, 0.05, flags)
        assert abs(ref[0] - got[0]) <= 1e-13 * abs(ref[0])
        np.testing.assert_allclose(got[1], ref[1], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(got[2], ref[2], rtol=1e-12, atol=1e-14)
        assert abs(ref[3] - got[3]) <= 1e-13
        np.testing.assert_allclose(got[4], ref[4], rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------ input generators
def test_synthetic_inputs_have_the_stated_statistics():
    g = wl.LCGeom(B=3, H=32, W=32, C=3, R=8, S=4, F=4)
    x, w, dy = wl.lc_inputs(g, "pink", seed=0)
    assert x.dtype == w.dtype == dy.dtype == np.float32
    flat = x.reshape(g.B, -1).astype(np.float64)
    np.testing.assert_allclose(flat.mean(axis=1), 0.0, atol=1e-6)
    np.testing.assert_allclose(flat.std(axis=1), 1.0, rtol=1e-5)
    # 1/f amplitude: low frequencies carry more energy than high ones
    spec = np.abs(np.fft.fft2(x[0, :, :, 0].astype(np.float64)))
    assert spec[1:3, 1:3].mean() > 4 * spec[12:16, 12:16].mean()
    assert abs(w.astype(np.float64).std() * np.sqrt(g.K) - 1.0) < 0.05
    x2, _, _ = wl.lc_inputs(g, "pink", seed=0)
    np.testing.assert_array_equal(x, x2)
    h = wl.halfnormal_maps(np.random.default_rng(0), 2, 8, 8, 4)
    assert h.min() >= 0
    bits = wl.to_bf16_round(np.array([1.0, 1.00390625, 1.005859375], dtype=np.float32))
    assert list(bits) == [0x3F80, 0x3F80, 0x3F81]
