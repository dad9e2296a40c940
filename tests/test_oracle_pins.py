"""Pins of the CPU oracle's primitives against what the mathematics fixes (no GPU).

The paper (LAMP, arXiv 2006.12575) prints no numeric value for any layer of the per-device path,
so each primitive is pinned by closed forms, special cases that reduce to a library routine,
independent brute-force forms, adjoint/bilinear identities and finite differences, chosen so a
dropped term, a wrong sign/index or a transposed operand fails at least one of them.
"""
import itertools

import numpy as np
import pytest

import oracle as O


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ------------------------------------------------------------------------------ O1 conv forward

def conv_scatter_form(x, w, b):
    """Independent second form: every input voxel scatters into its (up to) 27 outputs."""
    N, D, H, W, Ci = x.shape
    Co = w.shape[0]
    z = np.zeros((N, D, H, W, Co))
    if b is not None:
        z += b
    for n, i, j, k in itertools.product(range(N), range(D), range(H), range(W)):
        for kd, kh, kw in itertools.product(range(3), repeat=3):
            d, h, wv = i - (kd - 1), j - (kh - 1), k - (kw - 1)
            if 0 <= d < D and 0 <= h < H and 0 <= wv < W:
                z[n, d, h, wv, :] += w[:, kd, kh, kw, :] @ x[n, i, j, k, :]
    return z


@pytest.mark.parametrize("shape", [(1, 1, 1, 1, 2, 3), (2, 3, 4, 5, 3, 2), (1, 6, 5, 4, 1, 4), (1, 2, 2, 2, 5, 1)])
def test_conv_fwd_vs_scatter_bruteforce(shape):
    N, D, H, W, Ci, Co = shape
    r = rng(1)
    x = r.standard_normal((N, D, H, W, Ci))
    w = r.standard_normal((Co, 3, 3, 3, Ci))
    b = r.standard_normal(Co)
    np.testing.assert_allclose(O.conv3d_fwd(x, w, b), conv_scatter_form(x, w, b), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(O.conv3d_fwd(x, w, None), conv_scatter_form(x, w, None), rtol=1e-12, atol=1e-12)


def test_conv_fwd_delta_kernel_identity_and_shift():
    r = rng(2)
    N, D, H, W, C = 1, 5, 6, 7, 3
    x = r.standard_normal((N, D, H, W, C))
    for kd, kh, kw in itertools.product(range(3), repeat=3):
        w = np.zeros((C, 3, 3, 3, C))
        for c in range(C):
            w[c, kd, kh, kw, c] = 1.0
        z = O.conv3d_fwd(x, w)
        # z[d,h,w] = x[d+kd-1, h+kh-1, w+kw-1] with zero fill
        exp = np.zeros_like(x)
        for d, h, wv in itertools.product(range(D), range(H), range(W)):
            i, j, k = d + kd - 1, h + kh - 1, wv + kw - 1
            if 0 <= i < D and 0 <= j < H and 0 <= k < W:
                exp[0, d, h, wv] = x[0, i, j, k]
        np.testing.assert_array_equal(z, exp)


def test_conv_fwd_channel_orientation():
    # W[co,...,ci] maps input channel ci to output channel co (not the transpose)
    x = np.zeros((1, 3, 3, 3, 2))
    x[0, 1, 1, 1, 1] = 1.0
    w = np.zeros((3, 3, 3, 3, 2))
    w[2, 1, 1, 1, 1] = 5.0
    z = O.conv3d_fwd(x, w)
    assert z[0, 1, 1, 1, 2] == 5.0 and np.count_nonzero(z) == 1


def test_conv_fwd_all_ones_closed_form():
    D, H, W, Ci, Co = 4, 5, 6, 3, 2
    z = O.conv3d_fwd(np.ones((1, D, H, W, Ci)), np.ones((Co, 3, 3, 3, Ci)))

    def m(i, L):
        return 2 if (i == 0 or i == L - 1) else 3

    for d, h, w in itertools.product(range(D), range(H), range(W)):
        assert z[0, d, h, w, 0] == Ci * m(d, D) * m(h, H) * m(w, W)
    assert z[0, 1, 1, 1, 1] == 27 * Ci and z[0, 0, 0, 0, 0] == 8 * Ci


def test_conv_fwd_centre_tap_is_matmul():
    r = rng(3)
    x = r.standard_normal((2, 3, 4, 5, 6))
    m = r.standard_normal((7, 6))
    w = np.zeros((7, 3, 3, 3, 6))
    w[:, 1, 1, 1, :] = m
    np.testing.assert_allclose(O.conv3d_fwd(x, w), x @ m.T, rtol=1e-13, atol=1e-13)


def test_conv_fwd_linearity_and_bias():
    r = rng(4)
    x1, x2 = r.standard_normal((2, 1, 4, 4, 4, 3))
    w1, w2 = r.standard_normal((2, 2, 3, 3, 3, 3))
    b = r.standard_normal(2)
    a, c = 0.7, -1.3
    np.testing.assert_allclose(O.conv3d_fwd(a * x1 + c * x2, w1), a * O.conv3d_fwd(x1, w1) + c * O.conv3d_fwd(x2, w1), atol=1e-12)
    np.testing.assert_allclose(O.conv3d_fwd(x1, a * w1 + c * w2), a * O.conv3d_fwd(x1, w1) + c * O.conv3d_fwd(x1, w2), atol=1e-12)
    np.testing.assert_allclose(O.conv3d_fwd(x1, w1, b), O.conv3d_fwd(x1, w1) + b, atol=1e-13)


def test_conv_fwd_translation_equivariance_interior():
    r = rng(5)
    x = np.zeros((1, 10, 10, 10, 2))
    x[0, 3:6, 3:6, 3:6] = r.standard_normal((3, 3, 3, 2))
    w = r.standard_normal((2, 3, 3, 3, 2))
    z = O.conv3d_fwd(x, w)
    xs = np.roll(x, (1, 2, -1), axis=(1, 2, 3))
    np.testing.assert_allclose(O.conv3d_fwd(xs, w), np.roll(z, (1, 2, -1), axis=(1, 2, 3)), atol=1e-13)


# ------------------------------------------------------------------------------ O2 dgrad

@pytest.mark.parametrize("shape", [(2, 3, 4, 5, 3, 2), (1, 1, 1, 2, 2, 3), (1, 5, 5, 5, 4, 4)])
def test_dgrad_adjoint_identity(shape):
    N, D, H, W, Ci, Co = shape
    r = rng(6)
    x = r.standard_normal((N, D, H, W, Ci))
    y = r.standard_normal((N, D, H, W, Co))
    w = r.standard_normal((Co, 3, 3, 3, Ci))
    lhs = np.sum(O.conv3d_fwd(x, w) * y)
    rhs = np.sum(x * O.conv3d_dgrad(y, w))
    assert abs(lhs - rhs) <= 1e-11 * max(1.0, abs(lhs))


def test_dgrad_is_conv_with_flipped_transposed_weights():
    r = rng(7)
    dz = r.standard_normal((1, 4, 5, 6, 3))
    w = r.standard_normal((3, 3, 3, 3, 2))
    wf = np.ascontiguousarray(np.transpose(w[:, ::-1, ::-1, ::-1, :], (4, 1, 2, 3, 0)))
    np.testing.assert_allclose(O.conv3d_dgrad(dz, w), O.conv3d_fwd(dz, wf), atol=1e-12)


def test_dgrad_single_impulse():
    # an impulse in dz at voxel p, channel co spreads W[co,kd,kh,kw,:] to voxel p + (k-1)
    w = rng(8).standard_normal((2, 3, 3, 3, 3))
    dz = np.zeros((1, 5, 5, 5, 2))
    dz[0, 2, 2, 2, 1] = 1.0
    dx = O.conv3d_dgrad(dz, w)
    for kd, kh, kw in itertools.product(range(3), repeat=3):
        np.testing.assert_array_equal(dx[0, 2 + kd - 1, 2 + kh - 1, 2 + kw - 1, :], w[1, kd, kh, kw, :])


# ------------------------------------------------------------------------------ O3 wgrad

@pytest.mark.parametrize("shape", [(2, 3, 4, 5, 3, 2), (1, 2, 2, 2, 1, 4)])
def test_wgrad_bilinear_identity_and_fd(shape):
    N, D, H, W, Ci, Co = shape
    r = rng(9)
    x = r.standard_normal((N, D, H, W, Ci))
    dz = r.standard_normal((N, D, H, W, Co))
    w = r.standard_normal((Co, 3, 3, 3, Ci))
    dw, db = O.conv3d_wgrad(x, dz, want_db=True)
    lhs = np.sum(dz * O.conv3d_fwd(x, w))
    assert abs(lhs - np.sum(dw * w)) <= 1e-11 * max(1.0, abs(lhs))
    np.testing.assert_allclose(db, dz.reshape(-1, Co).sum(0), atol=1e-12)
    # central finite differences of L(W) = <dz, conv(x;W)> on a few entries (L is linear in W)
    hh = 1e-3
    for idx in [(0, 0, 0, 0, 0), (Co - 1, 2, 2, 2, Ci - 1), (0, 1, 1, 1, 0), (Co - 1, 0, 2, 1, 0), (0, 2, 0, 1, Ci - 1)]:
        wp, wm = w.copy(), w.copy()
        wp[idx] += hh
        wm[idx] -= hh
        fd = (np.sum(dz * O.conv3d_fwd(x, wp)) - np.sum(dz * O.conv3d_fwd(x, wm))) / (2 * hh)
        assert abs(fd - dw[idx]) <= 1e-7 * max(1.0, abs(fd))


def test_wgrad_batch_additivity_beta():
    r = rng(10)
    x = r.standard_normal((2, 3, 3, 4, 2))
    dz = r.standard_normal((2, 3, 3, 4, 3))
    full, fullb = O.conv3d_wgrad(x, dz, want_db=True)
    a, ab = O.conv3d_wgrad(x[:1], dz[:1], want_db=True)
    acc, accb = O.conv3d_wgrad(x[1:], dz[1:], dw_prev=a, db_prev=ab, beta=1.0, want_db=True)
    np.testing.assert_allclose(acc, full, atol=1e-12)
    np.testing.assert_allclose(accb, fullb, atol=1e-12)
    # beta = 0 ignores (even NaN) previous contents
    junk = np.full_like(a, np.nan)
    over, _ = O.conv3d_wgrad(x, dz, dw_prev=junk, beta=0.0)
    np.testing.assert_allclose(over, full, atol=1e-12)


def test_sampled_forms_match_full():
    r = rng(11)
    x = r.standard_normal((2, 4, 5, 6, 3))
    w = r.standard_normal((4, 3, 3, 3, 3))
    b = r.standard_normal(4)
    dz = r.standard_normal((2, 4, 5, 6, 4))
    coords = [(0, 0, 0, 0), (1, 3, 4, 5), (0, 2, 2, 2), (1, 0, 4, 0), (0, 3, 0, 5)]
    z = O.conv3d_fwd(x, w, b)
    np.testing.assert_allclose(O.conv3d_fwd_at(x, w, b, coords), np.stack([z[c] for c in coords]), atol=1e-12)
    dx = O.conv3d_dgrad(dz, w)
    np.testing.assert_allclose(O.conv3d_dgrad_at(dz, w, coords), np.stack([dx[c] for c in coords]), atol=1e-12)
    dw, _ = O.conv3d_wgrad(x, dz)
    ent = [(0, 0, 0, 0, 0), (3, 2, 2, 2, 2), (1, 1, 1, 1, 1), (2, 0, 2, 1, 0), (3, 2, 0, 0, 2)]
    np.testing.assert_allclose(O.conv3d_wgrad_at(x, dz, ent), np.array([dw[e] for e in ent]), atol=1e-12)


# ------------------------------------------------------------------------------ O4 / O5 instance norm + ReLU

def test_inorm_moments_invariance_constant():
    r = rng(12)
    z = r.standard_normal((2, 3, 4, 5, 3)) * 2.5 + 1.0
    eps = 1e-5
    u, st = O.inorm_relu(z, eps=eps, relu=False)
    var = z.reshape(2, -1, 3).var(axis=1)
    np.testing.assert_allclose(u.reshape(2, -1, 3).mean(axis=1), 0.0, atol=1e-13)
    np.testing.assert_allclose(u.reshape(2, -1, 3).var(axis=1), var / (var + eps), rtol=1e-12)
    np.testing.assert_allclose(st[..., 0], z.reshape(2, -1, 3).mean(axis=1), atol=1e-13)
    np.testing.assert_allclose(st[..., 1], 1 / np.sqrt(var + eps), rtol=1e-12)
    # positive affine re-scaling of the input changes nothing up to eps
    u2, _ = O.inorm_relu(3.0 * z + 7.0, eps=0.0, relu=False)
    u0, _ = O.inorm_relu(z, eps=0.0, relu=False)
    np.testing.assert_allclose(u2, u0, atol=1e-12)
    # ReLU and affine parameters
    g, b = r.uniform(0.5, 1.5, 3), r.uniform(-0.5, 0.5, 3)
    y, _ = O.inorm_relu(z, g, b, eps)
    np.testing.assert_allclose(y, np.maximum(0.0, g * u + b), atol=1e-13)
    # constant input -> max(0, beta)
    yc, _ = O.inorm_relu(np.full((1, 2, 2, 2, 3), 4.2), g, b, eps)
    np.testing.assert_allclose(yc, np.broadcast_to(np.maximum(0, b), yc.shape), atol=1e-6)
    # a per-channel constant added before the norm (a conv bias) is removed exactly
    y3, _ = O.inorm_relu(z + np.array([1.0, -2.0, 3.0]), g, b, eps)
    np.testing.assert_allclose(y3, y, atol=1e-12)


def test_inorm_bwd_fd_and_orthogonality():
    r = rng(13)
    z = r.standard_normal((2, 2, 3, 4, 3))
    dy = r.standard_normal(z.shape)
    g, b = r.uniform(0.5, 1.5, 3), r.uniform(-0.5, 0.5, 3)
    eps = 1e-5
    dz, dg, db = O.inorm_relu_bwd(dy, z, g, b, eps)
    y0, _ = O.inorm_relu(z, g, b, eps)
    u0, _ = O.inorm_relu(z, g, b, eps, relu=False)

    def L(zz, gg=g, bb=b):
        return np.sum(dy * O.inorm_relu(zz, gg, bb, eps)[0])

    hh = 1e-6
    cnt = 0
    for idx in itertools.product(range(2), range(2), range(3), range(4), range(3)):
        if cnt >= 25:
            break
        # keep away from ReLU kinks anywhere in this (n,c) slab
        if np.min(np.abs(u0[idx[0], ..., idx[4]])) < 1e-3:
            continue
        zp, zm = z.copy(), z.copy()
        zp[idx] += hh
        zm[idx] -= hh
        fd = (L(zp) - L(zm)) / (2 * hh)
        assert abs(fd - dz[idx]) <= 1e-6 * max(1.0, abs(fd)), idx
        cnt += 1
    assert cnt >= 5
    for c in range(3):
        gp, gm = g.copy(), g.copy()
        gp[c] += hh
        gm[c] -= hh
        assert abs((L(z, gp) - L(z, gm)) / (2 * hh) - dg[c]) <= 1e-6 * max(1.0, abs(dg[c]))
        bp, bm = b.copy(), b.copy()
        bp[c] += hh
        bm[c] -= hh
        assert abs((L(z, g, bp) - L(z, g, bm)) / (2 * hh) - db[c]) <= 1e-6 * max(1.0, abs(db[c]))
    # dz is orthogonal to 1 and to z-hat per (n,c)
    zh, _ = O.inorm_relu(z, eps=eps, relu=False)
    np.testing.assert_allclose(dz.reshape(2, -1, 3).sum(1), 0.0, atol=1e-12)
    # (exactly so only for eps = 0, since sum zh^2 = V*var/(var+eps))
    dz0, _, _ = O.inorm_relu_bwd(dy, z, g, b, 0.0)
    zh0, _ = O.inorm_relu(z, eps=0.0, relu=False)
    np.testing.assert_allclose((dz0 * zh0).reshape(2, -1, 3).sum(1), 0.0, atol=1e-11)
    var = z.reshape(2, -1, 3).var(axis=1)
    resid = (dz * zh).reshape(2, -1, 3).sum(1)
    sgz = (dy * (y0 > 0) * zh).reshape(2, -1, 3).sum(1)
    np.testing.assert_allclose(resid, g / np.sqrt(var + eps) * sgz * (eps / (var + eps)), atol=1e-12)
    # mask: where y == 0 the upstream gradient must not contribute to dbeta
    np.testing.assert_allclose(db, (dy * (y0 > 0)).reshape(-1, 3).sum(0), atol=1e-12)


# ------------------------------------------------------------------------------ O6 max pool

def test_maxpool_bruteforce_ramp_routing():
    r = rng(14)
    x = r.standard_normal((2, 4, 6, 8, 3))
    y = O.maxpool2_fwd(x)
    exp = x.reshape(2, 2, 2, 3, 2, 4, 2, 3).max(axis=(2, 4, 6))
    np.testing.assert_array_equal(y, exp)
    dy = r.standard_normal(y.shape)
    dx = O.maxpool2_bwd(x, dy)
    np.testing.assert_allclose(dx.reshape(2, 2, 2, 3, 2, 4, 2, 3).sum(axis=(2, 4, 6)), dy, atol=0)
    assert np.count_nonzero(dx) == dy.size
    # gradient sits exactly where x equals the window max
    up = np.repeat(np.repeat(np.repeat(y, 2, 1), 2, 2), 2, 3)
    assert np.all((dx != 0) <= (x == up))
    # strictly increasing ramp: arg-max is the (1,1,1) corner
    ramp = np.arange(4 * 4 * 4, dtype=np.float64).reshape(1, 4, 4, 4, 1)
    dr = O.maxpool2_bwd(ramp, np.ones((1, 2, 2, 2, 1)))
    assert np.all(dr[0, 1::2, 1::2, 1::2, 0] == 1) and dr.sum() == 8
    # ties: the first position in (i,j,k) raster order wins
    dt = O.maxpool2_bwd(np.zeros((1, 2, 2, 2, 1)), np.ones((1, 1, 1, 1, 1)))
    assert dt[0, 0, 0, 0, 0] == 1 and dt.sum() == 1


# ------------------------------------------------------------------------------ O7 transposed conv

def test_convtr_delta_is_nearest_upsampling_and_matmul_form():
    r = rng(15)
    x = r.standard_normal((2, 2, 3, 4, 3))
    wt = np.zeros((3, 2, 2, 2, 3))
    for c in range(3):
        wt[c, :, :, :, c] = 1.0
    y = O.convtr3d_fwd(x, wt)
    np.testing.assert_array_equal(y, np.repeat(np.repeat(np.repeat(x, 2, 1), 2, 2), 2, 3))
    # general weights: a matrix product [V,Ci]x[Ci,8Co] followed by a fixed permutation
    wt = r.standard_normal((3, 2, 2, 2, 5))
    b = r.standard_normal(5)
    y = O.convtr3d_fwd(x, wt, b)
    m = (x.reshape(-1, 3) @ wt.reshape(3, 40)).reshape(2, 2, 3, 4, 2, 2, 2, 5)
    exp = np.transpose(m, (0, 1, 4, 2, 5, 3, 6, 7)).reshape(2, 4, 6, 8, 5) + b
    np.testing.assert_allclose(y, exp, atol=1e-13)


def test_convtr_bwd_adjoint_bilinear():
    r = rng(16)
    x = r.standard_normal((2, 2, 3, 2, 4))
    wt = r.standard_normal((4, 2, 2, 2, 3))
    dy = r.standard_normal((2, 4, 6, 4, 3))
    dx, dwt, db = O.convtr3d_bwd(x, wt, dy)
    y = O.convtr3d_fwd(x, wt)
    L = np.sum(y * dy)
    assert abs(L - np.sum(x * dx)) < 1e-11 * max(1, abs(L))
    assert abs(L - np.sum(wt * dwt)) < 1e-11 * max(1, abs(L))
    np.testing.assert_allclose(db, dy.reshape(-1, 3).sum(0), atol=1e-12)
    # position orientation: an impulse in dy at an odd/even sub-position picks that tap only
    dyi = np.zeros_like(dy)
    dyi[0, 1, 2, 3, 2] = 1.0  # d=0,i=1 ; h=1,j=0 ; w=1,k=1
    dxi, dwi, _ = O.convtr3d_bwd(x, wt, dyi)
    np.testing.assert_allclose(dxi[0, 0, 1, 1, :], wt[:, 1, 0, 1, 2], atol=0)
    assert np.count_nonzero(dxi) == 4
    np.testing.assert_allclose(dwi[:, 1, 0, 1, 2], x[0, 0, 1, 1, :], atol=0)
    # beta accumulation
    _, acc, accb = O.convtr3d_bwd(x, wt, dy, want_dx=False, dwt_prev=dwt, db_prev=db, beta=1.0)
    np.testing.assert_allclose(acc, 2 * dwt, atol=1e-12)
    np.testing.assert_allclose(accb, 2 * db, atol=1e-12)


# ------------------------------------------------------------------------------ head / softmax / CE / bf16

def test_softmax_ce_closed_forms():
    V, K = 24, 10
    loss, d = O.cross_entropy(np.zeros((1, 2, 3, 4, K)), np.arange(V).reshape(1, 2, 3, 4) % K)
    assert abs(loss - np.log(10.0)) < 1e-14
    np.testing.assert_allclose(d.sum(-1), 0, atol=1e-16)
    loss5, _ = O.cross_entropy(np.full((1, 1, 1, 2, 5), 3.3), np.zeros((1, 1, 1, 2), dtype=np.int32))
    assert abs(loss5 - 1.6094379124341003) < 1e-14
    r = rng(17)
    lg = r.standard_normal((1, 2, 2, 2, 4)) * 3
    lab = r.integers(0, 4, (1, 2, 2, 2))
    loss, d = O.cross_entropy(lg, lab)
    hh = 1e-6
    for idx in [(0, 0, 0, 0, 0), (0, 1, 1, 1, 3), (0, 0, 1, 0, 2)]:
        lp, lm = lg.copy(), lg.copy()
        lp[idx] += hh
        lm[idx] -= hh
        fd = (O.cross_entropy(lp, lab)[0] - O.cross_entropy(lm, lab)[0]) / (2 * hh)
        assert abs(fd - d[idx]) < 1e-8
    # shift invariance and large-logit stability
    assert abs(O.cross_entropy(lg + 1000.0, lab)[0] - loss) < 1e-9


def test_head_is_centre_tap_conv_and_adjoint():
    r = rng(18)
    y = r.standard_normal((1, 3, 3, 3, 4))
    wh = r.standard_normal((5, 4))
    bh = r.standard_normal(5)
    w = np.zeros((5, 3, 3, 3, 4))
    w[:, 1, 1, 1, :] = wh
    np.testing.assert_allclose(O.head_fwd(y, wh, bh), O.conv3d_fwd(y, w, bh), atol=1e-13)
    dl = r.standard_normal((1, 3, 3, 3, 5))
    dy, dwh, dbh = O.head_bwd(y, wh, dl)
    L = np.sum(O.head_fwd(y, wh) * dl)
    assert abs(L - np.sum(dy * y)) < 1e-12 * max(1, abs(L)) and abs(L - np.sum(dwh * wh)) < 1e-12 * max(1, abs(L))
    np.testing.assert_allclose(dbh, dl.reshape(-1, 5).sum(0))


def test_round_bf16_known_values():
    # 1 + 2^-8 is a tie between 1 and 1+2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1+2^-6
    vals = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.3, 3.0e38 * 0 + 65504.0])
    out = O.round_bf16(vals)
    assert out[0] == 1.0 and out[1] == 1.0 and out[2] == 1.0 + 2 ** -7 and out[3] == 1.0 + 2 ** -6
    assert abs(out[4] + 0.3) <= 0.3 * 2 ** -8
    import torch

    t = torch.randn(1000, dtype=torch.float64, generator=torch.Generator().manual_seed(0))
    np.testing.assert_array_equal(O.round_bf16(t.numpy()), t.float().to(torch.bfloat16).double().numpy())


def test_rmsprop_matches_an_independent_implementation():
    """The oracle's RMSProp step against torch.optim.RMSprop (CPU, fp64) over several steps, and a
    closed form: with a constant gradient c and v0 = 0, v_t = (1 - alpha^t) c^2."""
    import torch
    r = np.random.Generator(np.random.PCG64(5))
    w0 = r.standard_normal((7, 5))
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.RMSprop([p], lr=1e-3, alpha=0.99, eps=1e-8)
    w, v = w0.copy(), np.zeros_like(w0)
    for step in range(5):
        g = r.standard_normal(w0.shape) * (10.0 ** (step - 2))
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, v = O.rmsprop_step(w, v, g, lr=1e-3, alpha=0.99, eps=1e-8)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-13, atol=1e-15)
    c, a = 0.3, 0.9
    w, v = np.zeros(3), np.zeros(3)
    for t in range(1, 6):
        w_prev = w
        w, v = O.rmsprop_step(w, v, np.full(3, c), lr=0.1, alpha=a, eps=0.0)
        np.testing.assert_allclose(v, (1 - a ** t) * c * c, rtol=1e-13)
        np.testing.assert_allclose(w_prev - w, 0.1 / np.sqrt(1 - a ** t), rtol=1e-13)


# ------------------------------------------------- squeeze-and-excitation on InstanceNorm + ReLU

def _se_case(seed, N=2, shape=(3, 4, 5), C=6, Cr=3):
    r = rng(seed)
    z = r.standard_normal((N,) + shape + (C,))
    gamma, beta = r.uniform(0.5, 1.5, C), r.uniform(-0.5, 0.5, C)
    w1, b1 = r.standard_normal((Cr, C)), r.uniform(0.1, 0.5, Cr)   # positive biases keep the hidden units off their kink
    w2, b2 = r.standard_normal((C, Cr)), r.standard_normal(C) * 0.3
    return r, z, gamma, beta, w1, b1, w2, b2


def test_se_gate_and_squeeze_by_explicit_loops():
    r, z, gamma, beta, w1, b1, w2, b2 = _se_case(61)
    res = r.standard_normal(z.shape)
    y, c = O.inorm_relu_se(z, gamma, beta, w1, b1, w2, b2, residual=res)
    a, _ = O.inorm_relu(z, gamma, beta)
    N, C, Cr = z.shape[0], z.shape[-1], w1.shape[0]
    V = z.size // (N * C)
    for n in range(N):
        m = [sum(a[n].reshape(V, C)[v, ch] for v in range(V)) / V for ch in range(C)]
        h = [max(0.0, sum(w1[j, ch] * m[ch] for ch in range(C)) + b1[j]) for j in range(Cr)]
        e = [1.0 / (1.0 + np.exp(-(sum(w2[ch, j] * h[j] for j in range(Cr)) + b2[ch]))) for ch in range(C)]
        assert all(0.0 < v < 1.0 for v in e)
        np.testing.assert_allclose(c["m"][n], m, rtol=1e-12)
        np.testing.assert_allclose(c["e"][n], e, rtol=1e-12)
        for ch in range(C):
            np.testing.assert_allclose(y[n, ..., ch], a[n, ..., ch] * e[ch] + res[n, ..., ch], rtol=1e-12, atol=1e-15)


def test_se_special_cases_reduce_to_plain_inorm_relu():
    r, z, gamma, beta, w1, b1, w2, b2 = _se_case(62)
    a, _ = O.inorm_relu(z, gamma, beta)
    # second layer switched off: the gate is sigmoid(0) = 1/2 everywhere
    y, _ = O.inorm_relu_se(z, gamma, beta, w1, b1, np.zeros_like(w2), np.zeros_like(b2))
    np.testing.assert_allclose(y, 0.5 * a, rtol=1e-14)
    # saturated gate: the block is InstanceNorm + ReLU itself, forward and backward
    big = np.full_like(b2, 40.0)
    y, _ = O.inorm_relu_se(z, gamma, beta, w1, b1, w2, big)
    np.testing.assert_allclose(y, a, rtol=1e-12)
    dy = r.standard_normal(z.shape)
    dz, dg, db, dw1, db1, dw2, db2 = O.inorm_relu_se_bwd(dy, z, gamma, beta, w1, b1, w2, big)
    dz0, dg0, db0 = O.inorm_relu_bwd(dy, z, gamma, beta)
    np.testing.assert_allclose(dz, dz0, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(dg, dg0, rtol=1e-9)
    assert np.abs(dw1).max() < 1e-12 and np.abs(dw2).max() < 1e-12   # a saturated gate passes no gradient


def test_se_backward_by_finite_differences():
    r, z, gamma, beta, w1, b1, w2, b2 = _se_case(63)
    res = r.standard_normal(z.shape)
    R = r.standard_normal(z.shape)          # L = <y, R>: upstream gradient dy = R
    grads = O.inorm_relu_se_bwd(R, z, gamma, beta, w1, b1, w2, b2)
    params = [z, gamma, beta, w1, b1, w2, b2]
    names = ["z", "gamma", "beta", "w1", "b1", "w2", "b2"]

    def loss():
        return float(np.sum(O.inorm_relu_se(z, gamma, beta, w1, b1, w2, b2, residual=res)[0] * R))

    hh = 1e-6
    for name, p, g in zip(names, params, grads):
        flat, gflat = p.reshape(-1), g.reshape(-1)
        for idx in r.choice(flat.size, size=min(6, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + hh
            lp = loss()
            flat[idx] = old - hh
            lm = loss()
            flat[idx] = old
            fd = (lp - lm) / (2 * hh)
            assert abs(fd - gflat[idx]) <= 1e-5 * max(1.0, abs(fd)), (name, idx, fd, gflat[idx])
    # the residual enters by plain addition: its gradient is the upstream gradient
    flat = res.reshape(-1)
    old = flat[7]
    flat[7] = old + hh
    lp = loss()
    flat[7] = old - hh
    lm = loss()
    flat[7] = old
    assert abs((lp - lm) / (2 * hh) - R.reshape(-1)[7]) < 1e-6
