"""Pins of the network-level oracle (Sec. 2.2 Eq. 2-3, Sec. 3 channel schedule) and of the
sliding-window oracle.  CPU only."""
import numpy as np
import pytest

import lamp_synth as S
import oracle as O
from oracle import sliding, unet


def make(levels, base, in_ch, classes, shape, seed, affine=True):
    r_p, r_x, r_l = S.streams(seed, 3)
    p = {k: v.astype(np.float64) for k, v in S.unet_params(r_p, levels, base, in_ch, classes, affine, test_mode=True).items()}
    x = r_x.standard_normal((shape[0],) + tuple(shape[1:]) + (in_ch,))
    lab = r_l.integers(0, classes, shape)
    return p, x, lab


def test_shape_walk_and_channel_schedule():
    # five encoder blocks, four skips, filters doubling from the first block (Sec. 2.2, Sec. 3)
    levels, base = 5, 2
    p, x, lab = make(levels, base, 1, 10, (1, 16, 16, 32), 1, affine=False)
    logits, cache = unet.forward(p, x, levels)
    assert logits.shape == (1, 16, 16, 32, 10)
    for l in range(1, levels + 1):
        C = base * 2 ** (l - 1)
        s = (1, 16 >> (l - 1), 16 >> (l - 1), 32 >> (l - 1))
        assert cache[f"enc{l}.conv1"]["z"].shape == s + (C,)
        assert cache[f"enc{l}.conv2"]["y"].shape == s + (C,)
        assert p[f"enc{l}.conv2.w"].shape == (C, 3, 3, 3, C)
    for l in range(1, levels):
        C = base * 2 ** (l - 1)
        assert cache[f"dec{l}.conv1"]["x"].shape[-1] == 2 * C  # concat of skip and upsampled
        assert p[f"dec{l}.up.w"].shape == (2 * C, 2, 2, 2, C)
        # skip occupies the first C channels of the concat
        np.testing.assert_array_equal(cache[f"dec{l}.conv1"]["x"][..., :C], cache[f"enc{l}.conv2"]["y"])
    assert "dec5.conv1" not in cache  # d_5 is the encoder output itself
    n_params = sum(v.size for v in S.unet_params(S.streams(0, 1)[0], 5, 32, 1, 10).values())
    assert n_params == 22_572_682  # 22.57 M for base 32, 10 classes


def test_tiny_config_param_count():
    # 3 levels, base 8, 1 input channel, 5 classes, no affine
    n = sum(v.size for v in S.unet_params(S.streams(0, 1)[0], 3, 8, 1, 5).values())
    conv = 27 * (1 * 8 + 8 * 8 + 8 * 16 + 16 * 16 + 16 * 32 + 32 * 32 + 32 * 16 + 16 * 16 + 16 * 8 + 8 * 8)
    up = 8 * (32 * 16 + 16 * 8) + 16 + 8
    head = 8 * 5 + 5
    assert n == conv + up + head == 84_893


def test_uniform_logits_loss_and_gradient_sum():
    levels = 2
    p, x, lab = make(levels, 2, 1, 5, (1, 4, 4, 4), 2)
    p["head.w"][:] = 0.0
    p["head.b"][:] = 0.7
    loss, grads, logits, _ = unet.loss_and_grads(p, x, lab, levels)
    assert abs(loss - np.log(5.0)) < 1e-12
    # with a zero head weight no gradient reaches the body
    assert all(np.all(grads[k] == 0) for k in grads if not k.startswith("head"))
    np.testing.assert_allclose(grads["head.b"].sum(), 0.0, atol=1e-14)


def test_whole_net_finite_differences_every_layer():
    levels = 3
    p, x, lab = make(levels, 2, 1, 3, (1, 8, 8, 8), 3)
    loss, grads, _, _ = unet.loss_and_grads(p, x, lab, levels)
    assert set(grads.keys()) == set(p.keys())
    r = np.random.Generator(np.random.PCG64(5))
    hh = 1e-6
    worst = 0.0
    for name in p:
        flat = p[name].reshape(-1)
        gflat = grads[name].reshape(-1)
        for idx in r.choice(flat.size, size=min(2, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + hh
            lp = O.cross_entropy(unet.forward(p, x, levels)[0], lab)[0]
            flat[idx] = old - hh
            lm = O.cross_entropy(unet.forward(p, x, levels)[0], lab)[0]
            flat[idx] = old
            fd = (lp - lm) / (2 * hh)
            err = abs(fd - gflat[idx]) / max(1e-4, abs(fd))
            worst = max(worst, err)
            assert err < 2e-4, (name, idx, fd, gflat[idx])
    assert worst < 2e-4


def make_se(levels, base, classes, shape, seed, ratio=2, affine=True):
    r_p, r_x, r_l = S.streams(seed, 3)
    p = {k: v.astype(np.float64)
         for k, v in S.unet_params(r_p, levels, base, 1, classes, affine, test_mode=True, se_ratio=ratio).items()}
    x = r_x.standard_normal((shape[0],) + tuple(shape[1:]) + (1,))
    lab = r_l.integers(0, classes, shape)
    return p, x, lab


def test_se_net_finite_differences_every_parameter():
    """The squeeze-and-excitation variant of the net (a reading of the cited block: gate on the second conv unit,
    first unit's output as the shortcut): gradients of every parameter tensor, the gate's included, against central
    finite differences of the loss."""
    levels = 3
    p, x, lab = make_se(levels, 4, 3, (2, 8, 8, 8), 13)
    assert sum(k.endswith(".se.w1") for k in p) == 2 * levels - 1      # one gate per block
    assert p["enc2.se.w1"].shape == (4, 8) and p["enc2.se.w2"].shape == (8, 4)
    loss, grads, _, _ = unet.loss_and_grads(p, x, lab, levels)
    assert set(grads.keys()) == set(p.keys())
    r = np.random.Generator(np.random.PCG64(15))
    hh = 1e-6
    for name in p:
        flat = p[name].reshape(-1)
        gflat = grads[name].reshape(-1)
        for idx in r.choice(flat.size, size=min(2, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + hh
            lp = O.cross_entropy(unet.forward(p, x, levels)[0], lab)[0]
            flat[idx] = old - hh
            lm = O.cross_entropy(unet.forward(p, x, levels)[0], lab)[0]
            flat[idx] = old
            fd = (lp - lm) / (2 * hh)
            assert abs(fd - gflat[idx]) / max(1e-4, abs(fd)) < 2e-4, (name, idx, fd, gflat[idx])


def test_se_net_closed_and_open_gate_special_cases():
    """Gate closed (b2 -> -inf, e = 0): every block returns its first unit's output, so the second convs and the
    gate's first layer get no gradient.  Gate saturated open (e = 1): the block is the plain residual block
    a1 + a2, written out here with the plain InstanceNorm + ReLU oracle."""
    levels = 2
    p, x, lab = make_se(levels, 4, 3, (1, 4, 4, 8), 17, affine=False)
    for k in p:
        if k.endswith(".se.w2"):
            p[k][:] = 0.0
        if k.endswith(".se.b2"):
            p[k][:] = -800.0
    loss, grads, logits, cache = unet.loss_and_grads(p, x, lab, levels)
    for blk in ("enc1", "enc2", "dec1"):
        np.testing.assert_array_equal(cache[f"{blk}.conv2"]["y"], cache[f"{blk}.conv1"]["y"])
        assert np.all(grads[f"{blk}.conv2.w"] == 0) and np.all(grads[f"{blk}.se.w1"] == 0)
    for k in p:
        if k.endswith(".se.b2"):
            p[k][:] = 800.0
    logits_open, cache = unet.forward(p, x, levels)
    a1 = cache["enc1.conv1"]["y"]
    a2, _ = O.inorm_relu(O.conv3d_fwd(a1, p["enc1.conv2.w"]))
    np.testing.assert_allclose(cache["enc1.conv2"]["y"], a1 + a2, rtol=0, atol=1e-13)


def test_stage_composition_equals_whole_net():
    # Eq. 3 == Eq. 2: cutting the sequence after encoder block 2 and carrying e_{1,1}, e_{2,1}
    levels = 3
    p, x, lab = make(levels, 2, 1, 3, (1, 8, 8, 8), 4)
    logits, cache = unet.forward(p, x, levels)
    (pooled, skips), scache = unet.forward(p, x, levels, first_level=1, last_level=2)
    np.testing.assert_array_equal(skips[0], cache["enc1.conv2"]["y"])
    np.testing.assert_array_equal(skips[1], cache["enc2.conv2"]["y"])
    np.testing.assert_array_equal(pooled, cache["enc3.conv1"]["x"])
    # stage backward with the gradients the rest of the net would hand back equals the whole-net grads
    loss, dl = O.cross_entropy(logits, lab)
    grads = unet.backward(p, cache, dl, levels)
    # recover upstream gradients of the stage outputs by finite-difference-free means: run the
    # remaining part's backward by hand
    g = {}
    gy, g["head.w"], g["head.b"] = O.head_bwd(cache["head"]["x"], p["head.w"], dl)
    skip_g = {}
    for l in (1, 2):
        gy = unet._block_bwd(p, f"dec{l}", gy, 1e-5, lambda a: a, cache, g)
        C = gy.shape[-1] // 2
        skip_g[l] = gy[..., :C]
        gy, _, _ = O.convtr3d_bwd(cache[f"dec{l}.up"]["x"], p[f"dec{l}.up.w"], np.ascontiguousarray(gy[..., C:]))
    g3 = unet._block_bwd(p, "enc3", gy, 1e-5, lambda a: a, cache, g)
    sg, _ = unet.stage_backward(p, scache, g3, [skip_g[1], skip_g[2]], 1, 2, levels)
    for k in sg:
        np.testing.assert_allclose(sg[k], grads[k], rtol=1e-10, atol=1e-14)


@pytest.mark.parametrize("cut", [1, 2])
def test_tail_after_stage_equals_whole_net(cut):
    # Eq. 3 == Eq. 2 for the other side of the cut: partition 0 followed by the tail is the whole net,
    # forward and backward, whose gradients the finite-difference pin above fixes
    levels = 3
    p, x, lab = make(levels, 2, 1, 3, (2, 8, 8, 8), 6)
    loss, grads, logits, _ = unet.loss_and_grads(p, x, lab, levels)
    (pooled, skips), c0 = unet.forward(p, x, levels, first_level=1, last_level=cut)
    tl, c1 = unet.tail_forward(p, pooled, skips, cut + 1, levels)
    np.testing.assert_array_equal(tl, logits)
    _, dl = O.cross_entropy(tl, lab)
    g1, g_pooled, g_skips = unet.tail_backward(p, c1, dl, cut + 1, levels)
    g0, _ = unet.stage_backward(p, c0, g_pooled, g_skips, 1, cut, levels)
    assert set(g0) | set(g1) == set(grads) and not set(g0) & set(g1)
    assert all(k.startswith(tuple(f"enc{l}." for l in range(1, cut + 1))) for k in g0)
    for k, v in {**g0, **g1}.items():
        np.testing.assert_allclose(v, grads[k], rtol=1e-10, atol=1e-14, err_msg=k)


def test_tail_input_gradients_by_finite_differences():
    # the gradients that cross the cut backwards (of the pooled tensor and of each skip copy e_{l,1})
    levels, cut = 3, 2
    p, x, lab = make(levels, 2, 1, 3, (1, 8, 8, 8), 8)
    (pooled, skips), _ = unet.forward(p, x, levels, first_level=1, last_level=cut)
    logits, c1 = unet.tail_forward(p, pooled, skips, cut + 1, levels)
    _, dl = O.cross_entropy(logits, lab)
    _, g_pooled, g_skips = unet.tail_backward(p, c1, dl, cut + 1, levels)
    r = np.random.Generator(np.random.PCG64(9))
    hh = 1e-6
    for t, g in [(pooled, g_pooled), (skips[0], g_skips[0]), (skips[1], g_skips[1])]:
        assert g.shape == t.shape
        flat, gflat = t.reshape(-1), g.reshape(-1)
        for idx in r.choice(flat.size, size=3, replace=False):
            old = flat[idx]
            flat[idx] = old + hh
            lp = O.cross_entropy(unet.tail_forward(p, pooled, skips, cut + 1, levels)[0], lab)[0]
            flat[idx] = old - hh
            lm = O.cross_entropy(unet.tail_forward(p, pooled, skips, cut + 1, levels)[0], lab)[0]
            flat[idx] = old
            fd = (lp - lm) / (2 * hh)
            assert abs(fd - gflat[idx]) <= 2e-4 * max(1e-4, abs(fd)), (idx, fd, gflat[idx])


@pytest.mark.parametrize("M", [2, 4])
def test_micro_batches_add_up_to_the_mini_batch(M):
    # Sec. 2.1: splitting the mini-batch into micro-batches changes nothing here because the
    # normalisation is per sample: loss and accumulated gradients equal the whole mini-batch's
    levels = 3
    p, x, lab = make(levels, 2, 1, 3, (4, 8, 8, 8), 7)
    loss, grads, _, _ = unet.loss_and_grads(p, x, lab, levels)
    pl, pg = unet.pipeline_loss_and_grads(p, x, lab, levels, cut=1, micro_batches=M)
    assert abs(pl - loss) <= 1e-12 * abs(loss)
    assert set(pg) == set(grads)
    for k in grads:
        np.testing.assert_allclose(pg[k], grads[k], rtol=1e-9, atol=1e-14, err_msg=k)


def test_bias_free_blocks_are_exact():
    # InstanceNorm removes a per-channel constant: adding a conv bias would change nothing
    levels = 2
    p, x, lab = make(levels, 2, 1, 3, (1, 4, 4, 4), 6)
    z = O.conv3d_fwd(x, p["enc1.conv1.w"])
    y0, _ = O.inorm_relu(z)
    y1, _ = O.inorm_relu(O.conv3d_fwd(x, p["enc1.conv1.w"], np.array([0.3, -1.1])))
    np.testing.assert_allclose(y0, y1, atol=1e-12)


def test_storage_emulation_rounds_only_storage():
    levels = 2
    p, x, lab = make(levels, 4, 1, 3, (1, 4, 4, 4), 7)
    pb = {k: O.round_bf16(v) for k, v in p.items()}
    xb = O.round_bf16(x)
    lg64, _ = unet.forward(pb, xb, levels)
    lgbf, cache = unet.forward(pb, xb, levels, store=O.round_bf16)
    z = cache["enc1.conv1"]["z"]
    np.testing.assert_array_equal(z, O.round_bf16(z))
    e = np.max(np.abs(lg64 - lgbf)) / np.max(np.abs(lg64))
    assert 0 < e < 5e-2


# ---------------------------------------------------------------------------------- sliding window

def test_window_grid_of_large_input_config():
    # 256 x 256 x 160 with 64^3 windows and 0.25 overlap: 5*5*3 = 75 windows, exact cover
    assert sliding.window_starts(256, 64) == [0, 48, 96, 144, 192]
    assert sliding.window_starts(160, 64) == [0, 48, 96]
    assert sliding.window_starts(64, 64) == [0]
    assert sliding.window_starts(100, 64) == [0, 36]
    n = len(sliding.window_starts(256, 64)) ** 2 * len(sliding.window_starts(160, 64))
    assert n == 75
    assert 75 * 64 ** 3 / (256 * 256 * 160) == 1.875


def test_gaussian_map_symmetry_and_extremes():
    g = sliding.gaussian_map(64)
    np.testing.assert_array_equal(g, g[::-1, ::-1, ::-1])
    np.testing.assert_allclose(g, np.transpose(g, (2, 0, 1)), rtol=1e-14)
    assert g.max() == g[31, 31, 31] == g[32, 32, 32]
    assert abs(g[31, 31, 31] - np.exp(-0.5 * 3 * 0.25 / 64.0)) < 1e-15
    assert abs(g.min() / np.exp(-0.5 * 3 * 31.5 ** 2 / 64.0) - 1) < 1e-12 and 7e-11 < g.min() < 9e-11


def test_blend_reproduces_per_voxel_maps_exactly():
    r = np.random.Generator(np.random.PCG64(8))
    vol = r.standard_normal((1, 20, 12, 16, 2))
    m = r.standard_normal((3, 2))

    def net(win):  # per-voxel map: sum(g f(v)) / sum(g) = f(v)
        return np.tanh(win @ m.T)

    out = sliding.sliding_window(net, vol, patch=8)
    np.testing.assert_allclose(out, net(vol), rtol=1e-12, atol=1e-13)


def test_blend_weights_windows_by_gaussian():
    # two windows along one axis (length 12, patch 8, starts 0 and 4) with constant outputs 1 and 3
    calls = []

    def net(win):
        calls.append(1)
        return np.full(win.shape[:-1] + (1,), 1.0 if len(calls) == 1 else 3.0)

    out = sliding.sliding_window(net, np.zeros((1, 8, 8, 12, 1)), patch=8, overlap=0.5)
    assert len(calls) == 2
    g1 = np.exp(-0.5 * ((np.arange(8) - 3.5) / 1.0) ** 2)
    for w in range(12):
        a = g1[w] if w < 8 else 0.0
        b = g1[w - 4] if w >= 4 else 0.0
        assert abs(out[0, 3, 3, w, 0] - (a * 1 + b * 3) / (a + b)) < 1e-12
