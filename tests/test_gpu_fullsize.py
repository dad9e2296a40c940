"""Parity at the benchmark's full size and launch configuration: the conv block of the headline
workload (1 x 128^3 x 64 -> 64, bf16 storage / fp32 accumulation, InstanceNorm + ReLU) forward,
data-gradient and weight-gradient, exactly the calls bench.py times.

The O(V * 27 * C^2) results are checked on sampled outputs the oracle computes one by one (>= 4096
voxels x all channels, forcing the 8 corners, edges, faces and coordinates on both sides of every
kind of tile boundary); the O(V) results (statistics, normalise+ReLU, its backward) in full.
"""
import os

import numpy as np
import pytest
import torch

import lamp_synth as S
import oracle as O
from gpu_util import DEV, as64, check

pytestmark = pytest.mark.gpu
BF, F32 = torch.bfloat16, torch.float32
D = 128
C = 64


@pytest.fixture(scope="module")
def L():
    import paper_2006_12575_amd as L
    L.lib()
    return L


@pytest.fixture(scope="module")
def block(L):
    rx, rw, rg = S.streams(1002, 3)

    def normal_dev(rng, shape):
        t = torch.empty(shape, dtype=BF, device=DEV)
        for d in range(shape[1]):
            t[:, d] = torch.from_numpy(S.normal(rng, (shape[0],) + tuple(shape[2:]))).to(BF).to(DEV)
        return t

    x = normal_dev(rx, (1, D, D, D, C))
    dy = normal_dev(rg, (1, D, D, D, C))
    w = torch.from_numpy(S.kaiming_conv(rw, C, C)).to(BF).to(DEV)
    z, y, dz, dx = (torch.empty_like(x) for _ in range(4))
    dw = torch.empty(w.shape, dtype=F32, device=DEV)
    st = torch.empty((1, C, 2), dtype=F32, device=DEV)
    L.lamp_conv3d_fwd(x, w, z, stats_out=st)
    L.lamp_inorm_relu(z, y, st, stats_given=True)
    L.lamp_inorm_relu_bwd(dy, z, st, dz)
    L.lamp_conv3d_dgrad(dz, w, dx)
    L.lamp_conv3d_wgrad(x, dz, dw)
    torch.cuda.synchronize()
    return dict(x=x, dy=dy, w=w, z=z, y=y, dz=dz, dx=dx, dw=dw, st=st)


def sample_coords(rng, n_random=3900):
    special = [0, 1, 7, 8, 9, 15, 16, 17, 63, 64, 65, 119, 120, 126, 127]  # borders and tile edges (8 / 16)
    pts = set()
    for d in (0, D - 1):
        for h in (0, D - 1):
            for w in (0, D - 1):
                pts.add((0, d, h, w))
    for a in special:
        for b in special[::3]:
            pts.add((0, a, b, 0)); pts.add((0, 0, a, b)); pts.add((0, b, D - 1, a)); pts.add((0, a, 64, b)); pts.add((0, 64, b, a))
    target = len(pts) + n_random
    while len(pts) < target:
        pts.add((0,) + tuple(int(v) for v in rng.integers(0, D, 3)))
    return sorted(pts)


def test_conv_fwd_sampled(block):
    r = np.random.Generator(np.random.PCG64(31))
    coords = sample_coords(r)
    assert len(coords) >= 4096
    x = block["x"].cpu().float().numpy()
    z = block["z"].cpu().float().numpy()
    ref = O.conv3d_fwd_at(x, as64(block["w"]), None, coords)
    got = np.stack([z[c] for c in coords]).astype(np.float64)
    e = check(got, ref, BF, "full-size conv fwd (sampled)")
    print(f"conv fwd sampled {len(coords)} voxels x {C} ch: E_inf = {e:.2e}")


def test_stats_and_inorm_relu_full(block):
    z = block["z"].cpu().float().numpy().astype(np.float64).reshape(-1, C)
    mean, var = z.mean(0), z.var(0)
    st = as64(block["st"])[0]
    np.testing.assert_allclose(st[:, 0], mean, atol=2e-5)
    np.testing.assert_allclose(st[:, 1], 1.0 / np.sqrt(var + 1e-5), rtol=1e-4)
    y_ref = np.maximum((z - mean) / np.sqrt(var + 1e-5), 0.0)
    check(block["y"].cpu().float().numpy().reshape(-1, C), y_ref, BF, "full-size inorm+relu")


def test_inorm_bwd_full(block):
    z = block["z"].cpu().float().numpy().astype(np.float64)
    dy = block["dy"].cpu().float().numpy().astype(np.float64)
    dz_ref, _, _ = O.inorm_relu_bwd(dy, z)
    u_ref, _ = O.inorm_relu(z, relu=False)
    near = np.abs(u_ref) <= 1e-3
    check(block["dz"].cpu().float().numpy(), dz_ref, BF, "full-size inorm bwd", ignore=near)
    assert near.mean() < 2e-3


def test_conv_dgrad_sampled(block):
    r = np.random.Generator(np.random.PCG64(32))
    coords = sample_coords(r)
    dz = block["dz"].cpu().float().numpy()
    dx = block["dx"].cpu().float().numpy()
    ref = O.conv3d_dgrad_at(dz, as64(block["w"]), coords)
    got = np.stack([dx[c] for c in coords]).astype(np.float64)
    e = check(got, ref, BF, "full-size conv dgrad (sampled)")
    print(f"conv dgrad sampled {len(coords)} voxels: E_inf = {e:.2e}")


def test_conv_wgrad_sampled(block):
    r = np.random.Generator(np.random.PCG64(33))
    x = block["x"].cpu().float().numpy()
    dz = block["dz"].cpu().float().numpy()
    # every tap at every combination of the channels next to the 32-channel block boundaries (the weight-gradient
    # kernel's workgroup blocks of input channels and fragment blocks of output channels), then random entries
    edge = (0, 31, 32, C - 1)
    ent = {(co, t // 9, (t // 3) % 3, t % 3, ci) for t in range(27) for co in edge for ci in edge}
    rc = [int(v) for v in r.integers(0, C, 6)]
    while len(ent) < 27 * 16 + 120:
        ent.add((rc[int(r.integers(6))], int(r.integers(3)), int(r.integers(3)), int(r.integers(3)), rc[int(r.integers(6))]))
    ent = sorted(ent)
    ref = O.conv3d_wgrad_at(x, dz, ent)
    dw = as64(block["dw"])
    got = np.array([dw[e] for e in ent])
    scale = np.abs(dw).max()
    err = np.max(np.abs(got - ref)) / scale
    print(f"conv wgrad sampled {len(ent)} entries: E_inf = {err:.2e}")
    assert err <= 2e-3
    assert np.all(np.isfinite(dw))


def test_full_size_determinism(L, block):
    z2 = torch.empty_like(block["z"])
    st2 = torch.empty_like(block["st"])
    dw2 = torch.empty_like(block["dw"])
    dx2 = torch.empty_like(block["dx"])
    L.lamp_conv3d_fwd(block["x"], block["w"], z2, stats_out=st2)
    L.lamp_conv3d_dgrad(block["dz"], block["w"], dx2)
    L.lamp_conv3d_wgrad(block["x"], block["dz"], dw2)
    assert torch.equal(z2, block["z"]) and torch.equal(st2, block["st"])
    assert torch.equal(dx2, block["dx"]) and torch.equal(dw2, block["dw"])


def test_se_block_fullsize(L, block):
    """The squeeze-and-excitation block at the size bench.py's se_block workload runs it (1 x 128^3 x
    64, bf16, reduction ratio 16, with residual): z and its statistics are the conv block's own, the
    block input serves as the residual.  O(V) work, so every output is checked in full."""
    z, st, dy, res = block["z"], block["st"], block["dy"], block["x"]
    Cr = C // 16
    r = np.random.Generator(np.random.PCG64(41))
    w1 = torch.from_numpy(r.standard_normal((Cr, C)) / np.sqrt(C)).to(F32).to(DEV)
    b1 = torch.from_numpy(r.uniform(0.2, 0.6, Cr)).to(F32).to(DEV)
    w2 = torch.from_numpy(r.standard_normal((C, Cr)) / np.sqrt(Cr)).to(F32).to(DEV)
    b2 = torch.from_numpy(r.standard_normal(C) * 0.3).to(F32).to(DEV)
    y, dz = torch.empty_like(z), torch.empty_like(z)
    save = torch.empty((1, 4 * C + Cr), dtype=F32, device=DEV)
    g = dict(dw1=torch.empty_like(w1), db1=torch.empty_like(b1), dw2=torch.empty_like(w2), db2=torch.empty_like(b2))
    L.lamp_inorm_relu_se(z, st, w1, w2, y, save, b1=b1, b2=b2, residual=res)
    L.lamp_inorm_relu_se_bwd(dy, z, st, w1, w2, save, dz, **g)
    z64 = z.cpu().float().numpy().astype(np.float64)
    res64 = res.cpu().float().numpy().astype(np.float64)
    y_ref, c = O.inorm_relu_se(z64, None, None, as64(w1), as64(b1), as64(w2), as64(b2), residual=res64)
    check(y.cpu().float().numpy(), y_ref, BF, "full-size se forward")
    del y_ref, res64
    np.testing.assert_allclose(as64(save)[0, :C], c["m"][0], rtol=1e-4)
    np.testing.assert_allclose(as64(save)[0, C:2 * C], c["e"][0], rtol=1e-4)
    dy64 = dy.cpu().float().numpy().astype(np.float64)
    ref = O.inorm_relu_se_bwd(dy64, z64, None, None, as64(w1), as64(b1), as64(w2), as64(b2))
    u_ref, _ = O.inorm_relu(z64, relu=False)
    near = np.abs(u_ref) <= 1e-3
    del u_ref
    check(dz.cpu().float().numpy(), ref[0], BF, "full-size se backward dz", ignore=near)
    for name, rf in zip(["dw1", "db1", "dw2", "db2"], ref[3:]):
        check(as64(g[name]), rf, F32, f"full-size se {name}", tol=2e-3)


@pytest.mark.timeout(900)
def test_unet_train_fullsize_sampled(L):
    """The whole-volume training workload at its full size (5 levels, base 32, 2 x 128^3 CT-like
    volumes with organ labels, 10 classes, bf16): (a) the layer-by-layer chain, every layer checked
    against the oracle on the GPU's own inputs of that layer -- 3x3x3 convolutions on sampled
    outputs, every O(V) op in full; (b) the whole-network entry point, as bench.py calls it, equal
    to that chain bit for bit (logits, loss, every gradient)."""
    from gpu_chain import Chain
    from test_gpu_unet import make_net
    levels, base, K, dims = 5, 32, 10, (2, 128, 128, 128)
    N, Dd, H, W = dims
    names, dev, _ = make_net(levels, base, 1, K, False, BF, 1004)
    rx, rl = S.streams(1004, 3)[1:]
    x = torch.from_numpy(S.ct_volume(rx, N, Dd, H, W)).to(BF).to(DEV).reshape(N, Dd, H, W, 1)
    lab = torch.from_numpy(S.organ_labels(rl, N, Dd, H, W, K)).to(DEV)
    ud = L.unet_desc(levels, base, 1, K, N, Dd, H, W, BF)
    logits = torch.empty((N, Dd, H, W, K), dtype=F32, device=DEV)
    loss = torch.empty((), dtype=F32, device=DEV)
    grads = [torch.empty(t.shape, dtype=F32, device=DEV) for t in dev]
    L.lamp_unet_fwd_bwd(ud, dev, x, lab, loss, grads, logits=logits)
    ch = Chain(L, levels, base, 1, K, False, BF, names, dev, verify="sampled")
    lg = ch.forward(x)
    print("forward checked:", ch.checked, flush=True)
    assert torch.equal(lg, logits), "whole-net logits differ from the layer-by-layer chain"
    loss_c, g_c = ch.backward(lab)
    assert torch.equal(loss_c, loss)
    for k, g in zip(names, grads):
        assert torch.equal(g_c[k], g), f"whole-net grad {k} differs from the layer-by-layer chain"
    print("checked ops:", ch.checked)
    print("worst teacher-forced E_inf per op:", {k: f"{v:.1e}" for k, v in ch.worst.items()})
    assert ch.checked["conv fwd"] == 18 and ch.checked["conv dgrad"] == 17 and ch.checked["conv wgrad"] == 18


@pytest.mark.timeout(600)
def test_pipeline_fullsize_vs_whole_net(L):
    """The training mini-batch (2 x 128^3, 5 levels, base 32) as bench.py's pipeline workload runs it:
    two partitions (cut after encoder block 2) on two streams, one sample per micro-batch.
    (a) Exact: with two micro-batches every gradient is half the sum of the two samples' own
    whole-net gradients, accumulated in the schedule's order (halving is exact in binary floating
    point, so the comparison is bit for bit).  (b) Against the whole-net call on the mini-batch of
    two, the call the sampled chain test verifies: logits to the bf16 bound, gradients by direction
    (the end-to-end gradients of two bf16 realisations drift apart through near-tie flips)."""
    from test_gpu_unet import make_net
    levels, base, K, cut, M = 5, 32, 10, 2, 2
    N, Dd, H, W = 2, 128, 128, 128
    names, dev, _ = make_net(levels, base, 1, K, False, BF, 1004)
    rx, rl = S.streams(1004, 3)[1:]
    x = torch.from_numpy(S.ct_volume(rx, N, Dd, H, W)).to(BF).to(DEV).reshape(N, Dd, H, W, 1)
    lab = torch.from_numpy(S.organ_labels(rl, N, Dd, H, W, K)).to(DEV)
    mb = L.unet_desc(levels, base, 1, K, 1, Dd, H, W, BF)
    aux = torch.cuda.Stream()
    g = [torch.full(t.shape, float("nan"), dtype=F32, device=DEV) for t in dev]
    loss = torch.full((), float("nan"), dtype=F32, device=DEV)
    lg = torch.empty((N, Dd, H, W, K), dtype=F32, device=DEV)
    L.lamp_unet_pipeline_fwd_bwd(mb, cut, M, dev, x, lab, loss, g, aux, logits=lg)
    torch.cuda.current_stream().synchronize()
    # (a) the samples one at a time through the whole-net entry point, last micro-batch first
    g1 = [torch.empty(t.shape, dtype=F32, device=DEV) for t in dev]
    l1 = [torch.empty((), dtype=F32, device=DEV) for _ in range(M)]
    lg1 = torch.empty_like(lg)
    for i, m in enumerate(reversed(range(M))):
        L.lamp_unet_fwd_bwd(mb, dev, x[m:m + 1], lab[m:m + 1], l1[m], g1, logits=lg1[m:m + 1], beta=0.0 if i == 0 else 1.0)
    assert torch.equal(lg, lg1), "pipeline logits differ from the per-sample whole-net runs"
    assert abs(loss.item() - 0.5 * (l1[0].item() + l1[1].item())) <= 1e-6 * loss.item()
    for k, a, b in zip(names, g, g1):
        assert torch.equal(a, 0.5 * b), f"pipeline grad {k} is not half the sum of the per-sample gradients"
    # (b) the mini-batch in one whole-net call
    full = L.unet_desc(levels, base, 1, K, N, Dd, H, W, BF)
    gf = [torch.empty(t.shape, dtype=F32, device=DEV) for t in dev]
    lf = torch.empty((), dtype=F32, device=DEV)
    L.lamp_unet_fwd_bwd(full, dev, x, lab, lf, gf, logits=lg1)
    check(as64(lg[:, ::4, ::4, ::4]), as64(lg1[:, ::4, ::4, ::4]), BF, "pipeline logits vs mini-batch run")
    assert abs(loss.item() - lf.item()) <= 1e-3 * lf.item()
    for k, a, b in zip(names, g, gf):   # two bf16 realisations of a deep net (the kernels' tiling follows the batch)
        a, b = as64(a).ravel(), as64(b).ravel()
        cos = float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))
        assert cos > 0.95, f"pipeline grad {k} vs mini-batch run: cosine {cos:.4f}"


@pytest.mark.timeout(900)
@pytest.mark.parametrize("dims,seed", [((256, 256, 160), 1005), ((352, 256, 288), 1008)], ids=["256x256x160", "352x256x288"])
def test_unet_infer_fullsize_sampled(L, dims, seed):
    """Large-input inference at its full size (1 x 256 x 256 x 160 CT-like volume, 5 levels, base 32,
    bf16): the layer-by-layer forward chain with sampled / full oracle checks of every layer, and
    the whole-network forward entry point equal to it bit for bit.  The whole head-and-neck sized
    volume with unequal axes (352 x 256 x 288, Sec. 3) is the second case."""
    from gpu_chain import Chain
    from test_gpu_unet import make_net
    levels, base, K = 5, 32, 10
    N, (Dd, H, W) = 1, dims
    names, dev, _ = make_net(levels, base, 1, K, False, BF, seed)
    x = torch.from_numpy(S.ct_volume(S.streams(seed, 2)[1], N, Dd, H, W)).to(BF).to(DEV)
    ud = L.unet_desc(levels, base, 1, K, N, Dd, H, W, BF)
    logits = torch.empty((N, Dd, H, W, K), dtype=F32, device=DEV)
    L.lamp_unet_fwd(ud, dev, x, logits)
    ch = Chain(L, levels, base, 1, K, False, BF, names, dev, verify="sampled")
    lg = ch.forward(x)
    assert torch.equal(lg, logits), "whole-net logits differ from the layer-by-layer chain"
    print("checked ops:", ch.checked)
    print("worst teacher-forced E_inf per op:", {k: f"{v:.1e}" for k, v in ch.worst.items()})
    assert ch.checked["conv fwd"] == 18 and ch.checked["convtr fwd"] == 4 and ch.checked["pool fwd"] == 4


@pytest.mark.timeout(900)
def test_sliding_window_fullsize(L):
    """Sliding-window inference at its full size (75 windows of 64^3, overlap 0.25, over
    256 x 256 x 160): window enumeration, extraction, Gaussian weights, blending and normalisation
    against the oracle's sliding-window routine.  The oracle's `net` argument is the GPU patch
    network run on the windows the ORACLE's enumeration extracts (same batch as the entry point
    uses), so this isolates everything the sliding-window path adds to the patch network, whose
    own parity the chain tests cover."""
    from oracle import sliding
    from test_gpu_unet import make_net
    levels, base, K, P = 5, 32, 10, 64
    Dd, H, W = 256, 256, 160
    names, dev, _ = make_net(levels, base, 1, K, False, BF, 1005)
    vol = torch.from_numpy(S.ct_volume(S.streams(1005, 2)[1], 1, Dd, H, W)).to(BF).to(DEV)
    cnt = L.lamp_sliding_window_count(Dd, H, W, P, 0.25)
    starts = [sliding.window_starts(n, P) for n in (Dd, H, W)]
    assert cnt == len(starts[0]) * len(starts[1]) * len(starts[2]) == 75
    pd = L.unet_desc(levels, base, 1, K, cnt, P, P, P, BF)
    out = torch.empty((1, Dd, H, W, K), dtype=F32, device=DEV)
    L.lamp_sliding_window_fwd(pd, dev, vol, out)
    # patch logits of the oracle-enumerated windows, one batched GPU forward
    wins = torch.stack([vol[0, d0:d0 + P, h0:h0 + P, w0:w0 + P, :] for d0 in starts[0] for h0 in starts[1] for w0 in starts[2]])
    plog = torch.empty((cnt, P, P, P, K), dtype=F32, device=DEV)
    L.lamp_unet_fwd(pd, dev, wins.contiguous(), plog)
    plog_h, wins_h = as64(plog), as64(wins)
    k = [0]

    def net(win):
        i = k[0]
        k[0] += 1
        np.testing.assert_array_equal(win[0], wins_h[i])
        return plog_h[i:i + 1]

    ref = sliding.sliding_window(net, as64(vol), patch=P)
    assert k[0] == cnt
    e = check(as64(out), ref, F32, "full-size sliding-window logits", tol=1e-4)
    print(f"sliding window, {cnt} windows: E_inf = {e:.2e}")
    # cross-check with the one-pass forward: both segment the volume alike away from near-ties
    ud = L.unet_desc(levels, base, 1, K, 1, Dd, H, W, BF)
    whole = torch.empty_like(out)
    L.lamp_unet_fwd(ud, dev, vol, whole)
    agree = (whole.argmax(-1) == out.argmax(-1)).float().mean().item()
    print(f"arg-max agreement one pass vs sliding windows: {agree:.4f}")


@pytest.mark.timeout(900)
def test_stage_fullsize_sampled(L):
    """One pipeline partition (encoder blocks 1-2, base 64; Sec. 2.1 / Eq. 3) at its full size,
    1 x 192^3 CT-like input, bf16, forward + backward as bench.py times it: the partition's
    outputs and gradients equal, bit for bit, the layer-by-layer chain whose layers are checked
    against the oracle (3x3x3 convolutions on sampled outputs, O(V) ops in full)."""
    from gpu_chain import Chain
    from test_gpu_unet import make_net
    levels, base, K = 3, 64, 10
    N, Dd, H, W = 1, 192, 192, 192
    names, dev, _ = make_net(levels, base, 1, K, False, BF, 1003)
    sp = dev[:4]
    rx, rg = S.streams(1003, 3)[1:]
    x = torch.from_numpy(S.ct_volume(rx, N, Dd, H, W)).to(BF).to(DEV)
    ud = L.unet_desc(levels, base, 1, K, N, Dd, H, W, BF)
    ws = torch.empty(L.lamp_unet_stage_workspace_bytes(ud, 1, 2), dtype=torch.uint8, device=DEV)
    pooled = torch.empty((N, Dd // 4, H // 4, W // 4, 2 * base), dtype=BF, device=DEV)
    skips = [torch.empty((N, Dd, H, W, base), dtype=BF, device=DEV),
             torch.empty((N, Dd // 2, H // 2, W // 2, 2 * base), dtype=BF, device=DEV)]
    L.lamp_unet_stage_fwd(ud, 1, 2, sp, x, pooled, skips, ws)
    ch = Chain(L, levels, base, 1, K, False, BF, names, dev, verify="sampled")
    ch.nsample = 256
    # blocks 1-2 of the chain (forward of the whole net is not needed)
    ch.enc, ch.pooled = {}, {}
    cur = x
    for l in (1, 2):
        ch.enc[l] = ch.block(f"enc{l}", cur)
        yv = ch.enc[l][1]["y"]
        p = torch.empty((N, yv.shape[1] // 2, yv.shape[2] // 2, yv.shape[3] // 2, yv.shape[4]), dtype=BF, device=DEV)
        L.lamp_maxpool2_fwd(yv, p)
        np.testing.assert_array_equal(as64(p), O.maxpool2_fwd(as64(yv)))
        ch.pooled[l] = cur = p
    assert torch.equal(skips[0], ch.enc[1][1]["y"]) and torch.equal(skips[1], ch.enc[2][1]["y"])
    assert torch.equal(pooled, ch.pooled[2])
    print("stage forward checked:", ch.checked, flush=True)

    def dev_normal(shape):
        t = torch.empty(shape, dtype=BF, device=DEV)
        for d in range(shape[1]):
            t[:, d] = torch.from_numpy(S.normal(rg, (shape[0],) + tuple(shape[2:]))).to(BF).to(DEV)
        return t

    gp = dev_normal(pooled.shape)
    gs = [dev_normal(s.shape) for s in skips]
    grads = [torch.empty(t.shape, dtype=F32, device=DEV) for t in sp]
    L.lamp_unet_stage_bwd(ud, 1, 2, sp, x, skips, gp, gs, grads, ws)
    cg = {}
    g = gp
    for l in (2, 1):
        c1, c2 = ch.enc[l]
        gy = torch.empty(c2["y"].shape, dtype=BF, device=DEV)
        L.lamp_maxpool2_bwd(c2["y"], g, gy, add=gs[l - 1])
        ref = O.maxpool2_bwd(as64(c2["y"]), as64(g)) + as64(gs[l - 1])
        check(as64(gy), ref, BF, f"pool bwd: enc{l}", tol=4e-3)
        del ref
        g = ch.conv_bwd(c2, gy, cg, True, below=c1)
        g = ch.conv_bwd(c1, g, cg, l > 1, dz_ready=True)
    for kname, gr in zip(names[:4], grads):
        assert torch.equal(gr, cg[kname]), f"stage grad {kname} differs from the chain"
    print("checked ops:", ch.checked)
    print("worst teacher-forced E_inf per op:", {k_: f"{v:.1e}" for k_, v in ch.worst.items()})


# bench.py times the wide nets on 2 x 128^3 (base 64) and 1 x 128^3 (base 128); the routine suite checks them
# on half / an eighth of that (same kernels: the ring kernel at level 1 of base 64, every 1024- and
# 2048-channel layer); LAMP_TEST_WIDE_FULL=1 runs the bench sizes (4 minutes: passed when this was written).
import os
_WIDE = ([(64, (2, 128, 128, 128), 1006), (128, (1, 128, 128, 128), 1007)] if os.environ.get("LAMP_TEST_WIDE_FULL")
         else [(64, (1, 128, 128, 128), 1006), (128, (1, 64, 64, 64), 1007)])


@pytest.mark.timeout(900)
@pytest.mark.parametrize("base,dims,seed", _WIDE, ids=["base64", "base128"])
def test_wide_unet_train_sampled(L, base, dims, seed):
    """The paper's wider nets (Sec. 3: 64 and 128 base filters, up to 1024 / 2048 channels):
    layer-by-layer chain with sampled oracle checks of the 3x3x3 convolutions and full checks of
    the O(V) ops, whole-network entry point equal to it bit for bit."""
    from gpu_chain import Chain
    from test_gpu_unet import make_net
    levels, K = 5, 10
    N, Dd, H, W = dims
    names, dev, _ = make_net(levels, base, 1, K, False, BF, seed)
    rx, rl = S.streams(seed, 3)[1:]
    x = torch.from_numpy(S.ct_volume(rx, N, Dd, H, W)).to(BF).to(DEV)
    lab = torch.from_numpy(S.organ_labels(rl, N, Dd, H, W, K)).to(DEV)
    ud = L.unet_desc(levels, base, 1, K, N, Dd, H, W, BF)
    logits = torch.empty((N, Dd, H, W, K), dtype=F32, device=DEV)
    loss = torch.empty((), dtype=F32, device=DEV)
    grads = [torch.empty(t.shape, dtype=F32, device=DEV) for t in dev]
    L.lamp_unet_fwd_bwd(ud, dev, x, lab, loss, grads, logits=logits)
    ch = Chain(L, levels, base, 1, K, False, BF, names, dev, verify="sampled")
    ch.nsample = 256
    lg = ch.forward(x)
    print("forward checked:", ch.checked, flush=True)
    assert torch.equal(lg, logits), "whole-net logits differ from the layer-by-layer chain"
    loss_c, g_c = ch.backward(lab)
    assert torch.equal(loss_c, loss)
    for k, g in zip(names, grads):
        assert torch.equal(g_c[k], g), f"whole-net grad {k} differs from the layer-by-layer chain"
    print("checked ops:", ch.checked)
    print("worst teacher-forced E_inf per op:", {k: f"{v:.1e}" for k, v in ch.worst.items()})
    assert ch.checked["conv fwd"] == 18 and ch.checked["conv dgrad"] == 17 and ch.checked["conv wgrad"] == 18


@pytest.mark.timeout(600)
@pytest.mark.parametrize("shape", [(1, 8, 8, 8, 2048, 2048), (1, 16, 16, 16, 2048, 1024), (2, 8, 8, 8, 1024, 1024)],
                         ids=["base128-level5", "base128-dec4", "base64-level5"])
def test_wide_layers_at_bench_size(L, shape):
    """The 1024- and 2048-channel convolutions of the wide nets at exactly the shapes bench.py times them on
    (base 128 on 1 x 128^3: 8^3 and 16^3 voxels at levels 5 and 4; base 64 on 2 x 128^3: 2 x 8^3): forward with
    fused statistics, data gradient and weight gradient through the layer entry points, checked on sampled
    outputs (at least 128 voxels x all channels; every tap and block boundary of the weight gradient) that the
    oracle computes one by one from the same inputs."""
    from gpu_chain import Chain
    N, D, H, W, Ci, Co = shape
    r = np.random.Generator(np.random.PCG64(4000 + Ci + Co))
    x = torch.from_numpy(S.normal(r, (N, D, H, W, Ci))).to(BF).to(DEV)
    w = torch.from_numpy(S.kaiming_conv(r, Co, Ci)).to(BF).to(DEV)
    dz = torch.from_numpy(S.normal(r, (N, D, H, W, Co))).to(BF).to(DEV)
    z = torch.empty((N, D, H, W, Co), dtype=BF, device=DEV)
    st = torch.empty((N, Co, 2), dtype=F32, device=DEV)
    dx = torch.empty_like(x)
    dw = torch.empty(w.shape, dtype=F32, device=DEV)
    L.lamp_conv3d_fwd(x, w, z, stats_out=st)
    L.lamp_conv3d_dgrad(dz, w, dx)
    L.lamp_conv3d_wgrad(x, dz, dw)
    ch = Chain(L, 1, 32, 1, 2, False, BF, [], [], verify="sampled")
    ch.nsample = 128
    ch._sampled_conv("fwd", f"wide {shape}", x, w, z)
    ch._sampled_conv("dgrad", f"wide {shape}", dz, w, dx)
    ch._sampled_wgrad(f"wide {shape}", x, dz, dw)
    _, st_ref = O.inorm_relu(as64(z))
    np.testing.assert_allclose(as64(st)[..., 0], st_ref[..., 0], atol=1e-4 * np.abs(st_ref[..., 0]).max() + 1e-5)
    np.testing.assert_allclose(as64(st)[..., 1], st_ref[..., 1], rtol=2e-4)
    print("worst sampled E_inf per op:", {k: f"{v:.1e}" for k, v in ch.worst.items()})
