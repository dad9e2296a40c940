"""Parity at the benchmark's full size and launch configuration: the conv block of the headline
workload (1 x 128^3 x 64 -> 64, bf16 storage / fp32 accumulation, InstanceNorm + ReLU) forward,
data-gradient and weight-gradient, exactly the calls bench.py times.

The O(V * 27 * C^2) results are checked on sampled outputs the oracle computes one by one (>= 4096
voxels x all channels, forcing the 8 corners, edges, faces and coordinates on both sides of every
kind of tile boundary); the O(V) results (statistics, normalise+ReLU, its backward) in full.
"""
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
    ent = [(0, 0, 0, 0, 0), (C - 1, 2, 2, 2, C - 1), (31, 1, 1, 1, 32), (32, 0, 2, 1, 31), (5, 2, 0, 0, 63)]
    ent += [tuple(int(v) for v in (r.integers(0, C), r.integers(0, 3), r.integers(0, 3), r.integers(0, 3), r.integers(0, C)))
            for _ in range(120)]
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
