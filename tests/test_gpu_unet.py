"""GPU parity of the network-level entry points (whole U-Net forward / forward+backward, one
encoder partition, sliding-window inference) against the network oracle.

bf16 runs are compared with the oracle that rounds every stored activation / gradient tensor to
bf16 at the same tensor boundaries (storage emulation); fp32 runs with the pure fp64 oracle.
End-to-end gradients are judged on the weight gradients and on the loss.  Two bf16 realisations of a deep net
drift apart through ReLU-mask and arg-max flips at near-ties, by an amount the oracle itself can measure: the
bound on each gradient tensor's relative L2 distance to the storage-emulating oracle is calibrated on the
distance between perturbed runs of that oracle (gpu_util.realisation_spread).
"""
import numpy as np
import pytest
import torch

import lamp_synth as S
import oracle as O
from gpu_util import DEV, TOL, as64, check, check_e2_calibrated, e2, realisation_spread, to_dev
from oracle import sliding, unet

pytestmark = pytest.mark.gpu
BF, F32 = torch.bfloat16, torch.float32
# End-to-end weight gradients of the fp32 path against the pure fp64 oracle: the path's stated bound (E_inf relative to
# the tensor's largest entry).  Measured on the MI355X: 5e-8 ... 1.5e-6 on every gradient tensor of the fp32 net.
FP32_GRAD_TOL = 1e-4


@pytest.fixture(scope="module")
def L():
    import paper_2006_12575_amd as L
    L.lib()
    return L


def make_net(levels, base, in_ch, classes, affine, dtype, seed, se_ratio=0):
    rp = S.streams(seed, 1)[0]
    p = S.unet_params(rp, levels, base, in_ch, classes, affine, test_mode=True, se_ratio=se_ratio)
    dev, ora = [], {}
    for k, v in p.items():
        small = k.endswith((".b", ".gamma", ".beta")) or ".se." in k
        t = to_dev(v, F32 if small else dtype)
        dev.append(t)
        ora[k] = as64(t)
    return list(p.keys()), dev, ora


def test_config1_tiny_unet_forward_fp32(L):
    """Tiny 3-level base-8 U-Net forward in fp32 on 1x1x32x32x32 N(0,1) voxels, 5 classes."""
    rx = S.streams(1001, 2)[0]
    names, dev, ora = make_net(3, 8, 1, 5, False, F32, 1001)
    x = to_dev(S.normal(rx, (1, 32, 32, 32, 1)), F32)
    ud = L.unet_desc(3, 8, 1, 5, 1, 32, 32, 32, F32)
    logits = torch.empty((1, 32, 32, 32, 5), dtype=F32, device=DEV)
    L.lamp_unet_fwd(ud, dev, x, logits)
    ref, _ = unet.forward(ora, as64(x), 3)
    e = check(as64(logits), ref, F32, "config 1 logits")
    print(f"config1 E_inf={e:.2e} E2={e2(as64(logits), ref):.2e}")
    # run-to-run determinism
    l2 = torch.empty_like(logits)
    L.lamp_unet_fwd(ud, dev, x, l2)
    assert torch.equal(l2, logits)


@pytest.mark.parametrize("cfg", [
    dict(levels=3, base=32, in_ch=1, classes=10, affine=False, dtype=BF, dims=(2, 16, 16, 32)),
    dict(levels=2, base=8, in_ch=2, classes=5, affine=True, dtype=F32, dims=(1, 8, 12, 16)),
    dict(levels=3, base=32, in_ch=1, classes=4, affine=True, dtype=BF, dims=(1, 16, 24, 16)),
    dict(levels=1, base=32, in_ch=1, classes=3, affine=False, dtype=BF, dims=(1, 8, 8, 16)),
    # 16 channels at level 1: generic kernels and a materialised concat buffer in bf16
    dict(levels=2, base=16, in_ch=1, classes=3, affine=False, dtype=BF, dims=(2, 8, 8, 16)),
    # many tiny samples: the convs run on one packed volume (also the decoder conv that reads its concat from two tensors)
    dict(levels=2, base=32, in_ch=1, classes=3, affine=False, dtype=BF, dims=(8, 4, 4, 4)),
], ids=["bf16-3lvl", "f32-affine", "bf16-affine", "bf16-1lvl", "bf16-base16", "bf16-8x4cubed"])
def test_unet_fwd_bwd(L, cfg):
    """(a) every layer of the replayed chain matches the oracle given the GPU's own inputs,
    (b) lamp_unet_fwd_bwd reproduces the chain bit for bit, (c) end to end, logits and loss match the
    storage-emulating oracle to the path's tolerance; end-to-end gradients are only sanity-checked
    (two bf16 realisations of a deep net drift apart through mask / arg-max flips at near-ties)."""
    from gpu_chain import Chain
    levels, dtype = cfg["levels"], cfg["dtype"]
    N, D, H, W = cfg["dims"]
    names, dev, ora = make_net(levels, cfg["base"], cfg["in_ch"], cfg["classes"], cfg["affine"], dtype, 77)
    rx, rl = S.streams(78, 2)
    x = to_dev(S.ct_volume(rx, N, D, H, W) if cfg["in_ch"] == 1 else S.normal(rx, (N, D, H, W, cfg["in_ch"])), dtype)
    lab = torch.from_numpy(S.organ_labels(rl, N, D, H, W, cfg["classes"])).to(DEV)
    ud = L.unet_desc(levels, cfg["base"], cfg["in_ch"], cfg["classes"], N, D, H, W, dtype, affine=cfg["affine"])
    grads = [torch.full(t.shape, float("nan"), dtype=F32, device=DEV) for t in dev]
    loss = torch.empty((), dtype=F32, device=DEV)
    logits = torch.empty((N, D, H, W, cfg["classes"]), dtype=F32, device=DEV)
    L.lamp_unet_fwd_bwd(ud, dev, x, lab, loss, grads, logits=logits)
    # (a) + (b)
    ch = Chain(L, levels, cfg["base"], cfg["in_ch"], cfg["classes"], cfg["affine"], dtype, names, dev)
    lg_chain = ch.forward(x)
    loss_chain, g_chain = ch.backward(lab)
    assert torch.equal(lg_chain, logits), "whole-net logits differ from the layer-by-layer chain"
    assert torch.equal(loss_chain, loss)
    for k, g in zip(names, grads):
        assert torch.equal(g_chain[k], g), f"whole-net grad {k} differs from the layer-by-layer chain"
    print("worst teacher-forced E_inf per op:", {k: f"{v:.1e}" for k, v in ch.worst.items()})
    # (c)
    store = O.round_bf16 if dtype == BF else (lambda a: a)
    run = lambda st: unet.loss_and_grads(ora, as64(x), lab.cpu().numpy(), levels, store=st)
    loss_ref, g_ref, lg_ref, _ = run(store)
    check(as64(logits), lg_ref, dtype, "logits", tol=1e-2 if dtype == BF else 1e-4)
    assert abs(loss.item() - loss_ref) <= 1e-3 * abs(loss_ref)
    if dtype == F32:
        for k, g in zip(names, grads):
            check(as64(g), g_ref[k], dtype, f"grad {k}", tol=FP32_GRAD_TOL)
    else:
        spread = realisation_spread(lambda st: run(st)[1], g_ref)
        rep = {}
        for k, g in zip(names, grads):
            rep[k] = check_e2_calibrated(as64(g), g_ref[k], spread[k], f"grad {k}")
        print("end-to-end grad E2 (bound):", {k: f"{e:.1e} ({b:.1e})" for k, (e, b) in rep.items()})
    # forward-only entry point gives the same logits; beta=1 accumulates
    l2 = torch.empty_like(logits)
    L.lamp_unet_fwd(ud, dev, x, l2)
    assert torch.equal(l2, logits)
    g2 = [g.clone() for g in grads]
    L.lamp_unet_fwd_bwd(ud, dev, x, lab, loss, g2, beta=1.0)
    for a, b in zip(grads, g2):
        assert torch.allclose(b, 2 * a, rtol=1e-6, atol=0)


@pytest.mark.parametrize("cfg", [
    dict(levels=3, base=8, in_ch=2, classes=5, affine=True, dtype=F32, dims=(2, 8, 12, 16), ratio=4),
    dict(levels=2, base=8, in_ch=1, classes=3, affine=False, dtype=F32, dims=(1, 8, 8, 8), ratio=16),   # one hidden unit
    dict(levels=3, base=32, in_ch=1, classes=10, affine=False, dtype=BF, dims=(2, 16, 16, 32), ratio=16),
    dict(levels=2, base=32, in_ch=1, classes=4, affine=True, dtype=BF, dims=(1, 16, 24, 16), ratio=8),
], ids=["f32-affine-r4", "f32-r16", "bf16-r16", "bf16-affine-r8"])
def test_seunet_fwd_bwd(L, cfg):
    """The squeeze-and-excitation variant of the net (se_ratio > 0: every block out = a1 + gate(mean a2) * a2) through
    the whole-network entry points against the network oracle.  fp32: logits and EVERY gradient tensor, the gate's
    included, within 1e-4 of the pure fp64 oracle, which pins the composition (shortcut add, the gate's backward, the
    parameter order).  bf16: logits and loss to the path's bound, gradients to the calibrated realisation bound."""
    levels, dtype, ratio = cfg["levels"], cfg["dtype"], cfg["ratio"]
    N, D, H, W = cfg["dims"]
    names, dev, ora = make_net(levels, cfg["base"], cfg["in_ch"], cfg["classes"], cfg["affine"], dtype, 177, se_ratio=ratio)
    rx, rl = S.streams(178, 2)
    x = to_dev(S.ct_volume(rx, N, D, H, W) if cfg["in_ch"] == 1 else S.normal(rx, (N, D, H, W, cfg["in_ch"])), dtype)
    lab = torch.from_numpy(S.organ_labels(rl, N, D, H, W, cfg["classes"])).to(DEV)
    ud = L.unet_desc(levels, cfg["base"], cfg["in_ch"], cfg["classes"], N, D, H, W, dtype, affine=cfg["affine"], se_ratio=ratio)
    assert L.lamp_unet_param_count(ud) == len(names)
    for i, t in enumerate(dev):
        assert L.lamp_unet_param_numel(ud, i) == t.numel(), names[i]
    grads = [torch.full(t.shape, float("nan"), dtype=F32, device=DEV) for t in dev]
    loss = torch.empty((), dtype=F32, device=DEV)
    logits = torch.empty((N, D, H, W, cfg["classes"]), dtype=F32, device=DEV)
    L.lamp_unet_fwd_bwd(ud, dev, x, lab, loss, grads, logits=logits)
    store = O.round_bf16 if dtype == BF else (lambda a: a)
    run = lambda st: unet.loss_and_grads(ora, as64(x), lab.cpu().numpy(), levels, store=st)
    loss_ref, g_ref, lg_ref, _ = run(store)
    check(as64(logits), lg_ref, dtype, "SE net logits")
    assert abs(loss.item() - loss_ref) <= 1e-3 * abs(loss_ref)
    if dtype == F32:
        for k, g in zip(names, grads):
            check(as64(g), g_ref[k], dtype, f"SE net grad {k}", tol=FP32_GRAD_TOL)
    else:
        spread = realisation_spread(lambda st: run(st)[1], g_ref)
        for k, g in zip(names, grads):
            check_e2_calibrated(as64(g), g_ref[k], spread[k], f"SE net grad {k}")
    # the forward-only entry point gives the same logits; a second call is bit-identical; beta = 1 accumulates
    l2 = torch.empty_like(logits)
    L.lamp_unet_fwd(ud, dev, x, l2)
    assert torch.equal(l2, logits)
    g2 = [g.clone() for g in grads]
    L.lamp_unet_fwd_bwd(ud, dev, x, lab, loss, g2, beta=1.0)
    for a, b in zip(grads, g2):
        assert torch.allclose(b, 2 * a, rtol=1e-6, atol=0)
    g3 = [torch.empty_like(g) for g in grads]
    L.lamp_unet_fwd_bwd(ud, dev, x, lab, loss, g3)
    for a, b in zip(grads, g3):
        assert torch.equal(a, b)
    # the partition entry points serve the plain U-Net only
    assert L.lamp_unet_stage_workspace_bytes(ud, 1, 1) == 0


def test_stage_partition_fwd_bwd(L):
    """One pipeline partition = encoder blocks 1-2 (Sec. 2.1 / Eq. 3): outputs pool(e_2), e_1, e_2;
    backward from N(0,1) upstream gradients of all three outputs.  The partition must reproduce the
    whole net's own tensors bit for bit (Eq. 3 == Eq. 2), and its backward the layer-by-layer chain."""
    from gpu_chain import Chain
    levels, base, dtype = 3, 32, BF
    N, D, H, W = 1, 16, 16, 32
    names, dev, ora = make_net(levels, base, 1, 4, False, dtype, 5)
    sp = dev[:4]
    rx, rg = S.streams(6, 2)
    x = to_dev(S.ct_volume(rx, N, D, H, W), dtype)
    ud = L.unet_desc(levels, base, 1, 4, N, D, H, W, dtype)
    ws = torch.empty(L.lamp_unet_stage_workspace_bytes(ud, 1, 2), dtype=torch.uint8, device=DEV)
    pooled = torch.empty((N, D // 4, H // 4, W // 4, 2 * base), dtype=dtype, device=DEV)
    skips = [torch.empty((N, D, H, W, base), dtype=dtype, device=DEV),
             torch.empty((N, D // 2, H // 2, W // 2, 2 * base), dtype=dtype, device=DEV)]
    L.lamp_unet_stage_fwd(ud, 1, 2, sp, x, pooled, skips, ws)
    ch = Chain(L, levels, base, 1, 4, False, dtype, names, dev)
    ch.forward(x)  # whole net, every layer verified against the oracle
    assert torch.equal(skips[0], ch.enc[1][1]["y"]) and torch.equal(skips[1], ch.enc[2][1]["y"])
    assert torch.equal(pooled, ch.pooled[2])
    (p_ref, s_ref), cache = unet.forward(ora, as64(x), levels, store=O.round_bf16, first_level=1, last_level=2)
    check(as64(pooled), p_ref, dtype, "stage pooled")
    check(as64(skips[0]), s_ref[0], dtype, "stage skip 1")
    check(as64(skips[1]), s_ref[1], dtype, "stage skip 2")
    gp = to_dev(S.normal(rg, pooled.shape), dtype)
    gs = [to_dev(S.normal(rg, s.shape), dtype) for s in skips]
    grads = [torch.empty(t.shape, dtype=F32, device=DEV) for t in sp]
    L.lamp_unet_stage_bwd(ud, 1, 2, sp, x, skips, gp, gs, grads, ws)
    # the same backward replayed layer by layer (each layer verified), then bitwise comparison
    cg = {}
    g = gp
    for l in (2, 1):
        c1, c2 = ch.enc[l]
        gy = torch.empty(c2["y"].shape, dtype=dtype, device=DEV)
        L.lamp_maxpool2_bwd(c2["y"], g, gy, add=gs[l - 1])
        np.testing.assert_allclose(as64(gy), O.maxpool2_bwd(as64(c2["y"]), as64(g)) + as64(gs[l - 1]), rtol=2 ** -8, atol=1e-30)
        g = ch.conv_bwd(c2, gy, cg, True, below=c1)
        g = ch.conv_bwd(c1, g, cg, l > 1, dz_ready=True)
    for k, gr in zip(names[:4], grads):
        assert torch.equal(gr, cg[k]), f"stage grad {k} differs from the chain"
    def stage_grads(st):
        _, c = unet.forward(ora, as64(x), levels, store=st, first_level=1, last_level=2)
        return unet.stage_backward(ora, c, as64(gp), [as64(t) for t in gs], 1, 2, levels, store=st)[0]
    g_ref = stage_grads(O.round_bf16)
    spread = realisation_spread(stage_grads, g_ref)
    for k, gr in zip(names[:4], grads):
        check_e2_calibrated(as64(gr), g_ref[k], spread[k], f"stage grad {k}")


def _stage_shapes(N, D, H, W, base, cut):
    sk = [(N, D >> (l - 1), H >> (l - 1), W >> (l - 1), base << (l - 1)) for l in range(1, cut + 1)]
    return (N, D >> cut, H >> cut, W >> cut, base << (cut - 1)), sk


@pytest.mark.parametrize("cut,affine", [(1, False), (2, False), (1, True)], ids=["cut1", "cut2", "cut1-affine"])
def test_tail_partition_fwd_bwd(L, cut, affine):
    """The net cut after encoder block `cut` (Sec. 2.2 Eq. 3): partition 0 forward, the tail forward
    and backward, partition 0 backward.  Every result must equal the whole net's bit for bit (the
    whole net is itself verified layer by layer against the oracle); the gradients that cross the cut
    are compared with the oracle's, computed from the GPU's own partition-0 outputs."""
    levels, base, K, dtype = 3, 32, 5, BF
    N, D, H, W = 2, 16, 16, 32
    names, dev, ora = make_net(levels, base, 1, K, affine, dtype, 21)
    rx, rl = S.streams(22, 2)
    x = to_dev(S.ct_volume(rx, N, D, H, W), dtype)
    lab = torch.from_numpy(S.organ_labels(rl, N, D, H, W, K)).to(DEV)
    ud = L.unet_desc(levels, base, 1, K, N, D, H, W, dtype, affine=affine)
    grads = [torch.empty(t.shape, dtype=F32, device=DEV) for t in dev]
    loss = torch.empty((), dtype=F32, device=DEV)
    logits = torch.empty((N, D, H, W, K), dtype=F32, device=DEV)
    L.lamp_unet_fwd_bwd(ud, dev, x, lab, loss, grads, logits=logits)

    toff = L.lamp_unet_tail_param_offset(ud, cut + 1)
    assert toff == 2 * cut * (3 if affine else 1)
    pshape, sshapes = _stage_shapes(N, D, H, W, base, cut)
    pooled = torch.empty(pshape, dtype=dtype, device=DEV)
    skips = [torch.empty(sh, dtype=dtype, device=DEV) for sh in sshapes]
    ws0 = torch.empty(L.lamp_unet_stage_workspace_bytes(ud, 1, cut), dtype=torch.uint8, device=DEV)
    L.lamp_unet_stage_fwd(ud, 1, cut, dev[:toff], x, pooled, skips, ws0)
    # forward only
    lt = torch.empty_like(logits)
    L.lamp_unet_tail_fwd(ud, cut + 1, dev[toff:], pooled, skips, lt)
    assert torch.equal(lt, logits), "tail logits differ from the whole net's"
    # forward + backward
    gt = [torch.full(t.shape, float("nan"), dtype=F32, device=DEV) for t in dev[toff:]]
    d_x = torch.full(pshape, float("nan"), dtype=dtype, device=DEV)
    d_skips = [torch.full(sh, float("nan"), dtype=dtype, device=DEV) for sh in sshapes]
    loss_t = torch.empty((), dtype=F32, device=DEV)
    lt.zero_()
    L.lamp_unet_tail_fwd_bwd(ud, cut + 1, dev[toff:], pooled, skips, lab, loss_t, gt, d_skips, d_x=d_x, logits=lt)
    assert torch.equal(lt, logits) and torch.equal(loss_t, loss)
    for k, a, b in zip(names[toff:], gt, grads[toff:]):
        assert torch.equal(a, b), f"tail grad {k} differs from the whole net's"
    gs = [torch.full(t.shape, float("nan"), dtype=F32, device=DEV) for t in dev[:toff]]
    L.lamp_unet_stage_bwd(ud, 1, cut, dev[:toff], x, skips, d_x, d_skips, gs, ws0)
    for k, a, b in zip(names[:toff], gs, grads[:toff]):
        assert torch.equal(a, b), f"partition-0 grad {k} (from the tail's cut gradients) differs from the whole net's"
    # the cut-crossing gradients against the oracle's tail, fed with the GPU's partition-0 outputs
    def tail_cut_grads(st):
        lg, c = unet.tail_forward(ora, as64(pooled), [as64(t) for t in skips], cut + 1, levels, store=st)
        _, dl = O.cross_entropy(lg, lab.cpu().numpy())
        _, gp_r, gsk_r = unet.tail_backward(ora, c, dl, cut + 1, levels, store=st)
        return dict([("d_x", gp_r)] + [(f"d_skip{i + 1}", r) for i, r in enumerate(gsk_r)]), lg
    cut_ref, lg_ref = tail_cut_grads(O.round_bf16)
    check(as64(lt), lg_ref, dtype, "tail logits")
    spread = realisation_spread(lambda st: tail_cut_grads(st)[0], cut_ref)
    for nm, a in [("d_x", d_x)] + [(f"d_skip{i + 1}", t) for i, t in enumerate(d_skips)]:
        check_e2_calibrated(as64(a), cut_ref[nm], spread[nm], f"tail {nm}")
    # argument errors are found on the host
    with pytest.raises(RuntimeError):
        L.lamp_unet_tail_fwd(ud, 1, dev, pooled, skips, lt)          # first_level 1 is the whole net
    assert L.lamp_unet_tail_workspace_bytes(L.unet_desc(levels, 16, 1, K, N, D, H, W, dtype), cut + 1) == 0
    assert L.lamp_unet_tail_workspace_bytes(L.unet_desc(levels, base, 1, K, N, D, H, W, F32), cut + 1) == 0


@pytest.mark.parametrize("cut,n,M,affine", [(1, 1, 2, False), (2, 2, 3, False), (1, 2, 1, False), (2, 1, 2, True)],
                         ids=["cut1-1x2", "cut2-2x3", "cut1-2x1", "cut2-1x2-affine"])
def test_pipeline_two_partitions_micro_batches(L, cut, n, M, affine):
    """Partition 0 and the tail on two streams, M micro-batches of n samples in the pipeline order
    (Sec. 2.1).  The result is the mini-batch's loss and gradients: compared with lamp_unet_fwd_bwd
    on the whole mini-batch (bit for bit when M == 1: same kernels on the same shapes; as two bf16
    realisations otherwise, since tile counts, hence the split of the reductions, depend on the batch)
    and with the oracle's micro-batch pipeline."""
    levels, base, K, dtype = 3, 32, 4, BF
    D, H, W = 16, 16, 16
    N = n * M
    names, dev, ora = make_net(levels, base, 1, K, affine, dtype, 31)
    rx, rl = S.streams(32 + cut, 2)
    x = to_dev(S.ct_volume(rx, N, D, H, W), dtype)
    lab = torch.from_numpy(S.organ_labels(rl, N, D, H, W, K)).to(DEV)
    full = L.unet_desc(levels, base, 1, K, N, D, H, W, dtype, affine=affine)
    g_full = [torch.empty(t.shape, dtype=F32, device=DEV) for t in dev]
    loss_full = torch.empty((), dtype=F32, device=DEV)
    lg_full = torch.empty((N, D, H, W, K), dtype=F32, device=DEV)
    L.lamp_unet_fwd_bwd(full, dev, x, lab, loss_full, g_full, logits=lg_full)

    mb = L.unet_desc(levels, base, 1, K, n, D, H, W, dtype, affine=affine)
    aux = torch.cuda.Stream()
    ws = torch.empty(L.lamp_unet_pipeline_workspace_bytes(mb, cut, M), dtype=torch.uint8, device=DEV)
    runs = []
    for rep in range(2):
        ws.fill_(0xFF)   # NaN patterns: nothing may be read before it is written
        g = [torch.full(t.shape, float("nan"), dtype=F32, device=DEV) for t in dev]
        loss = torch.full((), float("nan"), dtype=F32, device=DEV)
        lg = torch.full((N, D, H, W, K), float("nan"), dtype=F32, device=DEV)
        L.lamp_unet_pipeline_fwd_bwd(mb, cut, M, dev, x, lab, loss, g, aux, logits=lg, ws=ws)
        torch.cuda.current_stream().synchronize()   # the contract: the caller's stream alone
        runs.append((loss.clone(), [t.clone() for t in g], lg.clone()))
    loss, g, lg = runs[0]
    assert torch.equal(loss, runs[1][0]) and torch.equal(lg, runs[1][2])
    for a, b in zip(g, runs[1][1]):
        assert torch.equal(a, b), "pipeline results differ from run to run"
    if M == 1:
        assert torch.equal(loss, loss_full) and torch.equal(lg, lg_full)
        for k, a, b in zip(names, g, g_full):
            assert torch.equal(a, b), f"pipeline grad {k} differs from the whole net's"
    else:
        # Two bf16 realisations of the same quantities: the batch size decides the tiling, the packed layout of
        # the small levels and with them the summation order of the statistics, and one activation rounded the
        # other way is amplified by the normalisation of the 4^3 level.  Logits: each within the bound of the
        # exact result, so twice the bound; gradients: direction, as against the oracle.
        check(as64(lg), as64(lg_full), dtype, "pipeline logits vs mini-batch run", tol=2 * TOL[dtype])
        assert abs(loss.item() - loss_full.item()) <= 1e-3 * abs(loss_full.item())
    pipe = lambda st: unet.pipeline_loss_and_grads(ora, as64(x), lab.cpu().numpy(), levels, cut, M, store=st)
    loss_ref, g_ref = pipe(O.round_bf16)
    assert abs(loss.item() - loss_ref) <= 1e-3 * abs(loss_ref)
    spread = realisation_spread(lambda st: pipe(st)[1], g_ref)
    for k, a, b in zip(names, g, g_full):
        check_e2_calibrated(as64(a), g_ref[k], spread[k], f"pipeline grad {k}")
        # the one-call mini-batch run is one more realisation of the same quantities
        check_e2_calibrated(as64(b), g_ref[k], spread[k], f"mini-batch grad {k} against the oracle's pipeline")
    # beta = 1 accumulates onto what is there
    g2 = [t.clone() for t in g]
    L.lamp_unet_pipeline_fwd_bwd(mb, cut, M, dev, x, lab, loss, g2, aux, beta=1.0, ws=ws)
    torch.cuda.current_stream().synchronize()
    for a, b in zip(g, g2):   # fp32 sums taken in another order: bound relative to the tensor's scale
        assert (b - 2 * a).abs().max().item() <= 1e-5 * a.abs().max().item()
    with pytest.raises(RuntimeError):   # the two partitions need two different streams
        L.lamp_unet_pipeline_fwd_bwd(mb, cut, M, dev, x, lab, loss, g2, torch.cuda.current_stream(), ws=ws)


@pytest.mark.parametrize("dtype", [F32, BF], ids=["f32", "bf16"])
def test_sliding_window_vs_oracle(L, dtype):
    levels, base, K, P = 2, 8 if dtype == F32 else 32, 3, 8
    D, H, W = 20, 8, 12
    names, dev, ora = make_net(levels, base, 1, K, False, dtype, 11)
    vol = to_dev(S.ct_volume(S.streams(12, 1)[0], 1, D, H, W), dtype)
    cnt = L.lamp_sliding_window_count(D, H, W, P, 0.25)
    assert cnt == len(sliding.window_starts(D, P)) * len(sliding.window_starts(H, P)) * len(sliding.window_starts(W, P)) == 6
    pd = L.unet_desc(levels, base, 1, K, cnt, P, P, P, dtype)
    out = torch.empty((1, D, H, W, K), dtype=F32, device=DEV)
    L.lamp_sliding_window_fwd(pd, dev, vol, out)
    store = O.round_bf16 if dtype == BF else (lambda a: a)
    ref = sliding.sliding_window(lambda win: unet.forward(ora, win, levels, store=store)[0], as64(vol), patch=P)
    check(as64(out), ref, dtype, "sliding-window logits")


def test_unet_forward_as_captured_graph(L):
    """The whole-network forward only enqueues kernels (no allocation, no memset, no synchronisation), so
    it can be captured as one HIP graph.  Every replay -- with eager work, new inputs and synchronisations
    between the replays -- must reproduce the eager result bit for bit."""
    names, dev, _ = make_net(3, 8, 1, 5, False, F32, 1001)
    ud = L.unet_desc(3, 8, 1, 5, 1, 32, 32, 32, F32)
    x = torch.empty((1, 32, 32, 32, 1), dtype=F32, device=DEV)
    logits = torch.empty((1, 32, 32, 32, 5), dtype=F32, device=DEV)
    ws = torch.empty(L.lamp_unet_workspace_bytes(ud, False), dtype=torch.uint8, device=DEV)
    eager_out = torch.empty_like(logits)
    rx = S.streams(1001, 4)
    x.copy_(to_dev(S.normal(rx[0], x.shape), F32))
    L.lamp_unet_fwd(ud, dev, x, eager_out, ws=ws)       # also takes the one-time set-up out of the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        L.lamp_unet_fwd(ud, dev, x, logits, ws=ws)
    for i in range(4):
        x.copy_(to_dev(S.normal(rx[i], x.shape), F32))  # new input in place, eager work between the replays
        L.lamp_unet_fwd(ud, dev, x, eager_out, ws=ws)
        torch.cuda.synchronize()
        logits.fill_(float("nan"))
        ws.fill_(0xFF)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(logits, eager_out), f"replay {i} differs from the eager forward"
