"""Network-level oracle (TEST INFRASTRUCTURE ONLY): the 3D U-Net of Sec. 2.2, Eq. 2.

Topology as the paper states it: an encoder of L blocks e_1..e_L applied in sequence, skip
connections s_l that concatenate e_l with the decoder feature coming from below along the channel
axis, decoder blocks d_{L-1}..d_1, and a softmax after the decoder.  Channel schedule from Sec. 3:
the first block has `base` filters, doubled at every further encoder block, decoder symmetric.

Readings where the paper is silent (each also listed in the design notes):
  * d_L is the encoder output itself; there are L-1 real decoder blocks.
  * block(Ca->Cb) = [conv3x3x3 -> InstanceNorm -> ReLU] twice; no conv bias inside blocks.
  * 2x2x2 max-pool after every encoder block but the last.
  * d_l = block(concat[e_l , up(d_{l+1})]) with up = 2x2x2 stride-2 transposed conv (with bias)
    halving the channels; skip first in the concat, in the argument order of s_l(e_l, d_{l+1}).
  * 1x1x1 head with bias to `classes` logits; loss = mean softmax cross entropy over all voxels.
  * Gradient of e_l = pool-path gradient + concat-slice gradient (the two copies e_{l,0}, e_{l,1}
    of Eq. 3 are the same tensor).

`store` is applied to every activation / gradient tensor the GPU path keeps in its storage
dtype (identity for the pure fp64 oracle, oracle.round_bf16 to emulate bf16 storage).

The squeeze-and-excitation variant (Sec. 1 names "SEU-Net" through its citations only; Tables 2, 3 and 5 report
it): a block whose parameters include `<block>.se.w1` is read as a squeeze-and-excitation residual block,
    a1 = unit1(x),  a2 = ReLU(InstanceNorm(conv2(a1))),  out = a1 + gate(mean_v a2) * a2,
with the gate of oracle.se_gate (FC C -> C/r, ReLU, FC C/r -> C, logistic sigmoid).  Where the cited network
puts the gate and the shortcut inside its block is not in the paper: this placement is a reading
(parity unpinned against the paper; pinned by finite differences in tests/test_oracle_unet.py).

Parameters are a dict by name:
  enc{l}.conv{1,2}.w [Co,3,3,3,Ci]   (+ .gamma [Co], .beta [Co] when affine)
  (+ <block>.se.w1 [C/r,C], .se.b1 [C/r], .se.w2 [C,C/r], .se.b2 [C] for the squeeze-and-excitation variant)
  dec{l}.up.w [2C_l,2,2,2,C_l], dec{l}.up.b [C_l], dec{l}.conv{1,2}.w (+ gamma/beta)
  head.w [classes,C_1], head.b [classes]
"""
from __future__ import annotations

import numpy as np

import oracle as O


def _ident(a):
    return a


def _se(params, prefix):
    return [params[f"{prefix}.se.{k}"] for k in ("w1", "b1", "w2", "b2")] if f"{prefix}.se.w1" in params else None


def _block_fwd(params, prefix, a, eps, store, cache):
    se = _se(params, prefix)
    for i in (1, 2):
        name = f"{prefix}.conv{i}"
        z = store(O.conv3d_fwd(a, params[name + ".w"]))
        if se is not None and i == 2:   # gate on the second unit, the first unit's output as the shortcut
            y, _ = O.inorm_relu_se(z, params.get(name + ".gamma"), params.get(name + ".beta"), *se, residual=a, eps=eps)
            stats = None
        else:
            y, stats = O.inorm_relu(z, params.get(name + ".gamma"), params.get(name + ".beta"), eps)
        y = store(y)
        cache[name] = dict(x=a, z=z, y=y, stats=stats)
        a = y
    return a


def forward(params, x, levels, eps=1e-5, store=_ident, first_level=1, last_level=None):
    """Whole net (default) -> (logits, cache).  With first_level/last_level set to an encoder
    range it runs only that pipeline partition (Sec. 2.1: a part = consecutive layers) and
    returns ((pooled_output, [skips...]), cache)."""
    cache = {}
    a = np.asarray(x, dtype=np.float64)
    skips = {}
    enc_last = levels if last_level is None else last_level
    for l in range(first_level, enc_last + 1):
        a = _block_fwd(params, f"enc{l}", a, eps, store, cache)
        if l < levels:
            skips[l] = a
            p = store(O.maxpool2_fwd(a))
            cache[f"pool{l}"] = dict(x=a)
            a = p
    if last_level is not None and last_level < levels:
        return (a, [skips[l] for l in range(first_level, enc_last + 1)]), cache
    for l in range(levels - 1, 0, -1):
        up = store(O.convtr3d_fwd(a, params[f"dec{l}.up.w"], params[f"dec{l}.up.b"]))
        cache[f"dec{l}.up"] = dict(x=a)
        cat = np.concatenate([skips[l], up], axis=-1)
        a = _block_fwd(params, f"dec{l}", cat, eps, store, cache)
    logits = O.head_fwd(a, params["head.w"], params["head.b"])
    cache["head"] = dict(x=a)
    return logits, cache


def _block_bwd(params, prefix, g, eps, store, cache, grads, need_dx=True):
    se = _se(params, prefix)
    shortcut = None
    for i in (2, 1):
        name = f"{prefix}.conv{i}"
        c = cache[name]
        if se is not None and i == 2:
            shortcut = g   # out = a1 + gate * a2: the block's upstream gradient reaches a1 unchanged
            dz, dgam, dbet, dw1, db1, dw2, db2 = O.inorm_relu_se_bwd(g, c["z"], params.get(name + ".gamma"),
                                                                     params.get(name + ".beta"), *se, eps=eps)
            for k, v in zip(("w1", "b1", "w2", "b2"), (dw1, db1, dw2, db2)):
                grads[f"{prefix}.se.{k}"] = v
        else:
            dz, dgam, dbet = O.inorm_relu_bwd(g, c["z"], params.get(name + ".gamma"), params.get(name + ".beta"), eps)
        dz = store(dz)
        if name + ".gamma" in params:
            grads[name + ".gamma"] = dgam
            grads[name + ".beta"] = dbet
        grads[name + ".w"], _ = O.conv3d_wgrad(c["x"], dz)
        if i == 1 and not need_dx:
            return None
        g = store(O.conv3d_dgrad(dz, params[name + ".w"]))
        if i == 2 and shortcut is not None:
            g = store(g + shortcut)
    return g


def backward(params, cache, dlogits, levels, eps=1e-5, store=_ident):
    """Reverse composition of the adjoints; returns grads dict with the names of params."""
    grads = {}
    g, grads["head.w"], grads["head.b"] = O.head_bwd(cache["head"]["x"], params["head.w"], dlogits)
    g = store(g)
    skip_g = {}
    for l in range(1, levels):
        g = _block_bwd(params, f"dec{l}", g, eps, store, cache, grads)
        C = g.shape[-1] // 2
        skip_g[l] = g[..., :C]
        gup = np.ascontiguousarray(g[..., C:])
        c = cache[f"dec{l}.up"]
        g, grads[f"dec{l}.up.w"], grads[f"dec{l}.up.b"] = O.convtr3d_bwd(c["x"], params[f"dec{l}.up.w"], gup)
        g = store(g)
    for l in range(levels, 0, -1):
        if l < levels:
            g = O.maxpool2_bwd(cache[f"pool{l}"]["x"], g) + skip_g[l]
            g = store(g)
        g = _block_bwd(params, f"enc{l}", g, eps, store, cache, grads, need_dx=(l > 1))
    return grads


def loss_and_grads(params, x, labels, levels, eps=1e-5, store=_ident):
    logits, cache = forward(params, x, levels, eps, store)
    loss, dlogits = O.cross_entropy(logits, labels)
    grads = backward(params, cache, dlogits, levels, eps, store)
    return loss, grads, logits, cache


def stage_backward(params, cache, g_pool, g_skips, first_level, last_level, levels, eps=1e-5, store=_ident):
    """Backward of an encoder-only partition given upstream gradients for its pooled output and
    for each skip output (the e_{l,1} copies of Eq. 3).  Returns grads of its conv weights."""
    grads = {}
    g = g_pool
    for l in range(last_level, first_level - 1, -1):
        g = O.maxpool2_bwd(cache[f"pool{l}"]["x"], g) + g_skips[l - first_level]
        g = store(g)
        g = _block_bwd(params, f"enc{l}", g, eps, store, cache, grads, need_dx=(l > first_level or first_level > 1))
    return grads, g


# ---- the sequential form of Eq. 3: the net cut after encoder block `cut` -------------------------
# Partition 0 = encoder blocks 1..cut (forward(..., first_level=1, last_level=cut) / stage_backward);
# partition 1 ("tail") = encoder blocks cut+1..L, the decoder and the softmax head.  The skip copies
# e_{l,1}, l <= cut, cross the cut next to the pooled tensor and come back as gradients.

def tail_forward(params, pooled, skips, first_level, levels, eps=1e-5, store=_ident):
    """pooled = pool(e_{first_level-1}); skips[l-1] = e_l for l < first_level.  -> (logits, cache)."""
    cache = {}
    a = np.asarray(pooled, dtype=np.float64)
    sk = {l: np.asarray(skips[l - 1], dtype=np.float64) for l in range(1, first_level)}
    for l in range(first_level, levels + 1):
        a = _block_fwd(params, f"enc{l}", a, eps, store, cache)
        if l < levels:
            sk[l] = a
            p = store(O.maxpool2_fwd(a))
            cache[f"pool{l}"] = dict(x=a)
            a = p
    for l in range(levels - 1, 0, -1):
        up = store(O.convtr3d_fwd(a, params[f"dec{l}.up.w"], params[f"dec{l}.up.b"]))
        cache[f"dec{l}.up"] = dict(x=a)
        a = _block_fwd(params, f"dec{l}", np.concatenate([sk[l], up], axis=-1), eps, store, cache)
    cache["head"] = dict(x=a)
    return O.head_fwd(a, params["head.w"], params["head.b"]), cache


def tail_backward(params, cache, dlogits, first_level, levels, eps=1e-5, store=_ident):
    """-> (grads of the tail's parameters, gradient of `pooled`, [gradient of e_l for l < first_level])."""
    grads = {}
    g, grads["head.w"], grads["head.b"] = O.head_bwd(cache["head"]["x"], params["head.w"], dlogits)
    g = store(g)
    skip_g = {}
    for l in range(1, levels):
        g = _block_bwd(params, f"dec{l}", g, eps, store, cache, grads)
        C = g.shape[-1] // 2
        skip_g[l] = np.ascontiguousarray(g[..., :C])
        c = cache[f"dec{l}.up"]
        g, grads[f"dec{l}.up.w"], grads[f"dec{l}.up.b"] = O.convtr3d_bwd(c["x"], params[f"dec{l}.up.w"],
                                                                        np.ascontiguousarray(g[..., C:]))
        g = store(g)
    for l in range(levels, first_level - 1, -1):
        if l < levels:
            g = store(O.maxpool2_bwd(cache[f"pool{l}"]["x"], g) + skip_g[l])
        g = _block_bwd(params, f"enc{l}", g, eps, store, cache, grads, need_dx=True)
    return grads, g, [skip_g[l] for l in range(1, first_level)]


def pipeline_loss_and_grads(params, x, labels, levels, cut, micro_batches, eps=1e-5, store=_ident):
    """The mini-batch x (leading axis = micro_batches * n samples) run as the paper's pipeline does
    (Sec. 2.1): split into micro-batches, each taken through partition 0 and the tail and back, the
    weight gradients accumulated over the micro-batches.  Loss and gradients are those of the mean
    cross entropy over the whole mini-batch, so each micro-batch's dlogits carry 1/(M n V)."""
    M = micro_batches
    n = x.shape[0] // M
    assert n * M == x.shape[0]
    total, loss = {}, 0.0
    for m in range(M):
        xm, lm = x[m * n:(m + 1) * n], labels[m * n:(m + 1) * n]
        (pooled, skips), c0 = forward(params, xm, levels, eps, store, first_level=1, last_level=cut)
        logits, c1 = tail_forward(params, pooled, skips, cut + 1, levels, eps, store)
        l_m, dlogits = O.cross_entropy(logits, lm)
        loss += l_m / M
        g1, g_pooled, g_skips = tail_backward(params, c1, dlogits / M, cut + 1, levels, eps, store)
        g0, _ = stage_backward(params, c0, g_pooled, g_skips, 1, cut, levels, eps, store)
        for k, v in {**g0, **g1}.items():
            total[k] = total[k] + v if k in total else v
    return loss, total
