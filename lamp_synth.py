"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds none of the method's arithmetic: it only draws random numbers and paints
shapes.  The datasets the paper measures on (head-and-neck CT, liver CT; Sec. 3) are not
available; the volumes below take their shapes and value ranges and stand in for them:
single-channel CT-like volumes with Hounsfield-like values scaled to [-1,1], ellipsoid
"organs" over Gaussian noise, and integer label volumes of ellipsoid organs.

All draws come from numpy Generator(PCG64(seed)) child streams, in float64 (cast by the caller).
"""
from __future__ import annotations

import numpy as np


def streams(seed: int, n: int):
    """n independent child generators of one seed."""
    return [np.random.Generator(np.random.PCG64(s)) for s in np.random.SeedSequence(seed).spawn(n)]


def normal(rng, shape, std=1.0, dtype=np.float32):
    return (rng.standard_normal(shape) * std).astype(dtype)


def kaiming_conv(rng, co, ci, k=3, dtype=np.float32):
    """Conv weight [Co,k,k,k,Ci] ~ N(0, 2/fan_in), fan_in = k^3*Ci."""
    return normal(rng, (co, k, k, k, ci), np.sqrt(2.0 / (k ** 3 * ci)), dtype)


def kaiming_convtr(rng, ci, co, dtype=np.float32):
    """Transposed-conv weight [Ci,2,2,2,Co] ~ N(0, 2/(8*Ci))."""
    return normal(rng, (ci, 2, 2, 2, co), np.sqrt(2.0 / (8 * ci)), dtype)


def _ellipsoid_mask(shape, centre, semi):
    D, H, W = shape
    d = (np.arange(D, dtype=np.float32)[:, None, None] - centre[0]) / semi[0]
    h = (np.arange(H, dtype=np.float32)[None, :, None] - centre[1]) / semi[1]
    w = (np.arange(W, dtype=np.float32)[None, None, :] - centre[2]) / semi[2]
    return d * d + h * h + w * w <= 1.0


def ct_volume(rng, n, d, h, w, n_blobs=10, dtype=np.float32):
    """[n,d,h,w,1] CT-like: N(-800,100^2) HU background noise, n_blobs random ellipsoids of
    amplitude U(600,1700) HU added, clipped to [-1000,1000] HU and divided by 1000."""
    out = np.empty((n, d, h, w, 1), dtype=dtype)
    dims = np.array([d, h, w], dtype=np.float64)
    for i in range(n):
        v = (rng.standard_normal((d, h, w)).astype(np.float32) * 100.0) - 800.0
        for _ in range(n_blobs):
            c = rng.uniform(0, 1, 3) * dims
            s = rng.uniform(0.05, 0.25, 3) * dims
            amp = rng.uniform(600.0, 1700.0)
            v[_ellipsoid_mask((d, h, w), c, s)] += np.float32(amp)
        out[i, ..., 0] = np.clip(v, -1000.0, 1000.0) / 1000.0
    return out


def organ_labels(rng, n, d, h, w, classes=10, n_organs=10):
    """int32 [n,d,h,w]: background 0, n_organs ellipsoids each with a label drawn from
    [0,classes); later ellipsoids overwrite earlier ones."""
    out = np.zeros((n, d, h, w), dtype=np.int32)
    dims = np.array([d, h, w], dtype=np.float64)
    for i in range(n):
        for _ in range(n_organs):
            c = rng.uniform(0, 1, 3) * dims
            s = rng.uniform(0.05, 0.25, 3) * dims
            lab = int(rng.integers(0, classes))
            out[i][_ellipsoid_mask((d, h, w), c, s)] = lab
    return out


def unet_param_names(levels, affine, se_ratio=0):
    """Parameter tensors of the U-Net in the library's documented order (se_ratio > 0: the squeeze-and-excitation
    variant, four gate tensors behind each block's convs)."""
    names = []

    def block(prefix):
        for i in (1, 2):
            names.append(f"{prefix}.conv{i}.w")
            if affine:
                names.append(f"{prefix}.conv{i}.gamma")
                names.append(f"{prefix}.conv{i}.beta")
        if se_ratio:
            names.extend(f"{prefix}.se.{k}" for k in ("w1", "b1", "w2", "b2"))

    for l in range(1, levels + 1):
        block(f"enc{l}")
    for l in range(levels - 1, 0, -1):
        names.append(f"dec{l}.up.w")
        names.append(f"dec{l}.up.b")
        block(f"dec{l}")
    names += ["head.w", "head.b"]
    return names


def unet_params(rng, levels, base, in_ch, classes, affine=False, test_mode=False, dtype=np.float32, se_ratio=0):
    """Ordered dict name -> array.  Kaiming-normal weights; biases 0 (benchmarks) or N(0,0.1^2)
    (test_mode); gamma U(0.5,1.5), beta U(-0.5,0.5) when affine.  se_ratio > 0 adds each block's gate:
    w1 [C/r, C] ~ N(0, 1/C), w2 [C, C/r] ~ N(0, 1/(C/r)) in float32, biases 0 or N(0, 0.1^2)."""
    p = {}
    ch = [base * 2 ** (l - 1) for l in range(1, levels + 1)]

    def block(prefix, ci, co):
        for i, cin in ((1, ci), (2, co)):
            p[f"{prefix}.conv{i}.w"] = kaiming_conv(rng, co, cin, 3, dtype)
            if affine:
                p[f"{prefix}.conv{i}.gamma"] = rng.uniform(0.5, 1.5, co).astype(np.float32)
                p[f"{prefix}.conv{i}.beta"] = rng.uniform(-0.5, 0.5, co).astype(np.float32)
        if se_ratio:
            cr = max(1, co // se_ratio)
            p[f"{prefix}.se.w1"] = normal(rng, (cr, co), np.sqrt(1.0 / co))
            p[f"{prefix}.se.b1"] = normal(rng, (cr,), 0.1) if test_mode else np.zeros(cr, np.float32)
            p[f"{prefix}.se.w2"] = normal(rng, (co, cr), np.sqrt(1.0 / cr))
            p[f"{prefix}.se.b2"] = normal(rng, (co,), 0.1) if test_mode else np.zeros(co, np.float32)

    for l in range(1, levels + 1):
        block(f"enc{l}", in_ch if l == 1 else ch[l - 2], ch[l - 1])
    for l in range(levels - 1, 0, -1):
        p[f"dec{l}.up.w"] = kaiming_convtr(rng, ch[l], ch[l - 1], dtype)
        p[f"dec{l}.up.b"] = (normal(rng, (ch[l - 1],), 0.1) if test_mode else np.zeros(ch[l - 1], np.float32))
        block(f"dec{l}", 2 * ch[l - 1], ch[l - 1])
    p["head.w"] = normal(rng, (classes, ch[0]), np.sqrt(2.0 / ch[0]), dtype)
    p["head.b"] = (normal(rng, (classes,), 0.1) if test_mode else np.zeros(classes, np.float32))
    assert list(p.keys()) == unet_param_names(levels, affine, se_ratio)
    return p
