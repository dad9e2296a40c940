"""Sliding-window inference oracle (TEST INFRASTRUCTURE ONLY).

The paper compares inference over fixed-size windows with one pass over the whole image
(Sec. 3, Tables 3 and 5) but states neither overlap nor blending; the reading used here is the
benchmark's: cubic windows of side P, overlap 0.25 (stride 0.75 P), the last window on each axis
clamped so the cover is exact, logits blended with a Gaussian importance map of sigma = P/8
centred on the window, accumulated and divided by the accumulated weight.  Every window is an
independent sample (its own InstanceNorm statistics).
"""
from __future__ import annotations

import math

import numpy as np


def window_starts(length: int, patch: int, overlap: float = 0.25):
    """Start offsets along one axis: stride = patch*(1-overlap); count = ceil((length-patch)/stride)+1;
    start_i = min(i*stride, length-patch)."""
    assert length >= patch
    stride = int(round(patch * (1.0 - overlap)))
    cnt = int(math.ceil((length - patch) / stride)) + 1
    return [min(i * stride, length - patch) for i in range(cnt)]


def gaussian_map(patch: int, sigma_scale: float = 0.125):
    """g(a,b,c) = exp(-((a-m)^2+(b-m)^2+(c-m)^2)/(2 sigma^2)), m = (patch-1)/2, sigma = sigma_scale*patch."""
    m = (patch - 1) / 2.0
    s = sigma_scale * patch
    a = np.arange(patch, dtype=np.float64)
    g1 = np.exp(-0.5 * ((a - m) / s) ** 2)
    return g1[:, None, None] * g1[None, :, None] * g1[None, None, :]


def sliding_window(net, vol, patch=64, overlap=0.25, sigma_scale=0.125):
    """vol [1,D,H,W,Cin]; net maps [B,P,P,P,Cin] -> logits [B,P,P,P,K].  Windows are enumerated
    d-major, then h, then w.  Returns blended logits [1,D,H,W,K]."""
    _, D, H, W, _ = vol.shape
    sd, sh, sw = window_starts(D, patch, overlap), window_starts(H, patch, overlap), window_starts(W, patch, overlap)
    g = gaussian_map(patch, sigma_scale)
    acc = None
    wsum = np.zeros((D, H, W))
    for d0 in sd:
        for h0 in sh:
            for w0 in sw:
                win = vol[:, d0:d0 + patch, h0:h0 + patch, w0:w0 + patch, :]
                lg = net(np.ascontiguousarray(win))[0]
                if acc is None:
                    acc = np.zeros((D, H, W, lg.shape[-1]))
                acc[d0:d0 + patch, h0:h0 + patch, w0:w0 + patch, :] += g[..., None] * lg
                wsum[d0:d0 + patch, h0:h0 + patch, w0:w0 + patch] += g
    return (acc / wsum[..., None])[None]
