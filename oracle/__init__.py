"""CPU oracle (TEST INFRASTRUCTURE ONLY) for the per-device compute path of LAMP's 3D U-Net.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  It shares no code with the HIP library; the product never imports it.

The primitives (conv, norm, pool, transposed conv) are the plain C definitions in
``lamp_oracle.c``; this module only marshals numpy float64 arrays into them and adds the few
operations that are one library call each (1x1x1 head = a matrix product, softmax, cross entropy).
The network composition (Sec. 2.2, Eq. 2) lives in ``oracle.unet``; sliding-window inference in
``oracle.sliding``.

All arrays are float64, dense, NDHWC.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lamp_oracle.c")
_LIB = os.path.join(_HERE, "liblamp_oracle.so")


def build(force: bool = False) -> str:
    """Compile lamp_oracle.c with gcc (OpenMP).  Building the checker is not using it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=native", "-fopenmp", "-fPIC", "-shared", "-std=c99",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None
_i64 = ctypes.c_int64
_dp = ctypes.POINTER(ctypes.c_double)


def _L():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.ora_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_L().ora_num_threads())


def _p(a):
    if a is None:
        return None
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_dp)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def conv3d_fwd(x, w, b=None):
    """O1.  x [N,D,H,W,Ci], w [Co,3,3,3,Ci], b [Co] or None -> z [N,D,H,W,Co]."""
    x, w, b = _f64(x), _f64(w), _f64(b)
    N, D, H, W, Ci = x.shape
    Co = w.shape[0]
    assert w.shape == (Co, 3, 3, 3, Ci)
    z = np.empty((N, D, H, W, Co), dtype=np.float64)
    _L().ora_conv3d_fwd(_p(x), _p(w), _p(b), _p(z), _i64(N), _i64(D), _i64(H), _i64(W), _i64(Ci), _i64(Co))
    return z


def conv3d_dgrad(dz, w):
    """O2.  dz [N,D,H,W,Co], w [Co,3,3,3,Ci] -> dx [N,D,H,W,Ci]."""
    dz, w = _f64(dz), _f64(w)
    N, D, H, W, Co = dz.shape
    Ci = w.shape[4]
    assert w.shape == (Co, 3, 3, 3, Ci)
    dx = np.empty((N, D, H, W, Ci), dtype=np.float64)
    _L().ora_conv3d_dgrad(_p(dz), _p(w), _p(dx), _i64(N), _i64(D), _i64(H), _i64(W), _i64(Ci), _i64(Co))
    return dx


def conv3d_wgrad(x, dz, dw_prev=None, db_prev=None, beta=0.0, want_db=False):
    """O3.  Returns (dW [Co,3,3,3,Ci], db [Co] or None).  beta=1 accumulates onto *_prev."""
    x, dz = _f64(x), _f64(dz)
    N, D, H, W, Ci = x.shape
    Co = dz.shape[4]
    assert dz.shape == (N, D, H, W, Co)
    dw = np.zeros((Co, 3, 3, 3, Ci)) if dw_prev is None else _f64(dw_prev).copy()
    db = None
    if want_db:
        db = np.zeros((Co,)) if db_prev is None else _f64(db_prev).copy()
    _L().ora_conv3d_wgrad(_p(x), _p(dz), _p(dw), _p(db), ctypes.c_double(beta),
                          _i64(N), _i64(D), _i64(H), _i64(W), _i64(Ci), _i64(Co))
    return dw, db


def inorm_relu(z, gamma=None, beta=None, eps=1e-5, relu=True):
    """O4.  Returns (y, stats[N,C,2] = (mean, rstd))."""
    z, gamma, beta = _f64(z), _f64(gamma), _f64(beta)
    N, C = z.shape[0], z.shape[-1]
    V = int(np.prod(z.shape[1:-1]))
    y = np.empty_like(z)
    stats = np.empty((N, C, 2))
    _L().ora_inorm_relu(_p(z), _p(gamma), _p(beta), ctypes.c_double(eps), _p(y), _p(stats),
                        _i64(N), _i64(V), _i64(C), ctypes.c_int(1 if relu else 0))
    return y, stats


def inorm_relu_bwd(dy, z, gamma=None, beta=None, eps=1e-5, relu=True):
    """O5.  Returns (dz, dgamma[C], dbeta[C])."""
    dy, z, gamma, beta = _f64(dy), _f64(z), _f64(gamma), _f64(beta)
    N, C = z.shape[0], z.shape[-1]
    V = int(np.prod(z.shape[1:-1]))
    dz = np.empty_like(z)
    dg, db = np.empty((C,)), np.empty((C,))
    _L().ora_inorm_relu_bwd(_p(dy), _p(z), _p(gamma), _p(beta), ctypes.c_double(eps), _p(dz), _p(dg), _p(db),
                            _i64(N), _i64(V), _i64(C), ctypes.c_int(1 if relu else 0))
    return dz, dg, db


def maxpool2_fwd(x):
    """O6."""
    x = _f64(x)
    N, D, H, W, C = x.shape
    assert D % 2 == 0 and H % 2 == 0 and W % 2 == 0
    y = np.empty((N, D // 2, H // 2, W // 2, C))
    _L().ora_maxpool2_fwd(_p(x), _p(y), _i64(N), _i64(D), _i64(H), _i64(W), _i64(C))
    return y


def maxpool2_bwd(x, dy):
    """O6 backward: first arg-max in (i,j,k) raster order gets dy."""
    x, dy = _f64(x), _f64(dy)
    N, D, H, W, C = x.shape
    dx = np.empty_like(x)
    _L().ora_maxpool2_bwd(_p(x), _p(dy), _p(dx), _i64(N), _i64(D), _i64(H), _i64(W), _i64(C))
    return dx


def convtr3d_fwd(x, wt, b=None):
    """O7.  x [N,D,H,W,Ci], wt [Ci,2,2,2,Co] -> y [N,2D,2H,2W,Co]."""
    x, wt, b = _f64(x), _f64(wt), _f64(b)
    N, D, H, W, Ci = x.shape
    Co = wt.shape[4]
    assert wt.shape == (Ci, 2, 2, 2, Co)
    y = np.empty((N, 2 * D, 2 * H, 2 * W, Co))
    _L().ora_convtr3d_fwd(_p(x), _p(wt), _p(b), _p(y), _i64(N), _i64(D), _i64(H), _i64(W), _i64(Ci), _i64(Co))
    return y


def convtr3d_bwd(x, wt, dy, want_dx=True, dwt_prev=None, db_prev=None, beta=0.0):
    """O7 backward.  Returns (dx or None, dWt, db)."""
    x, wt, dy = _f64(x), _f64(wt), _f64(dy)
    N, D, H, W, Ci = x.shape
    Co = wt.shape[4]
    assert dy.shape == (N, 2 * D, 2 * H, 2 * W, Co)
    dx = np.empty_like(x) if want_dx else None
    dwt = np.zeros_like(wt) if dwt_prev is None else _f64(dwt_prev).copy()
    db = np.zeros((Co,)) if db_prev is None else _f64(db_prev).copy()
    _L().ora_convtr3d_bwd(_p(x), _p(wt), _p(dy), _p(dx), _p(dwt), _p(db), ctypes.c_double(beta),
                          _i64(N), _i64(D), _i64(H), _i64(W), _i64(Ci), _i64(Co))
    return dx, dwt, db


# ---- one-library-call operations -------------------------------------------------------------

def head_fwd(y, wh, bh=None):
    """1x1x1 convolution to class logits: a matrix product over the channel axis.
    y [...,C], wh [classes,C], bh [classes] -> logits [...,classes]."""
    out = np.asarray(y, dtype=np.float64) @ np.asarray(wh, dtype=np.float64).T
    if bh is not None:
        out = out + np.asarray(bh, dtype=np.float64)
    return out


def softmax(logits):
    """Softmax over the last axis (added after the decoder, Sec. 2.2)."""
    m = logits.max(axis=-1, keepdims=True)
    e = np.exp(logits - m)
    return e / e.sum(axis=-1, keepdims=True)


def cross_entropy(logits, labels):
    """Mean over all voxels of -log softmax(logits)[label].  Returns (loss, dlogits)."""
    p = softmax(logits)
    V = labels.size
    flat = p.reshape(V, -1)
    lab = labels.reshape(V).astype(np.int64)
    loss = -np.mean(np.log(flat[np.arange(V), lab]))
    d = flat.copy()
    d[np.arange(V), lab] -= 1.0
    return float(loss), (d / V).reshape(logits.shape)


def head_bwd(y, wh, dlogits):
    """Adjoints of head_fwd: returns (dy, dWh, dbh)."""
    C = y.shape[-1]
    K = wh.shape[0]
    dl = dlogits.reshape(-1, K)
    dy = (dl @ wh).reshape(y.shape)
    dwh = dl.T @ y.reshape(-1, C)
    dbh = dl.sum(axis=0)
    return dy, dwh, dbh


def round_bf16(a):
    """Round float64/float32 values to the nearest bfloat16 (ties to even), returned as float64.
    Used only by the storage-emulating switch of the network oracle."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(a))


# ---- single-output evaluation for sampled parity at full size -----------------------------------

def conv3d_fwd_at(x, w, b, coords):
    """O1 evaluated only at the listed output voxels.  coords: int array [S,4] of (n,d,h,w).
    x may be any float dtype (it is widened per patch); returns [S,Co] float64."""
    N, D, H, W, Ci = x.shape
    w = np.asarray(w, dtype=np.float64)
    Co = w.shape[0]
    out = np.zeros((len(coords), Co))
    for s, (n, d, h, wv) in enumerate(coords):
        acc = np.zeros(Co) if b is None else np.asarray(b, dtype=np.float64).copy()
        for kd in range(3):
            for kh in range(3):
                for kw in range(3):
                    i, j, k = d + kd - 1, h + kh - 1, wv + kw - 1
                    if 0 <= i < D and 0 <= j < H and 0 <= k < W:
                        acc += w[:, kd, kh, kw, :] @ x[n, i, j, k, :].astype(np.float64)
        out[s] = acc
    return out


def conv3d_dgrad_at(dz, w, coords):
    """O2 evaluated only at the listed input voxels.  Returns [S,Ci]."""
    N, D, H, W, Co = dz.shape
    w = np.asarray(w, dtype=np.float64)
    Ci = w.shape[4]
    out = np.zeros((len(coords), Ci))
    for s, (n, i, j, k) in enumerate(coords):
        acc = np.zeros(Ci)
        for kd in range(3):
            for kh in range(3):
                for kw in range(3):
                    od, oh, ow = i - kd + 1, j - kh + 1, k - kw + 1
                    if 0 <= od < D and 0 <= oh < H and 0 <= ow < W:
                        acc += dz[n, od, oh, ow, :].astype(np.float64) @ w[:, kd, kh, kw, :]
        out[s] = acc
    return out


def conv3d_wgrad_at(x, dz, entries):
    """O3 evaluated only at the listed weight entries.  entries: [S,5] of (co,kd,kh,kw,ci).
    Each is a full reduction over the volume (a shifted dot product of one channel of dz with one
    channel of x); a channel's plane is gathered from the NDHWC tensor once and kept for the
    entries that share it."""
    N, D, H, W, Ci = x.shape
    out = np.zeros(len(entries))
    gp, xp = {}, {}
    for s, (co, kd, kh, kw, ci) in enumerate(entries):
        if co not in gp:
            gp[co] = np.ascontiguousarray(dz[..., co], dtype=np.float64)
        if ci not in xp:
            xp[ci] = np.ascontiguousarray(x[..., ci], dtype=np.float64)
        # output voxel (d,h,w) pairs with input voxel (d+kd-1, h+kh-1, w+kw-1)
        od0, od1 = max(0, 1 - kd), min(D, D + 1 - kd)
        oh0, oh1 = max(0, 1 - kh), min(H, H + 1 - kh)
        ow0, ow1 = max(0, 1 - kw), min(W, W + 1 - kw)
        g = gp[co][:, od0:od1, oh0:oh1, ow0:ow1]
        xx = xp[ci][:, od0 + kd - 1:od1 + kd - 1, oh0 + kh - 1:oh1 + kh - 1, ow0 + kw - 1:ow1 + kw - 1]
        out[s] = float(np.einsum("ndhw,ndhw->", g, xx))
    return out


# ---- optimiser (Sec. 3: RMSProp, learning rate 1e-3) -----------------------------------------------

def rmsprop_step(w, v, g, lr=1e-3, alpha=0.99, eps=1e-8):
    """One RMSProp update in fp64 (no momentum, not centred):
    v' = alpha v + (1 - alpha) g^2,  w' = w - lr g / (sqrt(v') + eps).  Returns (w', v')."""
    w = np.asarray(w, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    v2 = alpha * v + (1.0 - alpha) * g * g
    return w - lr * g / (np.sqrt(v2) + eps), v2


# ---- squeeze-and-excitation on top of InstanceNorm + ReLU (the SEU-Net variant named in Sec. 1) -----
# The paper names the block only through its citations; this is the published squeeze-and-excitation
# gate written out: squeeze = per-sample, per-channel mean of the activated feature map over the
# volume, excitation = two small fully connected layers (ReLU between them, logistic sigmoid after),
# the feature map scaled channel-wise by the gate, and an optional residual tensor added.
# Relative to the paper itself this block is "parity unpinned" (the paper prints neither its definition nor
# any value of it); the functions are pinned by the mathematics of this definition (tests/test_oracle_pins.py).

def se_gate(m, w1, b1, w2, b2):
    """m [N,C] -> (e [N,C] in (0,1), h [N,Cr]):  h = max(0, W1 m + b1),  e = sigmoid(W2 h + b2)."""
    m, w1, b1, w2, b2 = (np.asarray(t, dtype=np.float64) for t in (m, w1, b1, w2, b2))
    h = np.maximum(m @ w1.T + b1, 0.0)
    e = 1.0 / (1.0 + np.exp(-(h @ w2.T + b2)))
    return e, h


def inorm_relu_se(z, gamma, beta, w1, b1, w2, b2, residual=None, eps=1e-5):
    """a = max(0, gamma zhat + beta) (O4);  m = mean_v a;  e = gate(m);  y = a * e (+ residual).
    Returns (y, dict(a, m, e, h, stats))."""
    a, stats = inorm_relu(z, gamma, beta, eps)
    N, C = a.shape[0], a.shape[-1]
    m = a.reshape(N, -1, C).mean(axis=1)
    e, h = se_gate(m, w1, b1, w2, b2)
    y = a * e.reshape((N,) + (1,) * (a.ndim - 2) + (C,))
    if residual is not None:
        y = y + np.asarray(residual, dtype=np.float64)
    return y, dict(a=a, m=m, e=e, h=h, stats=stats)


def inorm_relu_se_bwd(dy, z, gamma, beta, w1, b1, w2, b2, eps=1e-5):
    """Adjoint of inorm_relu_se for upstream dy (the residual's gradient is dy itself).
    Returns (dz, dgamma, dbeta, dw1, db1, dw2, db2)."""
    dy = np.asarray(dy, dtype=np.float64)
    w1 = np.asarray(w1, dtype=np.float64)
    w2 = np.asarray(w2, dtype=np.float64)
    _, c = inorm_relu_se(z, gamma, beta, w1, b1, w2, b2, None, eps)
    a, m, e, h = c["a"], c["m"], c["e"], c["h"]
    N, C = a.shape[0], a.shape[-1]
    V = a.size // (N * C)
    bshape = (N,) + (1,) * (a.ndim - 2) + (C,)
    de = (dy * a).reshape(N, V, C).sum(axis=1)          # gradient of the gate
    dp2 = de * e * (1.0 - e)                            # through the sigmoid
    dw2, db2 = dp2.T @ h, dp2.sum(axis=0)
    dp1 = (dp2 @ w2) * (h > 0)                          # through the hidden ReLU
    dw1, db1 = dp1.T @ m, dp1.sum(axis=0)
    dm = dp1 @ w1                                       # gradient of the squeezed means
    da = dy * e.reshape(bshape) + dm.reshape(bshape) / V
    dz, dgamma, dbeta = inorm_relu_bwd(da, z, gamma, beta, eps)
    return dz, dgamma, dbeta, dw1, db1, dw2, db2
