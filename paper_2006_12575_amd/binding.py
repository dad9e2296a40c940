"""Thin ctypes binding over liblamp.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/lamp.h), takes torch
tensors that already live on the GPU, passes their data pointers and the current HIP stream, and
raises LampError on a non-zero status.  No arithmetic happens here; torch is used for device
memory and streams only.  The library must be present: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblamp.so")

F32, BF16 = 0, 1


class LampError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: lamp_status {status} ({status_string(status)})")


class TensorDesc(Structure):
    _fields_ = [("n", c_int32), ("d", c_int32), ("h", c_int32), ("w", c_int32), ("c", c_int32),
                ("ldc", c_int32), ("dtype", c_int32)]


class NormIn(Structure):
    _fields_ = [("mean_rstd", c_void_p), ("gamma", c_void_p), ("beta", c_void_p),
                ("c_norm", c_int32), ("relu", c_int32)]


class UnetDesc(Structure):
    _fields_ = [("levels", c_int32), ("base", c_int32), ("in_ch", c_int32), ("classes", c_int32),
                ("n", c_int32), ("d", c_int32), ("h", c_int32), ("w", c_int32),
                ("dtype", c_int32), ("eps", c_float), ("affine", c_int32), ("se_ratio", c_int32)]


_lib = None

_PD = POINTER(TensorDesc)
_PN = POINTER(NormIn)
_PU = POINTER(UnetDesc)
_VP = c_void_p

_SIGS = {
    "lamp_status_string": (c_char_p, [c_int]),
    "lamp_build_info": (c_char_p, []),
    "lamp_rmsprop_step": (c_int, [c_int, POINTER(ctypes.c_int64), _VP, _VP, _VP, _VP, POINTER(c_int32), c_float, c_float,
                                  c_float, _VP]),
    "lamp_conv3d_fwd_workspace_bytes": (c_size_t, [_PD, _PD, c_int]),
    "lamp_conv3d_fwd": (c_int, [_PD, _VP, _PN, _VP, _VP, _PD, _VP, _VP, c_float, _VP, c_size_t, _VP]),
    "lamp_conv3d_dgrad_workspace_bytes": (c_size_t, [_PD, _PD]),
    "lamp_conv3d_dgrad": (c_int, [_PD, _VP, _VP, _PD, _VP, _VP, c_size_t, _VP]),
    "lamp_conv3d_dgrad_inorm_relu_bwd_workspace_bytes": (c_size_t, [_PD, _PD]),
    "lamp_conv3d_dgrad_inorm_relu_bwd": (c_int, [_PD, _VP, _VP, _PD, _VP, _PD, _VP, _VP, _VP, _VP, _PD, _VP, _VP, _VP, c_float,
                                                  _VP, c_size_t, _VP]),
    "lamp_conv3d_wgrad_workspace_bytes": (c_size_t, [_PD, _PD]),
    "lamp_conv3d_wgrad": (c_int, [_PD, _VP, _PN, _PD, _VP, _VP, _VP, c_float, _VP, c_size_t, _VP]),
    "lamp_inorm_relu_workspace_bytes": (c_size_t, [_PD]),
    "lamp_inorm_relu": (c_int, [_PD, _VP, _VP, _VP, c_float, _PD, _VP, _VP, c_int, _VP, c_size_t, _VP]),
    "lamp_inorm_relu_noalloc": (c_int, [_PD, _VP, _VP, _VP, c_float, _PD, _VP, _VP, _VP]),
    "lamp_inorm_relu_bwd_workspace_bytes": (c_size_t, [_PD]),
    "lamp_inorm_relu_bwd": (c_int, [_PD, _VP, _PD, _VP, _VP, _VP, _VP, _PD, _VP, _VP, _VP, c_float, _VP, c_size_t, _VP]),
    "lamp_maxpool2_fwd": (c_int, [_PD, _VP, _PN, _PD, _VP, _VP]),
    "lamp_maxpool2_bwd": (c_int, [_PD, _VP, _PN, _PD, _VP, _PD, _VP, _PD, _VP, _VP]),
    "lamp_convtr3d_workspace_bytes": (c_size_t, [_PD, _PD]),
    "lamp_convtr3d": (c_int, [_PD, _VP, _PN, _VP, _VP, _PD, _VP, _VP, c_size_t, _VP]),
    "lamp_convtr3d_bwd_workspace_bytes": (c_size_t, [_PD, _PD]),
    "lamp_convtr3d_bwd": (c_int, [_PD, _VP, _PN, _VP, _PD, _VP, _PD, _VP, _VP, _VP, c_float, _VP, c_size_t, _VP]),
    "lamp_inorm_relu_se_workspace_bytes": (c_size_t, [_PD, c_int]),
    "lamp_inorm_relu_se": (c_int, [_PD, _VP, _VP, _VP, _VP, c_int, _VP, _VP, _VP, _VP, _PD, _VP, _PD, _VP, _VP, _VP, c_size_t, _VP]),
    "lamp_inorm_relu_se_bwd": (c_int, [_PD, _VP, _PD, _VP, _VP, _VP, _VP, c_int, _VP, _VP, _VP, _PD, _VP, _VP, _VP, _VP, _VP, _VP,
                                       _VP, c_float, _VP, c_size_t, _VP]),
    "lamp_head_ce_workspace_bytes": (c_size_t, [_PD, c_int]),
    "lamp_head_fwd": (c_int, [_PD, _VP, _PN, _VP, _VP, c_int, _VP, _VP]),
    "lamp_head_ce": (c_int, [_PD, _VP, _PN, _VP, _VP, c_int, _VP, _VP, _VP, _PD, _VP, _VP, _VP, c_float, _VP, c_size_t, _VP]),
    "lamp_unet_param_count": (c_int32, [_PU]),
    "lamp_unet_param_numel": (c_int64, [_PU, c_int32]),
    "lamp_unet_workspace_bytes": (c_size_t, [_PU, c_int]),
    "lamp_unet_fwd": (c_int, [_PU, POINTER(c_void_p), _VP, _VP, _VP, c_size_t, _VP]),
    "lamp_unet_fwd_bwd": (c_int, [_PU, POINTER(c_void_p), _VP, _VP, _VP, _VP, POINTER(c_void_p), c_float, _VP, c_size_t, _VP]),
    "lamp_unet_stage_workspace_bytes": (c_size_t, [_PU, c_int, c_int, c_int]),
    "lamp_unet_stage_fwd": (c_int, [_PU, c_int, c_int, POINTER(c_void_p), _VP, _VP, POINTER(c_void_p), _VP, c_size_t, _VP]),
    "lamp_unet_stage_bwd": (c_int, [_PU, c_int, c_int, POINTER(c_void_p), _VP, POINTER(c_void_p), _VP, POINTER(c_void_p),
                                    POINTER(c_void_p), c_float, _VP, _VP, c_size_t, _VP]),
    "lamp_unet_tail_param_offset": (c_int32, [_PU, c_int32]),
    "lamp_unet_tail_workspace_bytes": (c_size_t, [_PU, c_int, c_int]),
    "lamp_unet_tail_fwd": (c_int, [_PU, c_int, POINTER(c_void_p), _VP, POINTER(c_void_p), _VP, _VP, c_size_t, _VP]),
    "lamp_unet_tail_fwd_bwd": (c_int, [_PU, c_int, POINTER(c_void_p), _VP, POINTER(c_void_p), _VP, _VP, _VP,
                                       POINTER(c_void_p), c_float, _VP, POINTER(c_void_p), _VP, c_size_t, _VP]),
    "lamp_unet_pipeline_workspace_bytes": (c_size_t, [_PU, c_int, c_int]),
    "lamp_unet_pipeline_fwd_bwd": (c_int, [_PU, c_int, c_int, POINTER(c_void_p), _VP, _VP, _VP, _VP, POINTER(c_void_p),
                                           c_float, _VP, c_size_t, _VP, _VP]),
    "lamp_sliding_window_count": (c_int32, [c_int32, c_int32, c_int32, c_int32, c_float]),
    "lamp_sliding_window_workspace_bytes": (c_size_t, [_PU, c_int32, c_int32, c_int32]),
    "lamp_sliding_window_fwd": (c_int, [_PU, POINTER(c_void_p), _VP, c_int32, c_int32, c_int32, c_float, c_float, _VP, _VP,
                                        c_size_t, _VP]),
}

EXPORTS = tuple(_SIGS.keys())


def lib():
    """Load liblamp.so (once).  Raises if it has not been built: there is no CPU fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2006_12575_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().lamp_status_string(int(status)).decode()


def build_info() -> str:
    return lib().lamp_build_info().decode()


def _check(status, where):
    if status != 0:
        raise LampError(status, where)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def desc(t: torch.Tensor) -> TensorDesc:
    """Descriptor of a dense NDHWC tensor or of a channel slice buf[..., a:b] of one."""
    assert t.dim() == 5, "expected [N,D,H,W,C]"
    n, d, h, w, c = t.shape
    assert c == 1 or t.stride(4) == 1, "channels must be contiguous"
    ext = [d * h * w, h * w, w, 1]  # voxels spanned by one step of dims 0..3
    ldc = c
    for dim in (3, 2, 1, 0):
        if t.shape[dim] > 1:
            ldc = t.stride(dim) // ext[dim]
            break
    for dim in range(4):
        assert t.shape[dim] == 1 or t.stride(dim) == ldc * ext[dim], "not an NDHWC view with dense voxels"
    assert ldc >= c
    return TensorDesc(n, d, h, w, c, ldc, _dtype_code(t))


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream():
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _norm(nm):
    """nm: None or dict(mean_rstd=, gamma=, beta=, c_norm=, relu=)."""
    if nm is None:
        return None
    g, b = nm.get("gamma"), nm.get("beta")
    return ctypes.byref(NormIn(nm["mean_rstd"].data_ptr(), g.data_ptr() if g is not None else None,
                               b.data_ptr() if b is not None else None, int(nm["c_norm"]), int(nm.get("relu", 1))))


def _ws(nbytes, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _ptr_table(tensors):
    arr = (c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr()
    return arr


def lamp_rmsprop_step(w, v, g, w_out=None, lr=1e-3, alpha=0.99, eps=1e-8):
    """RMSProp update of the fp32 master tensors `w` (lists of tensors; running mean squares `v`, fp32
    gradients `g`), writing the working copies `w_out` (fp32 or bf16 tensors, entries may be None)."""
    n = len(w)
    numel = (ctypes.c_int64 * n)(*[int(t.numel()) for t in w])
    outs = list(w_out) if w_out is not None else [None] * n
    codes = (c_int32 * n)(*[_dtype_code(t) if t is not None else F32 for t in outs])
    out_tab = (c_void_p * n)()
    for i, t in enumerate(outs):
        out_tab[i] = t.data_ptr() if t is not None else None
    _check(lib().lamp_rmsprop_step(n, numel, _ptr_table(w), _ptr_table(v), _ptr_table(g), out_tab, codes, lr, alpha, eps,
                                   _stream()), "lamp_rmsprop_step")


# ---- layer calls ----------------------------------------------------------------------------------

def lamp_conv3d_fwd(x, w, z, bias=None, xnorm=None, stats_out=None, eps=1e-5, ws=None):
    xd, zd = desc(x), desc(z)
    need = lib().lamp_conv3d_fwd_workspace_bytes(ctypes.byref(xd), ctypes.byref(zd), 1 if stats_out is not None else 0)
    ws = ws if ws is not None else _ws(need, x.device)
    _check(lib().lamp_conv3d_fwd(ctypes.byref(xd), _ptr(x), _norm(xnorm), _ptr(w), _ptr(bias), ctypes.byref(zd), _ptr(z),
                                 _ptr(stats_out), eps, _ptr(ws), ws.numel(), _stream()), "lamp_conv3d_fwd")
    return z


def lamp_conv3d_dgrad(dz, w, dx, ws=None):
    dzd, dxd = desc(dz), desc(dx)
    need = lib().lamp_conv3d_dgrad_workspace_bytes(ctypes.byref(dzd), ctypes.byref(dxd))
    ws = ws if ws is not None else _ws(need, dz.device)
    _check(lib().lamp_conv3d_dgrad(ctypes.byref(dzd), _ptr(dz), _ptr(w), ctypes.byref(dxd), _ptr(dx), _ptr(ws), ws.numel(),
                                   _stream()), "lamp_conv3d_dgrad")
    return dx


def lamp_conv3d_dgrad_inorm_relu_bwd(dz, w, g, z, stats, dzb, gamma=None, beta=None, dgamma=None, dbeta=None, beta_acc=0.0, ws=None):
    """g = data gradient of the conv (dz, w); dzb = InstanceNorm + ReLU backward of g through the layer below (z, stats);
    dzb may be g."""
    dzd, gd, zd, dzbd = desc(dz), desc(g), desc(z), desc(dzb)
    need = lib().lamp_conv3d_dgrad_inorm_relu_bwd_workspace_bytes(ctypes.byref(dzd), ctypes.byref(gd))
    ws = ws if ws is not None else _ws(need, dz.device)
    _check(lib().lamp_conv3d_dgrad_inorm_relu_bwd(ctypes.byref(dzd), _ptr(dz), _ptr(w), ctypes.byref(gd), _ptr(g), ctypes.byref(zd),
                                                  _ptr(z), _ptr(stats), _ptr(gamma), _ptr(beta), ctypes.byref(dzbd), _ptr(dzb),
                                                  _ptr(dgamma), _ptr(dbeta), beta_acc, _ptr(ws), ws.numel(), _stream()),
           "lamp_conv3d_dgrad_inorm_relu_bwd")
    return dzb


def lamp_conv3d_wgrad(x, dz, dw, dbias=None, beta=0.0, xnorm=None, ws=None):
    xd, dzd = desc(x), desc(dz)
    need = lib().lamp_conv3d_wgrad_workspace_bytes(ctypes.byref(xd), ctypes.byref(dzd))
    ws = ws if ws is not None else _ws(need, x.device)
    _check(lib().lamp_conv3d_wgrad(ctypes.byref(xd), _ptr(x), _norm(xnorm), ctypes.byref(dzd), _ptr(dz), _ptr(dw),
                                   _ptr(dbias), beta, _ptr(ws), ws.numel(), _stream()), "lamp_conv3d_wgrad")
    return dw


def lamp_inorm_relu(z, y, stats, gamma=None, beta=None, eps=1e-5, stats_given=False, ws=None):
    zd, yd = desc(z), desc(y)
    need = lib().lamp_inorm_relu_workspace_bytes(ctypes.byref(zd))
    ws = ws if ws is not None else _ws(need, z.device)
    _check(lib().lamp_inorm_relu(ctypes.byref(zd), _ptr(z), _ptr(gamma), _ptr(beta), eps, ctypes.byref(yd), _ptr(y),
                                 _ptr(stats), 1 if stats_given else 0, _ptr(ws), ws.numel(), _stream()), "lamp_inorm_relu")
    return y


def lamp_inorm_relu_noalloc(z, y, stats, gamma=None, beta=None, eps=1e-5):
    """lamp_inorm_relu (statistics computed here) without a workspace: the library's fixed per-GPU scratch is used."""
    zd, yd = desc(z), desc(y)
    _check(lib().lamp_inorm_relu_noalloc(ctypes.byref(zd), _ptr(z), _ptr(gamma), _ptr(beta), eps, ctypes.byref(yd), _ptr(y),
                                         _ptr(stats), _stream()), "lamp_inorm_relu_noalloc")
    return y


def lamp_inorm_relu_bwd(dy, z, stats, dz, gamma=None, beta=None, dgamma=None, dbeta=None, beta_acc=0.0, ws=None):
    dyd, zd, dzd = desc(dy), desc(z), desc(dz)
    need = lib().lamp_inorm_relu_bwd_workspace_bytes(ctypes.byref(zd))
    ws = ws if ws is not None else _ws(need, z.device)
    _check(lib().lamp_inorm_relu_bwd(ctypes.byref(dyd), _ptr(dy), ctypes.byref(zd), _ptr(z), _ptr(stats), _ptr(gamma),
                                     _ptr(beta), ctypes.byref(dzd), _ptr(dz), _ptr(dgamma), _ptr(dbeta), beta_acc,
                                     _ptr(ws), ws.numel(), _stream()), "lamp_inorm_relu_bwd")
    return dz


def lamp_inorm_relu_se(z, stats, w1, w2, y, gate_save, b1=None, b2=None, gamma=None, beta=None, residual=None, ws=None):
    """y = max(0, gamma*zhat + beta) * e[n,c] (+ residual), e the squeeze-and-excitation gate; w1 [cr, C], w2 [C, cr]
    fp32; gate_save fp32 [N, 4C + cr] receives (means, gate, hidden, two mask sums) for the backward."""
    zd, yd = desc(z), desc(y)
    rd = desc(residual) if residual is not None else None
    cr = int(w1.shape[0])
    ws = ws if ws is not None else _ws(lib().lamp_inorm_relu_se_workspace_bytes(ctypes.byref(zd), cr), z.device)
    _check(lib().lamp_inorm_relu_se(ctypes.byref(zd), _ptr(z), _ptr(stats), _ptr(gamma), _ptr(beta), cr, _ptr(w1), _ptr(b1),
                                    _ptr(w2), _ptr(b2), ctypes.byref(rd) if rd is not None else None, _ptr(residual),
                                    ctypes.byref(yd), _ptr(y), _ptr(gate_save), _ptr(ws), ws.numel(), _stream()),
           "lamp_inorm_relu_se")
    return y


def lamp_inorm_relu_se_bwd(dy, z, stats, w1, w2, gate_save, dz, gamma=None, beta=None, dgamma=None, dbeta=None, dw1=None,
                           db1=None, dw2=None, db2=None, beta_acc=0.0, ws=None):
    dyd, zd, dzd = desc(dy), desc(z), desc(dz)
    cr = int(w1.shape[0])
    ws = ws if ws is not None else _ws(lib().lamp_inorm_relu_se_workspace_bytes(ctypes.byref(zd), cr), z.device)
    _check(lib().lamp_inorm_relu_se_bwd(ctypes.byref(dyd), _ptr(dy), ctypes.byref(zd), _ptr(z), _ptr(stats), _ptr(gamma),
                                        _ptr(beta), cr, _ptr(w1), _ptr(w2), _ptr(gate_save), ctypes.byref(dzd), _ptr(dz),
                                        _ptr(dgamma), _ptr(dbeta), _ptr(dw1), _ptr(db1), _ptr(dw2), _ptr(db2), beta_acc,
                                        _ptr(ws), ws.numel(), _stream()), "lamp_inorm_relu_se_bwd")
    return dz


def lamp_maxpool2_fwd(x, y, xnorm=None):
    xd, yd = desc(x), desc(y)
    _check(lib().lamp_maxpool2_fwd(ctypes.byref(xd), _ptr(x), _norm(xnorm), ctypes.byref(yd), _ptr(y), _stream()),
           "lamp_maxpool2_fwd")
    return y


def lamp_maxpool2_bwd(x, dy, dx, add=None, xnorm=None):
    xd, dyd, dxd = desc(x), desc(dy), desc(dx)
    addd = desc(add) if add is not None else None
    _check(lib().lamp_maxpool2_bwd(ctypes.byref(xd), _ptr(x), _norm(xnorm), ctypes.byref(dyd), _ptr(dy),
                                   ctypes.byref(addd) if addd is not None else None, _ptr(add), ctypes.byref(dxd), _ptr(dx),
                                   _stream()), "lamp_maxpool2_bwd")
    return dx


def lamp_convtr3d(x, wt, y, bias=None, xnorm=None, ws=None):
    xd, yd = desc(x), desc(y)
    need = lib().lamp_convtr3d_workspace_bytes(ctypes.byref(xd), ctypes.byref(yd))
    ws = ws if ws is not None else _ws(need, x.device)
    _check(lib().lamp_convtr3d(ctypes.byref(xd), _ptr(x), _norm(xnorm), _ptr(wt), _ptr(bias), ctypes.byref(yd), _ptr(y),
                               _ptr(ws), ws.numel(), _stream()), "lamp_convtr3d")
    return y


def lamp_convtr3d_bwd(x, wt, dy, dx=None, dwt=None, dbias=None, beta=0.0, xnorm=None, ws=None):
    xd, dyd = desc(x), desc(dy)
    dxd = desc(dx) if dx is not None else None
    need = lib().lamp_convtr3d_bwd_workspace_bytes(ctypes.byref(xd), ctypes.byref(dyd))
    ws = ws if ws is not None else _ws(need, x.device)
    _check(lib().lamp_convtr3d_bwd(ctypes.byref(xd), _ptr(x), _norm(xnorm), _ptr(wt), ctypes.byref(dyd), _ptr(dy),
                                   ctypes.byref(dxd) if dxd is not None else None, _ptr(dx), _ptr(dwt), _ptr(dbias), beta,
                                   _ptr(ws), ws.numel(), _stream()), "lamp_convtr3d_bwd")
    return dx, dwt, dbias


def lamp_head_fwd(x, wh, bh, logits, xnorm=None):
    xd = desc(x)
    _check(lib().lamp_head_fwd(ctypes.byref(xd), _ptr(x), _norm(xnorm), _ptr(wh), _ptr(bh), wh.shape[0], _ptr(logits),
                               _stream()), "lamp_head_fwd")
    return logits


def lamp_head_ce(x, wh, bh, labels, loss, logits=None, dx=None, dwh=None, dbh=None, beta=0.0, xnorm=None, ws=None):
    xd = desc(x)
    dxd = desc(dx) if dx is not None else None
    need = lib().lamp_head_ce_workspace_bytes(ctypes.byref(xd), wh.shape[0])
    ws = ws if ws is not None else _ws(need, x.device)
    _check(lib().lamp_head_ce(ctypes.byref(xd), _ptr(x), _norm(xnorm), _ptr(wh), _ptr(bh), wh.shape[0], _ptr(labels),
                              _ptr(logits), _ptr(loss), ctypes.byref(dxd) if dxd is not None else None, _ptr(dx), _ptr(dwh),
                              _ptr(dbh), beta, _ptr(ws), ws.numel(), _stream()), "lamp_head_ce")
    return loss


# ---- network calls --------------------------------------------------------------------------------

def unet_desc(levels, base, in_ch, classes, n, d, h, w, dtype, eps=1e-5, affine=False, se_ratio=0) -> UnetDesc:
    code = {torch.float32: F32, torch.bfloat16: BF16}[dtype]
    return UnetDesc(levels, base, in_ch, classes, n, d, h, w, code, eps, 1 if affine else 0, int(se_ratio))


def lamp_unet_param_count(ud):
    return int(lib().lamp_unet_param_count(ctypes.byref(ud)))


def lamp_unet_param_numel(ud, idx):
    return int(lib().lamp_unet_param_numel(ctypes.byref(ud), idx))


def lamp_unet_workspace_bytes(ud, with_backward):
    return int(lib().lamp_unet_workspace_bytes(ctypes.byref(ud), 1 if with_backward else 0))


def lamp_unet_fwd(ud, params, x, logits, ws=None):
    ws = ws if ws is not None else _ws(lamp_unet_workspace_bytes(ud, False), x.device)
    _check(lib().lamp_unet_fwd(ctypes.byref(ud), _ptr_table(params), _ptr(x), _ptr(logits), _ptr(ws), ws.numel(),
                               _stream()), "lamp_unet_fwd")
    return logits


def lamp_unet_fwd_bwd(ud, params, x, labels, loss, grads, logits=None, beta=0.0, ws=None):
    ws = ws if ws is not None else _ws(lamp_unet_workspace_bytes(ud, True), x.device)
    _check(lib().lamp_unet_fwd_bwd(ctypes.byref(ud), _ptr_table(params), _ptr(x), _ptr(labels), _ptr(logits), _ptr(loss),
                                   _ptr_table(grads), beta, _ptr(ws), ws.numel(), _stream()), "lamp_unet_fwd_bwd")
    return loss


def lamp_unet_stage_workspace_bytes(ud, first, last, with_backward=True):
    return int(lib().lamp_unet_stage_workspace_bytes(ctypes.byref(ud), first, last, 1 if with_backward else 0))


def lamp_unet_stage_fwd(ud, first, last, params, x, pooled, skips, ws):
    _check(lib().lamp_unet_stage_fwd(ctypes.byref(ud), first, last, _ptr_table(params), _ptr(x), _ptr(pooled),
                                     _ptr_table(skips), _ptr(ws), ws.numel(), _stream()), "lamp_unet_stage_fwd")


def lamp_unet_stage_bwd(ud, first, last, params, x, skips, d_pooled, d_skips, grads, ws, beta=0.0, dx=None):
    _check(lib().lamp_unet_stage_bwd(ctypes.byref(ud), first, last, _ptr_table(params), _ptr(x), _ptr_table(skips),
                                     _ptr(d_pooled), _ptr_table(d_skips), _ptr_table(grads), beta, _ptr(dx), _ptr(ws),
                                     ws.numel(), _stream()), "lamp_unet_stage_bwd")


def lamp_unet_tail_param_offset(ud, first):
    return int(lib().lamp_unet_tail_param_offset(ctypes.byref(ud), first))


def lamp_unet_tail_workspace_bytes(ud, first, with_backward=True):
    return int(lib().lamp_unet_tail_workspace_bytes(ctypes.byref(ud), first, 1 if with_backward else 0))


def lamp_unet_tail_fwd(ud, first, params, x, skips, logits, ws=None):
    """params: the whole net's table from lamp_unet_tail_param_offset(ud, first) on."""
    ws = ws if ws is not None else _ws(lamp_unet_tail_workspace_bytes(ud, first, False), x.device)
    _check(lib().lamp_unet_tail_fwd(ctypes.byref(ud), first, _ptr_table(params), _ptr(x), _ptr_table(skips), _ptr(logits),
                                    _ptr(ws), ws.numel(), _stream()), "lamp_unet_tail_fwd")
    return logits


def lamp_unet_tail_fwd_bwd(ud, first, params, x, skips, labels, loss, grads, d_skips, d_x=None, logits=None, beta=0.0,
                           ws=None):
    ws = ws if ws is not None else _ws(lamp_unet_tail_workspace_bytes(ud, first, True), x.device)
    _check(lib().lamp_unet_tail_fwd_bwd(ctypes.byref(ud), first, _ptr_table(params), _ptr(x), _ptr_table(skips), _ptr(labels),
                                        _ptr(logits), _ptr(loss), _ptr_table(grads), beta, _ptr(d_x), _ptr_table(d_skips),
                                        _ptr(ws), ws.numel(), _stream()), "lamp_unet_tail_fwd_bwd")
    return loss


def lamp_unet_pipeline_workspace_bytes(ud, cut, micro_batches):
    return int(lib().lamp_unet_pipeline_workspace_bytes(ctypes.byref(ud), cut, micro_batches))


def lamp_unet_pipeline_fwd_bwd(ud, cut, micro_batches, params, x, labels, loss, grads, aux_stream, logits=None, beta=0.0,
                               ws=None):
    """ud describes one micro-batch; x and labels hold micro_batches of them.  aux_stream: a
    torch.cuda.Stream (default priority) other than the current one."""
    ws = ws if ws is not None else _ws(lamp_unet_pipeline_workspace_bytes(ud, cut, micro_batches), x.device)
    _check(lib().lamp_unet_pipeline_fwd_bwd(ctypes.byref(ud), cut, micro_batches, _ptr_table(params), _ptr(x), _ptr(labels),
                                            _ptr(logits), _ptr(loss), _ptr_table(grads), beta, _ptr(ws), ws.numel(),
                                            _stream(), c_void_p(aux_stream.cuda_stream)), "lamp_unet_pipeline_fwd_bwd")
    return loss


def lamp_sliding_window_count(D, H, W, patch, overlap=0.25):
    return int(lib().lamp_sliding_window_count(D, H, W, patch, overlap))


def lamp_sliding_window_fwd(patch_ud, params, vol, out, overlap=0.25, sigma_scale=0.125, ws=None):
    _, D, H, W, _ = vol.shape
    need = lib().lamp_sliding_window_workspace_bytes(ctypes.byref(patch_ud), D, H, W)
    ws = ws if ws is not None else _ws(need, vol.device)
    _check(lib().lamp_sliding_window_fwd(ctypes.byref(patch_ud), _ptr_table(params), _ptr(vol), D, H, W, overlap,
                                         sigma_scale, _ptr(out), _ptr(ws), ws.numel(), _stream()), "lamp_sliding_window_fwd")
    return out
