"""Host-only checks of the C-ABI boundary: the library loads, exports every symbol that
include/lamp.h declares, and its host logic (parameter table, window count, argument errors that
are detected before any launch) behaves.  No compute call is made: no GPU is needed."""
import ctypes
import os
import re

import pytest
import torch

import lamp_synth as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    import paper_2006_12575_amd as L
    if not os.path.exists(L.LIB_PATH):
        from paper_2006_12575_amd import build
        build.build(verbose=False)
    return L


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "lamp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lamp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(L):
    lib = ctypes.CDLL(L.LIB_PATH)
    names = declared_symbols()
    assert len(names) >= 28
    for n in names:
        assert hasattr(lib, n), f"{n} declared in lamp.h but not exported"
    assert set(L.EXPORTS) == set(names), set(L.EXPORTS) ^ set(names)
    assert "gfx950" in L.build_info()


def test_param_table_matches_documented_order(L):
    for levels, base, in_ch, classes, affine in [(5, 32, 1, 10, False), (3, 8, 1, 5, False), (3, 4, 2, 3, True), (1, 8, 1, 2, True)]:
        ud = L.unet_desc(levels, base, in_ch, classes, 1, 16, 16, 16, torch.float32, affine=affine)
        p = S.unet_params(S.streams(0, 1)[0], levels, base, in_ch, classes, affine)
        assert L.lamp_unet_param_count(ud) == len(p)
        for i, (k, v) in enumerate(p.items()):
            assert L.lamp_unet_param_numel(ud, i) == v.size, (i, k)
        assert L.lamp_unet_param_numel(ud, len(p)) == 0 and L.lamp_unet_param_numel(ud, -1) == 0


def test_param_table_of_the_squeeze_and_excitation_variant(L):
    """se_ratio > 0: four gate tensors behind each block's convs, cr = max(1, C / ratio) hidden units."""
    for levels, base, affine, ratio in [(5, 32, False, 16), (3, 8, True, 4), (2, 8, False, 16)]:
        ud = L.unet_desc(levels, base, 1, 4, 1, 16, 16, 16, torch.float32, affine=affine, se_ratio=ratio)
        p = S.unet_params(S.streams(0, 1)[0], levels, base, 1, 4, affine, se_ratio=ratio)
        assert L.lamp_unet_param_count(ud) == len(p)
        for i, (k, v) in enumerate(p.items()):
            assert L.lamp_unet_param_numel(ud, i) == v.size, (i, k)
    bad = L.unet_desc(3, 8, 1, 4, 1, 16, 16, 16, torch.float32, se_ratio=-1)
    assert L.lamp_unet_param_count(bad) == 0 and L.lamp_unet_workspace_bytes(bad, False) == 0
    se = L.unet_desc(3, 32, 1, 4, 1, 16, 16, 16, torch.bfloat16, se_ratio=16)
    plain = L.unet_desc(3, 32, 1, 4, 1, 16, 16, 16, torch.bfloat16)
    assert L.lamp_unet_workspace_bytes(se, True) > L.lamp_unet_workspace_bytes(plain, True)
    # the partition entry points serve the plain U-Net only
    assert L.lamp_unet_stage_workspace_bytes(se, 1, 2) == 0 and L.lamp_unet_tail_workspace_bytes(se, 2) == 0
    assert L.lamp_unet_pipeline_workspace_bytes(se, 1, 2) == 0


def test_noalloc_entry_point_argument_errors(L):
    """lamp_inorm_relu_noalloc: NULL pointers, bad descriptors and requests beyond the fixed scratch are
    turned away on the host before the scratch is even looked up (no GPU needed)."""
    lib = L.lib()
    TD = L.binding.TensorDesc
    ok = TD(1, 8, 8, 8, 32, 32, 1)
    one = ctypes.c_void_p(16)
    call = lambda zd, z, yd, y, st: lib.lamp_inorm_relu_noalloc(ctypes.byref(zd), z, None, None, 1e-5, ctypes.byref(yd), y, st, None)
    assert call(ok, None, ok, one, one) == -1 and call(ok, one, ok, None, one) == -1 and call(ok, one, ok, one, None) == -1
    assert call(TD(1, 0, 8, 8, 32, 32, 1), one, ok, one, one) == -2
    assert call(TD(1, 8, 8, 8, 32, 16, 1), one, ok, one, one) == -2            # ldc < c
    big = TD(64, 128, 128, 128, 4096, 4096, 1)
    assert lib.lamp_inorm_relu_workspace_bytes(ctypes.byref(big)) > (8 << 20)
    assert call(big, one, big, one, one) == -5


def test_window_count(L):
    assert L.lamp_sliding_window_count(256, 256, 160, 64, 0.25) == 75
    assert L.lamp_sliding_window_count(64, 64, 64, 64, 0.25) == 1
    assert L.lamp_sliding_window_count(100, 64, 64, 64, 0.25) == 2
    assert L.lamp_sliding_window_count(32, 64, 64, 64, 0.25) == 0  # volume smaller than the patch


def test_workspace_queries_and_bad_descriptors(L):
    ud = L.unet_desc(5, 32, 1, 10, 2, 128, 128, 128, torch.bfloat16)
    fwd, bwd = L.lamp_unet_workspace_bytes(ud, False), L.lamp_unet_workspace_bytes(ud, True)
    assert 0 < fwd < bwd < 16 * 2 ** 30
    bad = L.unet_desc(5, 32, 1, 10, 2, 120, 128, 128, torch.bfloat16)  # 120 not divisible by 16
    assert L.lamp_unet_workspace_bytes(bad, False) == 0 and L.lamp_unet_param_count(bad) == 0
    assert L.status_string(0) == "ok" and "NULL" in L.status_string(-1)


def test_argument_errors_are_caught_on_the_host(L):
    """Every call below must return its error before touching the device (there is none here)."""
    lib = L.lib()
    TD = L.binding.TensorDesc
    d = TD(1, 4, 4, 4, 8, 8, L.binding.BF16)
    fake = ctypes.c_void_p(4096)  # 16-byte aligned, never dereferenced
    by = ctypes.byref
    # NULL required pointer
    assert lib.lamp_conv3d_fwd(by(d), None, None, fake, None, by(d), fake, None, 1e-5, None, 0, None) == -1
    # shape mismatch between x and z
    d2 = TD(1, 4, 4, 5, 8, 8, L.binding.BF16)
    assert lib.lamp_conv3d_fwd(by(d), fake, None, fake, None, by(d2), fake, None, 1e-5, None, 0, None) == -2
    # ldc < c
    d3 = TD(1, 4, 4, 4, 8, 4, L.binding.BF16)
    assert lib.lamp_conv3d_fwd(by(d3), fake, None, fake, None, by(d), fake, None, 1e-5, None, 0, None) == -2
    # dtype mismatch
    d4 = TD(1, 4, 4, 4, 8, 8, L.binding.F32)
    assert lib.lamp_conv3d_fwd(by(d), fake, None, fake, None, by(d4), fake, None, 1e-5, None, 0, None) == -4
    # misaligned bf16 pointer
    assert lib.lamp_conv3d_fwd(by(d), ctypes.c_void_p(4098), None, fake, None, by(d), fake, None, 1e-5, None, 0, None) == -3
    # statistics requested without a workspace
    assert lib.lamp_conv3d_fwd(by(d), fake, None, fake, None, by(d), fake, fake, 1e-5, None, 0, None) == -5
    # wgrad: beta other than 0/1
    assert lib.lamp_conv3d_wgrad(by(d), fake, None, by(d), fake, fake, None, 0.5, fake, 1 << 30, None) == -2
    # pool: odd dimension
    odd = TD(1, 3, 4, 4, 8, 8, L.binding.BF16)
    half = TD(1, 1, 2, 2, 8, 8, L.binding.BF16)
    assert lib.lamp_maxpool2_fwd(by(odd), fake, None, by(half), fake, None) == -2
    # head: too many classes
    assert lib.lamp_head_fwd(by(d), fake, None, fake, None, 17, fake, None) == -2
    # unet: spatial dims not divisible by 2^(levels-1); missing workspace
    ud = L.unet_desc(3, 8, 1, 5, 1, 30, 32, 32, torch.float32)
    tbl = (ctypes.c_void_p * 32)(*([4096] * 32))
    assert lib.lamp_unet_fwd(by(ud), tbl, fake, fake, fake, 1 << 40, None) == -2
    ud = L.unet_desc(3, 8, 1, 5, 1, 32, 32, 32, torch.float32)
    assert lib.lamp_unet_fwd(by(ud), tbl, fake, fake, fake, 16, None) == -5
    # sliding window: batch of the patch descriptor must equal the window count
    pd = L.unet_desc(3, 8, 1, 5, 7, 64, 64, 64, torch.float32)
    assert lib.lamp_sliding_window_fwd(by(pd), tbl, fake, 256, 256, 160, 0.25, 0.125, fake, fake, 1 << 40, None) == -2


def test_tail_pipeline_and_gate_queries_on_the_host(L):
    """Workspace queries and argument checks of the partition / pipeline / squeeze-and-excitation entry
    points: pure host logic, nothing is launched."""
    lib = L.lib()
    by = ctypes.byref
    fake = ctypes.c_void_p(4096)
    tbl = (ctypes.c_void_p * 64)(*([4096] * 64))
    ud = L.unet_desc(5, 32, 1, 10, 1, 128, 128, 128, torch.bfloat16)
    np_all = L.lamp_unet_param_count(ud)
    # the tail's parameters are the whole net's from the first block after the cut on
    assert [L.lamp_unet_tail_param_offset(ud, f) for f in (2, 3, 5)] == [2, 4, 8]
    assert L.lamp_unet_tail_param_offset(ud, 1) == -1 and L.lamp_unet_tail_param_offset(ud, 6) == -1
    affine = L.unet_desc(5, 32, 1, 10, 1, 128, 128, 128, torch.bfloat16, affine=True)
    assert L.lamp_unet_tail_param_offset(affine, 3) == 12 and np_all == 28
    # workspaces: a later cut leaves less to the tail; the pipeline holds every micro-batch's share
    t2, t4 = L.lamp_unet_tail_workspace_bytes(ud, 2), L.lamp_unet_tail_workspace_bytes(ud, 4)
    assert 0 < t4 < t2 < L.lamp_unet_workspace_bytes(ud, True)
    p1, p2 = L.lamp_unet_pipeline_workspace_bytes(ud, 2, 1), L.lamp_unet_pipeline_workspace_bytes(ud, 2, 2)
    assert p1 > t2 and abs(p2 - 2 * p1) <= 1024
    # the tail needs the concat read from two tensors: bf16 and a base that is a multiple of 32
    assert L.lamp_unet_tail_workspace_bytes(L.unet_desc(5, 32, 1, 10, 1, 128, 128, 128, torch.float32), 2) == 0
    assert L.lamp_unet_tail_workspace_bytes(L.unet_desc(5, 16, 1, 10, 1, 128, 128, 128, torch.bfloat16), 2) == 0
    assert L.lamp_unet_pipeline_workspace_bytes(ud, 5, 2) == 0 and L.lamp_unet_pipeline_workspace_bytes(ud, 2, 0) == 0
    # argument errors before any launch
    assert lib.lamp_unet_tail_fwd(by(ud), 1, tbl, fake, tbl, fake, fake, 1 << 40, None) == -2            # first_level 1
    assert lib.lamp_unet_tail_fwd(by(ud), 3, tbl, fake, None, fake, fake, 1 << 40, None) == -1           # no skips
    assert lib.lamp_unet_tail_fwd(by(ud), 3, tbl, fake, tbl, fake, fake, 16, None) == -5                 # workspace
    assert lib.lamp_unet_pipeline_fwd_bwd(by(ud), 2, 2, tbl, fake, fake, None, fake, tbl, 0.0, fake, 1 << 40, fake, fake) == -2  # one stream twice
    assert lib.lamp_unet_pipeline_fwd_bwd(by(ud), 2, 2, tbl, fake, fake, None, fake, tbl, 0.5, fake, 1 << 40, None, fake) == -2  # beta
    assert lib.lamp_unet_pipeline_fwd_bwd(by(ud), 2, 2, tbl, fake, fake, None, fake, tbl, 0.0, fake, 16, None, fake) == -5
    # squeeze-and-excitation gate
    TD = L.binding.TensorDesc
    d = TD(2, 8, 8, 8, 64, 64, L.binding.BF16)
    assert lib.lamp_inorm_relu_se_workspace_bytes(by(d), 4) > 0
    assert lib.lamp_inorm_relu_se_workspace_bytes(by(d), 0) == 0
    args = (by(d), fake, fake, None, None)
    assert lib.lamp_inorm_relu_se(*args, 0, fake, None, fake, None, None, None, by(d), fake, fake, fake, 1 << 30, None) == -2   # cr
    assert lib.lamp_inorm_relu_se(*args, 4, None, None, fake, None, None, None, by(d), fake, fake, fake, 1 << 30, None) == -1   # w1
    assert lib.lamp_inorm_relu_se(*args, 4, fake, None, fake, None, None, fake, by(d), fake, fake, fake, 1 << 30, None) == -1   # residual without descriptor
    assert lib.lamp_inorm_relu_se(*args, 4, fake, None, fake, None, None, None, by(d), fake, fake, fake, 16, None) == -5
