"""The allocation-free entry point (for callers that cannot call hipMalloc) against the entry point it is a variant of.

lamp_inorm_relu_noalloc keeps the partial moments of its statistics pass in a fixed device array inside the
library instead of a caller's workspace.  Same kernels, same order of additions: the outputs must be bit for
bit those of lamp_inorm_relu with a workspace, also on a second call with a smaller input (the scratch then
still holds the first call's partials beyond what the second one writes), and the oracle bounds hold as for
the workspace variant."""
import ctypes

import numpy as np
import pytest
import torch

import lamp_synth as S
import oracle as O
import paper_2006_12575_amd as L
from gpu_util import DEV, as64, check, to_dev

pytestmark = pytest.mark.gpu
BF, F32 = torch.bfloat16, torch.float32


def _pair(shape, dt, seed, affine):
    r = np.random.Generator(np.random.PCG64(seed))
    N, D, H, W, C = shape
    z = to_dev(S.normal(r, shape) * 1.5 + 0.3, dt)
    gamma = to_dev(r.uniform(0.5, 1.5, C), F32) if affine else None
    beta = to_dev(r.uniform(-0.5, 0.5, C), F32) if affine else None
    y0, y1 = torch.empty_like(z), torch.empty_like(z)
    s0 = torch.empty((N, C, 2), dtype=F32, device=DEV)
    s1 = torch.empty_like(s0)
    L.lamp_inorm_relu(z, y0, s0, gamma=gamma, beta=beta)
    L.lamp_inorm_relu_noalloc(z, y1, s1, gamma=gamma, beta=beta)
    torch.cuda.synchronize()
    assert torch.equal(s0, s1), "statistics differ from the workspace variant"
    assert torch.equal(y0, y1), "output differs from the workspace variant"
    y_ref, st_ref = O.inorm_relu(as64(z), None if gamma is None else as64(gamma), None if beta is None else as64(beta))
    check(as64(y1), y_ref, dt, f"noalloc inorm_relu {shape}")
    np.testing.assert_allclose(as64(s1)[..., 0], st_ref[..., 0], atol=1e-5 * (1 + np.abs(st_ref[..., 0]).max()))
    np.testing.assert_allclose(as64(s1)[..., 1], st_ref[..., 1], rtol=2e-4)


@pytest.mark.parametrize("dt", [BF, F32])
def test_noalloc_two_calls_in_a_row(dt):
    _pair((2, 24, 40, 48, 64), dt, 9100, True)    # first call: many row chunks
    _pair((1, 7, 9, 13, 32), dt, 9101, False)     # second, smaller: fewer chunks, stale partials behind them
    _pair((1, 5, 6, 7, 3), dt, 9102, True)        # odd channel count (scalar path)


def test_noalloc_rejects_more_than_the_fixed_scratch():
    """A request whose partials exceed the fixed scratch returns LAMP_ERR_WORKSPACE on the host: the descriptor
    alone decides, nothing is launched and no tensor of that size is needed."""
    lib = L.lib()
    zd = L.binding.TensorDesc(64, 128, 128, 128, 4096, 4096, 1)
    assert lib.lamp_inorm_relu_workspace_bytes(ctypes.byref(zd)) > (8 << 20)
    t = torch.empty(16, dtype=torch.uint8, device=DEV)
    st = lib.lamp_inorm_relu_noalloc(ctypes.byref(zd), t.data_ptr(), None, None, 1e-5, ctypes.byref(zd), t.data_ptr(),
                                     t.data_ptr(), None)
    assert st == -5, st
