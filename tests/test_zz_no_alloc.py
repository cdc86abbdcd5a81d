"""eqat_recon_loss_static: the reconstruction loss for callers that cannot allocate (its workgroup partials live in a
device array inside the library instead of a caller's workspace).

Checked through the C ABI against eqat_recon_loss on the same inputs: same kernels, so loss and dY must be bitwise
equal; and against the oracle to the bar of the loss tests (1e-5 on the loss, 1e-5 / 2e-2 on dY).  Two calls in a row,
the second on a smaller input, so that a stale partial of the first call would show in the second; the outputs are
pre-filled with a pattern and the device's allocator is watched across the calls.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2407_11062_amd as eq
from paper_2407_11062_amd import synth

pytestmark = pytest.mark.gpu
TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}


def _case(n, dt, seed):
    Y = synth.normal((n,), 1.0, synth.seed_of("static", n, seed, "Y"), dt)
    R = (Y.float() + synth.normal((n,), 0.3, synth.seed_of("static", n, seed, "R"))).to(dt)
    return Y, R


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_recon_loss_static_matches_workspace_entry_point_twice(dt):
    L = eq.lib()
    # first call: more elements than 2048 workgroups x 256 lanes x 8 (every partial in use, grid-stride loop runs);
    # second call: a few workgroups and a ragged tail
    for n in (2048 * 256 * 8 + 8 * 977 + 5, 8 * 256 * 3 + 3):
        Y, R = _case(n, dt, 1)
        Yd, Rd = Y.cuda(), R.cuda()
        ref_loss_t, ref_dY_t = eq.eqat_recon_loss(Yd, Rd)
        loss = torch.full((1,), -7.0, dtype=torch.float32, device="cuda")
        dY = torch.full_like(Yd, 3.0)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rc = L.eqat_recon_loss_static(n, eq._dt(Yd), ctypes.c_void_p(Yd.data_ptr()), ctypes.c_void_p(Rd.data_ptr()),
                                      ctypes.c_void_p(loss.data_ptr()), ctypes.c_void_p(dY.data_ptr()),
                                      ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0, L.eqat_status_string(rc)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(loss, ref_loss_t), (n, loss.item(), ref_loss_t.item())
        assert torch.equal(dY, ref_dY_t), n
        ref_loss, ref_dY = oracle.recon_loss(Y.float().numpy(), R.float().numpy())
        assert abs(loss.item() - ref_loss) <= 1e-5 * ref_loss
        got = dY.float().cpu().numpy().astype(np.float64)
        assert np.abs(got - ref_dY).max() <= TOL[dt] * np.abs(ref_dY).max()


def test_recon_loss_static_loss_only_and_argument_errors():
    L = eq.lib()
    Y, R = _case(4099, torch.bfloat16, 2)
    Yd, Rd = Y.cuda(), R.cuda()
    ref, _ = eq.eqat_recon_loss(Yd, Rd, want_dY=False)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    eq.eqat_recon_loss_static(Yd, Rd, loss)
    torch.cuda.synchronize()
    assert torch.equal(loss, ref)
    P = ctypes.c_void_p(Yd.data_ptr())
    assert L.eqat_recon_loss_static(0, eq.BF16, P, P, P, None, None) == 2       # EQAT_ERR_SHAPE
    assert L.eqat_recon_loss_static(64, 7, P, P, P, None, None) == 5            # EQAT_ERR_DTYPE
    assert L.eqat_recon_loss_static(64, eq.BF16, None, P, P, None, None) == 1   # EQAT_ERR_NULL
    assert L.eqat_recon_loss_static(64, eq.BF16, P, ctypes.c_void_p(Yd.data_ptr() + 2), P, None, None) == 6   # EQAT_ERR_ALIGN
