"""GPU parity of the Block-AP step glue (reconstruction loss, AdamW over {W, s, z}) against the CPU oracle.

The paper names neither the loss form nor the optimizer (Sec. 3.2, Sec. 4.1): mean squared error and AdamW are this
build's reading, pinned in the oracle against the library MSE / autograd and torch.optim.AdamW.  Tolerances: fp32 data
1e-5, bf16 data 2e-2, both as max|got - ref| / max|ref| per tensor; the second moment is quadratic in the gradient, so
where the gradient itself carries the bf16 bar it gets twice that.
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


def npf(t):
    return t.detach().float().cpu().numpy()


def f32(x):
    """The C ABI takes the optimizer constants as binary32: the oracle must be given the same rounded values
    (1 - 0.999 and 1 - float(0.999f) differ by 1.3e-5 of themselves)."""
    return float(np.float32(x))


def relerr(got, ref):
    got = npf(got).astype(np.float64) if isinstance(got, torch.Tensor) else np.asarray(got, np.float64)
    denom = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (denom if denom > 0 else 1.0))


# ---------------------------------------------------------------- reconstruction loss

LOSS_SHAPES = [(1,), (7,), (8,), (3, 5), (2049 * 8 + 3,), (300, 4096), (1111, 4099)]


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("shape", LOSS_SHAPES)
def test_recon_loss(shape, dt):
    Y = synth.normal(shape, 1.0, synth.seed_of("loss", shape, "Y"), dt)
    R = (Y.float() + synth.normal(shape, 0.3, synth.seed_of("loss", shape, "R"))).to(dt)
    ref_loss, ref_dY = oracle.recon_loss(npf(Y), npf(R))
    loss, dY = eq.eqat_recon_loss(Y.cuda(), R.cuda())
    torch.cuda.synchronize()
    assert abs(loss.item() - ref_loss) <= 1e-5 * ref_loss, (loss.item(), ref_loss)
    assert relerr(dY, ref_dY) <= TOL[dt]
    # the loss alone: same sum, same order
    loss2, none = eq.eqat_recon_loss(Y.cuda(), R.cuda(), want_dY=False)
    assert none is None and torch.equal(loss, loss2)


def test_recon_loss_of_equal_tensors_is_zero():
    Y = synth.normal((64, 96), 1.0, 5, torch.bfloat16).cuda()
    loss, dY = eq.eqat_recon_loss(Y, Y.clone())
    assert loss.item() == 0.0 and not dY.float().abs().sum().item()


# ---------------------------------------------------------------- AdamW over {W, s, z}

def _state(tag, O, I, g, wdt):
    G = I // g
    W = synth.normal((O, I), 0.02, synth.seed_of(tag, "W"), wdt)
    s = synth.uniform((O, G), 0.01, 0.05, synth.seed_of(tag, "s"))
    z = synth.uniform((O, G), 0.0, 3.0, synth.seed_of(tag, "z"))
    return W, s, z


def _grads(tag, step, O, I, g, wdt):
    G = I // g
    return (synth.normal((O, I), 0.5, synth.seed_of(tag, "dW", step), wdt),
            synth.normal((O, G), 2.0, synth.seed_of(tag, "ds", step)),
            synth.normal((O, G), 0.1, synth.seed_of(tag, "dz", step)))


@pytest.mark.parametrize("O,I,g,wdt", [(72, 160, 32, torch.float32), (264, 384, 64, torch.bfloat16),
                                       (9, 96, 32, torch.float32), (9, 96, 32, torch.bfloat16),
                                       (1024, 2048, 128, torch.float32)])
def test_adamw_update_three_steps(O, I, g, wdt):
    tag = ("adam", O, I, g, str(wdt))
    lr_w, lr_q, b1, b2, eps, wd_w, wd_q = (f32(x) for x in (2e-3, 1e-2, 0.9, 0.95, 1e-8, 0.05, 0.0))
    W, s, z = _state(tag, O, I, g, wdt)
    dev = {k: v.cuda() for k, v in dict(W=W, s=s, z=z).items()}
    mom = {k: torch.zeros(v.shape, dtype=torch.float32, device="cuda") for k, v in dev.items()}
    mom2 = {k: torch.zeros_like(v) for k, v in mom.items()}
    ref = {k: npf(v).astype(np.float64) for k, v in dict(W=W, s=s, z=z).items()}
    rm = {k: np.zeros_like(v) for k, v in ref.items()}
    rv = {k: np.zeros_like(v) for k, v in ref.items()}
    for step in (1, 2, 3):
        gW, gs, gz = _grads(tag, step, O, I, g, wdt)
        h = eq.AdamW(lr_w, lr_q, b1, b2, eps, wd_w, wd_q, step)
        eq.eqat_block_ap_update(h, 2, g, W=dev["W"], dW=gW.cuda(), mW=mom["W"], vW=mom2["W"],
                                s=dev["s"], ds=gs.cuda(), ms=mom["s"], vs=mom2["s"],
                                z=dev["z"], dz=gz.cuda(), mz=mom["z"], vz=mom2["z"])
        torch.cuda.synchronize()
        for k, gr, lr, wd in (("W", gW, lr_w, wd_w), ("s", gs, lr_q, wd_q), ("z", gz, lr_q, wd_q)):
            # the reference continues from ITS OWN state; a bf16 parameter is rounded after every step on both sides
            ref[k], rm[k], rv[k] = oracle.adamw(ref[k], npf(gr), rm[k], rv[k], lr, b1, b2, eps, wd, step,
                                                p_min=oracle.S_MIN if k == "s" else -np.inf)
            if k == "W" and wdt == torch.bfloat16:
                ref[k] = npf(torch.from_numpy(ref[k]).to(torch.bfloat16)).astype(np.float64)
        for k in ("W", "s", "z"):
            tol = TOL[wdt] if k == "W" else TOL[torch.float32]
            assert relerr(dev[k], ref[k]) <= tol, (step, k)
            assert relerr(mom[k], rm[k]) <= 1e-5, (step, k, "m")
            assert relerr(mom2[k], rv[k]) <= 1e-5, (step, k, "v")
    if wdt == torch.bfloat16:
        # rounding the reference after every step keeps the two sides within a bf16 unit of the largest weight
        assert relerr(dev["W"], ref["W"]) <= 2.0 ** -7


def test_update_holds_step_sizes_at_their_floor():
    # a step that would carry s through zero (gradient positive, learning rate larger than s) leaves it at 1e-10, the
    # floor of the min/max initialisation; z and W have no bound.  After it the layer still quantizes: codes in range.
    O, I, g, bits = 8, 128, 64, 2
    W = synth.normal((O, I), 0.02, 91, torch.float32).cuda()
    s = torch.full((O, 2), 1e-3, dtype=torch.float32, device="cuda")
    z = torch.ones((O, 2), dtype=torch.float32, device="cuda")
    gs = torch.ones_like(s); gz = torch.ones_like(z); gW = torch.ones_like(W)
    zeros = lambda t: torch.zeros(t.shape, dtype=torch.float32, device="cuda")
    h = eq.AdamW(1e-4, 0.5, 0.9, 0.999, 1e-8, 0.0, 0.0, 1)
    s_ref = oracle.adamw(npf(s), npf(gs), np.zeros(s.shape), np.zeros(s.shape), f32(0.5), f32(0.9), f32(0.999), f32(1e-8), 0.0, 1,
                         p_min=oracle.S_MIN)[0]
    z_ref = oracle.adamw(npf(z), npf(gz), np.zeros(z.shape), np.zeros(z.shape), f32(0.5), f32(0.9), f32(0.999), f32(1e-8), 0.0, 1)[0]
    eq.eqat_block_ap_update(h, bits, g, W=W, dW=gW, mW=zeros(W), vW=zeros(W), s=s, ds=gs, ms=zeros(s), vs=zeros(s),
                            z=z, dz=gz, mz=zeros(z), vz=zeros(z))
    torch.cuda.synchronize()
    assert np.all(s_ref == oracle.S_MIN) and np.array_equal(npf(s).astype(np.float64), s_ref)
    assert np.all(z_ref < 0.6) and relerr(z, z_ref) <= 1e-5
    Wp, zp = eq.eqat_pack(W, s, z, bits, g)
    codes, _ = eq.eqat_unpack(Wp, zp, I, bits, g)
    c_ref, _ = oracle.quantize(npf(W), npf(s), npf(z), bits, g)
    assert np.array_equal(codes.cpu().numpy(), c_ref)


def test_adamw_update_of_a_subset_leaves_the_rest_alone():
    O, I, g = 40, 128, 64
    W, s, z = _state("subset", O, I, g, torch.float32)
    gW, gs, gz = _grads("subset", 1, O, I, g, torch.float32)
    sd = s.cuda()
    ms, vs = torch.zeros_like(sd), torch.zeros_like(sd)
    h = eq.AdamW(2e-5, 1e-4, 0.9, 0.999, 1e-8, 0.0, 0.0, 1)
    eq.eqat_block_ap_update(h, 2, g, s=sd, ds=gs.cuda(), ms=ms, vs=vs, shape=(O, I))      # E2E-QP: step sizes only
    torch.cuda.synchronize()
    lr_w, lr_q, b1, b2, eps = f32(2e-5), f32(1e-4), f32(0.9), f32(0.999), f32(1e-8)
    p, m, v = oracle.adamw(npf(s), npf(gs), np.zeros(s.shape), np.zeros(s.shape), lr_q, b1, b2, eps, 0.0, 1, p_min=oracle.S_MIN)
    assert relerr(sd, p) <= 1e-5 and relerr(ms, m) <= 1e-5 and relerr(vs, v) <= 1e-5
    # W and z alone, in one launch; s untouched
    Wd, zd = W.cuda(), z.cuda()
    s_before = sd.clone()
    mW, vW, mz, vz = (torch.zeros_like(Wd), torch.zeros_like(Wd), torch.zeros_like(zd), torch.zeros_like(zd))
    eq.eqat_block_ap_update(h, 2, g, W=Wd, dW=gW.cuda(), mW=mW, vW=vW, z=zd, dz=gz.cuda(), mz=mz, vz=vz)
    torch.cuda.synchronize()
    assert torch.equal(sd, s_before)
    pW = oracle.adamw(npf(W), npf(gW), np.zeros(W.shape), np.zeros(W.shape), lr_w, b1, b2, eps, 0.0, 1)[0]
    pz = oracle.adamw(npf(z), npf(gz), np.zeros(z.shape), np.zeros(z.shape), lr_q, b1, b2, eps, 0.0, 1)[0]
    assert relerr(Wd, pW) <= 1e-5 and relerr(zd, pz) <= 1e-5


# ---------------------------------------------------------------- the glue in place: whole Block-AP steps of one linear

def test_block_ap_steps_of_one_linear_against_the_oracle_and_the_loss_goes_down():
    """fwd -> reconstruction loss against the full-precision linear -> bwd -> AdamW, 2-bit, bf16 activations, fp32 master
    weights, the paper's learning rates (Sec. 4.1).  Step 1 is checked against the same chain in the oracle; then the
    chain runs on for a few steps on the same batch and the loss must fall."""
    T, I, O, bits, g = 256, 256, 128, 2, 64
    lr_w, lr_q = 2e-5, 1e-4
    X = synth.normal((T, I), 1.0, synth.seed_of("chain", "X"), torch.bfloat16)
    W = synth.normal((O, I), 0.02, synth.seed_of("chain", "W"), torch.float32)
    Yref = (X.float() @ W.t()).to(torch.bfloat16)                     # the teacher: the same linear, not quantized
    s0, z0 = oracle.init_minmax(npf(W), bits, g)
    Xd, Wd, Yrd = X.cuda(), W.cuda(), Yref.cuda()
    sd, zd = torch.from_numpy(s0).cuda(), torch.from_numpy(z0).cuda()
    mom = [torch.zeros_like(t) for t in (Wd, Wd, sd, sd, zd, zd)]

    # the oracle's chain, one step
    Y_o = oracle.fq_linear_fwd(npf(X), npf(W), s0, z0, bits, g)
    loss_o, dY_o = oracle.recon_loss(Y_o.astype(np.float32), npf(Yref))
    gr_o = oracle.fq_linear_bwd(npf(X), npf(W), s0, z0, dY_o.astype(np.float32), bits, g, want=("dW", "ds", "dz"))

    losses = []
    for step in range(1, 13):
        Y = eq.eqat_fq_linear_fwd(Xd, Wd, sd, zd, bits, g)
        loss, dY = eq.eqat_recon_loss(Y, Yrd)
        out = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dY, bits, g, want=("dW", "ds", "dz"))
        if step == 1:
            torch.cuda.synchronize()
            assert abs(loss.item() - loss_o) <= 2e-2 * loss_o
            assert relerr(out["dW"], gr_o["dW"]) <= 2e-2 and relerr(out["ds"], gr_o["ds"]) <= 2e-2
            assert relerr(out["dz"], gr_o["dz"]) <= 2e-2
        if step == 1:
            g_gpu = {k: npf(out[k]) for k in ("dW", "ds", "dz")}          # the gradients the update is about to consume
        h = eq.AdamW(lr_w, lr_q, 0.9, 0.999, 1e-8, 0.0, 0.0, step)
        eq.eqat_block_ap_update(h, bits, g, W=Wd, dW=out["dW"], mW=mom[0], vW=mom[1], s=sd, ds=out["ds"], ms=mom[2],
                                vs=mom[3], z=zd, dz=out["dz"], mz=mom[4], vz=mom[5])
        if step == 1:
            torch.cuda.synchronize()
            for name, got, p0, gk, lr in (("W", Wd, npf(W), "dW", lr_w), ("s", sd, s0, "ds", lr_q), ("z", zd, z0, "dz", lr_q)):
                p, m, v = oracle.adamw(p0, gr_o[gk].astype(np.float32), np.zeros(p0.shape), np.zeros(p0.shape), f32(lr),
                                       f32(0.9), f32(0.999), f32(1e-8), 0.0, 1, p_min=oracle.S_MIN if name == "s" else -np.inf)
                # The first Adam step moves every parameter by lr * g / (|g| + eps), i.e. by lr in the direction of the
                # gradient's sign.  Against the oracle's own chain the two sides can therefore differ by at most 2 lr
                # (where bf16 gradients next to zero disagree on the sign), and by nothing else:
                diff = np.abs(npf(got).astype(np.float64) - p)
                assert diff.max() <= 2.001 * lr + 2.0 ** -22 * np.abs(p).max(), name
                # ... and fed the very gradients the GPU computed, the oracle's update reproduces the GPU's to the
                # fp32 bar (1e-5 of the step, which is what the update changes; plus the parameter's own rounding)
                q = oracle.adamw(p0, g_gpu[gk], np.zeros(p0.shape), np.zeros(p0.shape), f32(lr), f32(0.9), f32(0.999), f32(1e-8),
                                 0.0, 1, p_min=oracle.S_MIN if name == "s" else -np.inf)[0]
                moved = np.abs(npf(got).astype(np.float64) - q)
                tiny = np.abs(g_gpu[gk]) < 1e-6          # lr * g / (|g| + eps) is steep where |g| is of eps's size (1e-8)
                if (~tiny).any():       # (dz is all zeros here: right after min/max initialisation nothing is clamped)
                    assert moved[~tiny].max() <= 1e-5 * lr + 2.0 ** -23 * np.abs(q).max(), name
        losses.append(loss)
    torch.cuda.synchronize()
    losses = [l.item() for l in losses]
    assert losses[-1] < losses[0], losses


# ---------------------------------------------------------------- at the sizes bench.py times

def test_loss_and_update_at_full_size():
    """The loss over one [8192, 4096] bf16 output of the 7B block (the workspace's 2048 partial sums in full use) and the
    AdamW launch over a 4096 x 4096 linear with its 262144 step sizes and zero points, compared in full."""
    T, O, I, g = 8192, 4096, 4096, 64
    Y = synth.normal((T, O), 1.0, synth.seed_of("fullglue", "Y"), torch.bfloat16)
    R = (Y.float() + synth.normal((T, O), 0.2, synth.seed_of("fullglue", "R"))).to(torch.bfloat16)
    ref_loss, ref_dY = oracle.recon_loss(npf(Y), npf(R))
    loss, dY = eq.eqat_recon_loss(Y.cuda(), R.cuda())
    torch.cuda.synchronize()
    assert abs(loss.item() - ref_loss) <= 1e-5 * ref_loss
    assert relerr(dY, ref_dY) <= TOL[torch.bfloat16]
    del Y, R, dY, ref_dY

    tag = "fullglue"
    lr_w, lr_q, b1, b2, eps = (f32(x) for x in (2e-5, 1e-4, 0.9, 0.999, 1e-8))
    W, s, z = _state(tag, O, I, g, torch.bfloat16)
    gW, gs, gz = _grads(tag, 1, O, I, g, torch.bfloat16)
    Wd, sd, zd = W.cuda(), s.cuda(), z.cuda()
    mom = [torch.zeros(t.shape, dtype=torch.float32, device="cuda") for t in (Wd, Wd, sd, sd, zd, zd)]
    # two steps, so that the second starts from non-zero moments
    ref = {"W": npf(W).astype(np.float64), "s": npf(s).astype(np.float64), "z": npf(z).astype(np.float64)}
    rm = {k: np.zeros_like(v) for k, v in ref.items()}
    rv = {k: np.zeros_like(v) for k, v in ref.items()}
    for step in (1, 2):
        h = eq.AdamW(lr_w, lr_q, b1, b2, eps, 0.0, 0.0, step)
        eq.eqat_block_ap_update(h, 2, g, W=Wd, dW=gW.cuda(), mW=mom[0], vW=mom[1], s=sd, ds=gs.cuda(), ms=mom[2], vs=mom[3],
                                z=zd, dz=gz.cuda(), mz=mom[4], vz=mom[5])
        for k, gr, lr in (("W", gW, lr_w), ("s", gs, lr_q), ("z", gz, lr_q)):
            ref[k], rm[k], rv[k] = oracle.adamw(ref[k], npf(gr), rm[k], rv[k], lr, b1, b2, eps, 0.0, step,
                                                p_min=oracle.S_MIN if k == "s" else -np.inf)
        ref["W"] = npf(torch.from_numpy(ref["W"]).to(torch.bfloat16)).astype(np.float64)
    torch.cuda.synchronize()
    assert relerr(Wd, ref["W"]) <= 2.0 ** -7
    assert relerr(sd, ref["s"]) <= 1e-5 and relerr(zd, ref["z"]) <= 1e-5
    assert relerr(mom[0], rm["W"]) <= 1e-5 and relerr(mom[1], rv["W"]) <= 1e-5
    assert relerr(mom[2], rm["s"]) <= 1e-5 and relerr(mom[5], rv["z"]) <= 1e-5
