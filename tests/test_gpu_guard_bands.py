"""No entry point writes outside what it is given: every output tensor and every workspace of the calls below sits
between two guard bands filled with a pattern, and the bands are compared after each call.

The shapes are the awkward ones: ragged in every dimension against the 256 x 256 / 128 x 128 tiles and the 64-wide K
tiles, one token, one group per row, groups wider than a tile, tiles cut along K, the fp32 path, the few-token kernel.
All kernels run their normal, bounds-checked code: nothing here provokes a fault, the test only looks at bytes the
kernels must not have touched.  (Reads outside an input cannot be seen this way; the buffer descriptors the kernels load
through are sized to the tensor and return zeros beyond it.)
"""
import ctypes

import numpy as np
import pytest
import torch

import paper_2407_11062_amd as eq
from paper_2407_11062_amd import synth

pytestmark = pytest.mark.gpu
GUARD = 4096
PATTERN = 0xC3


class Guarded:
    """Tensors carved out of byte buffers with a guard band on either side."""

    def __init__(self):
        self.bufs = []

    def new(self, shape, dtype, fill=None):
        n = int(np.prod(shape)) * torch.empty(0, dtype=dtype).element_size()
        pad = (-n) % 256
        raw = torch.full((GUARD + n + pad + GUARD,), PATTERN, dtype=torch.uint8, device="cuda")
        assert raw.data_ptr() % 256 == 0
        t = raw[GUARD:GUARD + n].view(dtype).view(shape)
        if fill is not None:
            t.copy_(fill)
        self.bufs.append((raw, n))
        return t

    def check(self, what):
        torch.cuda.synchronize()
        for k, (raw, n) in enumerate(self.bufs):
            lo, hi = raw[:GUARD], raw[GUARD + n:]
            assert bool((lo == PATTERN).all()) and bool((hi == PATTERN).all()), f"{what}: guard band of buffer {k} ({n} bytes) was written"


CASES = [
    # tag, T, I, O, bits, g, act, wdt
    ("ragged", 300, 384, 264, 2, 64, torch.bfloat16, torch.bfloat16),
    ("ragged3", 257, 512, 136, 3, 128, torch.bfloat16, torch.float32),
    ("one_token", 1, 128, 16, 2, 64, torch.bfloat16, torch.bfloat16),
    ("per_channel", 150, 384, 40, 2, -1, torch.bfloat16, torch.bfloat16),
    ("wide_group", 64, 512, 8, 4, 256, torch.bfloat16, torch.float32),
    ("fp32_path", 70, 160, 56, 4, 32, torch.float32, torch.float32),
    ("cut_tiles", 4400, 512, 4104, 2, 64, torch.bfloat16, torch.bfloat16),
    ("walk_odd_k", 4400, 320, 4104, 2, 64, torch.bfloat16, torch.bfloat16),
    ("split_dw_tiles", 2100, 4352, 4104, 3, 64, torch.bfloat16, torch.bfloat16),     # 289 dW tiles, 33 K tiles: split along the tokens
]


@pytest.mark.parametrize("tag,T,I,O,bits,g,act,wdt", CASES)
def test_nothing_is_written_outside_outputs_and_workspaces(tag, T, I, O, bits, g, act, wdt):
    G = 1 if g == -1 else I // g
    gd = Guarded()
    W = gd.new((O, I), wdt, synth.normal((O, I), 0.02, synth.seed_of("guard", tag, "W"), wdt).cuda())
    X = gd.new((T, I), act, synth.normal((T, I), 1.0, synth.seed_of("guard", tag, "X"), act).cuda())
    dY = gd.new((T, O), act, synth.normal((T, O), 1.0, synth.seed_of("guard", tag, "dY"), act).cuda())
    s, z = gd.new((O, G), torch.float32), gd.new((O, G), torch.float32)
    eq.eqat_init_minmax(W, bits, g, s=s, z=z)
    gd.check("eqat_init_minmax")
    u, d = synth.trained_state_noise((O, G), synth.seed_of("guard", tag, "sz"))
    s.mul_(u.cuda()); z.add_(d.cuda())

    dsc = eq.make_desc(T, I, O, bits, g, eq._dt(X), eq._dt(W))
    ws_bytes = [eq.lib().eqat_workspace_bytes(ctypes.byref(dsc), op) for op in range(6)]
    ws = [gd.new((max(n, 256),), torch.uint8) for n in ws_bytes]
    Y = gd.new((T, O), act)
    out = {"dX": gd.new((T, I), act), "dW": gd.new((O, I), wdt), "ds": gd.new((O, G), torch.float32),
           "dz": gd.new((O, G), torch.float32)}
    eq.eqat_fq_linear_fwd(X, W, s, z, bits, g, Y=Y, ws=ws[eq.OP_FQ_FWD])
    gd.check("eqat_fq_linear_fwd")
    eq.eqat_fq_linear_bwd(X, W, s, z, dY, bits, g, out=out, ws=ws[eq.OP_FQ_BWD])
    gd.check("eqat_fq_linear_bwd")
    eq.eqat_fq_linear_fwd(X, W, s, z, bits, g, Y=Y, ws=ws[eq.OP_FQ_BWD], keep=True)
    eq.eqat_fq_linear_bwd(X, W, s, z, dY, bits, g, out=out, ws=ws[eq.OP_FQ_BWD], kept=True)
    gd.check("eqat_fq_linear_fwd_keep / _bwd_kept")
    eq.eqat_fq_quantize_batched(eq.Batch([dsc], W=[W], s=[s], z=[z], ws=[ws[eq.OP_FQ_BWD]]))
    eq.eqat_fq_linear_fwd(X, W, s, z, bits, g, Y=Y, ws=ws[eq.OP_FQ_BWD], kept=True)
    gd.check("eqat_fq_quantize_batched / eqat_fq_linear_fwd_kept")

    Wp = gd.new((O, I * bits // 8), torch.uint8)
    zp = gd.new((O, 4 * ((G * bits + 31) // 32)), torch.uint8)
    eq.eqat_pack(W, s, z, bits, g, Wpacked=Wp, zpacked=zp)
    gd.check("eqat_pack")
    eq.eqat_pack_batched(eq.Batch([dsc], W=[W], s=[s], z=[z], Wpacked=[Wp], zpacked=[zp]))
    gd.check("eqat_pack_batched")
    outq = {"dX": out["dX"], "ds": out["ds"]}
    eq.eqat_qlinear_fwd(X, Wp, s, zp, bits, g, Y=Y, ws=ws[eq.OP_Q_FWD])
    gd.check("eqat_qlinear_fwd")
    eq.eqat_qlinear_bwd(X, Wp, s, zp, dY, I, bits, g, out=outq, ws=ws[eq.OP_Q_BWD])
    gd.check("eqat_qlinear_bwd")
    zf = gd.new((O, G), torch.float32, z.clamp(0, 2 ** bits - 1) + 0.25)
    eq.eqat_qlinear_fwd_z(X, Wp, s, zf, bits, g, Y=Y, ws=ws[eq.OP_Q_FWD])
    eq.eqat_qlinear_bwd_z(X, Wp, s, zf, dY, I, bits, g, out={"dX": out["dX"], "ds": out["ds"], "dz": out["dz"]}, ws=ws[eq.OP_Q_BWD])
    gd.check("eqat_qlinear_fwd_z / _bwd_z")
    pbytes = eq.lib().eqat_prepared_bytes(ctypes.byref(dsc))
    prep = gd.new((pbytes,), torch.uint8)
    eq.eqat_qlinear_prepare(Wp, zp, I, bits, g, act_dtype=eq._dt(X), prepared=prep)
    gd.check("eqat_qlinear_prepare")
    eq.eqat_qlinear_fwd_prepared(X, prep, s, O, bits, g, Y=Y, ws=ws[eq.OP_QP_FWD])
    eq.eqat_qlinear_bwd_prepared(X, prep, s, dY, I, bits, g, z=zf, want=("dX", "ds", "dz"), out=out, ws=ws[eq.OP_QP_BWD])
    gd.check("eqat_qlinear_fwd_prepared / _bwd_prepared")
    eq.eqat_qlinear_fwd_prepared(X, prep, s, O, bits, g, z=zf, Y=Y, ws=ws[eq.OP_QP_BWD], keep=True)
    eq.eqat_qlinear_bwd_prepared(X, prep, s, dY, I, bits, g, z=zf, want=("dX", "ds", "dz"), out=out, ws=ws[eq.OP_QP_BWD], kept=True)
    gd.check("eqat_qlinear_fwd_prepared_keep / _bwd_prepared_kept")

    # the step glue on the same tensors
    loss = gd.new((1,), torch.float32)
    dYl = gd.new((T, O), act)
    lws = gd.new((eq.lib().eqat_recon_loss_workspace_bytes(),), torch.uint8)
    eq.eqat_recon_loss(Y, dY, loss=loss, dY=dYl, ws=lws)
    gd.check("eqat_recon_loss")
    eq.eqat_recon_loss_static(Y, dY, loss, dYl)
    gd.check("eqat_recon_loss_static")
    mom = {k: (gd.new(t.shape, torch.float32, torch.zeros(t.shape)), gd.new(t.shape, torch.float32, torch.zeros(t.shape)))
           for k, t in (("W", W), ("s", s), ("z", z))}
    eq.eqat_block_ap_update(eq.AdamW(1e-5, 1e-4, 0.9, 0.999, 1e-8, 0.0, 0.0, 1), bits, g, W=W, dW=out["dW"], mW=mom["W"][0],
                            vW=mom["W"][1], s=s, ds=out["ds"], ms=mom["s"][0], vs=mom["s"][1], z=z, dz=out["dz"],
                            mz=mom["z"][0], vz=mom["z"][1])
    gd.check("eqat_block_ap_update")


@pytest.mark.parametrize("T,I,O,bits,g", [(1, 4096, 136, 2, 64), (5, 1184, 72, 3, 32), (16, 2048, 24, 4, 128), (3, 576, 40, 2, 96)])
def test_few_token_forward_stays_inside_y(T, I, O, bits, g):
    gd = Guarded()
    gen = torch.Generator(device="cuda"); gen.manual_seed(T * 1000 + O)
    Wp = torch.randint(0, 256, (O, I * bits // 8), dtype=torch.uint8, device="cuda", generator=gen)
    G = I // g
    zp = torch.randint(0, 256, (O, 4 * ((G * bits + 31) // 32)), dtype=torch.uint8, device="cuda", generator=gen)
    s = torch.empty((O, G), dtype=torch.float32, device="cuda").uniform_(0.005, 0.02, generator=gen)
    X = gd.new((T, I), torch.bfloat16, torch.randn((T, I), device="cuda", generator=gen).bfloat16())
    Y = gd.new((T, O), torch.bfloat16)
    eq.eqat_qlinear_fwd(X, Wp, s, zp, bits, g, Y=Y)
    gd.check("eqat_qlinear_fwd, few tokens")
    assert bool(torch.isfinite(Y.float()).all())
