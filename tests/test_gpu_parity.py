"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Sizes are chosen so that the fp64 oracle finishes in seconds while the GPU kernels still run several
tiles with ragged edges in every dimension.  Bars: integer codes / packed bytes / s, z of the min-max
initialisation bit-exact; floating-point outputs max|gpu - ref| / max|ref| <= 2e-2 on the bf16 MFMA
path and <= 1e-5 on the fp32 path.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2407_11062_amd as eq
from paper_2407_11062_amd import synth

pytestmark = pytest.mark.gpu

TOL = {torch.bfloat16: 2e-2, torch.float32: 1e-5}


def dev(t):
    return t.cuda().contiguous()


def npf(t):
    return t.detach().float().cpu().numpy()


def relerr(got, ref):
    got = npf(got).astype(np.float64)
    denom = np.abs(ref).max()
    if denom == 0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / denom)


def make_case(tag, T, I, O, bits, g, act, wdt, trained=True, w_std=0.02):
    G = 1 if g == -1 else I // g
    W = synth.normal((O, I), w_std, synth.seed_of(tag, "W"), wdt)
    X = synth.normal((T, I), 1.0, synth.seed_of(tag, "X"), act)
    dY = synth.normal((T, O), 1.0, synth.seed_of(tag, "dY"), act)
    s, z = oracle.init_minmax(npf(W), bits, g)
    if trained:
        u, d = synth.trained_state_noise((O, G), synth.seed_of(tag, "sz"))
        s = (s * u.numpy()).astype(np.float32)
        z = (z + d.numpy()).astype(np.float32)
    return X, W, torch.from_numpy(s), torch.from_numpy(z), dY


BF16_CASES = [
    # tag, T, I, O, bits, g, w dtype
    ("b2g64", 300, 384, 264, 2, 64, torch.bfloat16),
    ("b3g128", 257, 512, 136, 3, 128, torch.bfloat16),
    ("b4g32", 130, 160, 72, 4, 32, torch.bfloat16),
    ("b2g64w32", 200, 256, 128, 2, 64, torch.float32),
    ("b2perchan", 150, 384, 40, 2, -1, torch.bfloat16),
    ("b3g96", 96, 192, 64, 3, 96, torch.bfloat16),
    ("b4g256", 64, 512, 8, 4, 256, torch.float32),
    ("t1", 1, 128, 16, 2, 64, torch.bfloat16),
]


# --------------------------------------------------------------------------- elementwise passes

@pytest.mark.parametrize("bits,g,wdt", [(2, 64, torch.bfloat16), (3, 128, torch.float32), (4, 32, torch.bfloat16),
                                        (2, 512, torch.bfloat16), (4, 96, torch.float32), (3, -1, torch.bfloat16)])
def test_init_minmax_bit_exact(bits, g, wdt):
    O, I = 67, 1536
    W = synth.normal((O, I), 0.02, synth.seed_of("init", bits, g), wdt)
    W[3, :64] = 0.125                                  # a constant group: the 1e-10 floor
    s_ref, z_ref = oracle.init_minmax(npf(W), bits, g)
    s, z = eq.eqat_init_minmax(dev(W), bits, g)
    assert np.array_equal(npf(s), s_ref)
    assert np.array_equal(npf(z), z_ref)


@pytest.mark.parametrize("bits,g,wdt", [(2, 64, torch.bfloat16), (3, 128, torch.bfloat16), (4, 32, torch.float32),
                                        (3, 32, torch.float32), (2, -1, torch.bfloat16), (4, 128, torch.bfloat16)])
def test_pack_bytes_bit_exact_and_unpack(bits, g, wdt):
    O, I = 93, 1024
    X, W, s, z, dY = make_case(("pack", bits, g), 1, I, O, bits, g, torch.float32, wdt)
    z[0, 0] = -2.0                                      # zero points outside the code range are clamped when packed
    z[1, 0] = 2 ** bits + 1.0
    Wp_ref, zp_ref = oracle.pack(npf(W), s.numpy(), z.numpy(), bits, g)
    Wp, zp = eq.eqat_pack(dev(W), dev(s), dev(z), bits, g)
    assert Wp.shape == Wp_ref.shape and zp.shape == zp_ref.shape
    assert np.array_equal(Wp.cpu().numpy(), Wp_ref)
    assert np.array_equal(zp.cpu().numpy(), zp_ref)
    codes, zc = eq.eqat_unpack(Wp, zp, I, bits, g)
    c_ref, z_refc = oracle.unpack(Wp_ref, zp_ref, I, bits, g)
    assert np.array_equal(codes.cpu().numpy(), c_ref) and np.array_equal(zc.cpu().numpy(), z_refc)
    c_direct, _ = oracle.quantize(npf(W), s.numpy(), z.numpy(), bits, g)
    assert np.array_equal(codes.cpu().numpy(), c_direct)


def test_codes_exact_near_rounding_ties():
    # weights placed within a few ulp of every rounding tie of their group: the cheap reciprocal path must
    # hand these to the exact division
    bits, g, O, I = 4, 32, 64, 1024
    rng = np.random.default_rng(5)
    s = rng.uniform(0.001, 0.01, (O, I // g)).astype(np.float32)
    z = np.full((O, I // g), 8.0, np.float32)
    k = rng.integers(-8, 8, (O, I)) + 0.5
    W = (k * np.repeat(s, g, 1)).astype(np.float32)
    bump = rng.integers(-2, 3, (O, I)).astype(np.int32)
    W = (W.view(np.int32) + bump).view(np.float32)
    c_ref, _ = oracle.quantize(W, s, z, bits, g)
    Wp, zp = eq.eqat_pack(dev(torch.from_numpy(W)), dev(torch.from_numpy(s)), dev(torch.from_numpy(z)), bits, g)
    codes, _ = eq.eqat_unpack(Wp, zp, I, bits, g)
    assert np.array_equal(codes.cpu().numpy(), c_ref)


@pytest.mark.parametrize("bits,wdt,groups", [(2, torch.bfloat16, (64, 64, 64)), (3, torch.float32, (128, 32, -1)),
                                             (4, torch.bfloat16, (32, 96, 256))])
def test_batched_passes_equal_the_single_calls(bits, wdt, groups):
    """Several matrices in one launch (min/max, pack, Eq.(1) before a Block-AP step): bitwise what one call per matrix
    gives, which the tests around hold against the oracle.  Shapes and group sizes differ inside a batch."""
    shapes = [(72, 512), (136, 384), (8, 768)]
    T = 50
    Ws = [dev(synth.normal(sh, 0.02, synth.seed_of("batch", bits, k), wdt)) for k, sh in enumerate(shapes)]
    descs = [eq.make_desc(T, I, O, bits, g, eq.BF16, eq._dt(Ws[0])) for (O, I), g in zip(shapes, groups)]
    Gs = [1 if g == -1 else I // g for (O, I), g in zip(shapes, groups)]
    ss = [torch.empty((O, G), dtype=torch.float32, device="cuda") for (O, I), G in zip(shapes, Gs)]
    zs = [torch.empty_like(t) for t in ss]
    eq.eqat_init_minmax_batched(eq.Batch(descs, W=Ws, s=ss, z=zs))
    for W, s, z, g in zip(Ws, ss, zs, groups):
        s1, z1 = eq.eqat_init_minmax(W, bits, g)
        assert torch.equal(s, s1) and torch.equal(z, z1)
    for k, (s, z) in enumerate(zip(ss, zs)):      # a trained state, some zero points outside the N-bit range
        u, dlt = synth.trained_state_noise(tuple(s.shape), synth.seed_of("batch", bits, k, "sz"))
        s.mul_(u.cuda()); z.add_(dlt.cuda())
    Wps = [torch.empty((O, I * bits // 8), dtype=torch.uint8, device="cuda") for O, I in shapes]
    zps = [torch.empty((O, 4 * ((G * bits + 31) // 32)), dtype=torch.uint8, device="cuda") for (O, I), G in zip(shapes, Gs)]
    eq.eqat_pack_batched(eq.Batch(descs, W=Ws, s=ss, z=zs, Wpacked=Wps, zpacked=zps))
    for W, s, z, g, Wp, zp in zip(Ws, ss, zs, groups, Wps, zps):
        Wp1, zp1 = eq.eqat_pack(W, s, z, bits, g)
        assert torch.equal(Wp, Wp1) and torch.equal(zp, zp1)
    wss = [eq.workspace(d, eq.OP_FQ_BWD, "cuda").fill_(0xEE) for d in descs]
    eq.eqat_fq_quantize_batched(eq.Batch(descs, W=Ws, s=ss, z=zs, ws=wss))
    for (O, I), W, s, z, g, ws in zip(shapes, Ws, ss, zs, groups, wss):
        X = dev(synth.normal((T, I), 1.0, synth.seed_of("batch", O, "X"), torch.bfloat16))
        dY = dev(synth.normal((T, O), 1.0, synth.seed_of("batch", O, "dY"), torch.bfloat16))
        Y = eq.eqat_fq_linear_fwd(X, W, s, z, bits, g, ws=ws, kept=True)
        out = eq.eqat_fq_linear_bwd(X, W, s, z, dY, bits, g, ws=ws, kept=True)
        assert torch.equal(Y, eq.eqat_fq_linear_fwd(X, W, s, z, bits, g))
        ref = eq.eqat_fq_linear_bwd(X, W, s, z, dY, bits, g)
        for k in ref:
            assert torch.equal(out[k], ref[k]), k
        c_ref, side = oracle.quantize(npf(W), npf(s), npf(z), bits, g)
        codes, clamped, _ = eq.eqat_unpack_state(eq.STATE_FQ_KEPT, ws, O, I, bits, g, want_clamped=True)
        assert np.array_equal(codes.cpu().numpy(), c_ref) and np.array_equal(clamped.cpu().numpy(), (side != 0).astype(np.uint8))


# --------------------------------------------------------------------------- Block-AP

def check_block_ap(X, W, s, z, dY, bits, g, tol):
    Xn, Wn, sn, zn, dYn = npf(X), npf(W), s.numpy(), z.numpy(), npf(dY)
    Y_ref = oracle.fq_linear_fwd(Xn, Wn, sn, zn, bits, g)
    ref = oracle.fq_linear_bwd(Xn, Wn, sn, zn, dYn, bits, g)
    Xd, Wd, sd, zd, dYd = dev(X), dev(W), dev(s), dev(z), dev(dY)
    Y = eq.eqat_fq_linear_fwd(Xd, Wd, sd, zd, bits, g)
    out = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, bits, g)
    torch.cuda.synchronize()
    errs = {"Y": relerr(Y, Y_ref)}
    for k in ("dX", "dW", "ds", "dz"):
        errs[k] = relerr(out[k], ref[k])
    assert all(e <= tol for e in errs.values()), errs
    # the STE mask itself is an integer decision: dW must be exactly zero where, and only where, Eq.(1) clamped
    _, side = oracle.quantize(Wn, sn, zn, bits, g)
    dWn = npf(out["dW"])
    assert not dWn[side != 0].any()
    nz_ref = (ref["dW"] != 0) & (np.abs(ref["dW"]) > 1e-3 * np.abs(ref["dW"]).max())
    assert np.all(dWn[nz_ref] != 0)
    return errs


@pytest.mark.parametrize("trained", [False, True])
def test_block_ap_fp32_single_linear(trained):
    w = synth.WORKLOADS["single_fp32_w4g128"]
    lin = w.layers[0]
    X, W, s, z, dY = make_case(("cfg1", trained), w.tokens, lin.in_features, lin.out_features, w.bits, w.group,
                               torch.float32, torch.float32, trained)
    check_block_ap(X, W, s, z, dY, w.bits, w.group, TOL[torch.float32])


def test_block_ap_fp32_ragged():
    X, W, s, z, dY = make_case("f32ragged", 77, 96, 50, 3, 32, torch.float32, torch.float32)
    check_block_ap(X, W, s, z, dY, 3, 32, TOL[torch.float32])


@pytest.mark.parametrize("tag,T,I,O,bits,g,wdt", BF16_CASES)
def test_block_ap_bf16(tag, T, I, O, bits, g, wdt):
    X, W, s, z, dY = make_case(tag, T, I, O, bits, g, torch.bfloat16, wdt)
    check_block_ap(X, W, s, z, dY, bits, g, TOL[torch.bfloat16])


# More output tiles than the chip holds workgroups: every workgroup of the fwd / dX kernel then walks several tiles with
# its K loop running through the tile boundaries.  Ragged in every dimension, K-tile counts 5 (odd: one padding K tile
# per output tile) and 6; the third case walks with the small (128 x 128) tile (144 big tiles = 576 small ones).
WALK_CASES = [
    ("walk_fwd", 4400, 320, 4104, 2, 64),      # fwd: 18 x 17 = 306 tiles of 256 x 256
    ("walk_dx", 4400, 4128, 328, 3, 32),       # dX: 18 x 17 tiles, K = O = 328
    ("walk_small", 4096, 256, 2304, 4, 128),   # fwd: 32 x 18 = 576 tiles of 128 x 128
    ("walk_k64", 4400, 64, 4104, 2, 64),       # fwd: one K tile per output tile (the start-up loads already reach into the next)
    ("walk_dx_k128", 4400, 4128, 128, 2, 32),  # dX: two K tiles per output tile
]


@pytest.mark.parametrize("tag,T,I,O,bits,g", WALK_CASES)
def test_block_ap_bf16_more_tiles_than_resident_workgroups(tag, T, I, O, bits, g):
    X, W, s, z, dY = make_case(tag, T, I, O, bits, g, torch.bfloat16, torch.bfloat16)
    check_block_ap(X, W, s, z, dY, bits, g, TOL[torch.bfloat16])


# Tile counts that do not fill whole rounds of the resident workgroups, with K long enough to be cut: the last 1.x
# rounds of tiles are then shared out along K, and a tile's parts are added up by whichever contributor arrives last.
SPLIT_CASES = [
    ("cut_fwd", 4400, 512, 4104, 2, 64),       # fwd: 18 x 17 = 306 tiles of 256 x 256, 4 K-tile pairs each
    ("cut_dx", 4400, 4128, 520, 3, 32),        # dX: 306 tiles, K = O = 520: 5 pairs, the last one half past the end
    ("cut_dw", 600, 4416, 4104, 2, 64),        # dW: 18 x 17 tiles, K = T = 600
    ("cut_small", 4096, 512, 2304, 4, 128),    # fwd: 576 tiles of 128 x 128 on 512 resident workgroups
    ("cut_dw_perchan", 520, 4352, 4096, 2, -1),  # dW, 17 x 16 tiles, one group per row (partials + reduce kernel)
    # few tiles beyond the first round and a long K: a whole tile per workgroup, then every remaining tile split among
    # four (small tiles: eight) workgroups, whose parts the first of them adds up in their order
    ("split_fwd", 4400, 2048, 4104, 2, 64),    # fwd: 306 tiles, 16 K-tile pairs
    ("split_dx", 4400, 4128, 2056, 3, 32),     # dX: 306 tiles, K = O = 2056: 17 pairs (uneven pieces, ragged last K tile)
    ("split_small", 4096, 2048, 2304, 4, 128), # fwd: 576 tiles of 128 x 128, 16 pairs, eight contributors
    ("split_3r", 4400, 2048, 8440, 2, 64),     # fwd: 18 x 33 = 594 tiles (not a multiple of 8): two whole rounds, then 10 or 11 tiles per XCD split two ways
    ("split_dw", 2100, 4352, 4104, 3, 64),     # dW: 17 x 17 = 289 tiles, K = T = 2100: 17 pairs, six contributors per split tile
    ("split_dw_small", 2100, 2304, 4096, 4, 128), # dW: 18 x 32 = 576 tiles of 128 x 128 on 512 resident workgroups, eight contributors
    ("split_dw_perchan", 2100, 4352, 4096, 2, -1),  # dW: 17 x 16 tiles, one group per row (per-block partials + reduce kernel), eight contributors
]


@pytest.mark.parametrize("tag,T,I,O,bits,g", SPLIT_CASES)
def test_block_ap_and_e2e_with_tiles_cut_along_k(tag, T, I, O, bits, g):
    X, W, s, z, dY = make_case(tag, T, I, O, bits, g, torch.bfloat16, torch.bfloat16)
    check_block_ap(X, W, s, z, dY, bits, g, TOL[torch.bfloat16])
    check_e2e(X, W, s, z, dY, bits, g, TOL[torch.bfloat16])


def test_block_ap_with_fp32_master_weights_and_dw_tiles_split_along_the_tokens():
    # 17 x 16 tiles of dW; W and dW in fp32 (the epilogue moves four units of W rows per wave instead of two)
    X, W, s, z, dY = make_case("split_dw_f32w", 2100, 4352, 4096, 3, 128, torch.bfloat16, torch.float32)
    check_block_ap(X, W, s, z, dY, 3, 128, TOL[torch.bfloat16])


@pytest.mark.parametrize("case", [2, 5, 6, 9], ids=lambda c: SPLIT_CASES[c][0])
def test_cut_tiles_are_deterministic_and_ignore_what_the_workspace_held(case):
    tag, T, I, O, bits, g = SPLIT_CASES[case]
    X, W, s, z, dY = make_case(tag, T, I, O, bits, g, torch.bfloat16, torch.bfloat16)
    Xd, Wd, sd, zd, dYd = dev(X), dev(W), dev(s), dev(z), dev(dY)
    d = eq.make_desc(T, I, O, bits, g, eq.BF16, eq.BF16)
    ws = eq.workspace(d, eq.OP_FQ_BWD, Xd.device)
    outs = []
    for fill in (0, 255, 171):
        ws.fill_(fill)
        Y = eq.eqat_fq_linear_fwd(Xd, Wd, sd, zd, bits, g, ws=ws, keep=True)
        out = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, bits, g, ws=ws, kept=True)
        out2 = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, bits, g, ws=ws, kept=True)      # counters were left at zero
        torch.cuda.synchronize()
        for k in out:
            assert torch.equal(out[k], out2[k]), k
        outs.append((Y, out))
    for Y, out in outs[1:]:
        assert torch.equal(Y, outs[0][0])
        for k in out:
            assert torch.equal(out[k], outs[0][1][k]), k


@pytest.mark.parametrize("I,O", [(352, 200), (320, 192), (96, 72)])
def test_a_non_finite_token_does_not_leak_into_its_neighbour(I, O):
    """K tiles are 64 wide and two are multiplied per trip: with a contraction length that is not a multiple of 128 the
    last K tile (and a padding tile) reach past the end of an activation row, i.e. into the next row.  The weights there
    are zero, but 0 * Inf is NaN: the chunks past K must not be loaded at all.  Row 7 of X and of dY carries Inf and
    NaN; every other row of Y (fwd, K = I) and of dX (K = O) must come out as without them."""
    T, bits, g = 40, 2, 32
    X, W, s, z, dY = make_case(("leak", I, O), T, I, O, bits, g, torch.bfloat16, torch.bfloat16)
    Xd, Wd, sd, zd, dYd = dev(X), dev(W), dev(s), dev(z), dev(dY)
    Y0 = eq.eqat_fq_linear_fwd(Xd, Wd, sd, zd, bits, g)
    dX0 = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, bits, g, want=("dX",))["dX"]
    Xb, dYb = Xd.clone(), dYd.clone()
    Xb[7, :] = float("inf"); Xb[7, 1] = float("nan")
    dYb[7, :] = float("-inf"); dYb[7, 0] = float("nan")
    Y1 = eq.eqat_fq_linear_fwd(Xb, Wd, sd, zd, bits, g)
    dX1 = eq.eqat_fq_linear_bwd(Xb, Wd, sd, zd, dYb, bits, g, want=("dX",))["dX"]
    Wp, zp = eq.eqat_pack(Wd, sd, zd, bits, g)
    Yq1 = eq.eqat_qlinear_fwd(Xb, Wp, sd, zp, bits, g)
    torch.cuda.synchronize()
    keep = [t for t in range(T) if t != 7]
    assert torch.equal(Y1[keep], Y0[keep]) and torch.equal(dX1[keep], dX0[keep]) and torch.equal(Yq1[keep], Y0[keep])
    assert not torch.isfinite(Y1[7].float()).any() and not torch.isfinite(dX1[7].float()).any()


def test_block_ap_outputs_are_optional_and_deterministic():
    X, W, s, z, dY = make_case("opt", 140, 256, 136, 2, 64, torch.bfloat16, torch.bfloat16)
    Xd, Wd, sd, zd, dYd = dev(X), dev(W), dev(s), dev(z), dev(dY)
    full = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, 2, 64)
    again = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, 2, 64)
    for k in full:
        assert torch.equal(full[k], again[k]), k
    only_ds = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, 2, 64, want=("ds",))
    assert set(only_ds) == {"ds"} and torch.equal(only_ds["ds"], full["ds"])
    only_dx = eq.eqat_fq_linear_bwd(None, Wd, sd, zd, dYd, 2, 64, want=("dX",))
    assert torch.equal(only_dx["dX"], full["dX"])


@pytest.mark.parametrize("tag,T,I,O,bits,g,wdt", [c for c in BF16_CASES if c[0] in ("b2g64", "b3g128", "b2g64w32", "b2perchan", "t1")])
def test_forward_that_keeps_its_quantization_for_the_backward(tag, T, I, O, bits, g, wdt):
    """eqat_fq_linear_fwd_keep + eqat_fq_linear_bwd_kept run Eq.(1) once per step instead of twice: bitwise the results of
    the plain pair (which the tests above hold against the oracle)."""
    X, W, s, z, dY = make_case(tag, T, I, O, bits, g, torch.bfloat16, wdt)
    Xd, Wd, sd, zd, dYd = dev(X), dev(W), dev(s), dev(z), dev(dY)
    d = eq.make_desc(T, I, O, bits, g, eq.BF16, eq._dt(Wd))
    ws = eq.workspace(d, eq.OP_FQ_BWD, Xd.device)
    ws.random_(0, 256)                                    # nothing may depend on what the workspace held before
    Y = eq.eqat_fq_linear_fwd(Xd, Wd, sd, zd, bits, g, ws=ws, keep=True)
    out = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, bits, g, ws=ws, kept=True)
    again = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, bits, g, ws=ws, kept=True, want=("ds", "dX"))   # the kept state survives a backward
    assert torch.equal(Y, eq.eqat_fq_linear_fwd(Xd, Wd, sd, zd, bits, g))
    ref = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, bits, g)
    for k in ("dX", "dW", "ds", "dz"):
        assert torch.equal(out[k], ref[k]), k
    assert torch.equal(again["ds"], ref["ds"]) and torch.equal(again["dX"], ref["dX"])
    # and against the oracle directly
    r = oracle.fq_linear_bwd(npf(X), npf(W), s.numpy(), z.numpy(), npf(dY), bits, g, want=("ds", "dz"))
    assert relerr(out["ds"], r["ds"]) <= TOL[torch.bfloat16] and relerr(out["dz"], r["dz"]) <= TOL[torch.bfloat16]


def test_keep_with_no_tokens_still_leaves_a_usable_workspace():
    X, W, s, z, dY = make_case("keep0", 4, 128, 16, 2, 64, torch.bfloat16, torch.bfloat16)
    Wd, sd, zd = dev(W), dev(s), dev(z)
    d = eq.make_desc(0, 128, 16, 2, 64, eq.BF16, eq.BF16)
    ws = eq.workspace(d, eq.OP_FQ_BWD, Wd.device)
    ws.fill_(255)
    Xe = torch.empty((0, 128), dtype=torch.bfloat16, device="cuda")
    dYe = torch.empty((0, 16), dtype=torch.bfloat16, device="cuda")
    eq.eqat_fq_linear_fwd(Xe, Wd, sd, zd, 2, 64, ws=ws, keep=True)
    out = eq.eqat_fq_linear_bwd(Xe, Wd, sd, zd, dYe, 2, 64, ws=ws, kept=True)
    torch.cuda.synchronize()
    for k in ("dW", "ds", "dz"):
        assert not out[k].float().abs().sum().item() and torch.isfinite(out[k].float()).all(), k


def test_empty_token_batch():
    X, W, s, z, dY = make_case("empty", 4, 128, 16, 2, 64, torch.bfloat16, torch.bfloat16)
    Wd, sd, zd = dev(W), dev(s), dev(z)
    Xe = torch.empty((0, 128), dtype=torch.bfloat16, device="cuda")
    dYe = torch.empty((0, 16), dtype=torch.bfloat16, device="cuda")
    assert eq.eqat_fq_linear_fwd(Xe, Wd, sd, zd, 2, 64).shape == (0, 16)
    out = eq.eqat_fq_linear_bwd(Xe, Wd, sd, zd, dYe, 2, 64)
    torch.cuda.synchronize()
    assert out["dX"].shape == (0, 128)
    for k in ("dW", "ds", "dz"):
        assert not out[k].float().abs().sum().item(), k


# --------------------------------------------------------------------------- E2E-QP

def check_e2e(X, W, s, z, dY, bits, g, tol):
    I = W.shape[1]
    # z as Block-AP left it, -1 and Qmax + 1 included: Eqs.(1),(2) and the packed file use the same N-bit zero point
    Xn, Wn, sn, zn, dYn = npf(X), npf(W), s.numpy(), z.numpy(), npf(dY)
    Wp_ref, zp_ref = oracle.pack(Wn, sn, zn, bits, g)
    Y_ref = oracle.qlinear_fwd(Xn, Wp_ref, sn, zp_ref, bits, g)
    ref = oracle.qlinear_bwd(Xn, Wp_ref, sn, zp_ref, dYn, I, bits, g)
    Xd, sd, dYd = dev(X), dev(s), dev(dY)
    Wp, zp = eq.eqat_pack(dev(W), sd, dev(z), bits, g)
    assert np.array_equal(Wp.cpu().numpy(), Wp_ref) and np.array_equal(zp.cpu().numpy(), zp_ref)
    Y = eq.eqat_qlinear_fwd(Xd, Wp, sd, zp, bits, g)
    out = eq.eqat_qlinear_bwd(Xd, Wp, sd, zp, dYd, I, bits, g)
    torch.cuda.synchronize()
    errs = {"Y": relerr(Y, Y_ref), "dX": relerr(out["dX"], ref["dX"]), "ds": relerr(out["ds"], ref["ds"])}
    assert all(e <= tol for e in errs.values()), errs
    only_ds = eq.eqat_qlinear_bwd(Xd, Wp, sd, zp, dYd, I, bits, g, want=("ds",))
    assert torch.equal(only_ds["ds"], out["ds"])


@pytest.mark.parametrize("tag,T,I,O,bits,g,wdt", BF16_CASES)
def test_e2e_qp_bf16(tag, T, I, O, bits, g, wdt):
    X, W, s, z, dY = make_case(tag, T, I, O, bits, g, torch.bfloat16, wdt)
    check_e2e(X, W, s, z, dY, bits, g, TOL[torch.bfloat16])


@pytest.mark.parametrize("bits,g", [(4, 128), (3, 32), (2, -1)])
def test_e2e_qp_fp32(bits, g):
    X, W, s, z, dY = make_case(("e2e32", bits, g), 70, 256, 44, bits, g, torch.float32, torch.float32)
    check_e2e(X, W, s, z, dY, bits, g, TOL[torch.float32])


@pytest.mark.parametrize("act", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("bits,g", [(2, 64), (3, 128), (4, 32)])
def test_packed_layer_is_the_layer_block_ap_trained_for_any_zero_point(bits, g, act):
    # Sec. 3.3: E2E-QP starts from the Block-AP result.  With zero points that left the N-bit range during training
    # (-1.4, -1, Qmax + 1, Qmax + 2.5) the packed layer must give the very Y and dX of the fake-quant layer: both GEMM
    # paths consume the same codes and the same (s, zbar) pairs, so the comparison is bitwise.
    T, I, O = 140, 256, 72
    qmax = 2 ** bits - 1
    X, W, s, z, dY = make_case(("handoff", bits, g), T, I, O, bits, g, act, act)
    z[0::5] = -1.0
    z[1::5] = qmax + 1.0
    z[2::5, 0] = -1.4
    z[3::5, 0] = qmax + 2.5
    Xd, Wd, sd, zd, dYd = dev(X), dev(W), dev(s), dev(z), dev(dY)
    Wp, zp = eq.eqat_pack(Wd, sd, zd, bits, g)
    Wp_ref, zp_ref = oracle.pack(npf(W), s.numpy(), z.numpy(), bits, g)
    assert np.array_equal(Wp.cpu().numpy(), Wp_ref) and np.array_equal(zp.cpu().numpy(), zp_ref)
    Y_fq = eq.eqat_fq_linear_fwd(Xd, Wd, sd, zd, bits, g)
    Y_q = eq.eqat_qlinear_fwd(Xd, Wp, sd, zp, bits, g)
    dX_fq = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, bits, g, want=("dX",))["dX"]
    dX_q = eq.eqat_qlinear_bwd(Xd, Wp, sd, zp, dYd, I, bits, g, want=("dX",))["dX"]
    torch.cuda.synchronize()
    if act == torch.bfloat16:
        assert torch.equal(Y_fq, Y_q) and torch.equal(dX_fq, dX_q)
    else:       # the fp32 path multiplies (q - z) * s in both, in the same order, from different kernels' operands
        assert relerr(Y_q, npf(Y_fq).astype(np.float64)) <= 1e-6 and relerr(dX_q, npf(dX_fq).astype(np.float64)) <= 1e-6
    assert relerr(Y_q, oracle.fq_linear_fwd(npf(X), npf(W), s.numpy(), z.numpy(), bits, g)) <= TOL[act]
    ref = oracle.fq_linear_bwd(npf(X), npf(W), s.numpy(), z.numpy(), npf(dY), bits, g)
    out = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, bits, g)
    for k in ("dX", "dW", "ds", "dz"):
        assert relerr(out[k], ref[k]) <= TOL[act], k


@pytest.mark.parametrize("tag,T,I,O,bits,g,wdt", [c for c in BF16_CASES if c[0] in ("b2g64", "b3g128", "b4g32", "b2perchan")])
def test_e2e_forward_that_keeps_its_prepared_codes_for_the_backward(tag, T, I, O, bits, g, wdt):
    X, W, s, z, dY = make_case(tag, T, I, O, bits, g, torch.bfloat16, wdt)
    z = z.clamp(0, 2 ** bits - 1)
    Xd, sd, dYd = dev(X), dev(s), dev(dY)
    Wp, zp = eq.eqat_pack(dev(W), sd, dev(z), bits, g)
    d = eq.make_desc(T, I, O, bits, g, eq.BF16, eq.BF16)
    ws = eq.workspace(d, eq.OP_Q_BWD, Xd.device)
    ws.random_(0, 256)
    Y = eq.eqat_qlinear_fwd(Xd, Wp, sd, zp, bits, g, ws=ws, keep=True)
    out = eq.eqat_qlinear_bwd(Xd, Wp, sd, zp, dYd, I, bits, g, ws=ws, kept=True)
    ref = eq.eqat_qlinear_bwd(Xd, Wp, sd, zp, dYd, I, bits, g)
    assert torch.equal(out["dX"], ref["dX"]) and torch.equal(out["ds"], ref["ds"])
    assert relerr(Y, oracle.qlinear_fwd(npf(X), Wp.cpu().numpy(), s.numpy(), zp.cpu().numpy(), bits, g)) <= TOL[torch.bfloat16]
    if T > 16:      # the plain forward runs the same GEMM (at most 16 tokens: its matrix-vector kernel)
        assert torch.equal(Y, eq.eqat_qlinear_fwd(Xd, Wp, sd, zp, bits, g))


# ---------------------------------------------------------------- E2E-QP with trained (floating-point) zero points

def check_e2e_trained_z(X, W, s, z, dY, bits, g, tol, seed):
    I = W.shape[1]
    qmax = 2 ** bits - 1
    Xn, Wn, sn, dYn = npf(X), npf(W), s.numpy(), npf(dY)
    Wp_ref, _ = oracle.pack(Wn, sn, z.clamp(0, qmax).numpy(), bits, g)
    # zero points after some end-to-end training: no longer integral, slightly outside [0, Qmax] allowed
    drift = synth.uniform(tuple(z.shape), -0.6, 0.6, seed)
    zf = (z.clamp(0, qmax) + drift).contiguous()
    zn = zf.numpy()
    Y_ref = oracle.qlinear_fwd_z(Xn, Wp_ref, sn, zn, bits, g)
    ref = oracle.qlinear_bwd_z(Xn, Wp_ref, sn, zn, dYn, I, bits, g)
    Xd, sd, zd, dYd = dev(X), dev(s), dev(zf), dev(dY)
    Wp = torch.from_numpy(Wp_ref).cuda()
    Y = eq.eqat_qlinear_fwd_z(Xd, Wp, sd, zd, bits, g)
    out = eq.eqat_qlinear_bwd_z(Xd, Wp, sd, zd, dYd, I, bits, g)
    torch.cuda.synchronize()
    errs = {"Y": relerr(Y, Y_ref), "dX": relerr(out["dX"], ref["dX"]), "ds": relerr(out["ds"], ref["ds"]),
            "dz": relerr(out["dz"], ref["dz"])}
    assert all(e <= tol for e in errs.values()), errs
    # outputs are optional and do not depend on which others were asked for
    only_dz = eq.eqat_qlinear_bwd_z(Xd, Wp, sd, zd, dYd, I, bits, g, want=("dz",))
    assert torch.equal(only_dz["dz"], out["dz"]) and "ds" not in only_dz
    only_ds = eq.eqat_qlinear_bwd_z(Xd, Wp, sd, zd, dYd, I, bits, g, want=("ds",))
    assert torch.equal(only_ds["ds"], out["ds"])


# --------------------------------------------------------------------------- E2E-QP on a layer prepared once

@pytest.mark.parametrize("tag,T,I,O,bits,g,wdt", [c for c in BF16_CASES if c[0] in ("b2g64", "b3g128", "b4g32", "b2perchan", "b3g96", "t1")]
                         + [("cut_small_p", 4096, 512, 2304, 4, 128, torch.bfloat16)])
def test_e2e_on_a_prepared_layer_is_bitwise_the_plain_call(tag, T, I, O, bits, g, wdt):
    """Sec. 3.3: the codes are frozen in this phase, so their re-layout is done once (eqat_qlinear_prepare); a step then
    runs only its GEMMs.  Same kernels on the same operands: Y, dX, ds (and dz with float zero points) must be bitwise
    those of eqat_qlinear_fwd / _bwd / _z, which the tests above hold against the oracle.  Two steps in a row on the
    same prepared layer (its counters must come back to zero)."""
    X, W, s, z, dY = make_case(tag, T, I, O, bits, g, torch.bfloat16, wdt)
    Xd, sd, dYd = dev(X), dev(s), dev(dY)
    Wp, zp = eq.eqat_pack(dev(W), sd, dev(z), bits, g)
    prep = eq.eqat_qlinear_prepare(Wp, zp, I, bits, g)
    Y_ref = eq.eqat_qlinear_fwd(Xd, Wp, sd, zp, bits, g) if T > 16 else None      # few tokens: the plain call runs another kernel
    ref = eq.eqat_qlinear_bwd(Xd, Wp, sd, zp, dYd, I, bits, g)
    zf = (dev(z).clamp(0, 2 ** bits - 1) + 0.3).contiguous()
    Yz_ref = eq.eqat_qlinear_fwd_z(Xd, Wp, sd, zf, bits, g) if T > 16 else None
    refz = eq.eqat_qlinear_bwd_z(Xd, Wp, sd, zf, dYd, I, bits, g)
    for step in range(2):
        Y = eq.eqat_qlinear_fwd_prepared(Xd, prep, sd, O, bits, g)
        out = eq.eqat_qlinear_bwd_prepared(Xd, prep, sd, dYd, I, bits, g)
        Yz = eq.eqat_qlinear_fwd_prepared(Xd, prep, sd, O, bits, g, z=zf)
        outz = eq.eqat_qlinear_bwd_prepared(Xd, prep, sd, dYd, I, bits, g, z=zf, want=("dX", "ds", "dz"))
        torch.cuda.synchronize()
        if T > 16:
            assert torch.equal(Y, Y_ref) and torch.equal(Yz, Yz_ref)
        else:
            assert relerr(Y, oracle.qlinear_fwd(npf(X), Wp.cpu().numpy(), s.numpy(), zp.cpu().numpy(), bits, g)) <= TOL[torch.bfloat16]
        for k in ("dX", "ds"):
            assert torch.equal(out[k], ref[k]), k
        for k in ("dX", "ds", "dz"):
            assert torch.equal(outz[k], refz[k]), k
        # the pairs the forward made kept for the backward: one workspace (backward-sized), garbage in it to begin with
        ws = torch.full_like(eq.workspace(eq.make_desc(T, I, O, bits, g, eq.BF16, eq.BF16), eq.OP_QP_BWD, Xd.device), 0xA5)
        Yk = eq.eqat_qlinear_fwd_prepared(Xd, prep, sd, O, bits, g, z=zf, ws=ws, keep=True)
        outk = eq.eqat_qlinear_bwd_prepared(Xd, prep, sd, dYd, I, bits, g, z=zf, want=("dX", "ds", "dz"), ws=ws, kept=True)
        torch.cuda.synchronize()
        assert torch.equal(Yk, Yz)
        for k in ("dX", "ds", "dz"):
            assert torch.equal(outk[k], refz[k]), k


def test_e2e_on_a_prepared_layer_fp32_activations():
    bits, g = 3, 32
    X, W, s, z, dY = make_case(("prep32", bits, g), 70, 128, 48, bits, g, torch.float32, torch.float32)
    Xd, sd, dYd = dev(X), dev(s), dev(dY)
    Wp, zp = eq.eqat_pack(dev(W), sd, dev(z), bits, g)
    prep = eq.eqat_qlinear_prepare(Wp, zp, 128, bits, g, act_dtype=eq.F32)
    Y = eq.eqat_qlinear_fwd_prepared(Xd, prep, sd, 48, bits, g)
    out = eq.eqat_qlinear_bwd_prepared(Xd, prep, sd, dYd, 128, bits, g)
    ref = eq.eqat_qlinear_bwd(Xd, Wp, sd, zp, dYd, 128, bits, g)
    assert torch.equal(Y, eq.eqat_qlinear_fwd(Xd, Wp, sd, zp, bits, g))
    assert torch.equal(out["dX"], ref["dX"]) and torch.equal(out["ds"], ref["ds"])
    ws = eq.workspace(eq.make_desc(70, 128, 48, bits, g, eq.F32, eq.F32), eq.OP_QP_BWD, Xd.device)
    Yk = eq.eqat_qlinear_fwd_prepared(Xd, prep, sd, 48, bits, g, ws=ws, keep=True)
    outk = eq.eqat_qlinear_bwd_prepared(Xd, prep, sd, dYd, 128, bits, g, ws=ws, kept=True)
    assert torch.equal(Yk, Y) and torch.equal(outk["dX"], ref["dX"]) and torch.equal(outk["ds"], ref["ds"])


# --------------------------------------------------------------------------- the integer state the GEMMs work from

@pytest.mark.parametrize("wdt", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("bits,g", [(2, 64), (3, 128), (4, 32), (2, -1), (3, 96)])
def test_state_the_gemms_read_is_bit_exact(bits, g, wdt):
    """Eq.(1)'s integers as the GEMM kernels see them (not the eqat_pack stream, which another instantiation of the
    quantize kernel writes): codes, clamp plane and zbar left by eqat_fq_linear_fwd_keep, codes and zero points left by
    eqat_qlinear_fwd_keep and by eqat_qlinear_prepare, each against oracle.quantize / the unpacked oracle stream."""
    T, I, O = 40, 384, 88
    qmax = 2 ** bits - 1
    X, W, s, z, dY = make_case(("state", bits, g), T, I, O, bits, g, torch.bfloat16, wdt)
    z[::3, 0] = -1.0
    z[1::3, 0] = qmax + 2.0
    c_ref, side = oracle.quantize(npf(W), s.numpy(), z.numpy(), bits, g)
    zb_ref = np.clip(np.rint(z.numpy()), 0, qmax).astype(np.float32)
    Xd, Wd, sd, zd = dev(X), dev(W), dev(s), dev(z)
    d = eq.make_desc(T, I, O, bits, g, eq.BF16, eq._dt(Wd))
    ws = eq.workspace(d, eq.OP_FQ_BWD, Xd.device)
    ws.fill_(0xA5)
    eq.eqat_fq_linear_fwd(Xd, Wd, sd, zd, bits, g, ws=ws, keep=True)
    codes, clamped, zbar = eq.eqat_unpack_state(eq.STATE_FQ_KEPT, ws, O, I, bits, g, want_clamped=True)
    assert np.array_equal(codes.cpu().numpy(), c_ref)
    assert np.array_equal(clamped.cpu().numpy(), (side != 0).astype(np.uint8))
    assert np.array_equal(zbar.cpu().numpy(), zb_ref)
    Wp, zp = eq.eqat_pack(Wd, sd, zd, bits, g)
    wsq = eq.workspace(d, eq.OP_Q_BWD, Xd.device)
    wsq.fill_(0x5A)
    eq.eqat_qlinear_fwd(Xd, Wp, sd, zp, bits, g, ws=wsq, keep=True)
    prep = eq.eqat_qlinear_prepare(Wp, zp, I, bits, g)
    for kind, state in ((eq.STATE_Q_KEPT, wsq), (eq.STATE_PREPARED, prep)):
        codes, _, zbar = eq.eqat_unpack_state(kind, state, O, I, bits, g)
        assert np.array_equal(codes.cpu().numpy(), c_ref), kind
        assert np.array_equal(zbar.cpu().numpy(), zb_ref), kind


@pytest.mark.parametrize("wdt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("bits,g", [(2, 64), (3, 128), (4, 32)])
def test_working_layout_codes_exact_near_rounding_ties(bits, g, wdt):
    # as test_codes_exact_near_rounding_ties, for the instantiations of the quantize kernel that the Block-AP calls run
    # (working layout, with and without the clamp plane); bf16 weights cannot sit a few ulp of binary32 from a tie, so
    # there the step sizes are chosen such that w/s lands on and around the ties exactly
    O, I = 64, 1024
    G = I // g
    qmax = 2 ** bits - 1
    rng = np.random.default_rng(7 + bits)
    z = np.full((O, G), float(qmax // 2), np.float32)
    k = rng.integers(-(qmax // 2) - 1, qmax - qmax // 2 + 1, (O, I)) + 0.5
    if wdt == torch.float32:
        s = rng.uniform(0.001, 0.01, (O, G)).astype(np.float32)
        W = (k * np.repeat(s, g, 1)).astype(np.float32)
        W = (W.view(np.int32) + rng.integers(-2, 3, (O, I)).astype(np.int32)).view(np.float32)
    else:
        s = (2.0 ** rng.integers(-9, -5, (O, G))).astype(np.float32) * rng.choice(np.array([1.0, 3.0, 5.0], np.float32), (O, G))
        W = torch.from_numpy((k * np.repeat(s, g, 1)).astype(np.float32)).bfloat16().float().numpy()
    c_ref, side = oracle.quantize(W, s, z, bits, g)
    Wd = dev(torch.from_numpy(W).to(wdt)); sd = dev(torch.from_numpy(s)); zd = dev(torch.from_numpy(z))
    Xd = torch.zeros((8, I), dtype=torch.bfloat16, device="cuda")
    d = eq.make_desc(8, I, O, bits, g, eq.BF16, eq._dt(Wd))
    for op, keep in ((eq.OP_FQ_BWD, True), (eq.OP_FQ_FWD, False)):
        ws = eq.workspace(d, op, Xd.device)
        eq.eqat_fq_linear_fwd(Xd, Wd, sd, zd, bits, g, ws=ws, keep=keep)
        if keep:
            codes, clamped, _ = eq.eqat_unpack_state(eq.STATE_FQ_KEPT, ws, O, I, bits, g, want_clamped=True)
            assert np.array_equal(clamped.cpu().numpy(), (side != 0).astype(np.uint8))
        else:       # the forward-only workspace starts with the same code array
            codes, _, _ = eq.eqat_unpack_state(eq.STATE_Q_KEPT, ws, O, I, bits, g)
        assert np.array_equal(codes.cpu().numpy(), c_ref), (op, int((codes.cpu().numpy() != c_ref).sum()))


@pytest.mark.parametrize("tag,T,I,O,bits,g,wdt", BF16_CASES)
def test_e2e_qp_trained_z_bf16(tag, T, I, O, bits, g, wdt):
    X, W, s, z, dY = make_case(tag, T, I, O, bits, g, torch.bfloat16, wdt)
    check_e2e_trained_z(X, W, s, z, dY, bits, g, TOL[torch.bfloat16], synth.seed_of(tag, "zdrift"))


@pytest.mark.parametrize("bits,g", [(4, 128), (3, 32), (2, -1)])
def test_e2e_qp_trained_z_fp32(bits, g):
    X, W, s, z, dY = make_case(("e2ez32", bits, g), 70, 256, 44, bits, g, torch.float32, torch.float32)
    check_e2e_trained_z(X, W, s, z, dY, bits, g, TOL[torch.float32], synth.seed_of("e2ez32", bits, g))


def test_e2e_qp_trained_z_with_integral_z_matches_the_packed_z_entry_points():
    X, W, s, z, dY = make_case("zint", 140, 256, 72, 3, 64, torch.bfloat16, torch.bfloat16)
    zc = z.clamp(0, 7)
    Xd, sd, dYd = dev(X), dev(s), dev(dY)
    Wp, zp = eq.eqat_pack(dev(W), sd, dev(zc), 3, 64)
    a = eq.eqat_qlinear_bwd(Xd, Wp, sd, zp, dYd, 256, 3, 64)
    b = eq.eqat_qlinear_bwd_z(Xd, Wp, sd, dev(zc), dYd, 256, 3, 64)
    assert torch.equal(eq.eqat_qlinear_fwd(Xd, Wp, sd, zp, 3, 64), eq.eqat_qlinear_fwd_z(Xd, Wp, sd, dev(zc), 3, 64))
    assert torch.equal(a["dX"], b["dX"]) and torch.equal(a["ds"], b["ds"])


# ---------------------------------------------------------------- E2E-QP forward for a few tokens (matrix-vector kernel)

GEMV_CASES = [
    # tag, T, I, O, bits, g
    ("v1", 1, 4096, 4096, 2, 64),          # the decode shape of the 7B attention projections
    ("v2", 2, 416, 200, 2, 32),            # I not a multiple of 128 (ragged last chunk), O not a multiple of 16
    ("v3", 5, 1024, 72, 3, 128),
    ("v4", 16, 512, 136, 4, 64),           # the most tokens the kernel takes
    ("v5", 3, 384, 40, 2, -1),             # one group per row
    ("v6", 1, 96, 8, 3, 96),               # a single, partly filled chunk; one 8-row block
    ("v7", 4, 2048, 264, 4, 32),
    ("v8", 7, 160, 24, 3, 32),
    # a row gets one wave per 1024 inputs, up to 16: five waves, eleven (the last run ragged), eight with 4-bit codes,
    # and more runs than waves (two trips for some waves: the down projection of the 70B block)
    ("v9", 2, 5120, 48, 2, 64),
    ("v10", 1, 11008, 40, 3, 128),
    ("v11", 3, 8192, 32, 4, 64),
    ("v12", 1, 28672, 24, 2, 64),
]


@pytest.mark.parametrize("tag,T,I,O,bits,g", GEMV_CASES)
def test_e2e_qp_forward_few_tokens(tag, T, I, O, bits, g):
    X, W, s, z, dY = make_case(tag, T, I, O, bits, g, torch.bfloat16, torch.bfloat16)
    qmax = 2 ** bits - 1
    z = z.clamp(0, qmax)
    Xn, sn = npf(X), s.numpy()
    Wp_ref, zp_ref = oracle.pack(npf(W), sn, z.numpy(), bits, g)
    Xd, sd = dev(X), dev(s)
    Wp, zp = torch.from_numpy(Wp_ref).cuda(), torch.from_numpy(zp_ref).cuda()
    Y = eq.eqat_qlinear_fwd(Xd, Wp, sd, zp, bits, g)
    e = relerr(Y, oracle.qlinear_fwd(Xn, Wp_ref, sn, zp_ref, bits, g))
    assert e <= TOL[torch.bfloat16], e
    # trained (floating-point) zero points through the same kernel
    zf = (z + synth.uniform(tuple(z.shape), -0.6, 0.6, synth.seed_of(tag, "zf"))).contiguous()
    Yz = eq.eqat_qlinear_fwd_z(Xd, Wp, sd, dev(zf), bits, g)
    e = relerr(Yz, oracle.qlinear_fwd_z(Xn, Wp_ref, sn, zf.numpy(), bits, g))
    assert e <= TOL[torch.bfloat16], e
    # deterministic, and rows do not leak into each other: token k alone gives the same row k
    assert torch.equal(Y, eq.eqat_qlinear_fwd(Xd, Wp, sd, zp, bits, g))
    if T > 1:
        Yk = eq.eqat_qlinear_fwd(Xd[T - 1:T].contiguous(), Wp, sd, zp, bits, g)
        assert relerr(Yk, npf(Y[T - 1:T]).astype(np.float64)) <= 1e-2


def test_few_token_kernel_and_gemm_agree_across_the_switch():
    # 16 tokens run the matrix-vector kernel, 17 the tiled GEMM: the first 16 rows must agree to bf16 accuracy
    X, W, s, z, dY = make_case("switch", 17, 512, 64, 2, 64, torch.bfloat16, torch.bfloat16)
    z = z.clamp(0, 3)
    sd = dev(s)
    Wp, zp = eq.eqat_pack(dev(W), sd, dev(z), 2, 64)
    Xd = dev(X)
    Y17 = eq.eqat_qlinear_fwd(Xd, Wp, sd, zp, 2, 64)
    Y16 = eq.eqat_qlinear_fwd(Xd[:16].contiguous(), Wp, sd, zp, 2, 64)
    assert relerr(Y16, npf(Y17[:16]).astype(np.float64)) <= 1e-2


# ---------------------------------------------------------------- the rest of the paper's (N, g) grid; stacked linears

# (N, g) pairs of the paper's bit-width / group-size tables that the cases above do not reach
GRID_REST = [(2, 32), (2, 128), (2, 256), (3, 64), (3, 256), (3, -1), (4, 64), (4, -1)]


@pytest.mark.parametrize("bits,g", GRID_REST)
def test_grid_rest_block_ap_and_e2e(bits, g):
    tag = ("grid", bits, g)
    X, W, s, z, dY = make_case(tag, 200, 512, 72, bits, g, torch.bfloat16, torch.bfloat16)
    check_block_ap(X, W, s, z, dY, bits, g, TOL[torch.bfloat16])
    check_e2e(X, W, s, z, dY, bits, g, TOL[torch.bfloat16])
    check_e2e_trained_z(X, W, s, z, dY, bits, g, TOL[torch.bfloat16], synth.seed_of(tag, "zdrift"))


def test_stacked_linears_equal_their_parts():
    """q|k|v (or gate|up) share their input; groups run along the input dimension, so the three weight matrices stacked
    along the output dimension are ONE quantized linear whose every per-row result is that of the part it came from."""
    bits, g, T, I = 2, 64, 300, 256
    parts = [("q", 264), ("k", 40), ("v", 40)]
    Xs = synth.normal((T, I), 1.0, synth.seed_of("stack", "X"), torch.bfloat16)
    Ws, ss, zs, dYs = [], [], [], []
    for name, O in parts:
        _, W, s, z, dY = make_case(("stack", name), T, I, O, bits, g, torch.bfloat16, torch.bfloat16)
        Ws.append(W), ss.append(s), zs.append(z), dYs.append(dY)
    Xd = dev(Xs)
    Wc, sc, zc, dYc = dev(torch.cat(Ws)), dev(torch.cat(ss)), dev(torch.cat(zs)), dev(torch.cat(dYs, dim=1))
    Y = eq.eqat_fq_linear_fwd(Xd, Wc, sc, zc, bits, g)
    out = eq.eqat_fq_linear_bwd(Xd, Wc, sc, zc, dYc, bits, g)
    Wp, zp = eq.eqat_pack(Wc, sc, zc.clamp(0, 3), bits, g)
    dX_sum = torch.zeros((T, I), dtype=torch.float64)
    r0 = 0
    for (name, O), W, s, z, dY in zip(parts, Ws, ss, zs, dYs):
        Wd, sd, zd, dYd = dev(W), dev(s), dev(z), dev(dY)
        rows = slice(r0, r0 + O)
        # every output element is accumulated over the same contraction in the same order: bitwise equal
        assert torch.equal(Y[:, rows], eq.eqat_fq_linear_fwd(Xd, Wd, sd, zd, bits, g)), name
        part = eq.eqat_fq_linear_bwd(Xd, Wd, sd, zd, dYd, bits, g)
        for k in ("dW", "ds", "dz"):
            assert torch.equal(out[k][rows], part[k]), (name, k)
        Wp1, zp1 = eq.eqat_pack(Wd, sd, zd.clamp(0, 3), bits, g)
        assert torch.equal(Wp[rows], Wp1) and torch.equal(zp[rows], zp1), name
        dX_sum += part["dX"].double().cpu()
        r0 += O
    # dX of the stack is the sum of the parts' dX (what the shared input receives), here up to bf16 rounding of the parts
    assert relerr(out["dX"], dX_sum.numpy()) <= TOL[torch.bfloat16]
    # and against the oracle on the stack itself
    ref = oracle.fq_linear_bwd(None, npf(Wc), sc.cpu().numpy(), zc.cpu().numpy(), npf(dYc), bits, g, want=("dX",))
    assert relerr(out["dX"], ref["dX"]) <= TOL[torch.bfloat16]
