"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares, sizes its
buffers as documented, and turns every bad argument into its status code on the host (nothing is launched:
each call below fails validation by construction)."""
import ctypes
import os
import re

import pytest

import paper_2407_11062_amd as eq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, NULL, SHAPE, BITS, GROUP, DTYPE, ALIGN, WORKSPACE, DEVICE = range(9)
P = 0x10000   # a fake, non-NULL, 256-byte aligned "device pointer"; never dereferenced on these paths


def d(T=16, I=128, O=64, bits=2, group=64, act=eq.BF16, w=eq.BF16):
    return eq.make_desc(T, I, O, bits, group, act, w)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "eqat.h")).read()
    declared = set(re.findall(r"\b(eqat_[a-z0-9_]+)\s*\(", header))
    assert declared == set(eq.EXPORTS)
    L = eq.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_header_is_plain_c_and_cxx(tmp_path):
    """The boundary is a C ABI: the header must compile on its own as C99 and as C++11, and a C program that calls the
    host-only helpers must link against the library and agree with the Python binding on the descriptor's layout."""
    import subprocess
    hdr = os.path.join(ROOT, "include", "eqat.h")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c", hdr], check=True)
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", hdr], check=True)
    src = tmp_path / "use.c"
    src.write_text(
        '#include <stdio.h>\n#include "eqat.h"\n'
        "int main(void) {\n"
        "  eqat_desc d = {8192, 4096, 11008, 2, 64, EQAT_BF16, EQAT_BF16};\n"
        '  printf("%d %zu %zu %zu %zu\\n", (int)eqat_validate_desc(&d), sizeof(eqat_desc), eqat_packed_w_bytes(&d),\n'
        "         eqat_packed_z_bytes(&d), eqat_workspace_bytes(&d, EQAT_OP_FQ_BWD));\n"
        "  d.bits = 5;\n"
        '  printf("%s\\n", eqat_status_string(eqat_validate_desc(&d)));\n'
        "  return 0;\n}\n")
    exe = tmp_path / "use"
    libdir = os.path.dirname(eq.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe), "-L", libdir,
                    "-l:" + os.path.basename(eq.LIB_PATH), "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    status, size, wb, zb, ws = (int(x) for x in out[0].split())
    dd = d(T=8192, I=4096, O=11008)
    L = eq.lib()
    assert status == OK and size == ctypes.sizeof(eq.Desc)
    assert wb == L.eqat_packed_w_bytes(ctypes.byref(dd)) == 11008 * 4096 * 2 // 8
    assert zb == L.eqat_packed_z_bytes(ctypes.byref(dd)) and ws == L.eqat_workspace_bytes(ctypes.byref(dd), eq.OP_FQ_BWD)
    assert out[1] == "bits must be 2, 3 or 4"


def test_status_strings():
    L = eq.lib()
    seen = {L.eqat_status_string(i) for i in range(10)}
    assert len(seen) == 10 and all(s for s in seen)
    assert L.eqat_status_string(99) == b"unknown status"


@pytest.mark.parametrize("kw,code", [
    (dict(bits=1), BITS), (dict(bits=5), BITS), (dict(bits=8), BITS),
    (dict(I=100), SHAPE), (dict(I=0), SHAPE), (dict(O=0), SHAPE), (dict(T=-1), SHAPE),
    (dict(O=12), SHAPE),                                  # bf16 activations need O % 8 == 0
    (dict(group=0), GROUP), (dict(group=48), GROUP), (dict(group=96), GROUP), (dict(group=-2), GROUP), (dict(group=16), GROUP),
    (dict(act=2), DTYPE), (dict(w=7), DTYPE),
    (dict(T=40000, I=28672), SHAPE),                      # X would be 2 GiB or more
    (dict(O=32768, I=32768, w=eq.F32), SHAPE),            # W would be 4 GiB
    (dict(T=8, O=8, I=1 << 22), SHAPE),                   # bf16 path: I, O < 2^22
    (dict(T=8, O=8, I=(1 << 22) - 32, group=-1), OK),
    (dict(), OK), (dict(group=-1), OK), (dict(O=12, act=eq.F32), OK), (dict(T=0), OK), (dict(I=96, group=96, bits=3), OK),
])
def test_descriptor_validation(kw, code):
    desc = d(**kw)
    assert eq.lib().eqat_validate_desc(ctypes.byref(desc)) == code
    assert eq.lib().eqat_validate_desc(None) == NULL


def test_packed_sizes():
    L = eq.lib()
    for bits, I, g, O in [(2, 4096, 64, 4096), (3, 5120, 128, 13824), (4, 128, 32, 8), (3, 96, 96, 5), (2, 8192, 64, 28672)]:
        desc = d(I=I, O=O, bits=bits, group=g)
        G = I // g
        assert L.eqat_packed_w_bytes(ctypes.byref(desc)) == O * I * bits // 8
        assert L.eqat_packed_z_bytes(ctypes.byref(desc)) == O * 4 * ((G * bits + 31) // 32)
    bad = d(bits=7)
    assert L.eqat_packed_w_bytes(ctypes.byref(bad)) == 0 and L.eqat_packed_z_bytes(ctypes.byref(bad)) == 0


def test_workspace_sizes_are_modest_and_monotone():
    L = eq.lib()
    desc = d(T=4096, I=4096, O=4096)
    w = [L.eqat_workspace_bytes(ctypes.byref(desc), op) for op in range(6)]
    wbytes = 4096 * 4096 * 2
    assert 0 < w[eq.OP_FQ_FWD] < wbytes // 4          # 2-bit codes + (s, z) pairs, a fraction of W itself
    assert w[eq.OP_FQ_FWD] < w[eq.OP_FQ_BWD] < wbytes // 2
    assert 0 < w[eq.OP_Q_FWD] <= w[eq.OP_Q_BWD] < wbytes // 4         # re-laid-out codes + zero points
    assert w[eq.OP_QP_FWD] == w[eq.OP_QP_BWD] == 4096 * 64 * 8        # a prepared layer: only the (s, z) pairs
    assert L.eqat_workspace_bytes(ctypes.byref(desc), 9) == 0
    f32 = d(T=256, I=512, O=512, bits=4, group=128, act=eq.F32, w=eq.F32)
    assert L.eqat_workspace_bytes(ctypes.byref(f32), eq.OP_FQ_FWD) == 0
    assert L.eqat_workspace_bytes(ctypes.byref(f32), eq.OP_FQ_BWD) >= 512 * 512 * 4


def test_null_alignment_and_workspace_errors_come_back_before_any_launch():
    L = eq.lib()
    desc = d()
    r = ctypes.byref(desc)
    ws_need = L.eqat_workspace_bytes(r, eq.OP_FQ_BWD)
    # NULL
    assert L.eqat_init_minmax(r, None, P, P, None) == NULL
    assert L.eqat_init_minmax(r, P, None, P, None) == NULL
    assert L.eqat_pack(r, P, P, P, None, P, None) == NULL
    assert L.eqat_fq_linear_fwd(r, None, P, P, P, P, P, 1 << 30, None) == NULL
    assert L.eqat_fq_linear_fwd(r, P, P, P, P, None, P, 1 << 30, None) == NULL
    assert L.eqat_fq_linear_bwd(r, P, P, P, P, None, P, P, P, P, P, 1 << 30, None) == NULL
    assert L.eqat_fq_linear_bwd(r, None, P, P, P, P, P, P, P, P, P, 1 << 30, None) == NULL   # dW wanted, X missing
    assert L.eqat_qlinear_fwd(r, P, None, P, P, P, P, 1 << 30, None) == NULL
    assert L.eqat_qlinear_bwd(r, None, P, P, P, P, None, P, P, 1 << 30, None) == NULL        # ds wanted, X missing
    assert L.eqat_unpack(r, None, P, P, None, None) == NULL
    # alignment
    assert L.eqat_init_minmax(r, P + 2, P, P, None) == ALIGN
    assert L.eqat_pack(r, P, P, P, P + 8, P, None) == ALIGN
    assert L.eqat_fq_linear_fwd(r, P, P, P, P, P + 4, P, 1 << 30, None) == ALIGN
    assert L.eqat_fq_linear_fwd(r, P, P, P, P, P, P + 16, 1 << 30, None) == ALIGN            # workspace: 256 bytes
    assert L.eqat_qlinear_bwd(r, P, P, P, P, P, P, P + 1, P, 1 << 30, None) == ALIGN
    # workspace
    assert ws_need > 0
    assert L.eqat_fq_linear_bwd(r, P, P, P, P, P, P, P, P, P, P, ws_need - 1, None) == WORKSPACE
    assert L.eqat_fq_linear_bwd(r, P, P, P, P, P, P, P, P, P, None, ws_need, None) == WORKSPACE
    assert L.eqat_fq_linear_fwd(r, P, P, P, P, P, P, 0, None) == WORKSPACE
    assert L.eqat_qlinear_fwd(r, P, P, P, P, P, None, 0, None) == WORKSPACE
    assert L.eqat_qlinear_bwd(r, P, P, P, P, P, P, P, P, 16, None) == WORKSPACE
    # the keep / kept pair checks like the plain pair, with the backward's workspace size for both
    ws_fwd = L.eqat_workspace_bytes(r, eq.OP_FQ_FWD)
    assert ws_fwd < ws_need
    assert L.eqat_fq_linear_fwd_keep(r, P, P, P, P, P, P, ws_fwd, None) == WORKSPACE
    assert L.eqat_fq_linear_fwd_keep(r, None, P, P, P, P, P, ws_need, None) == NULL
    assert L.eqat_fq_linear_bwd_kept(r, P, P, P, P, P, P, P, P, P, P, ws_need - 1, None) == WORKSPACE
    assert L.eqat_fq_linear_bwd_kept(r, P, P, P, P, None, P, P, P, P, P, ws_need, None) == NULL
    assert L.eqat_fq_linear_bwd_kept(r, P, P, P, P, P, None, None, None, None, P, ws_need, None) == OK      # nothing wanted
    wq_f, wq_b = L.eqat_workspace_bytes(r, eq.OP_Q_FWD), L.eqat_workspace_bytes(r, eq.OP_Q_BWD)
    assert wq_f <= wq_b
    assert L.eqat_qlinear_fwd_keep(r, P, P, P, P, P, P, wq_b - 1, None) == WORKSPACE
    assert L.eqat_qlinear_fwd_keep(r, P, None, P, P, P, P, wq_b, None) == NULL
    assert L.eqat_qlinear_bwd_kept(r, P, P, P, P, P, P, P, P, wq_b - 1, None) == WORKSPACE
    assert L.eqat_qlinear_bwd_kept(r, None, P, P, P, P, None, P, P, wq_b, None) == NULL      # ds wanted, X missing
    assert L.eqat_qlinear_bwd_kept(r, P, P, P, P, P, None, None, P, wq_b, None) == OK        # nothing wanted
    # the prepared-layer entry points
    pb = L.eqat_prepared_bytes(r)
    assert pb >= 64 * 128 * 2 // 8 + 64 * 2 * 4
    assert L.eqat_prepared_bytes(ctypes.byref(d(bits=7))) == 0
    assert L.eqat_qlinear_prepare(r, None, P, P, pb, None) == NULL
    assert L.eqat_qlinear_prepare(r, P, P, None, pb, None) == NULL
    assert L.eqat_qlinear_prepare(r, P, P, P, pb - 1, None) == WORKSPACE
    assert L.eqat_qlinear_prepare(r, P, P, P + 16, pb, None) == ALIGN
    wp_f, wp_b = L.eqat_workspace_bytes(r, eq.OP_QP_FWD), L.eqat_workspace_bytes(r, eq.OP_QP_BWD)
    assert wp_f <= wp_b < wq_b
    assert L.eqat_qlinear_fwd_prepared(r, P, None, P, None, P, P, 1 << 30, None) == NULL
    assert L.eqat_qlinear_fwd_prepared(r, P, P, None, None, P, P, 1 << 30, None) == NULL
    assert L.eqat_qlinear_fwd_prepared(r, P, P + 16, P, None, P, P, 1 << 30, None) == ALIGN
    assert L.eqat_qlinear_bwd_prepared(r, None, P, P, None, P, None, P, None, P, 1 << 30, None) == NULL      # ds wanted, X missing
    assert L.eqat_qlinear_bwd_prepared(r, P, P, P, None, P, None, None, None, P, 1 << 30, None) == OK        # nothing wanted
    per_chan = d(group=-1, I=256)           # one group per row: the backward needs room for per-32-column partial sums
    rp = ctypes.byref(per_chan)
    need = L.eqat_workspace_bytes(rp, eq.OP_QP_BWD)
    assert need > 0
    assert L.eqat_qlinear_bwd_prepared(rp, P, P, P, None, P, P, P, None, P, need - 1, None) == WORKSPACE
    # ... and the pair that keeps the (s, z) pairs between forward and backward: the forward takes the backward's workspace
    assert L.eqat_qlinear_fwd_prepared_keep(rp, P, P, P, None, P, P, need - 1, None) == WORKSPACE
    assert L.eqat_qlinear_fwd_prepared_keep(r, P, None, P, None, P, P, 1 << 30, None) == NULL
    assert L.eqat_qlinear_fwd_prepared_keep(r, P, P, None, None, P, P, 1 << 30, None) == NULL
    assert L.eqat_qlinear_bwd_prepared_kept(rp, P, P, P, None, P, P, P, None, P, need - 1, None) == WORKSPACE
    assert L.eqat_qlinear_bwd_prepared_kept(r, None, P, P, None, P, None, P, None, P, 1 << 30, None) == NULL  # ds wanted, X missing
    assert L.eqat_qlinear_bwd_prepared_kept(r, P, P, P, None, P, None, None, None, P, 1 << 30, None) == OK    # nothing wanted
    # the test aid
    assert L.eqat_unpack_state(r, 7, P, P, None, P, None) == SHAPE
    assert L.eqat_unpack_state(r, eq.STATE_PREPARED, None, P, None, P, None) == NULL
    assert L.eqat_unpack_state(r, eq.STATE_PREPARED, P, P, P, P, None) == NULL          # no clamp plane in a prepared layer
    assert L.eqat_unpack_state(ctypes.byref(d(act=eq.F32)), eq.STATE_FQ_KEPT, P, P, None, P, None) == DTYPE
    # several matrices in one launch
    two = (eq.Desc * 2)(d(), d(I=256, O=8))
    arr = (ctypes.c_void_p * 2)(P, P)
    sizes = (ctypes.c_size_t * 2)(1 << 30, 1 << 30)
    assert L.eqat_init_minmax_batched(0, two, arr, arr, arr, None) == SHAPE
    assert L.eqat_init_minmax_batched(9, two, arr, arr, arr, None) == SHAPE
    assert L.eqat_init_minmax_batched(2, None, arr, arr, arr, None) == NULL
    assert L.eqat_init_minmax_batched(2, two, None, arr, arr, None) == NULL
    assert L.eqat_init_minmax_batched(2, two, (ctypes.c_void_p * 2)(P, None), arr, arr, None) == NULL
    assert L.eqat_pack_batched(2, two, arr, arr, arr, (ctypes.c_void_p * 2)(P, P + 4), arr, None) == ALIGN
    assert L.eqat_pack_batched(2, (eq.Desc * 2)(d(), d(bits=3)), arr, arr, arr, arr, arr, None) == BITS
    assert L.eqat_pack_batched(2, (eq.Desc * 2)(d(), d(w=eq.F32)), arr, arr, arr, arr, arr, None) == DTYPE
    assert L.eqat_pack_batched(2, (eq.Desc * 2)(d(), d(group=48)), arr, arr, arr, arr, arr, None) == GROUP
    assert L.eqat_fq_quantize_batched(2, two, arr, arr, arr, arr, (ctypes.c_size_t * 2)(1 << 30, 16), None) == WORKSPACE
    assert L.eqat_fq_quantize_batched(2, two, arr, arr, arr, arr, None, None) == NULL
    assert L.eqat_fq_quantize_batched(2, (eq.Desc * 2)(d(act=eq.F32, w=eq.F32), d(act=eq.F32, w=eq.F32)), arr, arr, arr, arr, sizes, None) == OK
    assert L.eqat_fq_linear_fwd_kept(r, P, P, P, P, P, P, ws_need - 1, None) == WORKSPACE
    assert L.eqat_fq_linear_fwd_kept(r, P, P, P, P, None, P, ws_need, None) == NULL
    # descriptor errors win over everything else
    bad = d(bits=9)
    assert L.eqat_fq_linear_fwd(ctypes.byref(bad), None, None, None, None, None, None, 0, None) == BITS
    assert L.eqat_pack(ctypes.byref(d(group=50)), P, P, P, P, P, None) == GROUP


def test_every_kernel_class_has_a_name():
    L = eq.lib()
    names = [L.eqat_profile_kernel_name(k) for k in range(L.eqat_profile_kernels())]
    assert all(n and n != b"?" for n in names) and len(set(names)) == len(names)
    assert L.eqat_profile_kernel_name(len(names)) == b"?"


def test_step_glue_errors_come_back_before_any_launch():
    L = eq.lib()
    need = L.eqat_recon_loss_workspace_bytes()
    assert 0 < need <= 1 << 16
    assert L.eqat_recon_loss(0, eq.BF16, P, P, P, P, P, need, None) == SHAPE
    assert L.eqat_recon_loss(64, 5, P, P, P, P, P, need, None) == DTYPE
    assert L.eqat_recon_loss(64, eq.F32, None, P, P, P, P, need, None) == NULL
    assert L.eqat_recon_loss(64, eq.F32, P, P, None, P, P, need, None) == NULL
    assert L.eqat_recon_loss(64, eq.F32, P, P + 4, P, P, P, need, None) == ALIGN
    assert L.eqat_recon_loss(64, eq.F32, P, P, P, None, P, need - 1, None) == WORKSPACE
    assert L.eqat_recon_loss(64, eq.F32, P, P, P, None, None, need, None) == WORKSPACE
    r = ctypes.byref(d())
    ok = eq.AdamW(2e-5, 1e-4, 0.9, 0.999, 1e-8, 0.0, 0.0, 1)
    HYPER = eq.STATUS_NAMES.index("EQAT_ERR_HYPER")
    for bad in (eq.AdamW(2e-5, 1e-4, 1.0, 0.999, 1e-8, 0, 0, 1), eq.AdamW(2e-5, 1e-4, 0.9, -0.1, 1e-8, 0, 0, 1),
                eq.AdamW(2e-5, 1e-4, 0.9, 0.999, -1.0, 0, 0, 1), eq.AdamW(2e-5, 1e-4, 0.9, 0.999, 1e-8, 0, 0, 0),
                eq.AdamW(2e-5, 1e-4, float("nan"), 0.999, 1e-8, 0, 0, 1)):
        assert L.eqat_block_ap_update(r, ctypes.byref(bad), *([P] * 12), None) == HYPER
    assert L.eqat_block_ap_update(r, None, *([P] * 12), None) == NULL
    # a parameter that is given needs its gradient and both moments: W, s, z, dW, ds, dz, mW, vW, ms, vs, mz, vz
    assert L.eqat_block_ap_update(r, ctypes.byref(ok), P, None, None, None, None, None, P, P, None, None, None, None, None) == NULL
    assert L.eqat_block_ap_update(r, ctypes.byref(ok), None, P, None, None, P, None, None, None, P, None, None, None, None) == NULL
    assert L.eqat_block_ap_update(r, ctypes.byref(ok), None, None, P, None, None, P, None, None, None, None, P + 8, P, None) == ALIGN
    assert L.eqat_block_ap_update(ctypes.byref(d(bits=7)), ctypes.byref(ok), *([None] * 12), None) == BITS
    # nothing to update: fine, and nothing is launched
    assert L.eqat_block_ap_update(r, ctypes.byref(ok), *([None] * 12), None) == OK


def test_nothing_to_do_returns_ok_without_a_device():
    L = eq.lib()
    desc = d(T=0)
    r = ctypes.byref(desc)
    big = 1 << 30
    assert L.eqat_fq_linear_fwd(r, None, P, P, P, None, P, big, None) == OK          # T = 0: nothing to compute
    assert L.eqat_qlinear_fwd(r, None, P, P, P, None, P, big, None) == OK
    full = d()
    assert L.eqat_fq_linear_bwd(ctypes.byref(full), P, P, P, P, P, None, None, None, None, P, big, None) == OK   # no output wanted
    assert L.eqat_qlinear_bwd(ctypes.byref(full), P, P, P, P, P, None, None, P, big, None) == OK


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(eq, "_lib", None)
    monkeypatch.setattr(eq, "LIB_PATH", str(tmp_path / "libeqat.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        eq.lib()
