#!/usr/bin/env python3
"""Benchmark of the EfficientQAT quantized-linear hot path on one MI355X.

One "step" = one Block-AP pass (eqat_fq_linear_fwd + eqat_fq_linear_bwd with dX, dW, ds, dz) over the
seven linears of a Llama-2-7B-shaped decoder block, 8192 tokens, 2-bit codes, group 64, bf16 operands
(the configuration the headline metric is quoted on).  Inputs are synthetic, seeded, generated on the
device before the timed region; outputs and workspaces are pre-allocated.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline        the dominant kernel of the step against the bf16 MFMA peak (HIP events inside the library), and against
                  the rate a bare MFMA loop reaches on this chip in this run (measured_peaks),
  measured_peaks  a loop of nothing but MFMAs (zeros and random operands) and a plain device copy, timed in this run,
  cpu_baseline    the fp64 CPU oracle timed on a bounded sample of the same workload,
  rows            the other rows of the hot path and the other configurations, measured in the same run: E2E-QP on the
                  7B block; Block-AP, pack and E2E-QP on the 13B block (3 bit, group 128) and on the 70B block; pack, init,
                  loss, update (GB/s against the HBM peak and the measured copy rate); the few-token forward.
Step times: `value` / `ms_per_step` are the wall-clock mean over exactly --steps steps between two synchronisations;
`ms_per_step_median` / `_min` come from HIP events recorded between the steps on the stream the kernels run on.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
COPY_CALIBRATION_BYTES = 1 << 30


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=25)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama2_7b_block_ap_w2g64")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-rows", action="store_true", help="skip the rows beside the headline step")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a few 1 GiB device copies: the reference reading for the FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


def time_steps(torch, fn, steps, warmup):
    """`warmup` untimed calls of fn, then exactly `steps` timed ones between two synchronisations (wall clock), with a HIP
    event recorded on the current stream (the one the library launches on) before every step and after the last."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    for i in range(steps):
        ev[i].record()
        fn()
    ev[steps].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    return {"mean_ms": 1e3 * wall / steps, "median_ms": per[len(per) // 2], "min_ms": per[0]}


def profile_kernels(torch, eq, fn, steps):
    """Average launch duration of every kernel class of the library over `steps` calls of fn (HIP events inside the
    library, on the stream each kernel runs on; they cost a little, so step times are taken without them)."""
    eq.eqat_profile_start()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return eq.eqat_profile_stop()


def step_row(torch, eq, fn, flops, tokens, flop_per_launch, args, peaks):
    """One fwd+bwd step of a block: step time (mean / median / min), TFLOP/s, and the three GEMM kernels per launch."""
    t = time_steps(torch, fn, args.steps, 2)
    prof = profile_kernels(torch, eq, fn, max(5, args.steps // 2))
    tf = flops / (t["mean_ms"] * 1e-3) / 1e12
    row = {"tokens": tokens, "ms_per_step": round(t["mean_ms"], 4), "ms_per_step_median": round(t["median_ms"], 4),
           "ms_per_step_min": round(t["min_ms"], 4), "tflops": round(tf, 2),
           "tflops_at_median": round(flops / (t["median_ms"] * 1e-3) / 1e12, 2),
           "pct_of_bf16_mfma_peak": round(100 * tf / PEAK_BF16_TFLOPS, 2),
           "frac_of_measured_mfma_peak": frac_measured(tf, peaks),
           "tokens_per_s_per_layer": round(tokens / (t["mean_ms"] * 1e-3), 1),
           "kernels": kernel_table(prof, flop_per_launch, peaks)}
    return row


def frac_measured(tflops, peaks):
    m = peaks.get("mfma_bf16_random_operands_tflops") if peaks else None
    return round(tflops / m, 4) if m else None


def kernel_table(prof, flop_per_launch, peaks):
    out = {}
    for k, (ms, n) in prof.items():
        out[k] = {"launches": n, "avg_ms": round(ms / n, 4)}
        if k.startswith("gemm_"):
            tf = flop_per_launch / (ms / n * 1e-3) / 1e12
            out[k].update({"tflops": round(tf, 2), "frac": round(tf / PEAK_BF16_TFLOPS, 4),
                           "frac_of_measured_peak": frac_measured(tf, peaks)})
    return out


def peaks_lib():
    """The bench-only kernels (MFMA loop, copy, read): a library of their own, not part of libeqat.so."""
    import ctypes
    path = os.path.join(ROOT, "paper_2407_11062_amd", "libeqat_peaks.so")
    if not os.path.exists(path):
        return None
    L = ctypes.CDLL(path)
    vp = ctypes.c_void_p
    L.eqat_peak_mfma_flop.restype = ctypes.c_double
    L.eqat_peak_mfma_flop.argtypes = [ctypes.c_int, ctypes.c_int]
    L.eqat_peak_mfma_loop.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, vp, vp]
    L.eqat_peak_mfma16_flop.restype = ctypes.c_double
    L.eqat_peak_mfma16_flop.argtypes = [ctypes.c_int, ctypes.c_int]
    L.eqat_peak_mfma16_loop.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, vp, vp]
    L.eqat_peak_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    L.eqat_peak_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    return L


def measured_peaks(torch, dev, args):
    """What this chip gives, in this run: (a) a loop of nothing but v_mfma_f32_32x32x16_bf16, and one of nothing but
    v_mfma_f32_16x16x32_bf16 (the GEMM kernels use both shapes), two waves per SIMD on all compute units, on all-zero and
    on random bf16 operands (the clock the chip holds depends on the bits it multiplies); the better of the two shapes is
    the reference of every frac_of_measured_peak;
    (b) a plain copy kernel and the runtime's device copy on a 1 GiB buffer.  Bench-only kernels (libeqat_peaks.so)."""
    import ctypes
    L = peaks_lib()
    if L is None:
        return {"error": "libeqat_peaks.so not built"}
    vp = ctypes.c_void_p
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    groups, iters = cus, 20000                      # one workgroup of 8 waves per compute unit; about 1 ms per launch
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    out = {"compute_units": cus}
    stream = lambda: vp(torch.cuda.current_stream().cuda_stream)
    for name, data in (("zero", torch.zeros(1 << 20, dtype=torch.bfloat16, device=dev)),
                       ("random", torch.randn(1 << 20, device=dev).bfloat16())):
        def run():
            rc = L.eqat_peak_mfma_loop(vp(data.data_ptr()), data.numel() * 2, groups, iters, vp(sink.data_ptr()), stream())
            assert rc == 0

        def run16():
            rc = L.eqat_peak_mfma16_loop(vp(data.data_ptr()), data.numel() * 2, groups, iters, vp(sink.data_ptr()), stream())
            assert rc == 0
        t = time_steps(torch, run, 20, 3)
        a32 = round(L.eqat_peak_mfma_flop(groups, iters) / (t["median_ms"] * 1e-3) / 1e12, 1)
        t = time_steps(torch, run16, 20, 3)
        a16 = round(L.eqat_peak_mfma16_flop(groups, iters) / (t["median_ms"] * 1e-3) / 1e12, 1)
        out[f"mfma_32x32x16_bf16_{name}_operands_tflops"] = a32
        out[f"mfma_16x16x32_bf16_{name}_operands_tflops"] = a16
        out[f"mfma_bf16_{name}_operands_tflops"] = max(a32, a16)
    nbytes = 1 << 30
    src = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 256)
    dst = torch.empty_like(src)

    def kcopy():
        assert L.eqat_peak_copy(vp(dst.data_ptr()), vp(src.data_ptr()), nbytes, stream()) == 0

    t = time_steps(torch, kcopy, 20, 3)
    out["copy_kernel_gbs"] = round(2.0 * nbytes / (t["median_ms"] * 1e-3) / 1e9, 1)      # bytes read + bytes written
    t = time_steps(torch, lambda: dst.copy_(src), 20, 3)
    out["runtime_copy_gbs"] = round(2.0 * nbytes / (t["median_ms"] * 1e-3) / 1e9, 1)
    out["copy_gbs"] = max(out["copy_kernel_gbs"], out["runtime_copy_gbs"])      # the reference of every frac_of_measured_copy
    rsink = torch.zeros(1, dtype=torch.int32, device=dev)
    t = time_steps(torch, lambda: L.eqat_peak_read(vp(src.data_ptr()), nbytes, vp(rsink.data_ptr()), stream()), 20, 3)
    out["read_kernel_gbs"] = round(nbytes / (t["median_ms"] * 1e-3) / 1e9, 1)              # bytes read only
    out["note"] = ("median of 20 launches by HIP events; copy rates count bytes read plus bytes written of a 1 GiB buffer; "
                   "published peaks: 2500 TFLOP/s dense bf16, 8000 GB/s")
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2
    import torch
    import paper_2407_11062_amd as eq
    from paper_2407_11062_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    eq.lib()   # fail loudly if the HIP library was not built
    dev = torch.device("cuda:0")
    if args.copy_calibration:
        src = torch.empty(COPY_CALIBRATION_BYTES, dtype=torch.uint8, device=dev).random_(0, 256)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": COPY_CALIBRATION_BYTES, "copies": 4}))
        return 0
    wl = synth.WORKLOADS[args.workload]
    T, bits, g = wl.tokens, wl.bits, wl.group
    adt = synth.torch_dtype(wl.act_dtype)
    layers = build_layers(torch, eq, synth, wl, dev)
    sum_io = sum(L["O"] * L["I"] for L in layers)
    flops_step = 6.0 * T * sum_io

    def block_ap_step():
        run_block_ap_step(eq, layers, bits, g)

    # the headline: W warm-up steps, then exactly K steps between two synchronisations
    t = time_steps(torch, block_ap_step, args.steps, args.warmup)
    prof = profile_kernels(torch, eq, block_ap_step, args.steps)
    peaks = measured_peaks(torch, dev, args)
    ms_step = t["mean_ms"]
    tflops = flops_step / (ms_step * 1e-3) / 1e12

    # dominant kernel of the step: all three GEMM kernels do 2*T*I*O flop per launch
    gemms = {k: v for k, v in prof.items() if k.startswith("gemm_")}
    dom = max(gemms, key=lambda k: gemms[k][0])
    dom_ms, dom_n = gemms[dom]
    flop_per_launch = 2.0 * T * sum_io / len(layers)          # mean over the seven shapes
    dom_tflops = flop_per_launch / (dom_ms / dom_n * 1e-3) / 1e12
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(args.workload, {}).get(dom)
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(dom_tflops, 2), "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(dom_tflops / PEAK_BF16_TFLOPS, 4),
                "measured_peak": peaks.get("mfma_bf16_random_operands_tflops"),
                "frac_of_measured_peak": frac_measured(dom_tflops, peaks),
                "traffic": traffic, "traffic_source": "profiles/hbm_traffic.json (rocprofv3 --pmc runs of this bench, committed)",
                "avg_launch_ms": round(dom_ms / dom_n, 4), "launches": dom_n,
                "flop_per_launch": flop_per_launch}
    kernels = kernel_table(prof, flop_per_launch, peaks)
    if "quantize" in prof:
        # W and (s, z) in; codes, clamp bit-plane and (s, zbar) pairs out
        # (one launch per step over all linears of the block)
        qb = sum_io * (2 + 8.0 / g + bits / 8 + 1.0 / 8 + 8.0 / g)
        gbs = qb / (prof["quantize"][0] / args.steps * 1e-3) / 1e9
        kernels["quantize"].update({"approx_gbs": round(gbs, 1), "frac_of_hbm_peak": round(gbs / PEAK_HBM_GBS, 4),
                                    "frac_of_measured_copy": round(gbs / peaks["copy_gbs"], 4) if peaks.get("copy_gbs") else None})

    result = {
        "metric": "quantized-linear fwd+bwd TFLOP/s (% bf16 MFMA peak) and tokens/s per layer",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "phase": "block_ap", "tokens": T, "bits": bits, "group": g,
                   "layers": [[L["name"], L["O"], L["I"]] for L in layers], "flop_per_step": flops_step},
        "ms_per_step_median": round(t["median_ms"], 4), "ms_per_step_min": round(t["min_ms"], 4),
        "value_at_median": round(flops_step / (t["median_ms"] * 1e-3) / 1e12, 2),
        "pct_of_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "frac_of_measured_mfma_peak": frac_measured(tflops, peaks),
        "tokens_per_s_per_layer": round(T / (ms_step * 1e-3), 1),
        "roofline": roofline, "measured_peaks": peaks, "kernels": kernels,
    }

    if not args.no_rows:
        result["rows"] = measure_other_rows(torch, eq, layers, bits, g, adt, dev, args, peaks)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(result))
    return 0


def build_layers(torch, eq, synth, wl, dev, w_dtype=None):
    """Seeded synthetic tensors, trained-state (s, z), preallocated outputs and workspaces for every linear of a workload.
    w_dtype: dtype of W and dW (default: the activation dtype)."""
    T, bits, g = wl.tokens, wl.bits, wl.group
    adt = synth.torch_dtype(wl.act_dtype)
    wdt = adt if w_dtype is None else w_dtype
    gen = torch.Generator(device=dev)

    def randn(shape, std, seed, dtype):
        gen.manual_seed(seed)
        t = torch.empty(shape, dtype=torch.float32, device=dev).normal_(0.0, 1.0, generator=gen)
        return (t * std).to(dtype) if std != 1.0 else t.to(dtype)

    layers = []
    for lin in wl.layers:
        O, I = lin.out_features, lin.in_features
        L = {"name": lin.name, "O": O, "I": I}
        L["W"] = randn((O, I), wl.w_std, synth.seed_of(wl.name, lin.name, "W"), wdt)
        L["X"] = randn((T, I), 1.0, synth.seed_of(wl.name, lin.name, "X"), adt)
        L["dY"] = randn((T, O), 1.0, synth.seed_of(wl.name, lin.name, "dY"), adt)
        s, z = eq.eqat_init_minmax(L["W"], bits, g)
        # move the fresh min/max state into a "trained" one so that the clamped branches run
        gen.manual_seed(synth.seed_of(wl.name, lin.name, "sz"))
        u = torch.empty_like(s).uniform_(0.7, 1.1, generator=gen)
        d = torch.randint(-1, 2, s.shape, generator=gen, device=dev).float()
        L["s"], L["z"] = (s * u).contiguous(), (z + d).clamp_(0, 2 ** bits - 1).contiguous()
        G = s.shape[1]
        L["Y"] = torch.empty((T, O), dtype=adt, device=dev)
        L["out"] = {"dX": torch.empty((T, I), dtype=adt, device=dev), "dW": torch.empty((O, I), dtype=wdt, device=dev),
                    "ds": torch.empty((O, G), dtype=torch.float32, device=dev),
                    "dz": torch.empty((O, G), dtype=torch.float32, device=dev)}
        dsc = eq.make_desc(T, I, O, bits, g, eq._dt(L["X"]), eq._dt(L["W"]))
        L["ws_f"] = eq.workspace(dsc, eq.OP_FQ_FWD, dev)
        L["ws_b"] = eq.workspace(dsc, eq.OP_FQ_BWD, dev)
        layers.append(L)
    return layers


def block_batch(eq, layers, bits, g, T):
    """Pointer arrays for the one-launch passes over all linears of the block."""
    descs = [eq.make_desc(T, L["I"], L["O"], bits, g, eq._dt(L["X"]), eq._dt(L["W"])) for L in layers]
    return eq.Batch(descs, W=[L["W"] for L in layers], s=[L["s"] for L in layers], z=[L["z"] for L in layers],
                    ws=[L["ws_b"] for L in layers])


def run_block_ap_step(eq, layers, bits, g, batch=None):
    # as a training step runs them: Eq.(1) of all linears of the block in ONE launch (W, s, z do not change inside a
    # step), kept in each linear's workspace for its forward and its backward
    if batch is None:
        batch = layers[0].get("batch")
        if batch is None:
            batch = layers[0]["batch"] = block_batch(eq, layers, bits, g, layers[0]["X"].shape[0])
    eq.eqat_fq_quantize_batched(batch)
    for L in layers:
        eq.eqat_fq_linear_fwd(L["X"], L["W"], L["s"], L["z"], bits, g, Y=L["Y"], ws=L["ws_b"], kept=True)
        eq.eqat_fq_linear_bwd(L["X"], L["W"], L["s"], L["z"], L["dY"], bits, g, out=L["out"], ws=L["ws_b"], kept=True)


def pack_block(torch, eq, layers, bits, g, T2, dev):
    """The block after Block-AP: packed codes and zero points of every linear, each prepared once for E2E-QP (Sec. 3.3
    freezes W_q in that phase, so the re-layout of the codes is no part of a training step), with views and workspaces
    for a step on the first T2 tokens of the block's activations."""
    packed = []
    for L in layers:
        Wp, zp = eq.eqat_pack(L["W"], L["s"], L["z"], bits, g)
        dsc = eq.make_desc(T2, L["I"], L["O"], bits, g, eq.BF16, eq.BF16)
        packed.append({"Wp": Wp, "zp": zp, "prep": eq.eqat_qlinear_prepare(Wp, zp, L["I"], bits, g),
                       "X": L["X"][:T2], "dY": L["dY"][:T2], "Y": L["Y"][:T2],
                       "out": {"dX": L["out"]["dX"][:T2], "ds": L["out"]["ds"]},
                       "ws_b": eq.workspace(dsc, eq.OP_QP_BWD, dev)})
    return packed


def run_e2e_step(eq, layers, packed, bits, g, zf=None, outs=None):
    """fwd + bwd (dX, ds; with float zero points zf also dz) of every linear on its prepared layer; the (s, z) pairs the
    forward made are kept for the backward (one pairing launch per linear and step)."""
    for k, (L, P) in enumerate(zip(layers, packed)):
        z = None if zf is None else zf[k]
        eq.eqat_qlinear_fwd_prepared(P["X"], P["prep"], L["s"], L["O"], bits, g, z=z, Y=P["Y"], ws=P["ws_b"], keep=True)
        eq.eqat_qlinear_bwd_prepared(P["X"], P["prep"], L["s"], P["dY"], L["I"], bits, g, z=z,
                                     want=("dX", "ds") if z is None else ("dX", "ds", "dz"),
                                     out=P["out"] if outs is None else outs[k], ws=P["ws_b"], kept=True)


def hbm_row(torch, eq, fn, nbytes, args, peaks):
    """A memory-bound pass: summed GPU time of the library's kernels inside fn (HIP events), bytes / time against the
    published HBM peak and against the copy kernel's rate of this run."""
    for _ in range(2):
        fn()
    torch.cuda.synchronize()
    eq.eqat_profile_start()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fn()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / args.steps
    prof = eq.eqat_profile_stop()
    gpu = sum(v[0] for v in prof.values()) * 1e-3 / args.steps
    gbs = nbytes / gpu / 1e9
    return {"kernel_ms": round(gpu * 1e3, 4), "wall_ms": round(wall * 1e3, 4), "gbs": round(gbs, 1),
            "frac_of_hbm_peak": round(gbs / PEAK_HBM_GBS, 4),
            "frac_of_measured_copy": round(gbs / peaks["copy_gbs"], 4) if peaks.get("copy_gbs") else None,
            "bytes": nbytes, "kernels_ms": {k: round(v[0] / args.steps, 4) for k, v in prof.items()}}


def config_rows(torch, eq, synth, dev, args, peaks, name, phases=("block_ap", "eqat_pack", "e2e_qp")):
    """Another BASELINE configuration (workload `name`), every phase it names: the Block-AP step, eqat_pack of the block
    and the E2E-QP step, each timed like the headline and with its GEMM kernels per launch."""
    wl = synth.WORKLOADS[name]
    layers = build_layers(torch, eq, synth, wl, dev)
    T, bits, g = wl.tokens, wl.bits, wl.group
    sum_io = sum(L["O"] * L["I"] for L in layers)
    fpl = 2.0 * T * sum_io / len(layers)
    out = {"tokens": T, "bits": bits, "group": g, "linears": len(layers)}
    if "block_ap" in phases:
        out["block_ap"] = step_row(torch, eq, lambda: run_block_ap_step(eq, layers, bits, g), 6.0 * T * sum_io, T, fpl, args, peaks)
    packed = pack_block(torch, eq, layers, bits, g, T, dev)
    if "eqat_pack" in phases:
        pb = eq.Batch(layers[0]["batch"].descs if "batch" in layers[0] else block_batch(eq, layers, bits, g, T).descs,
                      W=[L["W"] for L in layers], s=[L["s"] for L in layers], z=[L["z"] for L in layers],
                      Wpacked=[P["Wp"] for P in packed], zpacked=[P["zp"] for P in packed])

        def pack_all():
            eq.eqat_pack_batched(pb)
        out["eqat_pack"] = hbm_row(torch, eq, pack_all, sum_io * (2 + 8.0 / g + bits / 8.0 + bits / (8.0 * g)), args, peaks)
    if "e2e_qp" in phases:
        out["e2e_qp"] = step_row(torch, eq, lambda: run_e2e_step(eq, layers, packed, bits, g), 6.0 * T * sum_io, T, fpl, args, peaks)
    del layers, packed
    torch.cuda.empty_cache()
    return out


def measure_other_rows(torch, eq, layers, bits, g, adt, dev, args, peaks):
    """The other rows of the hot path on the headline block, and the other BASELINE configurations."""
    from paper_2407_11062_amd import synth
    T2 = 4096
    rows = {}
    packed = pack_block(torch, eq, layers, bits, g, T2, dev)
    sum_io = sum(L["O"] * L["I"] for L in layers)
    fl = 6.0 * T2 * sum_io
    fpl = 2.0 * T2 * sum_io / len(layers)
    # BASELINE configuration 3: E2E-QP on the 7B block, 4096 tokens
    rows["e2e_qp_fwd_bwd"] = step_row(torch, eq, lambda: run_e2e_step(eq, layers, packed, bits, g), fl, T2, fpl, args, peaks)
    # the same step with step sizes AND zero points trained (zero points kept in floating point, dz from the same epilogue)
    zf = [(L["z"].clamp(0, 2 ** bits - 1) + 0.25).contiguous() for L in layers]
    outz = [{"dX": P["out"]["dX"], "ds": P["out"]["ds"], "dz": torch.empty_like(L["s"])} for L, P in zip(layers, packed)]

    rows["e2e_qp_fwd_bwd_trained_s_z"] = step_row(torch, eq, lambda: run_e2e_step(eq, layers, packed, bits, g, zf, outz),
                                                  fl, T2, fpl, args, peaks)
    wbytes = 2 if adt == torch.bfloat16 else 4

    descs = block_batch(eq, layers, bits, g, T2).descs
    pb = eq.Batch(descs, W=[L["W"] for L in layers], s=[L["s"] for L in layers], z=[L["z"] for L in layers],
                  Wpacked=[P["Wp"] for P in packed], zpacked=[P["zp"] for P in packed])

    def pack_all():         # the seven matrices of the block in one launch
        eq.eqat_pack_batched(pb)

    b = sum_io * (wbytes + 8.0 / g + bits / 8.0 + bits / (8.0 * g))
    rows["eqat_pack"] = hbm_row(torch, eq, pack_all, b, args, peaks)
    sz = [(torch.empty_like(L["s"]), torch.empty_like(L["z"])) for L in layers]
    ib = eq.Batch(descs, W=[L["W"] for L in layers], s=[a for a, _ in sz], z=[c for _, c in sz])

    def init_all():
        eq.eqat_init_minmax_batched(ib)

    b = sum_io * (wbytes + 8.0 / g)
    rows["eqat_init_minmax"] = hbm_row(torch, eq, init_all, b, args, peaks)

    def pack_one_by_one():
        for L, P in zip(layers, packed):
            eq.eqat_pack(L["W"], L["s"], L["z"], bits, g, Wpacked=P["Wp"], zpacked=P["zp"])

    rows["eqat_pack_one_launch_per_matrix"] = hbm_row(torch, eq, pack_one_by_one, sum_io * (wbytes + 8.0 / g + bits / 8.0 + bits / (8.0 * g)), args, peaks)

    # The 7B matrices are 34-90 MB: each launch lasts 10-25 us, a good part of it ramp-up and the timing events
    # themselves.  The same two passes on the largest matrix of the 70B block (gate/up, 28672 x 8192 = 470 MB, two
    # buffers alternating so that nothing is served from the 256 MB last-level cache) show the kernels' streaming rate.
    O2, I2 = 28672, 8192
    big = []
    for k in range(2):
        W = torch.empty((O2, I2), dtype=adt, device=dev).normal_(0.0, 0.015)
        s2, z2 = eq.eqat_init_minmax(W, bits, g)
        Wp, zp = eq.eqat_pack(W, s2, z2, bits, g)
        big.append((W, s2, z2, Wp, zp))

    def pack_big():
        for W, s2, z2, Wp, zp in big:
            eq.eqat_pack(W, s2, z2, bits, g, Wpacked=Wp, zpacked=zp)

    def init_big():
        for W, s2, z2, Wp, zp in big:
            eq.eqat_init_minmax(W, bits, g, s=s2, z=z2)

    n2 = 2.0 * O2 * I2
    rows["eqat_pack_28672x8192"] = hbm_row(torch, eq, pack_big, n2 * (wbytes + 8.0 / g + bits / 8.0 + bits / (8.0 * g)), args, peaks)
    rows["eqat_init_minmax_28672x8192"] = hbm_row(torch, eq, init_big, n2 * (wbytes + 8.0 / g), args, peaks)
    del big
    rows["qlinear_fwd_1_token"] = decode_rows(torch, eq, bits, g, dev, args)

    # Block-AP step glue on the same block: reconstruction loss over the seven output tensors, then one AdamW launch
    # per linear over {W, s, z} fed by the gradients of the last backward (copies of the parameters, so that the rows
    # above keep their inputs).  Bytes per element: loss 3 x the activation size (Y, Yref in, dY out); update
    # p, g in + p out in the parameter's dtype and two fp32 moments in and out.
    asz = 2 if adt == torch.bfloat16 else 4
    refs = [(L["Y"], torch.randn_like(L["Y"]), torch.empty_like(L["Y"])) for L in layers]
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    lws = torch.empty(eq.lib().eqat_recon_loss_workspace_bytes(), dtype=torch.uint8, device=dev)

    def loss_all():
        for Y, R, dY in refs:
            eq.eqat_recon_loss(Y, R, loss=loss, dY=dY, ws=lws)

    rows["eqat_recon_loss"] = hbm_row(torch, eq, loss_all, 3.0 * asz * sum(Y.numel() for Y, _, _ in refs), args, peaks)
    del refs
    st = [{"W": L["W"].clone(), "s": L["s"].clone(), "z": L["z"].clone(),
           "mW": torch.zeros(L["W"].shape, dtype=torch.float32, device=dev),
           "vW": torch.zeros(L["W"].shape, dtype=torch.float32, device=dev),
           "ms": torch.zeros_like(L["s"]), "vs": torch.zeros_like(L["s"]),
           "mz": torch.zeros_like(L["s"]), "vz": torch.zeros_like(L["s"])} for L in layers]
    hyper = eq.AdamW(2e-5, 1e-4, 0.9, 0.999, 1e-8, 0.0, 0.0, 1)      # Sec. 4.1: learning rates at 2 bit

    def update_all():
        for L, S in zip(layers, st):
            eq.eqat_block_ap_update(hyper, bits, g, W=S["W"], dW=L["out"]["dW"], mW=S["mW"], vW=S["vW"],
                                    s=S["s"], ds=L["out"]["ds"], ms=S["ms"], vs=S["vs"],
                                    z=S["z"], dz=L["out"]["dz"], mz=S["mz"], vz=S["vz"])

    n_sz = sum(L["s"].numel() for L in layers)
    rows["eqat_block_ap_update"] = hbm_row(torch, eq, update_all, sum_io * (3.0 * wbytes + 16.0) + 2 * n_sz * 28.0, args, peaks)
    del st
    rows["vendor_gemm_reference"] = vendor_gemm_rows(torch, layers, layers[0]["X"].shape[0], args)
    del packed, zf, outz, sz

    # BASELINE configuration 4: the 13B-shaped block, 3 bit, group 128, 4096 tokens: Block-AP, pack, E2E-QP
    rows["llama2_13b_w3g128"] = config_rows(torch, eq, synth, dev, args, peaks, "llama2_13b_w3g128")
    # BASELINE configuration 5: the 70B-shaped block (grouped-query attention: k, v 1024 x 8192), 2 bit, group 64,
    # 4096 tokens: both phases; and the Block-AP step with q|k|v and gate|up stacked along the output dimension
    rows["llama2_70b_w2g64"] = config_rows(torch, eq, synth, dev, args, peaks, "llama2_70b_w2g64")
    rows["llama2_70b_w2g64"]["block_ap_qkv_and_gate_up_stacked"] = config_rows(
        torch, eq, synth, dev, args, peaks, "llama2_70b_w2g64_fused", phases=("block_ap",))["block_ap"]
    # the headline block again with fp32 master weights, and with q|k|v and gate|up stacked (context: BASELINE's
    # configuration is the seven linears in bf16)
    rows["block_ap_llama2_7b_w2g64_fp32_weights"] = master_weight_row(torch, eq, dev, args, peaks, "llama2_7b_block_ap_w2g64")
    rows["block_ap_llama2_7b_w2g64_stacked"] = config_rows(
        torch, eq, synth, dev, args, peaks, "llama2_7b_block_ap_w2g64_fused", phases=("block_ap",))["block_ap"]
    return rows


def master_weight_row(torch, eq, dev, args, peaks, name):
    """The Block-AP step of workload `name` with W and dW in fp32 (master weights) and bf16 activations: the quantize pass
    reads twice the bytes and the dW epilogue reads and writes 4-byte weights; fwd and dX are unchanged."""
    from paper_2407_11062_amd import synth
    wl = synth.WORKLOADS[name]
    layers = build_layers(torch, eq, synth, wl, dev, w_dtype=torch.float32)
    sum_io = sum(L["O"] * L["I"] for L in layers)
    row = step_row(torch, eq, lambda: run_block_ap_step(eq, layers, wl.bits, wl.group), 6.0 * wl.tokens * sum_io, wl.tokens,
                   2.0 * wl.tokens * sum_io / len(layers), args, peaks)
    del layers
    torch.cuda.empty_cache()
    return row


def vendor_gemm_rows(torch, layers, T, args):
    """Context only, not part of the product path: the vendor GEMM library (torch.matmul, bf16) on the three plain GEMMs
    of the same seven linears with the weights already materialised in bf16: Y = X W^T (NT), dX = dY W (NN), dW = dY^T X (TN).
    It rebuilds no weights and has no Eq.(3)-(5) epilogue; it shows what this machine gives a tuned bf16 GEMM on this data."""
    out = {}
    ops = {"nt_like_fwd": lambda L: torch.matmul(L["X"], L["W"].t()),
           "nn_like_dx": lambda L: torch.matmul(L["dY"], L["W"]),
           "tn_like_dw": lambda L: torch.matmul(L["dY"].t(), L["X"])}
    flops = 2.0 * T * sum(L["O"] * L["I"] for L in layers)
    for name, fn in ops.items():
        for L in layers:
            fn(L)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            for L in layers:
                fn(L)
        e1.record(); torch.cuda.synchronize()
        out[name] = {"tflops": round(flops / (e0.elapsed_time(e1) * 1e-3 / args.steps) / 1e12, 1)}
    return out


# out_features x in_features of the paper's matrix-vector table (App. "Speedup with BitBLAS"), and the INT2 latencies it
# prints for an A100-80GB (context only: another machine, another kernel library)
DECODE_SHAPES = [(4096, 4096, 9), (11008, 4096, 21), (5120, 5120, 11), (13824, 5120, 26), (8192, 8192, 24), (28672, 8192, 67)]


def decode_rows(torch, eq, bits, g, dev, args):
    """eqat_qlinear_fwd on ONE token at the six shapes of the paper's matrix-vector table: HBM-bound, N/8 bytes per weight.
    Enough copies of each packed matrix are cycled through that nothing is served from the 256 MB last-level cache."""
    import ctypes
    out = {}
    L, vp = peaks_lib(), ctypes.c_void_p
    rsink = torch.zeros(1, dtype=torch.int32, device=dev)
    for O, I, a100_us in DECODE_SHAPES:
        G = I // g
        wb = O * I * bits // 8
        copies = max(2, min(160, int(640e6 // wb) + 1))
        gen = torch.Generator(device=dev); gen.manual_seed(O * 7 + I)
        Wps = [torch.randint(0, 256, (O, I * bits // 8), dtype=torch.uint8, device=dev, generator=gen) for _ in range(copies)]
        zp = torch.randint(0, 256, (O, 4 * ((G * bits + 31) // 32)), dtype=torch.uint8, device=dev, generator=gen)
        s = torch.empty((O, G), dtype=torch.float32, device=dev).uniform_(0.005, 0.02, generator=gen)
        x = torch.empty((1, I), dtype=torch.float32, device=dev).normal_(0, 1, generator=gen).bfloat16()
        y = torch.empty((1, O), dtype=torch.bfloat16, device=dev)
        ws = eq.workspace(eq.make_desc(1, I, O, bits, g, eq.BF16, eq.BF16), eq.OP_Q_FWD, dev)

        def run():
            for Wp in Wps:
                eq.eqat_qlinear_fwd(x, Wp, s, zp, bits, g, Y=y, ws=ws)

        # A launch lasts 5-25 us: host launch cost and per-kernel timing events would dominate, so one pass over all the
        # copies is captured in a HIP graph and replayed; the time per launch includes the gap between two kernels.
        def replay_us(fn):
            fn(); torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                fn()
            graph.replay(); torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 5
            e0.record()
            for _ in range(reps):
                graph.replay()
            e1.record(); torch.cuda.synchronize()
            del graph
            return e0.elapsed_time(e1) * 1e3 / (reps * copies)

        k_us = replay_us(run)
        nbytes = wb + O * G * 4 + O * 4 * ((G * bits + 31) // 32) + I * 2 + O * 2      # codes, s (fp32), z, x, y
        row = {"us_per_launch": round(k_us, 2), "gbs": round(nbytes / k_us / 1e3, 1),
               "frac_of_hbm_peak": round(nbytes / k_us / 1e3 / PEAK_HBM_GBS, 4), "bytes": nbytes,
               "paper_a100_int2_us": a100_us}
        del Wps
        if L is not None:
            # what a kernel that does nothing but read the same number of bytes once reaches, measured the same way
            rbytes = (nbytes + 15) // 16 * 16
            bufs = [torch.randint(0, 256, (rbytes,), dtype=torch.uint8, device=dev, generator=gen) for _ in range(copies)]

            def read_all():
                for b in bufs:
                    assert L.eqat_peak_read(vp(b.data_ptr()), rbytes, vp(rsink.data_ptr()), vp(torch.cuda.current_stream().cuda_stream)) == 0

            r_us = replay_us(read_all)
            row["read_only_kernel_us"] = round(r_us, 2)
            row["frac_of_read_only_kernel"] = round(r_us / k_us, 4)
            del bufs
        out[f"{O}x{I}"] = row
    return out


def cpu_baseline(wl):
    """The fp64 oracle on a bounded sample of the same workload: the q projection, a slab of token rows for
    Y and dX (against the full weight matrix) and a slab of output rows for dW/ds/dz (full token contraction)."""
    import torch
    import oracle
    from paper_2407_11062_amd import synth
    lin = wl.layers[0]
    O, I, T = lin.out_features, lin.in_features, wl.tokens
    n_tok, n_rows = T, O          # the whole projection: about 10 s on 16 host cores
    adt = synth.torch_dtype(wl.act_dtype)
    W = synth.normal((O, I), wl.w_std, 11, adt).float().numpy()
    Xs = synth.normal((n_tok, I), 1.0, 12, adt).float().numpy()
    dYs = synth.normal((n_tok, O), 1.0, 13, adt).float().numpy()
    Xf = synth.normal((T, I), 1.0, 14, adt).float().numpy()
    dYr = synth.normal((T, n_rows), 1.0, 15, adt).float().numpy()
    s, z = oracle.init_minmax(W, wl.bits, wl.group)
    t0 = time.perf_counter()
    oracle.fq_linear_fwd(Xs, W, s, z, wl.bits, wl.group)
    oracle.fq_linear_bwd(None, W, s, z, dYs, wl.bits, wl.group, want=("dX",))
    oracle.fq_linear_bwd(Xf, W[:n_rows], s[:n_rows], z[:n_rows], dYr, wl.bits, wl.group, want=("dW", "ds", "dz"))
    dt = time.perf_counter() - t0
    flops = 2.0 * n_tok * O * I * 2 + 2.0 * T * n_rows * I
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "seconds": round(dt, 3),
            "sample": f"q projection {O}x{I}, w{wl.bits}g{wl.group}: Y and dX for {n_tok} token rows against the full "
                      f"weight matrix, dW/ds/dz for {n_rows} output rows over all {T} tokens ({flops:.3e} flop, fp64)"}


if __name__ == "__main__":
    sys.exit(main())
