#!/usr/bin/env python3
"""Benchmark: one K-FAC step (curvature + inversion + precondition) of a BERT-Large pipeline stage.

A step is what one GPU of the paper's Chimera BERT-Large run has to do for
K-FAC (figure "chimera_timeline": 2 stages x 3 encoder blocks per GPU,
8 micro-batches of 32 x 128 tokens): for each of the 8 micro-batches one
curvature work item per factor (72 factors: A and B of 36 linears), then one
inversion per factor and one precondition per layer.  Inputs are synthetic
(seeded torch.randn on the device; GELU of it for the second feed-forward
linear's input; errors scaled by 1e-3) and are resident in HBM before the
timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_F32_MFMA_TFLOPS = 157.3  # MI355X published dense fp32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0  # MI355X published dense bf16 matrix peak
# HBM traffic of one curvature launch of the default workload, from the
# FETCH_SIZE / WRITE_SIZE counter runs summarised under profiles/ (None = not measured).
CURVATURE_TRAFFIC_BYTES_PER_LAUNCH = 12.57e9  # profiles/curvature_syrk_pmc.txt: 11.48 GB fetched + 1.09 GB written


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="workload id (4 = BERT-Large stage, the headline; 2, 3: one block; 5: bf16 stress block; "
                         "6, 7: BERT-Large-shaped block with 16384 / 65536 tokens)")
    ap.add_argument("--seed", type=int, default=221114133)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline", choices=["sample", "full"], default="sample",
                    help="sample: time the oracle on a bounded part of the workload (default, seconds); "
                         "full: run the oracle over the whole step (minutes)")
    ap.add_argument("--no-assignment", action="store_true",
                    help="skip the work-assignment block (it runs extra launches to time the chunks; leave them out of a "
                         "profile whose per-kernel averages should be those of the timed steps)")
    ap.add_argument("--streams", type=int, default=1, choices=[1, 2],
                    help="2: after the curvature, invert the small factors (and precondition the layers that only need "
                         "them) on one stream and the large factors on another (same results; default 1)")
    ap.add_argument("--curvature", choices=["f32", "split_bf16", "split_f16"], default="f32",
                    help="the float32 workloads' curvature on the 16-bit matrix core instead of the fp32 MFMA: split_bf16 = "
                         "KFAC_F32_BF16X3 (every value as three bfloat16 terms, six bf16 MFMA products per product), split_f16 = "
                         "KFAC_F32_F16X2 (every tensor scaled by a power of two, every value as two float16 terms, three f16 MFMA "
                         "products per product); fp32 accumulation in both; the default line reports both variants' curvature "
                         "times in blocks of their own either way")
    ap.add_argument("--precondition", choices=["f32", "split_f16"], default="f32",
                    help="split_f16: the precondition with its operands as two float16 terms on the f16 MFMA "
                         "(kfac_precondition_grouped_f16x2) instead of the fp32 MFMA; the default line reports this variant's "
                         "time in a block of its own either way")
    ap.add_argument("--phase", choices=["all", "curvature", "inversion", "precondition"], default="all",
                    help="for profiling: after one full untimed step, time only this phase (prints a short JSON "
                         "line that is not the benchmark line)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run plain 1 GiB device copies (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the K-FAC work; run it with --gpus 1 "
              "(this build has no multi-GPU path)", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2211_14133_amd import binding, synth

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU: there is no CPU fallback")
    lib = binding.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)  # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": src.numel() * 4, "copies": 3}))
        return
    cfg = synth.CONFIGS[args.config]
    bf16 = bool(cfg["bf16"])  # activations / errors in bfloat16 (the stress workload); everything else fp32
    in_dtype = binding.KFAC_BF16 if bf16 else binding.KFAC_F32
    split = args.curvature != "f32"
    products = 6.0 if args.curvature == "split_bf16" else 3.0  # 16-bit MFMA products per product of two float32 values
    if split:
        if bf16:
            raise SystemExit("--curvature %s is a mode for the float32 workloads" % args.curvature)
        in_dtype = binding.KFAC_F32_BF16X3 if args.curvature == "split_bf16" else binding.KFAC_F32_F16X2
    tokens, n_micro, blocks = cfg["tokens"], cfg["n_micro"], cfg["blocks"]
    damping = synth.DAMPING
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed)

    # ------------------------------------------------------------------ inputs
    layers = []  # (d_in, d_out)
    xs = [[] for _ in range(n_micro)]  # per micro-batch: list of [tokens, d] inputs, A then B per layer
    facs, invs, grads, outs = [], [], [], []
    for b in range(blocks):
        for (name, d_in, d_out, gelu) in cfg["layers"]:
            layers.append((d_in, d_out))
            g = torch.zeros(d_out, d_in, device=dev)
            for m in range(n_micro):
                x = torch.randn(tokens, d_in, device=dev, generator=gen)
                if gelu:
                    x = torch.nn.functional.gelu(x)
                e = torch.randn(tokens, d_out, device=dev, generator=gen) * 1e-3
                if bf16:
                    x, e = x.to(torch.bfloat16), e.to(torch.bfloat16)
                xs[m].append(x)
                xs[m].append(e)
                g.addmm_(e.float().t(), x.float(), alpha=1.0 / (tokens * n_micro))
            grads.append(g)
            outs.append(torch.empty_like(g))
            facs.append(torch.empty(d_in, d_in, device=dev))
            facs.append(torch.empty(d_out, d_out, device=dev))
            invs.append(torch.empty(d_in, d_in, device=dev))
            invs.append(torch.empty(d_out, d_out, device=dev))
    a_invs, b_invs = invs[0::2], invs[1::2]
    infos = torch.zeros(len(facs), dtype=torch.int32, device=dev)

    # ---------------------------------------------- marshal once, outside the loop
    curv_items = [binding._curv_items(xs[m], facs) for m in range(n_micro)]
    inv_items = binding._inv_items(facs, invs, infos)
    prec_items = binding._prec_items(b_invs, a_invs, grads, outs)
    nfac, nlay = len(facs), len(grads)
    prec_split = args.precondition == "split_f16"
    if prec_split and args.streams == 2:
        raise SystemExit("--precondition split_f16 is measured on one stream")
    prec_call = lib.kfac_precondition_grouped_f16x2 if prec_split else lib.kfac_precondition_grouped
    prec_ws = lib.kfac_precondition_grouped_f16x2_workspace if prec_split else lib.kfac_precondition_grouped_workspace
    ws_bytes = max(lib.kfac_curvature_grouped_workspace(curv_items[0], nfac, in_dtype),
                   lib.kfac_invert_batched_workspace(inv_items, nfac),
                   prec_ws(prec_items, nlay))
    ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device=dev)
    ws_ptr = (ws.data_ptr() + 255) // 256 * 256
    import ctypes

    wsp = ctypes.c_void_p(ws_ptr)
    stream = torch.cuda.current_stream()
    sp = ctypes.c_void_p(stream.cuda_stream)
    alpha = 1.0 / (tokens * n_micro)

    def check(st):
        if st != 0:
            raise RuntimeError("kfac call failed: %s" % lib.kfac_status_string(st).decode())

    # ---- optional two-stream split of inversion + precondition (small factors / large factors)
    if args.streams == 2:
        dsmall = min(f.shape[0] for f in facs)
        small = [i for i, f in enumerate(facs) if f.shape[0] == dsmall]
        large = [i for i, f in enumerate(facs) if f.shape[0] != dsmall]
        lay_small = [l for l, (di, do) in enumerate(layers) if di == dsmall and do == dsmall]
        lay_rest = [l for l in range(nlay) if l not in lay_small]
        sel = lambda seq, idx: [seq[i] for i in idx]  # noqa: E731
        inv_s = binding._inv_items(sel(facs, small), sel(invs, small), infos[:len(small)])
        inv_l = binding._inv_items(sel(facs, large), sel(invs, large), infos[len(small):])
        prec_s = binding._prec_items(sel(b_invs, lay_small), sel(a_invs, lay_small), sel(grads, lay_small), sel(outs, lay_small))
        prec_r = binding._prec_items(sel(b_invs, lay_rest), sel(a_invs, lay_rest), sel(grads, lay_rest), sel(outs, lay_rest))
        ws2_bytes = lib.kfac_invert_batched_workspace(inv_l, len(large))
        ws2 = torch.empty(ws2_bytes + 256, dtype=torch.uint8, device=dev)
        ws2p = ctypes.c_void_p((ws2.data_ptr() + 255) // 256 * 256)
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        s1p, s2p = ctypes.c_void_p(s1.cuda_stream), ctypes.c_void_p(s2.cuda_stream)
        ev_fork, ev_j1, ev_j2 = torch.cuda.Event(), torch.cuda.Event(), torch.cuda.Event()

        def invert_and_precondition_two_streams():
            ev_fork.record(stream)
            s1.wait_event(ev_fork)
            s2.wait_event(ev_fork)
            check(lib.kfac_invert_batched(inv_s, len(small), damping, wsp, ws_bytes, s1p))
            check(lib.kfac_precondition_grouped(prec_s, len(lay_small), wsp, ws_bytes, s1p))
            check(lib.kfac_invert_batched(inv_l, len(large), damping, ws2p, ws2_bytes, s2p))
            ev_j1.record(s1)
            ev_j2.record(s2)
            stream.wait_event(ev_j1)
            stream.wait_event(ev_j2)
            check(lib.kfac_precondition_grouped(prec_r, len(lay_rest), wsp, ws_bytes, sp))

    def step(events=None):
        if events is not None:
            events["t0"].record(stream)
        for m in range(n_micro):
            if events is not None:
                events["c0"][m].record(stream)
            check(lib.kfac_curvature_grouped(curv_items[m], nfac, in_dtype, alpha,
                                             0.0 if m == 0 else 1.0, wsp, ws_bytes, sp))
            if events is not None:
                events["c1"][m].record(stream)
        if args.streams == 2:
            invert_and_precondition_two_streams()
            if events is not None:
                events["t2"].record(stream)  # (the two phases overlap: only their sum is meaningful)
                events["t3"].record(stream)
            return
        check(lib.kfac_invert_batched(inv_items, nfac, damping, wsp, ws_bytes, sp))
        if events is not None:
            events["t2"].record(stream)
        check(prec_call(prec_items, nlay, wsp, ws_bytes, sp))
        if events is not None:
            events["t3"].record(stream)

    def phase_only(which):
        if which == "curvature":
            for m in range(n_micro):
                check(lib.kfac_curvature_grouped(curv_items[m], nfac, in_dtype, alpha,
                                                 0.0 if m == 0 else 1.0, wsp, ws_bytes, sp))
        elif which == "inversion":
            check(lib.kfac_invert_batched(inv_items, nfac, damping, wsp, ws_bytes, sp))
        else:
            check(prec_call(prec_items, nlay, wsp, ws_bytes, sp))

    if args.phase != "all":
        step()  # every buffer the phase reads holds real data
        for _ in range(args.warmup):
            phase_only(args.phase)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.steps):
            phase_only(args.phase)
        e1.record(stream)
        torch.cuda.synchronize()
        print(json.dumps({"phase": args.phase, "workload": cfg["name"], "repetitions": args.steps,
                          "ms": round(e0.elapsed_time(e1) / args.steps, 4)}))
        return

    def new_events():
        ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731
        return {"t0": ev(), "t2": ev(), "t3": ev(), "c0": [ev() for _ in range(n_micro)],
                "c1": [ev() for _ in range(n_micro)]}

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    all_events = [new_events() for _ in range(args.steps)]
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(all_events[i])
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    ms_per_step = (t_end - t_start) * 1e3 / args.steps
    if int(infos.abs().max().item()) != 0:
        raise RuntimeError("an inversion reported failure: %s" % infos.tolist())

    curv_launch_ms, per_step = [], {"curvature": [], "inversion": [], "precondition": [], "step": []}
    for ev in all_events:
        for m in range(n_micro):
            curv_launch_ms.append(ev["c0"][m].elapsed_time(ev["c1"][m]))
        per_step["curvature"].append(ev["t0"].elapsed_time(ev["c1"][n_micro - 1]))
        per_step["inversion"].append(ev["c1"][n_micro - 1].elapsed_time(ev["t2"]))
        per_step["precondition"].append(ev["t2"].elapsed_time(ev["t3"]))
        per_step["step"].append(ev["t0"].elapsed_time(ev["t3"]))
    curv_ms = sum(per_step["curvature"]) / args.steps
    inv_ms = sum(per_step["inversion"]) / args.steps
    prec_ms = sum(per_step["precondition"]) / args.steps

    def median(v):
        v = sorted(v)
        return 0.5 * (v[(len(v) - 1) // 2] + v[len(v) // 2])

    launch_ms = sum(curv_launch_ms) / len(curv_launch_ms)

    # ------------------------------------------------- algorithmic work (useful flops)
    f_curv_launch = sum(tokens * d * (d + 1) for (di, do) in layers for d in (di, do))
    f_curv = f_curv_launch * n_micro
    f_inv = sum(d ** 3 for (di, do) in layers for d in (di, do))
    f_prec = sum(2 * do * di * (di + do) for (di, do) in layers)
    f_total = f_curv + f_inv + f_prec
    in_bytes = 2 if bf16 else 4
    b_curv = sum(n_micro * tokens * d * in_bytes + (2 * n_micro - 1) * 4 * d * d for (di, do) in layers for d in (di, do))
    b_inv = sum(2 * 4 * d * d for (di, do) in layers for d in (di, do))
    b_prec = sum(4 * (do * do + di * di + 2 * do * di) for (di, do) in layers)
    achieved = f_curv_launch / (launch_ms * 1e-3) / 1e12
    peak = PEAK_BF16_MFMA_TFLOPS if (bf16 or split) else PEAK_F32_MFMA_TFLOPS
    if split:
        achieved *= products  # 16-bit MFMA products per product of two float32 values; the pre-passes are part of the launch

    # what the matrix cores sustain on this chip with nothing else in the way (register-only MFMA loop)
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    probe_flops = ctypes.c_double(0.0)
    probe_ms = []
    for _ in range(4):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        check(lib.kfac_mfma_probe(binding.KFAC_BF16 if split else in_dtype, 4000, ctypes.c_void_p(sink.data_ptr()),
                                  ctypes.byref(probe_flops), sp))
        e1.record(stream)
        torch.cuda.synchronize()
        probe_ms.append(e0.elapsed_time(e1))
    measured_peak = probe_flops.value / (min(probe_ms[1:]) * 1e-3) / 1e12
    # the same loop on operands with random sign and mantissa bits: the chip lowers its clock under the power the
    # matrix cores then draw, so this, not the constant-operand figure, is what real data can reach
    probe_ms = []
    for _ in range(4):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        check(lib.kfac_mfma_probe_data(binding.KFAC_BF16 if split else in_dtype, 1, 4000, ctypes.c_void_p(sink.data_ptr()),
                                       ctypes.byref(probe_flops), sp))
        e1.record(stream)
        torch.cuda.synchronize()
        probe_ms.append(e0.elapsed_time(e1))
    measured_peak_random = probe_flops.value / (min(probe_ms[1:]) * 1e-3) / 1e12

    result = {
        "metric": "kfac_step_ms_%s (curvature + inversion + precondition)" % cfg["name"].replace("-", "_"),
        "value": round(ms_per_step, 3),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if bf16 else ({"split_bf16": "f32 as 3 x bf16", "split_f16": "f32 as 2 x f16"}[args.curvature] if split else "f32"),
        "data": "synthetic",
        "config": {
            "workload": "%s: %d blocks x %d linears, %d micro-batches x %d tokens, %s, damping %g"
                        % (cfg["name"], blocks, len(cfg["layers"]), n_micro, tokens,
                           "bf16 activations and errors, fp32 factors / inverses / gradients" if bf16 else "fp32", damping),
            "factors": nfac,
            "layers": nlay,
            "streams": args.streams,
        },
        "useful_tflops": round(f_total / (ms_per_step * 1e-3) / 1e12, 2),
        "phases_ms": {"curvature": round(curv_ms, 3), "inversion": round(inv_ms, 3), "precondition": round(prec_ms, 3)},
        "phases_ms_median": {k2: round(median(v), 3) for k2, v in per_step.items()},
        "phases_ms_min": {k2: round(min(v), 3) for k2, v in per_step.items()},
        # minimum bytes each phase has to move (inputs once, factors / inverses / gradients read and written once)
        "phases_min_traffic_gbps": {
            "curvature": round(b_curv / (curv_ms * 1e-3) / 1e9, 1),
            "inversion": round(b_inv / (inv_ms * 1e-3) / 1e9, 1),
            "precondition": round(b_prec / (prec_ms * 1e-3) / 1e9, 1),
        },
        "phases_useful_tflops": {
            "curvature": round(f_curv / (curv_ms * 1e-3) / 1e12, 2),
            "inversion": round(f_inv / (inv_ms * 1e-3) / 1e12, 2),
            "precondition": round(f_prec / (prec_ms * 1e-3) / 1e12, 2),
        },
        # the curvature counted as a dense product (2 N d^2 per factor) instead of its triangle (N d (d+1))
        "curvature_dense_equivalent_tflops": round(
            sum(2 * tokens * d * d for (di, do) in layers for d in (di, do)) * n_micro / (curv_ms * 1e-3) / 1e12, 2),
        "roofline": {
            "kernel": "%s (one launch = all %d factors of the stage for one micro-batch)"
                      % ("curvature_syrk_bf16_256_rowmajor_kernel" if bf16 else
                         ({"split_bf16": "split3_pack_kernel + curvature_syrk_split3_256_kernel, 6 bf16 products per fp32 product",
                           "split_f16": "split2_amax_kernel + split2_pack_kernel + curvature_syrk_split2_256_kernel, "
                                        "3 f16 products per fp32 product"}[args.curvature]
                          if split else "curvature_syrk_kernel"), nfac),
            "bound": "mfma",
            "achieved": round(achieved, 2),
            "peak": peak,
            "unit": "TFLOP/s",
            "frac": round(achieved / peak, 4),
            "traffic": CURVATURE_TRAFFIC_BYTES_PER_LAUNCH if (args.config == 4 and not split) else None,
            "measured_mfma_peak": round(measured_peak, 1),
            "frac_of_measured_peak": round(achieved / measured_peak, 4),
            "measured_mfma_peak_random_operands": round(measured_peak_random, 1),
            "frac_of_measured_peak_random_operands": round(achieved / measured_peak_random, 4),
            "launch_ms": round(launch_ms, 4),
            "flops_per_launch": f_curv_launch,
        },
    }

    if not bf16 and not split:
        result["curvature_f32_as_3xbf16"] = split_curvature_variant(
            torch, binding, lib, check, xs, facs, n_micro, alpha, sp, stream, curv_ms, inv_ms, prec_ms, f_curv,
            binding.KFAC_F32_BF16X3)
        result["curvature_f32_as_2xf16"] = split_curvature_variant(
            torch, binding, lib, check, xs, facs, n_micro, alpha, sp, stream, curv_ms, inv_ms, prec_ms, f_curv,
            binding.KFAC_F32_F16X2)

    if not prec_split and args.streams == 1:
        result["precondition_f32_as_2xf16"] = split_precondition_variant(
            torch, lib, check, prec_items, outs, nlay, sp, stream, prec_ms, f_prec)

    if args.streams == 2:
        # the two phases overlap: report their sum, and none of the blocks that need them separately
        both = inv_ms + prec_ms
        result["phases_ms"] = {"curvature": round(curv_ms, 3), "inversion_plus_precondition": round(both, 3)}
        for key in ("phases_ms_median", "phases_ms_min", "phases_min_traffic_gbps", "phases_useful_tflops"):
            result.pop(key)
        result["inversion_plus_precondition_useful_tflops"] = round((f_inv + f_prec) / (both * 1e-3) / 1e12, 2)
        print(json.dumps(result))
        return

    # Section 3.3 of the paper with the measured K-FAC times.  T_f and T_b are NOT measured (no model is
    # run here): they are the stage's forward GEMM flops at the rate this engine reaches on the
    # precondition products, and twice that.
    f_fwd = sum(2 * tokens * di * do for (di, do) in layers)
    prec_ms_fp32 = prec_ms
    if prec_split:
        # the assumed forward / backward passes stay fp32 GEMMs: time the fp32 precondition for their rate
        need = lib.kfac_precondition_grouped_workspace(prec_items, nlay)
        if need > ws_bytes:
            raise RuntimeError("the workspace of the step is smaller than the fp32 precondition's")
        check(lib.kfac_precondition_grouped(prec_items, nlay, wsp, ws_bytes, sp))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(3):
            check(lib.kfac_precondition_grouped(prec_items, nlay, wsp, ws_bytes, sp))
        e1.record(stream)
        torch.cuda.synchronize()
        prec_ms_fp32 = e0.elapsed_time(e1) / 3
    t_f = f_fwd / (f_prec / (prec_ms_fp32 * 1e-3)) * 1e3
    t_b = 2.0 * t_f
    depth = 4
    c = n_micro + depth - 1
    model = binding.kfac_perf_model(c, c, t_f, t_b, n_micro, curv_ms / n_micro, inv_ms, prec_ms)
    result["pipefisher_model"] = {
        "assumed": "GPipe, depth %d, %d micro-batches (C_f = C_b = %d); T_f = forward GEMM flops of the stage / "
                   "measured rate of the fp32 precondition, T_b = 2 T_f (not measured)" % (depth, n_micro, c),
        "t_f_ms": round(t_f, 3), "t_b_ms": round(t_b, 3),
        "t_pipe_ms": round(model["t_pipe"], 3), "t_bubble_ms": round(model["t_bubble"], 3),
        "t_kfac_ms": round(model["t_kfac"], 3),
        "curvature_plus_inversion_over_bubble": round(model["ratio"], 3),
    }

    # Section 3.1 with measured durations: the work of the stage cut into chunks (one grouped curvature call per
    # micro-batch and side, every launch step of the inversion), each timed with HIP events, and assigned to the
    # bubbles of each GPipe stage under rules 1 - 3.  steps_per_refresh is the paper's refresh interval.
    if not args.no_assignment:
        result["pipefisher_assignment"] = work_assignment(
            binding, lib, check, xs, facs, invs, infos, ws, wsp, ws_bytes, sp, in_dtype, alpha, damping, nlay,
            n_micro, depth, t_f, t_b, prec_ms, step)

    if not args.no_cpu_baseline:
        if args.cpu_baseline == "full":
            result["cpu_baseline"] = cpu_baseline_full(xs, grads, layers, tokens, n_micro, damping)
        else:
            result["cpu_baseline"] = cpu_baseline(cfg, xs, grads, layers, tokens, n_micro, damping,
                                                  f_curv, f_inv, f_prec)
    print(json.dumps(result))


def split_curvature_variant(torch, binding, lib, check, xs, facs, n_micro, alpha, sp, stream, curv_ms, inv_ms, prec_ms, f_curv,
                            dt):
    """The curvature of the same step computed as KFAC_F32_BF16X3 (float32 values as three bfloat16 terms on the
    bf16 MFMA) or KFAC_F32_F16X2 (two float16 terms on the f16 MFMA), pre-passes included, timed with HIP events,
    and how far its factors are from the fp32 MFMA path's."""
    import ctypes

    bf = dt == binding.KFAC_F32_BF16X3
    products = 6 if bf else 3
    nfac = len(facs)
    items = [binding._curv_items(xs[m], facs) for m in range(n_micro)]
    need = lib.kfac_curvature_grouped_workspace(items[0], nfac, dt)
    ws = torch.empty(need + 256, dtype=torch.uint8, device=facs[0].device)
    wsp = ctypes.c_void_p((ws.data_ptr() + 255) // 256 * 256)
    biggest = max(range(nfac), key=lambda i: facs[i].shape[0])
    smallest = min(range(nfac), key=lambda i: facs[i].shape[0])
    ref = [f.clone() for f in facs]  # what the timed steps left: the fp32 MFMA path's factors

    def curvature():
        for m in range(n_micro):
            check(lib.kfac_curvature_grouped(items[m], nfac, dt, alpha, 0.0 if m == 0 else 1.0, wsp, need, sp))

    curvature()
    torch.cuda.synchronize()
    reps = 3
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        curvature()
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    diff = {i: float((facs[i].double() - ref[i].double()).norm() / ref[i].double().norm()) for i in (biggest, smallest)}
    for f, r in zip(facs, ref):  # leave the buffers as the timed steps left them
        f.copy_(r)
    return {
        "what": ("curvature of the same step with --curvature split_bf16 (KFAC_F32_BF16X3): pre-pass + bf16 MFMA kernel, "
                 "fp32 accumulation; not part of `value`") if bf else
                ("curvature of the same step with --curvature split_f16 (KFAC_F32_F16X2): largest-magnitude pass + pre-pass + "
                 "f16 MFMA kernel, fp32 accumulation; not part of `value`"),
        "curvature_ms": round(ms, 3),
        "launch_ms": round(ms / n_micro, 4),
        "speedup_over_fp32_mfma_curvature": round(curv_ms / ms, 3),
        "step_ms_with_it": round(ms + inv_ms + prec_ms, 3),
        "useful_tflops": round(f_curv / (ms * 1e-3) / 1e12, 2),
        "mfma_products_per_product": products,
        "mfma_16bit_tflops": round(products * f_curv / (ms * 1e-3) / 1e12, 1),
        "frac_of_16bit_mfma_peak": round(products * f_curv / (ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4),
        "rel_fro_difference_from_fp32_path": {"d=%d" % facs[i].shape[0]: float("%.3g" % diff[i]) for i in diff},
    }


def split_precondition_variant(torch, lib, check, prec_items, outs, nlay, sp, stream, prec_ms, f_prec):
    """The precondition of the same step with its operands as two float16 terms on the f16 MFMA
    (kfac_precondition_grouped_f16x2), timed with HIP events, and how far its result is from the fp32 MFMA path's."""
    import ctypes

    need = lib.kfac_precondition_grouped_f16x2_workspace(prec_items, nlay)
    ws = torch.empty(need + 256, dtype=torch.uint8, device=outs[0].device)
    wsp = ctypes.c_void_p((ws.data_ptr() + 255) // 256 * 256)
    ref = [o.clone() for o in outs]  # what the timed steps left
    check(lib.kfac_precondition_grouped_f16x2(prec_items, nlay, wsp, need, sp))
    torch.cuda.synchronize()
    reps = 5
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        check(lib.kfac_precondition_grouped_f16x2(prec_items, nlay, wsp, need, sp))
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    diff = max(float((o.double() - r.double()).norm() / r.double().norm()) for o, r in zip(outs, ref))
    # the same with the inverses' planes made once (they only change when the inverses are refreshed)
    pbytes = lib.kfac_precondition_f16x2_prepared_bytes(prec_items, nlay)
    prep = torch.empty(pbytes + 256, dtype=torch.uint8, device=outs[0].device)
    prepp = ctypes.c_void_p((prep.data_ptr() + 255) // 256 * 256)
    need2 = lib.kfac_precondition_grouped_f16x2_prepared_workspace(prec_items, nlay)
    e0.record(stream)
    check(lib.kfac_precondition_f16x2_prepare(prec_items, nlay, prepp, pbytes, sp))
    e1.record(stream)
    check(lib.kfac_precondition_grouped_f16x2_prepared(prec_items, nlay, prepp, pbytes, wsp, need2, sp))
    torch.cuda.synchronize()
    prepare_ms = e0.elapsed_time(e1)
    prepared_once = [o.clone() for o in outs]
    e0.record(stream)
    for _ in range(reps):
        check(lib.kfac_precondition_grouped_f16x2_prepared(prec_items, nlay, prepp, pbytes, wsp, need2, sp))
    e1.record(stream)
    torch.cuda.synchronize()
    ms_prepared = e0.elapsed_time(e1) / reps
    check(lib.kfac_precondition_grouped_f16x2(prec_items, nlay, wsp, need, sp))
    torch.cuda.synchronize()
    same = all(bool(torch.equal(o, r)) for o, r in zip(outs, prepared_once))
    for o, r in zip(outs, ref):
        o.copy_(r)
    return {
        "what": "precondition of the same step with --precondition split_f16 (kfac_precondition_grouped_f16x2): operands as two "
                "float16 terms, three f16 MFMA products per product, fp32 accumulation; not part of `value`",
        "precondition_ms": round(ms, 3),
        "speedup_over_fp32_mfma_precondition": round(prec_ms / ms, 3),
        "useful_tflops": round(f_prec / (ms * 1e-3) / 1e12, 2),
        "largest_rel_fro_difference_from_fp32_path": float("%.3g" % diff),
        "with_prepared_inverses": {
            "what": "kfac_precondition_f16x2_prepare once per refresh of the inverses, then "
                    "kfac_precondition_grouped_f16x2_prepared every step",
            "prepare_ms": round(prepare_ms, 3),
            "precondition_ms": round(ms_prepared, 3),
            "speedup_over_fp32_mfma_precondition": round(prec_ms / ms_prepared, 3),
            "same_bits_as_the_one_call_form": same,
        },
    }


def work_assignment(binding, lib, check, xs, facs, invs, infos, ws, wsp, ws_bytes, sp, in_dtype, alpha, damping, nlay,
                    n_micro, depth, t_f, t_b, prec_ms, step):
    from paper_2211_14133_amd import bubble_schedule as bs

    a_items = binding._curv_items(xs[0][0::2], facs[0::2])
    b_items = binding._curv_items(xs[0][1::2], facs[1::2])
    t_curv_a = bs.time_ms(lambda: check(lib.kfac_curvature_grouped(a_items, nlay, in_dtype, alpha, 0.0, wsp, ws_bytes, sp)))
    t_curv_b = bs.time_ms(lambda: check(lib.kfac_curvature_grouped(b_items, nlay, in_dtype, alpha, 0.0, wsp, ws_bytes, sp)))
    step()  # factors of the whole mini-batch again
    plan = binding.InvertPlan(facs, damping, invs, infos=infos, workspace=ws)
    chunk_ms = bs.measure_plan_steps(plan, reps=3)
    by_kind = {}
    for i, t in enumerate(chunk_ms):
        by_kind[plan.step_label(i)] = by_kind.get(plan.step_label(i), 0.0) + t
    refresh = []
    for stage in range(depth):
        tl = binding.kfac_gpipe_stage(stage, depth, n_micro, t_f, t_b)
        works = [bs.Work("A%d" % m, [None], [t_curv_a], release_ms=tl["forward_end"][m]) for m in range(n_micro)]
        works += [bs.Work("B%d" % m, [None], [t_curv_b], release_ms=tl["backward_end"][m]) for m in range(n_micro)]
        works.append(bs.Work("inversion", [None] * len(chunk_ms), chunk_ms, deps=list(range(2 * n_micro))))
        _, needed = bs.assign(tl, tl["t_step"] + prec_ms, works)
        refresh.append(needed)
    plan.close()
    return {
        "chunks": {"curvature_A_per_microbatch_ms": round(t_curv_a, 3), "curvature_B_per_microbatch_ms": round(t_curv_b, 3),
                   "inversion_steps": len(chunk_ms), "longest_inversion_step_ms": round(max(chunk_ms), 3)},
        "inversion_ms_by_kind_of_step": {k2: round(v, 3) for k2, v in by_kind.items()},
        "steps_per_refresh_by_gpipe_stage": refresh,
    }


def cpu_baseline(cfg, xs, grads, layers, tokens, n_micro, damping, f_curv, f_inv, f_prec):
    """Time the fp64 oracle, as it stands, on one layer of the workload and scale to a step."""
    from oracle import kfac_oracle as oracle

    # sample: every linear of the first two encoder blocks (or of the only one), micro-batch 0
    nl = len(cfg["layers"]) * min(2, cfg["blocks"])
    if cfg["bf16"]:
        nl = 4  # the attention linears only: the oracle needs minutes for one 8192-dimensional factor
    hx = [xs[0][2 * i].float().cpu().numpy() for i in range(nl)]
    he = [xs[0][2 * i + 1].float().cpu().numpy() for i in range(nl)]
    hg = [grads[i].cpu().numpy() for i in range(nl)]
    t0 = time.perf_counter()
    fa = [oracle.curvature_update(x, 1.0 / tokens, 0.0) for x in hx]
    fb = [oracle.curvature_update(e, 1.0 / tokens, 0.0) for e in he]
    t1 = time.perf_counter()
    ia = [oracle.invert(a, damping)[0] for a in fa]
    ib = [oracle.invert(b, damping)[0] for b in fb]
    t2 = time.perf_counter()
    for g, a_inv, b_inv in zip(hg, ia, ib):
        oracle.precondition(b_inv, g, a_inv)
    t3 = time.perf_counter()
    # the same sample through the HIP path, compared with what the oracle just computed
    import torch

    import paper_2211_14133_amd as k

    ga = [torch.empty(x.shape[1], x.shape[1], device="cuda") for x in hx]
    gb = [torch.empty(e.shape[1], e.shape[1], device="cuda") for e in he]
    k.kfac_curvature_grouped([xs[0][2 * i] for i in range(nl)] + [xs[0][2 * i + 1] for i in range(nl)], ga + gb, 1.0 / tokens, 0.0)
    gia, gib = [torch.empty_like(t) for t in ga], [torch.empty_like(t) for t in gb]
    k.kfac_invert_batched(ga + gb, damping, gia + gib)
    gp = [torch.empty_like(grads[i]) for i in range(nl)]
    k.kfac_precondition_grouped(gib, gia, [grads[i] for i in range(nl)], gp)
    torch.cuda.synchronize()
    worst = {"factor": 0.0, "inverse": 0.0, "preconditioned_gradient": 0.0}
    for i in range(nl):
        worst["factor"] = max(worst["factor"], oracle.rel_fro(ga[i].cpu().numpy(), fa[i]), oracle.rel_fro(gb[i].cpu().numpy(), fb[i]))
        worst["inverse"] = max(worst["inverse"], oracle.rel_fro(gia[i].cpu().numpy(), ia[i]), oracle.rel_fro(gib[i].cpu().numpy(), ib[i]))
        worst["preconditioned_gradient"] = max(worst["preconditioned_gradient"],
                                               oracle.rel_fro(gp[i].cpu().numpy(), oracle.precondition(ib[i], hg[i], ia[i])))
    s_curv = sum(tokens * (di * (di + 1) + do * (do + 1)) for di, do in layers[:nl])
    s_inv = sum(di ** 3 + do ** 3 for di, do in layers[:nl])
    s_prec = sum(2 * do * di * (di + do) for di, do in layers[:nl])
    est_ms = ((t1 - t0) * f_curv / s_curv + (t2 - t1) * f_inv / s_inv + (t3 - t2) * f_prec / s_prec) * 1e3
    return {
        "value": round(est_ms, 1),
        "unit": "ms",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": "fp64 oracle on the first %d linears of the stage, one micro-batch of %d tokens: curvature "
                  "%.2f s, inversion %.2f s, precondition %.2f s; each phase scaled by the step's useful flops "
                  "over the sample's" % (nl, tokens, t1 - t0, t2 - t1, t3 - t2),
        # worst relative Frobenius error of the HIP path against the oracle on that sample (gates: 1e-4 / 5e-3)
        "hip_vs_oracle_on_sample": {k2: float("%.3g" % v) for k2, v in worst.items()},
    }


def cpu_baseline_full(xs, grads, layers, tokens, n_micro, damping):
    """The fp64 oracle, as it stands, over the whole step: every factor from all micro-batches, every inverse,
    every preconditioned gradient (minutes; copies from the device are not counted)."""
    from oracle import kfac_oracle as oracle

    t_curv = t_inv = t_prec = 0.0
    for li in range(len(layers)):
        hx = [xs[m][2 * li].float().cpu().numpy() for m in range(n_micro)]
        he = [xs[m][2 * li + 1].float().cpu().numpy() for m in range(n_micro)]
        hg = grads[li].cpu().numpy()
        t0 = time.perf_counter()
        fa = fb = None
        for m in range(n_micro):
            fa = oracle.curvature_update(hx[m], 1.0 / (tokens * n_micro), 0.0 if m == 0 else 1.0, fa)
            fb = oracle.curvature_update(he[m], 1.0 / (tokens * n_micro), 0.0 if m == 0 else 1.0, fb)
        t1 = time.perf_counter()
        ia, ib = oracle.invert(fa, damping)[0], oracle.invert(fb, damping)[0]
        t2 = time.perf_counter()
        oracle.precondition(ib, hg, ia)
        t3 = time.perf_counter()
        t_curv, t_inv, t_prec = t_curv + (t1 - t0), t_inv + (t2 - t1), t_prec + (t3 - t2)
        print("cpu baseline: layer %d of %d done" % (li + 1, len(layers)), file=sys.stderr, flush=True)
    return {
        "value": round((t_curv + t_inv + t_prec) * 1e3, 1),
        "unit": "ms",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": "the whole step, not a sample: fp64 oracle on all %d layers and %d micro-batches: curvature "
                  "%.1f s, inversion %.1f s, precondition %.1f s" % (len(layers), n_micro, t_curv, t_inv, t_prec),
    }


if __name__ == "__main__":
    main()
