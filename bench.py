#!/usr/bin/env python3
"""Throughput benchmark of the pattern-sparse 3x3 convolution path on one MI355X.

Workload: the VGG-16-shaped 13-layer 3x3 stack at 3x224x224, fp32, batch 64 - the
throughput configuration (8-pattern library, connectivity keep ratio 1/3.6, first
layer dense, He-normal weights, every layer on a seeded input of its own shape).
A "step" is one pass over all 13 layers.  Inputs, weights and outputs are resident
in HBM before the timed region starts.

Prints ONE JSON line.  `value` is effective GFLOP/s over non-zero FLOPs
(2 x 4 x kept kernels x output pixels; 2 x 9 for the dense first layer).  Beside it:
the roofline of the dominant kernel, per-layer rows of this stack and of the
ResNet-50-shaped and MobileNet-V2-shaped (depthwise, HBM-bound) stacks, peaks measured
in the same run (stream copy, plain FMA loop), batch-1 stack latencies, the dense
comparison and the CPU oracle's rate.
"""

from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_VECTOR_TFLOPS = 157.3      # published; counts packed FP32 FMAs (2 per lane per clock)
PEAK_FP32_NONPACKED_TFLOPS = 78.6    # 256 CU x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz
PEAK_HBM_GBPS = 8000.0               # published HBM3E bandwidth


def _log(msg):
    print(msg, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5, help="workload configuration (5 = N=64 VGG stack)")
    ap.add_argument("--batch", type=int, default=None, help="override the batch size")
    ap.add_argument("--tune", action="store_true",
                    help="run the autotuner on every layer, also on those the configuration file covers")
    ap.add_argument("--no-tune", action="store_true",
                    help="never run the autotuner: layers the configuration file does not cover use the "
                         "library default (a profiler trace of such a run holds no tuner launches)")
    ap.add_argument("--configs", default=os.path.join(ROOT, "paper_2001_00138_amd", "tuned_configs.json"),
                    help="launch configurations per layer shape, as an earlier --save-configs run wrote "
                         "them (the tuner's result kept with the layer, as section 5.5 writes it back)")
    ap.add_argument("--save-configs", default=None,
                    help="write the launch configurations in use (loaded and tuned) to this JSON file")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense-compare", action="store_true")
    ap.add_argument("--no-latency", action="store_true", help="skip the batch-1 stack latency leg")
    ap.add_argument("--no-other-stacks", action="store_true",
                    help="skip the per-layer rows of the ResNet-50 / MobileNet-V2 shaped stacks")
    ap.add_argument("--no-peaks", action="store_true", help="skip the stream-copy and FMA-loop probes")
    ap.add_argument("--no-ablation", action="store_true",
                    help="skip the per-layer breakdown (No-opt / +reorder / +LRE / +tuning, CSR, dense)")
    ap.add_argument("--no-pattern-sweep", action="store_true",
                    help="skip the timing of one layer with pattern sets of 6 / 8 / 12 / 56 patterns")
    ap.add_argument("--only-timed", action="store_true",
                    help="the timed region only (for profiler runs): implies every --no-* leg above")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch the plain copy probe once on 256 MiB (for rocprofv3 --pmc runs: its "
                         "FETCH_SIZE / WRITE_SIZE readings calibrate the counters)")
    ap.add_argument("--traffic-json", default=os.path.join(ROOT, "profiles", "hbm_traffic.json"),
                    help="per-kernel HBM bytes per launch written by profile_summary.py from --pmc runs "
                         "of this same command; fills roofline.traffic when it names the dominant kernel")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "run it with --gpus 1", file=sys.stderr)
        return 2
    if args.only_timed:
        args.no_cpu_baseline = args.no_dense_compare = args.no_latency = True
        args.no_other_stacks = args.no_peaks = args.no_ablation = args.no_pattern_sweep = True

    import numpy as np
    import torch
    from paper_2001_00138_amd import binding as B
    from paper_2001_00138_amd import buildlib
    from paper_2001_00138_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    B.lib()
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()      # the stream every launch below goes to

    def variant_name(cfg):
        # variant -1: the library picks its default configuration at every call
        return B.patdnn_variant_name(cfg["variant"]) if cfg["variant"] >= 0 else "auto"

    # Workspace for the layers whose configuration splits the input channels (one buffer of
    # partial sums per slice); shared by every launch on `stream`, which run one after the other.
    ws = torch.empty(64 << 20, dtype=torch.float32, device="cuda")          # 256 MB

    saved = wl.load_tuned_configs(args.configs) if not args.tune else {}
    used_configs = dict(saved)
    names = {B.patdnn_variant_name(v): v for v in range(B.patdnn_num_variants())}

    def configure(L, spec, x, bias, out):
        """Launch configuration of one layer: from the file, tuned now, or the library default."""
        key = wl.shape_key(spec)
        c = saved.get(key)
        if c is not None and c["variant"] in names:
            L.set_config(names[c["variant"]], c["ck"], c["waves"], c["ksplit"])
        elif not args.no_tune:
            L.tune(x, bias, out, workspace=ws)
        cfg = L.get_config()
        if cfg["variant"] >= 0:
            used_configs[key] = dict(cfg, variant=B.patdnn_variant_name(cfg["variant"]))
        return cfg

    def timed_ms(fn, reps):
        """Milliseconds of each of `reps` runs of fn() on the stream (HIP events)."""
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e0, e1 in ev:
            e0.record(stream)
            fn()
            e1.record(stream)
        torch.cuda.synchronize()
        return [e0.elapsed_time(e1) for e0, e1 in ev]

    # ------------------------------------------------------------------ set-up
    def build_stack(cfg_no, batch, per_image_input=True):
        out = []
        for li in range(len(wl.config_layers(cfg_no))):
            d = wl.gen_layer(cfg_no, li, n=batch, with_input=False)
            spec = d["spec"]
            x = torch.empty((spec.n, spec.c_in, spec.h, spec.w), dtype=torch.float32, device="cuda")
            if per_image_input:
                for i in range(spec.n):
                    x[i].copy_(torch.from_numpy(wl.gen_input_image(spec, cfg_no, li, i)))
            else:
                # the seeded image 0, repeated: the timing does not depend on the values
                x[:] = torch.from_numpy(wl.gen_input_image(spec, cfg_no, li, 0)).cuda()[None]
            L = B.Layer.from_workload(d)
            bias = torch.from_numpy(d["bias"]).cuda()
            o = torch.empty(L.output_shape(spec.n, spec.h, spec.w), dtype=torch.float32, device="cuda")
            kept = int(L.stats()["kept_kernels"])
            cfg = configure(L, spec, x, bias, o)
            out.append(dict(spec=spec, d=d, L=L, x=x, bias=bias, out=o, kept=kept, cfg=cfg,
                            nz=wl.nz_flops(spec, kept), dense_eq=wl.dense_flops(spec),
                            bytes=wl.algorithmic_bytes(spec, kept)))
            _log(f"[setup] {spec.name}: {spec.c_in}->{spec.c_out} @{spec.h} s{spec.stride} N={spec.n} kept={kept} "
                 f"cfg={cfg} ({variant_name(cfg)})")
        return out

    def layer_row(ly, ms_list):
        spec = ly["spec"]
        ms_list = sorted(ms_list)
        med = ms_list[len(ms_list) // 2]
        t = med * 1e-3
        bound = "hbm" if (spec.depthwise or ly["bytes"] / PEAK_HBM_GBPS / 1e9 > ly["nz"] / PEAK_FP32_VECTOR_TFLOPS / 1e12) else "alu"
        return {
            "layer": spec.name, "shape": f"{spec.c_in}->{spec.c_out}@{spec.h}" + ("/s2" if spec.stride == 2 else ""),
            "n": spec.n, "kept": ly["kept"], "variant": variant_name(ly["cfg"]),
            "ck": ly["cfg"]["ck"], "waves": ly["cfg"]["waves"], "ksplit": ly["cfg"]["ksplit"],
            "ms": round(float(np.mean(ms_list)), 4), "ms_median": round(med, 4), "ms_min": round(ms_list[0], 4),
            "nz_gflops": round(ly["nz"] / t / 1e9, 1),
            "dense_eq_gflops": round(ly["dense_eq"] / t / 1e9, 1),
            "alg_gbps": round(ly["bytes"] / t / 1e9, 1),
            "bound": bound,
            "frac_alu_peak": round(ly["nz"] / t / 1e12 / PEAK_FP32_VECTOR_TFLOPS, 4),
            "frac_alu_nonpacked": round(ly["nz"] / t / 1e12 / PEAK_FP32_NONPACKED_TFLOPS, 4),
            "frac_hbm_peak": round(ly["bytes"] / t / 1e9 / PEAK_HBM_GBPS, 4),
        }

    t_setup = time.time()
    layers = build_stack(args.config, args.batch)
    torch.cuda.synchronize()
    _log(f"[setup] done in {time.time() - t_setup:.1f} s")

    def step(events=None):
        for k, ly in enumerate(layers):
            if events is not None:
                events[k][0].record(stream)
            ly["L"].conv2d_ws(ly["x"], ly["bias"], ly["out"], workspace=ws, relu=True)
            if events is not None:
                events[k][1].record(stream)

    probes = None
    if args.calibrate_copy or not args.no_peaks:
        probes = ctypes.CDLL(buildlib.PROBES_LIB)
        probes.patdnn_probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        probes.patdnn_probe_fma.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                            ctypes.POINTER(ctypes.c_double)]
    sptr = stream.cuda_stream or None
    if args.calibrate_copy:
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        assert probes.patdnn_probe_copy(dst.data_ptr(), src.data_ptr(), src.numel() * 4, sptr) == 0
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------ timed region
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in layers] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(ev[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    per_layer = [[ev[s][k][0].elapsed_time(ev[s][k][1]) for s in range(args.steps)] for k in range(len(layers))]
    per_layer_ms = [float(np.mean(v)) for v in per_layer]
    total_nz = sum(ly["nz"] for ly in layers)
    total_dense = sum(ly["dense_eq"] for ly in layers)
    value = total_nz / (ms_per_step * 1e-3) / 1e9

    # ------------------------------------------------------------------ roofline of the dominant kernel
    by_kernel = {}
    for k, ly in enumerate(layers):
        name = variant_name(ly["cfg"])
        if ly["spec"].dense or ly["spec"].depthwise:
            continue
        if ly["cfg"].get("ksplit", 1) > 1:
            # a channel-split layer is two launches (the split instantiation of the kernel, whose
            # slices store to the workspace, then sum + bias + ReLU): another kernel symbol, kept
            # apart from the unsplit launches
            name += "+split"
        agg = by_kernel.setdefault(name, dict(ms=0.0, flops=0, bytes=0, launches=0))
        agg["ms"] += per_layer_ms[k]
        agg["flops"] += ly["nz"]
        agg["bytes"] += ly["bytes"]
        agg["launches"] += 1
    roofline = None
    if by_kernel:
        kname, agg = max(by_kernel.items(), key=lambda kv: kv[1]["ms"])
        achieved = agg["flops"] / (agg["ms"] * 1e-3) / 1e12
        roofline = {
            "bound": "alu", "kernel": kname, "achieved": round(achieved, 3),
            "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
            "frac": round(achieved / PEAK_FP32_VECTOR_TFLOPS, 4),
            "peak_nonpacked": PEAK_FP32_NONPACKED_TFLOPS,
            "frac_nonpacked": round(achieved / PEAK_FP32_NONPACKED_TFLOPS, 4),
            "launches_per_step": agg["launches"],
            "avg_launch_ms": round(agg["ms"] / agg["launches"], 4),
            "algorithmic_gflop_per_launch": round(agg["flops"] / agg["launches"] / 1e9, 3),
            "algorithmic_gb_per_launch": round(agg["bytes"] / agg["launches"] / 1e9, 4),
            "hbm_gbps_at_algorithmic_bytes": round(agg["bytes"] / (agg["ms"] * 1e-3) / 1e9, 1),
            "traffic": None,
        }
        # HBM bytes per launch from hardware counters, if a counter run of this command was summarised
        try:
            ly0 = next(ly for ly in layers if variant_name(ly["cfg"]) == kname.replace("+split", ""))
            info = B.patdnn_tiled_info(ly0["L"].handle, ly0["cfg"]["variant"], ly0["cfg"]["ck"])
            sig = re.compile(rf"Geo<{info['G']}, {info['patch_rows']}, {info['patch_cols']}, {info['conv_stride']}, "
                             rf"{info['lanes_x']}, false, \d+, {info['mode']}>, {'true' if kname.endswith('+split') else 'false'}>")
            with open(args.traffic_json) as f:
                table = json.load(f)
            hit = [v for k, v in table.items() if sig.search(k) and "fetch_bytes" in v and "write_bytes" in v]
            if hit:
                roofline["traffic"] = round(hit[0]["fetch_bytes"] + hit[0]["write_bytes"])
                roofline["traffic_detail"] = {"fetch_bytes_per_launch": round(hit[0]["fetch_bytes"]),
                                              "write_bytes_per_launch": round(hit[0]["write_bytes"]),
                                              "source": os.path.relpath(args.traffic_json, ROOT)}
        except (OSError, ValueError, StopIteration, KeyError, B.PatdnnError):
            pass

    layer_rows = [layer_row(ly, per_layer[k]) for k, ly in enumerate(layers)]

    # ------------------------------------------------------------------ peaks measured in this run
    peaks = None
    if not args.no_peaks:
        nbytes = 1 << 30
        src = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        probes.patdnn_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, sptr)
        ms = sorted(timed_ms(lambda: probes.patdnn_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, sptr), 10))
        copy_gbps = 2 * nbytes / (ms[len(ms) // 2] * 1e-3) / 1e9
        del src, dst
        sink = torch.zeros(4, dtype=torch.float32, device="cuda")
        flops = ctypes.c_double()
        probes.patdnn_probe_fma(sink.data_ptr(), 256 * 32, 4096, sptr, ctypes.byref(flops))
        ms = sorted(timed_ms(lambda: probes.patdnn_probe_fma(sink.data_ptr(), 256 * 32, 4096, sptr, ctypes.byref(flops)), 10))
        fma_tflops = flops.value / (ms[len(ms) // 2] * 1e-3) / 1e12
        peaks = {"stream_copy_gbps": round(copy_gbps, 1), "stream_copy_bytes": 2 * nbytes,
                 "fma_loop_tflops": round(fma_tflops, 2),
                 "note": "read + written bytes of a plain 1 GiB device copy; 24 independent plain "
                         "(non-packed) fp32 FMA chains per lane, 8192 workgroups"}
        if roofline is not None:
            roofline["frac_of_measured_fma_loop"] = round(roofline["achieved"] / fma_tflops, 4)

    # ------------------------------------------------------------------ the same step as two half batches
    # The images of a batch are independent, so a caller may send one half of the batch through
    # all layers on one stream and the other half on a second one: the launches of one half then
    # cover the ends of the other half's launches, where the machine runs out of workgroups.
    # Reported beside the headline, which stays one stream (there a launch's duration is the
    # kernel's own, which is what the roofline row divides by).
    halves = None
    if not args.only_timed and layers[0]["spec"].n >= 2:
        n_img = layers[0]["spec"].n
        side = [torch.cuda.Stream(), torch.cuda.Stream()]
        side_ws = [ws[:ws.numel() // 2], ws[ws.numel() // 2:]]       # launches of the two streams overlap
        cut = [0, n_img // 2, n_img]

        def step_halves():
            fork = torch.cuda.Event()
            fork.record(stream)
            for p, st in enumerate(side):
                st.wait_event(fork)
                for ly in layers:
                    ly["L"].conv2d_ws(ly["x"][cut[p]:cut[p + 1]], ly["bias"], ly["out"][cut[p]:cut[p + 1]],
                                      workspace=side_ws[p], relu=True, stream=st)
                join = torch.cuda.Event()
                join.record(st)
                stream.wait_event(join)

        for _ in range(min(args.warmup, 3)):
            step_halves()
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(args.steps):
            step_halves()
        torch.cuda.synchronize()
        ms_h = (time.perf_counter() - c0) * 1e3 / args.steps
        halves = {"ms_per_step": round(ms_h, 4), "nz_gflops": round(total_nz / (ms_h * 1e-3) / 1e9, 1),
                  "note": "the batch as two halves on two streams, each half through all layers in order, "
                          "joined at the end of every step; same kernels and configurations"}

    # ------------------------------------------------------------------ the other stacks, per layer
    other = None
    if not args.no_other_stacks and args.config == 5:
        other = {}
        for key, cfg_no, batch in (("resnet50_3x3_n1", 3, 1), ("resnet50_3x3_n64", 3, 64),
                                   ("mobilenet_v2_depthwise_n1", 4, 1), ("mobilenet_v2_depthwise_n64", 4, 64)):
            try:
                st = build_stack(cfg_no, batch, per_image_input=False)
                rows = []
                for ly in st:
                    fn = lambda ly=ly: ly["L"].conv2d_ws(ly["x"], ly["bias"], ly["out"], workspace=ws, relu=True)
                    fn()
                    rows.append(layer_row(ly, timed_ms(fn, 20)))
                    if cfg_no == 4 and batch > 1:
                        # An HBM-bound row timed over and over on one pair of buffers may be served by
                        # the 256 MB Infinity Cache: time it again on a rotating set of input / output
                        # pairs larger than the cache (768 MB or more in all), so that every run
                        # really comes from and goes to HBM.
                        pair = ly["x"].numel() * 4 + ly["out"].numel() * 4
                        copies = int(min(64, max(2, -(-768 * 2 ** 20 // pair))))
                        xs = [ly["x"]] + [ly["x"].clone() for _ in range(copies - 1)]
                        os_ = [ly["out"]] + [torch.empty_like(ly["out"]) for _ in range(copies - 1)]
                        turn = [0]

                        def rot(ly=ly, xs=xs, os_=os_, turn=turn):
                            k = turn[0] % len(xs)
                            turn[0] += 1
                            ly["L"].conv2d_ws(xs[k], ly["bias"], os_[k], workspace=ws, relu=True)
                        for _ in range(copies):
                            rot()
                        ms = sorted(timed_ms(rot, max(20, copies)))
                        med = ms[len(ms) // 2]
                        rows[-1]["rotating_buffers"] = {
                            "pairs": copies, "ms_median": round(med, 4),
                            "alg_gbps": round(ly["bytes"] / (med * 1e-3) / 1e9, 1),
                            "frac_hbm_peak": round(ly["bytes"] / (med * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)}
                        del xs, os_
                tot_ms = sum(r["ms_median"] for r in rows)
                other[key] = {"workload": wl.CONFIG_NAMES[cfg_no].replace("N=1", f"N={batch}"), "batch": batch,
                              "layers": rows,
                              "sum_ms_median": round(tot_ms, 4),
                              "nz_gflops": round(sum(ly["nz"] for ly in st) / (tot_ms * 1e-3) / 1e9, 1),
                              "alg_gbps": round(sum(ly["bytes"] for ly in st) / (tot_ms * 1e-3) / 1e9, 1)}
                if cfg_no == 4 and batch > 1:
                    rot_ms = sum(r["rotating_buffers"]["ms_median"] for r in rows)
                    other[key]["rotating_buffers"] = {
                        "note": "every layer on a rotating set of input / output pairs larger than the "
                                "256 MB Infinity Cache: all traffic is HBM traffic",
                        "sum_ms_median": round(rot_ms, 4),
                        "alg_gbps": round(sum(ly["bytes"] for ly in st) / (rot_ms * 1e-3) / 1e9, 1)}
                    # the same layers on half-precision storage (section 6.1): half the bytes
                    rows16 = []
                    for ly in st:
                        x16, o16 = ly["x"].half(), ly["out"].half()
                        fn = lambda ly=ly, x16=x16, o16=o16: ly["L"].conv2d_f16(x16, ly["bias"], o16, relu=True)
                        fn()
                        ms = sorted(timed_ms(fn, 20))
                        med = ms[len(ms) // 2]
                        by16 = ly["bytes"] / 2
                        rows16.append({"layer": ly["spec"].name, "ms_median": round(med, 4), "ms_min": round(ms[0], 4),
                                       "alg_gbps": round(by16 / (med * 1e-3) / 1e9, 1),
                                       "frac_hbm_peak": round(by16 / (med * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)})
                        del x16, o16
                    tot16 = sum(r["ms_median"] for r in rows16)
                    other[key + "_f16_storage"] = {
                        "workload": other[key]["workload"] + ", binary16 weights / input / output, fp32 arithmetic",
                        "batch": batch, "layers": rows16, "sum_ms_median": round(tot16, 4),
                        "alg_gbps": round(sum(ly["bytes"] for ly in st) / 2 / (tot16 * 1e-3) / 1e9, 1),
                        "speedup_over_fp32_storage": round(tot_ms / tot16, 2)}
                for ly in st:
                    ly["L"].close()
                del st
            except Exception as exc:            # the throughput line must not depend on this leg
                other[key] = {"error": f"{type(exc).__name__}: {exc}"}

    # ------------------------------------------------------------------ batch-1 latency of the same stack
    # (the paper's headline scenario, section 6.2: one image through all CONV layers; reported
    # beside the throughput number, never instead of it)
    latency = None
    if not args.no_latency and args.config == 5:
        def stack_latency(cfg_no):
            """One image through every layer of a configuration, launches back to back."""
            one = build_stack(cfg_no, 1, per_image_input=False)
            run = lambda: [ly["L"].conv2d_ws(ly["x"], ly["bias"], ly["out"], workspace=ws, relu=True) for ly in one]
            for _ in range(3):
                run()
            torch.cuda.synchronize()
            reps = 20
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                run()
            e1.record(stream)
            torch.cuda.synchronize()
            ms1 = e0.elapsed_time(e1) / reps
            nz1 = sum(ly["nz"] for ly in one)
            by1 = sum(ly["bytes"] for ly in one)
            kernels = sorted({variant_name(ly["L"].get_config()) for ly in one})
            for ly in one:
                ly["L"].close()
            return {"workload": wl.CONFIG_NAMES[cfg_no], "layers": len(one), "ms_per_image": round(ms1, 4),
                    "nz_gflops": round(nz1 / (ms1 * 1e-3) / 1e9, 1),
                    "alg_gbps": round(by1 / (ms1 * 1e-3) / 1e9, 1), "kernels": kernels}

        def vgg_chained():
            """The VGG-16 shaped stack as a network: every layer reads what the one before wrote,
            ReLU + 2x2 max pooling fused into conv 2, 4, 7, 10 and 13; plain launches and one HIP
            graph launch per image (patdnn_stack_run)."""
            one = build_stack(2, 1, per_image_input=False)
            pool = [li in (1, 3, 6, 9, 12) for li in range(len(one))]
            st = B.Stack([(ly["L"], ly["bias"], True, p) for ly, p in zip(one, pool)], 1, one[0]["spec"].h,
                         one[0]["spec"].w)
            out = torch.empty(st.output_shape(), dtype=torch.float32, device="cuda")
            side = torch.cuda.Stream()
            res = {}
            with torch.cuda.stream(side):
                for key, graph in (("plain_ms_per_image", False), ("graph_ms_per_image", True)):
                    for _ in range(3):
                        st.run(one[0]["x"], out, graph=graph, stream=side)
                    side.synchronize()
                    reps = 50
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(side)
                    for _ in range(reps):
                        st.run(one[0]["x"], out, graph=graph, stream=side)
                    e1.record(side)
                    side.synchronize()
                    res[key] = round(e0.elapsed_time(e1) / reps, 4)
            st.close()
            for ly in one:
                ly["L"].close()
            res["note"] = ("13 layers chained on real activations, 5 fused ReLU + 2x2 max-pool epilogues "
                           "(a layer that splits its input channels is two launches: slices into the "
                           "stack's partial-sum buffers, then sum + bias + ReLU / pool); the graph run is "
                           "one hipGraphLaunch")
            return res

        def vgg_chained_batch():
            """The same network at the batch of the headline, on the headline's layer handles: what
            the fused pooling saves when the layers feed each other (the headline times every layer
            on its own buffers, un-pooled)."""
            pool = [li in (1, 3, 6, 9, 12) for li in range(len(layers))]
            n_img = layers[0]["spec"].n
            st = B.Stack([(ly["L"], ly["bias"], True, p) for ly, p in zip(layers, pool)], n_img,
                         layers[0]["spec"].h, layers[0]["spec"].w)
            out = torch.empty(st.output_shape(), dtype=torch.float32, device="cuda")
            for _ in range(3):
                st.run(layers[0]["x"], out, stream=stream)
            ms = sorted(timed_ms(lambda: st.run(layers[0]["x"], out, stream=stream), 20))
            st.close()
            med = ms[len(ms) // 2]
            return {"batch": n_img, "ms_per_batch": round(med, 4), "images_per_s": round(n_img / (med * 1e-3), 1),
                    "nz_gflops": round(total_nz / (med * 1e-3) / 1e9, 1),
                    "note": "13 layers chained, ReLU + 2x2 max pooling fused into conv 2, 4, 7, 10 and 13"}

        latency = {"note": "one image, all layers launched back to back on one stream, launch gaps included"}
        try:
            latency["vgg16_chained"] = vgg_chained()
        except Exception as exc:
            latency["vgg16_chained"] = {"error": f"{type(exc).__name__}: {exc}"}
        if args.config == 5:
            try:
                latency["vgg16_chained_batch"] = vgg_chained_batch()
            except Exception as exc:
                latency["vgg16_chained_batch"] = {"error": f"{type(exc).__name__}: {exc}"}
        for key, cfg_no in (("vgg16", 2), ("resnet50_3x3", 3), ("mobilenet_v2_depthwise", 4)):
            try:
                latency[key] = stack_latency(cfg_no)
            except Exception as exc:        # the throughput line must not depend on this leg
                latency[key] = {"error": f"{type(exc).__name__}: {exc}"}

    # ------------------------------------------------------------------ dense comparison (same shapes)
    dense_cmp = None
    if not args.no_dense_compare:
        rows = []
        for k, ly in enumerate(layers):
            spec = ly["spec"]
            if spec.depthwise:
                continue
            if spec.dense:
                rows.append({"layer": spec.name, "dense_ms": round(per_layer_ms[k], 4)})
                continue
            Ld = B.Layer(ly["d"]["weights"], None, None, None, stride=spec.stride, pad=spec.pad, dense=True)
            fn = lambda: Ld.conv2d(ly["x"], ly["bias"], ly["out"], relu=True)
            fn()
            ms = sorted(timed_ms(fn, 3))[1]
            rows.append({"layer": spec.name, "dense_ms": round(ms, 4),
                         "dense_gflops": round(ly["dense_eq"] / (ms * 1e-3) / 1e9, 1),
                         "speedup_pattern_vs_dense": round(ms / per_layer_ms[k], 2)})
            Ld.close()
        dense_cmp = rows

    # ------------------------------------------------------------------ per-layer breakdown (section 6.3)
    # No-opt -> +filter-kernel reorder -> +load-redundancy elimination -> +tuning on the unique
    # layer shapes of the stack, with the CSR control (section 6.2) and the dense kernel beside it
    ablation = None
    if not args.no_ablation and args.config == 5:
        names_ = {B.patdnn_variant_name(v): v for v in range(B.patdnn_num_variants())}
        rows, seen_shapes = [], set()
        for k, ly in enumerate(layers):
            spec = ly["spec"]
            if spec.dense or spec.depthwise or wl.shape_key(spec) in seen_shapes:
                continue
            seen_shapes.add(wl.shape_key(spec))
            L = ly["L"]
            tuned_cfg = L.get_config()
            run = lambda: L.conv2d_ws(ly["x"], ly["bias"], ly["out"], workspace=ws, relu=True)
            ms = {}
            for stage, (vname, ck, waves) in (("noopt", ("noopt", 0, 0)), ("reorder", ("fkw", 0, 0)),
                                              ("lre", ("t_g16_p7x1_s1_x16", 0, 0)), ("csr", ("csr", 0, 0))):
                L.set_config(names_[vname], ck, waves, 1)
                run()
                ms[stage] = sorted(timed_ms(run, 3))[1]
            L.set_config(tuned_cfg["variant"], tuned_cfg["ck"], tuned_cfg["waves"], tuned_cfg["ksplit"])
            run()
            ms["tuned"] = sorted(timed_ms(run, 5))[2]
            Ld = B.Layer(ly["d"]["weights"], None, None, None, stride=spec.stride, pad=spec.pad, dense=True)
            rund = lambda: Ld.conv2d(ly["x"], ly["bias"], ly["out"], relu=True)
            rund()
            ms["dense"] = sorted(timed_ms(rund, 3))[1]
            Ld.close()
            rows.append({"layer": spec.name, "shape": f"{spec.c_in}->{spec.c_out}@{spec.h}", "n": spec.n,
                         "ms": {kk: round(v, 4) for kk, v in ms.items()},
                         "speedup_reorder": round(ms["noopt"] / ms["reorder"], 2),
                         "speedup_lre": round(ms["reorder"] / ms["lre"], 2),
                         "speedup_tuning": round(ms["lre"] / ms["tuned"], 2),
                         "csr_over_dense": round(ms["csr"] / ms["dense"], 2),
                         "dense_over_pattern": round(ms["dense"] / ms["tuned"], 2)})
        ablation = {"note": "noopt: one lane per pixel, original filter / kernel order, pattern decided per "
                            "kernel in the inner loop; reorder: the same lane mapping over the FKW arrays; lre: "
                            "the tiled kernel in its default configuration; tuned: the autotuner's choice; csr: "
                            "one lane per pixel over CSR; dense: the dense direct kernel on unpruned weights",
                    "layers": rows}

    # ------------------------------------------------------------------ pattern-count sweep (section 6.6)
    # the same layer with libraries of 6 / 8 / 12 / 56 patterns: the kernels carry a code body for
    # every one of the 56 centre-keeping patterns, so the set size only changes the streams
    sweep = None
    if not args.no_pattern_sweep and args.config == 5:
        sweep = {"note": "128->128@112 and 512->512@28 at N=64, keep 1/3.6, pattern ids uniform over a seeded "
                         "library of k patterns; same launch configuration as the 8-pattern layer", "rows": []}
        for li in (3, 8):
            ly = layers[li]
            spec, d = ly["spec"], ly["d"]
            cfg0 = ly["L"].get_config()
            for kpat in (6, 8, 12, 56):
                lib_k = wl.pattern_library(wl.PATTERN_SEED, kpat)
                ids_k = np.random.default_rng(600 + kpat).integers(0, kpat, d["pattern_ids"].shape, dtype=np.uint8)
                Lk = B.Layer(d["weights"], ids_k, d["kernel_mask"], lib_k, stride=spec.stride, pad=spec.pad)
                Lk.set_config(cfg0["variant"], cfg0["ck"], cfg0["waves"], cfg0["ksplit"])
                runk = lambda: Lk.conv2d_ws(ly["x"], ly["bias"], ly["out"], workspace=ws, relu=True)
                runk()
                ms = sorted(timed_ms(runk, 7))[3]
                sweep["rows"].append({"layer": spec.name, "patterns": kpat, "ms": round(ms, 4),
                                      "nz_gflops": round(ly["nz"] / (ms * 1e-3) / 1e9, 1)})
                Lk.close()

    # ------------------------------------------------------------------ CPU oracle beside it
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ref
        done_flops, spent, images = 0, 0.0, 0
        # whole images of the stack, one after another, until the time budget is used
        while spent < args.cpu_seconds and images < layers[0]["spec"].n:
            for k, ly in enumerate(layers):
                spec, d = ly["spec"], ly["d"]
                x1 = ly["x"][images:images + 1].cpu().numpy()
                c0 = time.perf_counter()
                ref.conv2d(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"], x1,
                           d["bias"], stride=spec.stride, pad=spec.pad, relu=True, dense=spec.dense,
                           depthwise=spec.depthwise, skip_removed=True)
                spent += time.perf_counter() - c0
                done_flops += wl.nz_flops(spec, ly["kept"], n=1)
            images += 1
        cpu = {"value": round(done_flops / spent / 1e9, 3), "unit": "GFLOP/s", "cores": ref.num_threads(),
               "kind": "oracle",
               "sample": f"fp64 oracle (OpenMP), all {len(layers)} layers on {images} of the "
                         f"{layers[0]['spec'].n} images, {spent:.1f} s of CPU wall time"}

    if args.save_configs:
        with open(args.save_configs, "w") as f:
            json.dump(used_configs, f, indent=1, sort_keys=True)

    spec0 = layers[0]["spec"]
    result = {
        "metric": "effective GFLOP/s (non-zero FLOPs) over the pattern-sparse VGG-16 3x3 conv stack",
        "value": round(value, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.CONFIG_NAMES[args.config], "batch": spec0.n, "layers": len(layers),
                   "patterns": 8, "connectivity_keep": "1/3.6", "input": "3x224x224" if args.config in (2, 5) else "per layer"},
        "dense_equivalent_gflops": round(total_dense / (ms_per_step * 1e-3) / 1e9, 1),
        "nz_gflop_per_step": round(total_nz / 1e9, 2),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "measured_peaks": peaks,
        "two_stream_halves": halves,
        "batch1_stack_latency": latency,
        "layers": layer_rows,
        "other_stacks": other,
        "dense_compare": dense_cmp,
        "ablation": ablation,
        "pattern_count_sweep": sweep,
    }
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
