#!/usr/bin/env python3
"""Times one layer of a workload configuration in every launch configuration the library
offers - the autotuner's search space (paper section 5.5) written out as a table, for
choosing defaults and for reading alongside a rocprofv3 trace.

    python -m paper_2001_00138_amd.tune_report --config 5 --layer 3 [--batch 64]
        [--variants 1,2] [--ck 4,8,16] [--waves 2,4,8] [--reps 5] [--json]

Variants marked experimental are included only when PATDNN_EXPERIMENTAL=1 is set
(the library refuses them otherwise).  Every run goes through the C ABI; inputs are
the seeded synthetic tensors of ``workloads.py`` (weights, masks) and a random input.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def _ints(text):
    return [int(v) for v in text.split(",") if v != ""]


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--layer", type=int, default=3)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--variants", type=_ints, default=None, help="variant numbers (default: all that fit)")
    ap.add_argument("--names", default=None, help="regex over variant names")
    ap.add_argument("--ck", type=_ints, default=[4, 8, 16])
    ap.add_argument("--waves", type=_ints, default=[2, 4, 8])
    ap.add_argument("--ksplit", type=_ints, default=[1], help="input-channel slices (>1 needs PATDNN_EXPERIMENTAL=1)")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args(argv)

    import torch
    from paper_2001_00138_amd import binding as B
    from paper_2001_00138_amd import workloads as wl

    if not torch.cuda.is_available():
        print("tune_report: no GPU visible", file=sys.stderr)
        return 2
    B.lib()
    d = wl.gen_layer(args.config, args.layer, n=args.batch, with_input=False)
    spec = d["spec"]
    x = torch.randn((spec.n, spec.c_in, spec.h, spec.w), device="cuda")
    if spec.input_dist == "relu_normal":
        x.relu_()
    L = B.Layer.from_workload(d)
    bias = torch.from_numpy(d["bias"]).cuda()
    out = torch.empty(L.output_shape(spec.n, spec.h, spec.w), device="cuda")
    kept = int(L.stats()["kept_kernels"])
    nz = wl.nz_flops(spec, kept)
    rows = []
    variants = args.variants if args.variants is not None else list(range(B.patdnn_num_variants()))
    if args.names:
        import re
        variants = [v for v in variants if re.search(args.names, B.patdnn_variant_name(v))]
    for v in variants:
        name = B.patdnn_variant_name(v)
        combos = [(0, 0, 1)] if v == B.PATDNN_VARIANT_FKW else \
            [(c, w, k) for c in args.ck for w in args.waves for k in args.ksplit]
        for ck, waves, ksplit in combos:
            row = {"variant": v, "name": name, "ck": ck, "waves": waves, "ksplit": ksplit}
            try:
                L.set_config(v, ck, waves, ksplit)
                L.conv2d(x, bias, out, relu=True)
                torch.cuda.synchronize()
            except B.PatdnnError as e:
                if e.status != B.PATDNN_EUNSUPPORTED:
                    raise
                row["status"] = "unsupported"
                rows.append(row)
                continue
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.reps):
                L.conv2d(x, bias, out, relu=True)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.reps
            row.update(status="ok", ms=round(ms, 4), nz_tflops=round(nz / ms / 1e9, 2))
            rows.append(row)
            if not args.json:
                print(f"{spec.name} {spec.c_in}->{spec.c_out}@{spec.h} n={spec.n} {name} ck={ck} waves={waves} ksplit={ksplit}: "
                      f"{ms:.4f} ms  {nz / ms / 1e9:.2f} TFLOP/s nz", flush=True)
    L.close()
    if args.json:
        print(json.dumps({"layer": spec.name, "n": spec.n, "kept": kept, "rows": rows}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
