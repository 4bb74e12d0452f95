#!/usr/bin/env python3
"""Throughput of the direct sparse convolution hot path on one MI355X.

A step is one pass of the whole hot path (pad_in + sconv, every layer of the workload) over
one batch of seeded synthetic input already resident in HBM.  The default workload is the
ResNet-50-style set of 3x3 layers at 80 % weight sparsity, batch 32 (the layers the stated
target is quoted on).  Prints ONE JSON line: effective GFLOP/s counted as 2*nnz*E*F*N flops
per layer, the roofline of the dominant kernel (HIP-event durations measured here), and the
CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
FP32_VECTOR_PEAK_TFLOPS = 157.3  # 256 CU x 128 FMA/clk x 2.4 GHz x 2


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet",
                    help="one of workloads.CONFIG_LAYERS or a comma list of layer names")
    ap.add_argument("--path", default=os.environ.get("ESCOIN_BENCH_PATH", "auto"),
                    choices=["auto", "direct", "tiled"], help="which sconv entry point to time")
    ap.add_argument("--flags", type=int, default=0, help="1 = bias, 2 = relu (fused epilogue)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--cpu-images", type=int, default=0,
                    help="images per layer for the oracle sample (0 = auto, about 10-30 s)")
    ap.add_argument("--others", action="store_true",
                    help="after the timed workload, also time the other bundled workloads (50 steps "
                         "each) and report their GFLOP/s under `other_workloads`")
    ap.add_argument("--per-layer", action="store_true", help="also print a per-layer table to stderr")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: a few launches of a plain copy of known size "
                         "(pad_in with pad 0) and of every layer's kernels, nothing timed")
    return ap.parse_args()


def algorithmic_bytes(L, two_kernel: bool) -> int:
    """Bytes the method must move per layer call: input once, output once, CSR once
    ((2*nnz + M + 1)*4, Section 2.3); the separate pad_in adds one write and one read of the
    padded array."""
    s = L.spec
    b = 4 * s.N * s.C * s.H * s.W + 4 * s.N * s.M * s.E * s.F + 4 * (2 * L.nnz + s.M + 1)
    if two_kernel and s.pad > 0:
        b += 2 * 4 * s.N * s.C * s.Hp * s.Wp
    return b


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); the path shards over batch "
              "or output channels without any exchange step, but no multi-GPU figure is produced.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1802_10280_amd as esc
    from paper_1802_10280_amd import workloads as wl
    from paper_1802_10280_amd.runner import LayerRunner

    esc.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    names = wl.CONFIG_LAYERS.get(args.workload) or args.workload.split(",")
    layers = [wl.make_layer(n) for n in names]
    runners = [LayerRunner(L, path=args.path, flags=args.flags) for L in layers]
    flops = [2.0 * L.nnz * L.spec.E * L.spec.F * L.spec.N for L in layers]
    stream = torch.cuda.current_stream()

    def step():
        for r in runners:
            r.run()

    if args.traffic_probe:
        # the copy moves exactly 2 * 64 MiB: it calibrates what FETCH_SIZE / WRITE_SIZE read
        n = 16 * 1024 * 1024
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        d = esc.make_desc(1, 1, 4096, 4096, 1, 1, 1, 1, 0)
        for _ in range(3):
            esc.escoin_pad_in(d, src, dst)
            step()
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": "done", "copy_bytes_read": 4 * n, "copy_bytes_written": 4 * n,
                          "launch_order": ["copy"] + [L.spec.name for L in layers], "rounds": 3,
                          "layers": [{"layer": L.spec.name, "N": L.spec.N, "nnz": L.nnz,
                                      "kernel": r.sconv_kernel_name(),
                                      "plan": {k: r.plan_info[k] for k in ("K", "Q", "B", "WM", "CC", "NB", "TH")}
                                      if r.path == "tiled" else None}
                                     for L, r in zip(layers, runners)]}))
        return

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = sum(flops) / (dt / args.steps) / 1e9

    # Per-kernel durations with HIP events on the launch stream (torch's current stream is the
    # one handed to the library), over a second run of the same steps.
    nk = sum(len(r.kernels()) for r in runners)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(nk + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    for k in range(args.steps):
        i = 0
        evs[k][0].record(stream)
        for r in runners:
            for fn in r.kernels():
                fn()
                i += 1
                evs[k][i].record(stream)
    torch.cuda.synchronize()
    dur = np.array([[evs[k][i].elapsed_time(evs[k][i + 1]) for i in range(nk)]
                    for k in range(args.steps)])          # ms
    avg_ms = dur.mean(axis=0)

    rows, i = [], 0
    for L, r, fl in zip(layers, runners, flops):
        names_k = r.kernel_names()
        t = {nm: float(avg_ms[i + j]) for j, nm in enumerate(names_k)}
        i += len(names_k)
        t_sconv = t["sconv"]
        t_all = sum(t.values())
        comp = algorithmic_bytes(L, two_kernel=False)
        moved = algorithmic_bytes(L, two_kernel="pad_in" in t)
        t_alu = fl / (FP32_VECTOR_PEAK_TFLOPS * 1e12) * 1e3
        t_hbm = comp / (HBM_PEAK_GBPS * 1e9) * 1e3
        rows.append({
            "layer": L.spec.name, "kernel": r.sconv_kernel_name(), "nnz": L.nnz,
            "us_pad_in": round(t.get("pad_in", 0.0) * 1e3, 2), "us_sconv": round(t_sconv * 1e3, 2),
            "gflops_sconv": round(fl / t_sconv / 1e6, 1), "gflops_layer": round(fl / t_all / 1e6, 1),
            "gbps_compulsory": round(comp / t_all / 1e6, 1),
            "gbps_method": round(moved / t_all / 1e6, 1),
            "hbm_frac": round(comp / t_all / 1e6 / HBM_PEAK_GBPS, 4),
            "alu_frac": round(fl / t_sconv / 1e9 / FP32_VECTOR_PEAK_TFLOPS, 4),
            "binding": "alu" if t_alu >= t_hbm else "hbm",
            "binding_frac": round(max(t_alu, t_hbm) / t_all, 4),
        })
        # achieved GB/s: HBM-side bytes the counters recorded for this layer and tiling, if any
        moved_hw = r.measured_traffic()
        rows[-1]["traffic_bytes"] = moved_hw
        rows[-1]["gbps_measured"] = round(moved_hw / t_sconv / 1e6, 1) if moved_hw else None
    dom = max(range(len(rows)), key=lambda k: rows[k]["us_sconv"])
    Ld, rd = layers[dom], rows[dom]
    if rd["binding"] == "alu":
        achieved = flops[dom] / (rd["us_sconv"] * 1e-6) / 1e12
        roofline = {"bound": "alu", "achieved": round(achieved, 3), "peak": FP32_VECTOR_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(achieved / FP32_VECTOR_PEAK_TFLOPS, 4)}
    else:
        achieved = algorithmic_bytes(Ld, False) / (rd["us_sconv"] * 1e-6) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4)}
    roofline.update({"kernel": rd["kernel"], "layer": rd["layer"], "avg_us": rd["us_sconv"],
                     "traffic": runners[dom].measured_traffic()})

    out = {
        "metric": "effective GFLOP/s (2*nnz MACs) over pad_in+sconv of every layer; HBM GB/s per layer in `layers`",
        "value": round(value, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: " + ",".join(n for n in names),
                   "batch": layers[0].spec.N, "sparsity": layers[0].spec.sparsity,
                   "path": runners[0].path, "flags": args.flags},
        "hbm_gbps_compulsory": round(sum(algorithmic_bytes(L, False) for L in layers)
                                     / (dt / args.steps) / 1e9, 1),
        "roofline": roofline,
        "layers": rows,
    }

    if args.others:
        # context only: the same measurement, shorter, on the other bundled workloads
        del runners
        others = {}
        for w, ns in wl.CONFIG_LAYERS.items():
            if w == args.workload:
                continue
            ls = [wl.make_layer(n) for n in ns]
            rs = [LayerRunner(L, path=args.path, flags=args.flags) for L in ls]
            fl = sum(2.0 * L.nnz * L.spec.E * L.spec.F * L.spec.N for L in ls)
            for _ in range(5):
                for r in rs:
                    r.run()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(50):
                for r in rs:
                    r.run()
            torch.cuda.synchronize()
            t = (time.perf_counter() - t0) / 50
            others[w] = {"gflops": round(fl / t / 1e9, 1), "ms_per_step": round(t * 1e3, 4),
                         "layers": ",".join(ns)}
            del rs, ls
        out["other_workloads"] = others

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(layers, args.cpu_images)
    if args.per_layer:
        for r in rows:
            print(json.dumps(r), file=sys.stderr)
    print(json.dumps(out))


def cpu_baseline(layers, images):
    """The oracle as it stands, timed on this machine's host cores on the first `images` images of
    every layer of the workload (its work is linear in the batch)."""
    import oracle
    oracle.build(force=False)
    # dense inner iterations the oracle walks per image; aim at roughly 10-30 s in total
    per_img = sum(L.spec.M * L.spec.E * L.spec.F * L.spec.C * L.spec.R * L.spec.S for L in layers)
    if images <= 0:
        budget = 4.5e10 * max(1, oracle.threads()) / 8.0
        images = int(max(1, min(min(L.spec.N for L in layers), budget // per_img)))
    t_total, fl_total = 0.0, 0.0
    for L in layers:
        s = L.spec
        n = min(images, s.N)
        Wd = oracle.csr_to_dense(s.M, s.C, s.R, s.S, L.rowptr, L.colidx, L.value)
        x = np.ascontiguousarray(L.input[:n])
        t0 = time.perf_counter()
        oracle.conv(x, Wd, s.stride, s.pad)
        t_total += time.perf_counter() - t0
        fl_total += 2.0 * L.nnz * s.E * s.F * n
    return {"value": round(fl_total / t_total / 1e9, 3), "unit": "GFLOP/s",
            "cores": oracle.threads(), "kind": "oracle",
            "sample": f"first {images} image(s) of each layer, {t_total:.1f} s of oracle time; "
                      f"nproc={os.cpu_count()}"}


if __name__ == "__main__":
    main()
