#!/usr/bin/env python3
"""Throughput of the direct sparse convolution hot path on one MI355X.

A step is one pass of the whole hot path over one batch of seeded synthetic input already
resident in HBM: every layer of the workload through the LDS-tiled sconv, which pads while it
stages (the fused form of pad_in + sconv).  The default workload is the ResNet-50-style set of
3x3 layers at 80 % weight sparsity, batch 32 (the layers the stated target is quoted on).

Prints ONE JSON line:
  value            effective GFLOP/s (2*nnz*E*F*N flops per layer) over the timed steps, inputs
                   warm in the Infinity Cache (every step touches the same buffers);
  roofline         the kernel with the largest average duration: HIP-event durations taken here;
  layers           per layer: mean and median kernel time warm, median cold (caches flushed by a
                   large write before every step), both roofline fractions, and the paper's
                   two-kernel dataflow (pad_in, then sconv on the padded array) timed beside it;
  other_workloads  the remaining bundled workloads, shorter runs (100 steps) of the same measurement;
  cpu_baseline     the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
FP32_VECTOR_PEAK_TFLOPS = 157.3  # 256 CU x 128 FMA/clk x 2.4 GHz x 2
FLUSH_BYTES = 1 << 30            # written before every cold step: four times the Infinity Cache


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet",
                    help="one of workloads.CONFIG_LAYERS or a comma list of layer names; `chain` "
                         "feeds every layer's output (bias + ReLU fused) to the next layer")
    ap.add_argument("--path", default=os.environ.get("ESCOIN_BENCH_PATH", "auto"),
                    choices=["auto", "direct", "tiled"], help="which sconv entry point `value` times")
    ap.add_argument("--flags", type=int, default=0, help="1 = bias, 2 = relu (fused epilogue)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--cpu-images", type=int, default=0,
                    help="images per layer for the oracle sample (0 = auto, about 10-30 s)")
    ap.add_argument("--no-others", action="store_true", help="skip the other bundled workloads")
    ap.add_argument("--no-two-kernel", action="store_true", help="skip the pad_in + sconv leg")
    ap.add_argument("--no-cold", action="store_true", help="skip the flushed-cache timing")
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


def kernel_source_hash() -> str:
    """Identifies the code the recorded HBM counters were taken with."""
    h = hashlib.sha256()
    for f in ("sconv_tiled.hip", "plan.cpp", "plan.h"):
        h.update(open(os.path.join(ROOT, "paper_1802_10280_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


TRAFFIC_KEYS = ("K", "Q", "B", "WM", "WS", "CC", "CC0", "NB", "TH", "CS", "VW", "WW")


def measured_traffic(runner):
    """HBM bytes one launch of this layer's tiled kernel moved, read plus written, as the
    rocprofv3 FETCH_SIZE / WRITE_SIZE counters recorded it (profiles/hbm_traffic.json, written
    from the counter runs summarised beside it).  None unless a record matches this layer,
    batch size, every tiling knob and the kernel sources exactly."""
    table = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if runner.path != "tiled" or not os.path.exists(table):
        return None
    doc = json.load(open(table))
    if doc.get("kernel_source_hash") != kernel_source_hash():
        return None
    h, s = runner.plan_info, runner.layer.spec
    for rec in doc["records"]:
        if (rec["layer"] == s.name and rec["N"] == s.N and rec["nnz"] == runner.layer.nnz
                and all(rec["plan"].get(k) == h[k] for k in TRAFFIC_KEYS)):
            return rec["read_bytes"] + rec["written_bytes"]
    return None


def make_runners(wl, LayerRunner, workload, path, flags):
    """Layers and runners of a workload; `chain` links every output to the next input."""
    names = wl.CONFIG_LAYERS.get(workload) or workload.split(",")
    layers = [wl.make_layer(n) for n in names]
    runners = []
    for i, L in enumerate(layers):
        d_in = runners[-1].d_out if (workload == "chain" and i) else None
        runners.append(LayerRunner(L, path=path, flags=flags, d_in=d_in))
    return names, layers, runners


def time_kernels(torch, runners, steps, stream, flush=None):
    """HIP-event duration (ms) of every library call of every step: [steps, calls].  Events go
    on the stream the kernels are launched on.  With `flush`, a large buffer is overwritten
    before every step so that the step finds neither its inputs nor its plans in any cache."""
    nk = sum(len(r.kernels()) for r in runners)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(nk + 1)] for _ in range(steps)]
    torch.cuda.synchronize()
    for k in range(steps):
        if flush is not None:
            flush.add_(1)
        i = 0
        evs[k][0].record(stream)
        for r in runners:
            for fn in r.kernels():
                fn()
                i += 1
                evs[k][i].record(stream)
    torch.cuda.synchronize()
    return np.array([[evs[k][i].elapsed_time(evs[k][i + 1]) for i in range(nk)] for k in range(steps)])


def wall_time(torch, runners, steps, warmup):
    for _ in range(warmup):
        for r in runners:
            r.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        for r in runners:
            r.run()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


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

    flags = args.flags
    if args.workload == "chain" and not flags:
        flags = esc.F_BIAS | esc.F_RELU       # the layers of a chain hand post-ReLU maps on
    names, layers, runners = make_runners(wl, LayerRunner, args.workload, args.path, flags)
    flops = [2.0 * L.nnz * L.spec.E * L.spec.F * L.spec.N for L in layers]
    stream = torch.cuda.current_stream()

    if args.traffic_probe:
        # the copy moves exactly 2 * 64 MiB: it calibrates what FETCH_SIZE / WRITE_SIZE read
        n = 16 * 1024 * 1024
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        d = esc.make_desc(1, 1, 4096, 4096, 1, 1, 1, 1, 0)
        direct = [LayerRunner(L, path="direct", flags=flags) for L in layers]
        for _ in range(3):
            esc.escoin_pad_in(d, src, dst)
            for r in runners:
                r.run()
            for r in direct:
                r.run()
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": "done", "copy_bytes_read": 4 * n, "copy_bytes_written": 4 * n,
                          "launch_order": ["copy"] + [L.spec.name for L in layers]
                          + [f"{L.spec.name}:pad_in,{L.spec.name}:direct" for L in layers], "rounds": 3,
                          "kernel_source_hash": kernel_source_hash(),
                          "layers": [{"layer": L.spec.name, "N": L.spec.N, "nnz": L.nnz,
                                      "kernel": r.sconv_kernel_name(),
                                      "plan": {k: r.plan_info[k] for k in TRAFFIC_KEYS}
                                      if r.path == "tiled" else None}
                                     for L, r in zip(layers, runners)]}))
        return

    # ---- cold: every step starts from flushed caches (at least 20 steps for the median)
    cold_ms = None
    if not args.no_cold:
        for r in runners:
            r.run()
        flush = torch.zeros(FLUSH_BYTES // 4, dtype=torch.float32, device="cuda")
        cold_ms = np.median(time_kernels(torch, runners, max(20, min(args.steps, 50)), stream, flush), axis=0)
        del flush
    # ---- the paper's two-kernel dataflow on the same layers: pad_in, then sconv on the padded array
    two = None
    if not args.no_two_kernel and runners[0].path == "tiled":
        direct = []
        for i, L in enumerate(layers):
            d_in = direct[-1].d_out if (args.workload == "chain" and i) else None
            direct.append(LayerRunner(L, path="direct", flags=flags, d_in=d_in))
        n2 = max(20, min(args.steps, 30))
        for _ in range(3):
            for r in direct:
                r.run()
        two = np.median(time_kernels(torch, direct, n2, stream), axis=0).reshape(len(layers), 2)
        del direct

    # ---- value: W warm-up steps, then the wall clock over exactly K steps (warm).  The legs above
    # have run before it, so the clocks have left their idle state when the warm-up starts.
    sec_per_step = wall_time(torch, runners, args.steps, args.warmup)
    ms_per_step = sec_per_step * 1e3
    value = sum(flops) / sec_per_step / 1e9

    # ---- per-kernel durations, warm: a second run of the same steps with events
    dur = time_kernels(torch, runners, args.steps, stream)
    avg_ms, med_ms = dur.mean(axis=0), np.median(dur, axis=0)

    rows, i = [], 0
    for li, (L, r, fl) in enumerate(zip(layers, runners, flops)):
        names_k = r.kernel_names()
        t = {nm: float(avg_ms[i + j]) for j, nm in enumerate(names_k)}
        tm = {nm: float(med_ms[i + j]) for j, nm in enumerate(names_k)}
        tc = {nm: float(cold_ms[i + j]) for j, nm in enumerate(names_k)} if cold_ms is not None else None
        i += len(names_k)
        t_sconv, t_all = t["sconv"], sum(t.values())
        comp = algorithmic_bytes(L, two_kernel=False)
        moved = algorithmic_bytes(L, two_kernel="pad_in" in t)
        t_alu = fl / (FP32_VECTOR_PEAK_TFLOPS * 1e12) * 1e3
        t_hbm = comp / (HBM_PEAK_GBPS * 1e9) * 1e3
        row = {
            "layer": L.spec.name, "kernel": r.sconv_kernel_name(), "nnz": L.nnz,
            "us_pad_in": round(t.get("pad_in", 0.0) * 1e3, 2), "us_sconv": round(t_sconv * 1e3, 2),
            "us_sconv_median": round(tm["sconv"] * 1e3, 2),
            "us_layer_cold_median": round(sum(tc.values()) * 1e3, 2) if tc else None,
            "gflops_sconv": round(fl / t_sconv / 1e6, 1), "gflops_layer": round(fl / t_all / 1e6, 1),
            "gbps_compulsory": round(comp / t_all / 1e6, 1),
            "gbps_method": round(moved / t_all / 1e6, 1),
            "hbm_frac": round(comp / t_all / 1e6 / HBM_PEAK_GBPS, 4),
            "alu_frac": round(fl / t_sconv / 1e9 / FP32_VECTOR_PEAK_TFLOPS, 4),
            "binding": "alu" if t_alu >= t_hbm else "hbm",
            "binding_frac": round(max(t_alu, t_hbm) / t_all, 4),
        }
        if tc:
            row["hbm_frac_cold"] = round(comp / sum(tc.values()) / 1e6 / HBM_PEAK_GBPS, 4)
        if two is not None:
            s = L.spec
            t_pad, t_dir = float(two[li][0]), float(two[li][1])
            pad_bytes = 4 * s.N * s.C * (s.H * s.W + s.Hp * s.Wp)
            row["two_kernel"] = {
                "us_pad_in": round(t_pad * 1e3, 2), "us_sconv": round(t_dir * 1e3, 2),
                "pad_in_gbps": round(pad_bytes / t_pad / 1e6, 1),
                "pad_in_hbm_frac": round(pad_bytes / t_pad / 1e6 / HBM_PEAK_GBPS, 4),
                "gflops_sconv": round(fl / t_dir / 1e6, 1),
                "gflops_layer": round(fl / (t_pad + t_dir) / 1e6, 1),
                "gbps_method": round(algorithmic_bytes(L, True) / (t_pad + t_dir) / 1e6, 1),
            }
        # achieved GB/s: HBM-side bytes the counters recorded for this layer and tiling, if any
        moved_hw = measured_traffic(r)
        row["traffic_bytes"] = moved_hw
        row["gbps_measured"] = round(moved_hw / t_sconv / 1e6, 1) if moved_hw else None
        rows.append(row)

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
                     "median_us": rd["us_sconv_median"], "traffic": measured_traffic(runners[dom])})

    fused = runners[0].path == "tiled"
    out = {
        "metric": ("effective GFLOP/s (2*nnz MACs) of the sparse convolution of every layer"
                   + (", padding fused into the tiled sconv" if fused else ", pad_in + sconv")
                   + "; HBM GB/s per layer in `layers`"),
        "value": round(value, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: " + ",".join(n for n in names),
                   "batch": layers[0].spec.N, "sparsity": layers[0].spec.sparsity,
                   "path": runners[0].path, "flags": flags, "cache_state": "warm (Infinity Cache)"},
        "hbm_gbps_compulsory": round(sum(algorithmic_bytes(L, False) for L in layers) / sec_per_step / 1e9, 1),
        "value_median_kernels": round(sum(flops) / float(med_ms.sum()) / 1e6, 1),
        "roofline": roofline,
        "layers": rows,
    }
    if cold_ms is not None:
        out["cold"] = {"gflops": round(sum(flops) / float(cold_ms.sum()) / 1e6, 1),
                       "us_per_step_median": round(float(cold_ms.sum()) * 1e3, 2),
                       "how": f"{FLUSH_BYTES >> 20} MiB overwritten before every step; sum of per-kernel medians"}
    if two is not None:
        out["two_kernel"] = {"gflops": round(sum(flops) / float(two.sum()) / 1e6, 1),
                             "us_per_step_median": round(float(two.sum()) * 1e3, 2),
                             "what": "pad_in, then the general sconv on the padded array (Section 4.2's dataflow)"}

    if not args.no_others:
        # the same measurement, shorter, on the other bundled workloads
        del runners
        others = {}
        for w in wl.CONFIG_LAYERS:
            if w == args.workload:
                continue
            fl_w = esc.F_BIAS | esc.F_RELU if w == "chain" else args.flags
            ns, ls, rs = make_runners(wl, LayerRunner, w, args.path, fl_w)
            fl = [2.0 * L.nnz * L.spec.E * L.spec.F * L.spec.N for L in ls]
            # building the plans on the host has let the clocks drop: a longer warm-up than the
            # steps themselves would need
            sec = wall_time(torch, rs, 100, 40)
            med = np.median(time_kernels(torch, rs, 50, stream), axis=0)
            per, j = {}, 0
            for L, r in zip(ls, rs):
                n_k = len(r.kernel_names())
                per[L.spec.name] = round(float(med[j:j + n_k].sum()) * 1e3, 2)
                j += n_k
            others[w] = {"gflops": round(sum(fl) / sec / 1e9, 1), "ms_per_step": round(sec * 1e3, 4),
                         "us_median": per}
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
