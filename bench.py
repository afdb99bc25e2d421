#!/usr/bin/env python3
"""Benchmark of the sparse-convolution hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: build_index_grid -> build_kernel_map -> sparse_conv_fwd.  The headline value
is the paper's "effective TFLOP/s" (Sec. 4.1.3: 2 * active pairs * C_in * C_out) over the whole
step; the per-stage figures (conv-only TFLOP/s, kernel-map and grid-build Mvoxels/s) and the
roofline of the dominant kernel are reported in the same JSON line, next to the CPU oracle
timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0}
FP32_VALU_PEAK_TFLOPS = 157.3

WORKLOAD_DESC = {
    "sphere64": "config 1: sphere shell r=28 in 64^3, 3x3x3 submanifold, 32->32 fp32",
    "indoor4": "config 2: 4 indoor-like grids in 512^3, 3x3x3 submanifold, 64->64 fp16",
    "lidar1m": "config 3: LiDAR-like 2048x2048x64 grid (~1M voxels), 3x3x3 submanifold, 64->64 bf16",
    "lidar1m_down": "config 4: config-3 grid, 2x2x2 stride 2, 64->128 bf16 (coarse grid + map + conv)",
    "sheets4": "config 5: 4 random-walk sheet grids in 128^3, 3x3x3 submanifold, 256->256 bf16",
}


def accounting(n_in, n_out, pairs, k3, c_in, c_out, elem_bytes, out_bytes):
    """Algorithmic work of one step (what the method must compute / move, per the paper's
    effective-FLOP definition and the byte model of Sec. 3.5 scenario 1)."""
    flops = 2.0 * pairs * c_in * c_out
    conv_bytes = n_in * c_in * elem_bytes + n_out * c_out * out_bytes + k3 * c_in * c_out * elem_bytes
    kmap_bytes = n_out * k3 * 4                 # dense int32 map entries written by the lookup kernel
    grid_bytes = n_in * 12                      # ijk read once
    return flops, conv_bytes, kmap_bytes, grid_bytes


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="lidar1m", choices=sorted(WORKLOAD_DESC))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=300000)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards by grid of the batch; see DESIGN.md); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2407_01781_amd as fx
    from workloads import generators as G

    assert torch.cuda.is_available(), "no GPU visible"
    torch.cuda.set_device(0)
    w = G.workload(args.workload)
    ijk, joffsets = w.jagged_ijk()                                     # shuffled, no duplicates
    feat, wt = w.feats_weights()
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[w.dtype]
    d_ijk = torch.from_numpy(ijk).cuda()
    d_feat = torch.from_numpy(feat).to(tdt).cuda().contiguous()
    d_w = torch.from_numpy(wt).to(tdt).cuda().contiguous()
    elem = 4 if w.dtype == "f32" else 2

    def step(out=None):
        g = fx.build_index_grid(d_ijk, joffsets)
        km = fx.build_kernel_map(g, w.kernel_size, w.stride)
        y = fx.sparse_conv_fwd(km, d_feat, d_w, out=out)
        return g, km, y

    # ---- one untimed pass for sizes
    g, km, y = step()
    n_in, n_out = g.num_voxels, km.n_out
    pairs, _ = km.info()
    tstats = km.tile_stats()
    flops, conv_bytes, kmap_bytes, grid_bytes = accounting(n_in, n_out, pairs, w.k3, w.c_in, w.c_out, elem, elem)
    out_buf = torch.empty_like(y)
    del g, km, y

    # ---- warm-up + timed steps (whole hot path)
    for _ in range(args.warmup):
        step(out_buf)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(out_buf)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # ---- per-kernel times from HIP events on the launch stream (separate passes)
    fx.profile_enable(True)
    fx.profile_reset()
    n_prof = max(5, min(args.steps, 20))
    for _ in range(n_prof):
        step(out_buf)
    torch.cuda.synchronize()
    prof = fx.profile_read()
    fx.profile_enable(False)
    kern_ms = {k: v[0] / v[1] for k, v in prof.items()}
    launches_per_step = {k: v[1] / n_prof for k, v in prof.items()}
    per_step_ms = {k: v[0] / n_prof for k, v in prof.items()}

    # ---- per-stage wall time (events around each call, stages run back to back)
    def stage_times(reps=10):
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(reps)]
        for r in range(reps):
            ev[r][0].record()
            g = fx.build_index_grid(d_ijk, joffsets)
            ev[r][1].record()
            km = fx.build_kernel_map(g, w.kernel_size, w.stride)
            ev[r][2].record()
            fx.sparse_conv_fwd(km, d_feat, d_w, out=out_buf)
            ev[r][3].record()
        torch.cuda.synchronize()
        t = np.array([[ev[r][i].elapsed_time(ev[r][i + 1]) for i in range(3)] for r in range(reps)])
        return np.sort(t, axis=0)[: max(1, reps * 4 // 5)].mean(axis=0)   # mean of the best 80 %

    t_grid, t_kmap, t_conv = stage_times()

    # ---- warm, back-to-back convolution only (map reused, as across the layers of a network)
    g, km, _ = step(out_buf)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        fx.sparse_conv_fwd(km, d_feat, d_w, out=out_buf)
    e1.record()
    torch.cuda.synchronize()
    t_conv_b2b = e0.elapsed_time(e1) / 20

    dom = "k_conv_mfma" if "k_conv_mfma" in kern_ms else "k_conv_scalar"
    dom_ms = kern_ms[dom]
    if dom == "k_conv_mfma":
        peak = MFMA_PEAK_TFLOPS[w.dtype]
        roof = {"kernel": dom, "bound": "mfma", "achieved": flops / (dom_ms * 1e-3) / 1e12, "peak": peak,
                "unit": "TFLOP/s"}
    else:
        roof = {"kernel": dom, "bound": "alu", "achieved": flops / (dom_ms * 1e-3) / 1e12,
                "peak": FP32_VALU_PEAK_TFLOPS, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = None
    roof["avg_launch_ms"] = dom_ms
    roof["hbm_view"] = {"algorithmic_bytes": conv_bytes, "GB/s": conv_bytes / (dom_ms * 1e-3) / 1e9,
                        "frac_of_8TBs": conv_bytes / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    nb_ms = kern_ms.get("k_nbmap")
    kmap_roof = None
    if nb_ms:
        kmap_roof = {"kernel": "k_nbmap", "bound": "hbm", "achieved": kmap_bytes / (nb_ms * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "avg_launch_ms": nb_ms}
        kmap_roof["frac"] = kmap_roof["achieved"] / HBM_PEAK_GBS

    result = {
        "metric": "sparse conv effective TFLOP/s (active pairs), whole hot path: grid build + kernel map + conv",
        "value": flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload}: {WORKLOAD_DESC[args.workload]}", "n_voxels_in": n_in,
                   "n_voxels_out": n_out, "active_pairs": pairs, "kernel_size": w.kernel_size,
                   "stride": w.stride, "c_in": w.c_in, "c_out": w.c_out, "batch": len(w.grids)},
        "stages": {
            "grid_build_ms": float(t_grid), "kernel_map_ms": float(t_kmap), "conv_ms": float(t_conv),
            "conv_back_to_back_ms": float(t_conv_b2b),
            "conv_effective_TFLOPs": flops / (t_conv_b2b * 1e-3) / 1e12,
            "kernel_map_Mvoxels_per_s": n_out / (t_kmap * 1e-3) / 1e6,
            "grid_build_Mvoxels_per_s": n_in / (t_grid * 1e-3) / 1e6,
            "mfma_row_utilisation": (pairs / tstats["mfma_rows_issued"]) if tstats["mfma_rows_issued"] else None,
            "staged_rows_per_output": tstats["staged_rows"] / max(n_out, 1),
        },
        "kernels_ms_per_launch": kern_ms,
        "kernels_ms_per_step": per_step_ms,
        "roofline": roof,
        "roofline_kernel_map": kmap_roof,
    }

    # ---- CPU oracle on this machine's host cores (bounded sample, one thread)
    if not args.no_cpu_baseline:
        from oracle import cpu_oracle as O
        t = time.perf_counter()
        og = O.OracleGrid(ijk, joffsets)
        t_o1 = time.perf_counter() - t
        t = time.perf_counter()
        ogo = O.output_grid(og, w.kernel_size, w.stride)
        nb = O.kernel_map(og, ogo, w.kernel_size, w.stride)
        t_o2 = time.perf_counter() - t
        rows = min(args.cpu_sample_rows, n_out)
        f64, w64 = feat.astype(np.float64), wt.astype(np.float64)
        t = time.perf_counter()
        O.conv(og, ogo, w.kernel_size, w.stride, f64, w64, 0, rows)
        t_o3 = time.perf_counter() - t
        sample_pairs = int((nb[:rows] >= 0).sum())
        t_o3_full = t_o3 * pairs / max(sample_pairs, 1)
        result["cpu_baseline"] = {
            "value": flops / (t_o1 + t_o2 + t_o3_full) / 1e12, "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
            "sample": f"grid build and kernel map on the full input ({t_o1:.2f} s, {t_o2:.2f} s); convolution "
                      f"on the first {rows} of {n_out} output rows ({t_o3:.2f} s), scaled by active pairs",
            "conv_only_TFLOPs": 2.0 * sample_pairs * w.c_in * w.c_out / t_o3 / 1e12,
            "host_cpus": os.cpu_count(),
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
