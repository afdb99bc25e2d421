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
VALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12      # one vector instruction per SIMD every 4 cycles, 64 lanes each: 39.3
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "f32": 157.3}
FP32_VALU_PEAK_TFLOPS = 157.3

WORKLOAD_DESC = {
    "sphere64": "config 1: sphere shell r=28 in 64^3, 3x3x3 submanifold, 32->32 fp32",
    "indoor4": "config 2: 4 indoor-like grids in 512^3, 3x3x3 submanifold, 64->64 fp16",
    "lidar1m": "config 3: LiDAR-like 2048x2048x64 grid (~1M voxels), 3x3x3 submanifold, 64->64 bf16",
    "lidar1m_down": "config 4: config-3 grid, 2x2x2 stride 2, 64->128 bf16 (coarse grid + map + conv)",
    "sheets4": "config 5: 4 random-walk sheet grids in 128^3, 3x3x3 submanifold, 256->256 bf16",
    "lidar1m_down3": "config-3 grid, 3x3x3 stride 2, 64->128 bf16 (coarse grid + map + conv)",
    "volume1m": "volumetric class: solid balls and thick shells in 224^3 (~1M voxels, leaf occupancy 53 %), "
                "3x3x3 submanifold, 8->16 fp32",
    "volume1m_c64": "volumetric class: the volume1m grid, 3x3x3 submanifold, 64->64 bf16",
    "dense96": "dense class: a full 96^3 block (884 736 voxels), 3x3x3 submanifold, 64->64 bf16",
    "mixed1m": "mixed classes in one grid: LiDAR-like rings and boxes, thin shells and solid balls (697 301 voxels, 62 % of "
               "them in locally dense leaves), 3x3x3 submanifold, 64->64 bf16",
}


def accounting(n_in, n_out, pairs, k3, c_in, c_out, elem_bytes, out_bytes):
    """Algorithmic work of one step (what the method must compute / move, per the paper's
    effective-FLOP definition and the byte model of Sec. 3.5 scenario 1)."""
    flops = 2.0 * pairs * c_in * c_out
    conv_bytes = n_in * c_in * elem_bytes + n_out * c_out * out_bytes + k3 * c_in * c_out * elem_bytes
    kmap_bytes = n_out * k3 * 4                 # dense int32 map entries written by the lookup kernel
    grid_bytes = n_in * 12                      # ijk read once
    return flops, conv_bytes, kmap_bytes, grid_bytes


def pmc_summary(directory):
    """Per-kernel averages of the counters in a `rocprofv3 --pmc ... --output-format csv` run."""
    import collections
    import csv
    import glob
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        print(f"no *counter_collection.csv under {directory}", file=sys.stderr)
        sys.exit(1)
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for f in files:
        for row in csv.DictReader(open(f)):
            name = row["Kernel_Name"].replace("(anonymous namespace)::", "").split("(")[0]
            acc[name][row["Counter_Name"]].append(float(row["Counter_Value"]))
    for name in sorted(acc):
        for ctr, v in sorted(acc[name].items()):
            print(f"{name[:90]:90s} {ctr:28s} dispatches {len(v):4d}  mean {sum(v) / len(v):16.1f}  max {max(v):16.1f}")


KERNEL_SOURCES = {          # the files whose contents decide what a kernel moves through HBM
    "k_conv_mfma": ("conv.hip", "conv_common.h", "kmap.h"),
    "k_conv_gather": ("conv.hip", "conv_common.h", "kmap.h"),
    "k_build_tiles": ("kmap.hip", "kmap.h", "tree_device.h"),
}


def kernel_source_sha1(kernel):
    """Fingerprint of a kernel's sources: a committed counter summary is quoted only while it matches."""
    import hashlib
    h = hashlib.sha1()
    for f in KERNEL_SOURCES.get(kernel, ()):
        h.update(open(os.path.join(ROOT, "paper_2407_01781_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def committed_traffic(kernel, workload):
    """HBM bytes per launch measured with rocprofv3 counters (rocprofv3 cannot run inside this process; the
    FETCH_SIZE / WRITE_SIZE runs of this same command are summarised under profiles/ in
    <kernel>_<workload>_hbm_traffic.md: `traffic_bytes_per_launch: N` and `kernel_source_sha1: H`).  Returns
    (bytes, note): the figure is dropped, and the note says so, when the kernel's sources have changed since."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_hbm_traffic.md")
    traffic, sha = None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":", 1)[1])
            if line.startswith("kernel_source_sha1:"):
                sha = line.split(":", 1)[1].strip()
    except OSError:
        return None, "no counter summary committed for this kernel and workload"
    if traffic is None:
        return None, "no counter summary committed for this kernel and workload"
    if sha != kernel_source_sha1(kernel):
        return None, f"profiles/{os.path.basename(path)} was measured on other sources of this kernel ({sha}): not quoted"
    return traffic, f"profiles/{os.path.basename(path)}, sources {sha}"


def committed_valu_instructions(kernel, workload):
    """Vector-ALU wave instructions per launch from the committed SQ_INSTS_VALU summary of this command
    (profiles/<kernel>_<workload>_issue_counters.md: `valu_wave_instructions_per_launch: N` and the fingerprint of the
    kernel's sources); (None, note) when there is none or the sources have changed since."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_issue_counters.md")
    n, sha = None, None
    try:
        for line in open(path):
            if line.startswith("valu_wave_instructions_per_launch:"):
                n = float(line.split(":", 1)[1])
            if line.startswith("kernel_source_sha1:"):
                sha = line.split(":", 1)[1].strip()
    except OSError:
        return None, "no issue-counter summary committed for this kernel and workload"
    if n is None:
        return None, "no issue-counter summary committed for this kernel and workload"
    if sha != kernel_source_sha1(kernel):
        return None, f"profiles/{os.path.basename(path)} was measured on other sources of this kernel ({sha}): not quoted"
    return n, f"profiles/{os.path.basename(path)}, sources {sha}"


def gpu_clocks():
    """Current clock levels / power of the first GPU as the driver's sysfs files show them, when they are readable
    (plain file reads: no child process is started from a process that holds the GPU)."""
    import glob
    out = {}
    for card in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
        try:
            for key, name in (("sclk", "pp_dpm_sclk"), ("mclk", "pp_dpm_mclk"), ("fclk", "pp_dpm_fclk")):
                path = os.path.join(card, name)
                if os.path.exists(path):
                    cur = [l.split(":", 1)[1].replace("*", "").strip() for l in open(path) if "*" in l]
                    if cur:
                        out[key] = cur[0]
            perf = os.path.join(card, "power_dpm_force_performance_level")
            if os.path.exists(perf):
                out["performance_level"] = open(perf).read().strip()
            for hw in glob.glob(os.path.join(card, "hwmon", "hwmon*", "power1_average")):
                out["power_W"] = int(open(hw).read().strip()) / 1e6
        except OSError:
            continue
        if out:
            break
    return out or None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="lidar1m", choices=sorted(WORKLOAD_DESC))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-low-depth", action="store_true",
                    help="skip the extra section that times the map-free low-depth operator on the volumetric grid")
    ap.add_argument("--cpu-sample-rows", type=int, default=1000000)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch a plain elementwise copy kernel of known size (256 MiB read + 256 MiB "
                         "written), the yardstick for the FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--pmc-summary", metavar="DIR", help="print per-kernel counter averages of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.pmc_summary:
        pmc_summary(args.pmc_summary)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path would shard by grid of the batch, one grid per GPU, with no exchange in the forward pass); "
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

    if args.copy_calibration:
        src = torch.zeros(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)        # one vectorised elementwise kernel: 4 B read + 4 B written per element
        torch.cuda.synchronize()
        del src, dst

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
    tiled_bytes = km.tiled_bytes()
    n_leaf_out = km.g_out.counts()[0]
    flops, conv_bytes, kmap_bytes, grid_bytes = accounting(n_in, n_out, pairs, w.k3, w.c_in, w.c_out, elem, elem)
    out_buf = torch.empty_like(y)
    del g, km, y

    # ---- warm-up + timed steps (whole hot path).  The device's clocks climb for the first ~30 ms of continuous
    # work after an idle stretch (a 0.45 ms kernel measured 0.95, 0.50, 0.48, 0.46, 0.45 ms over its first fifty
    # launches), so the untimed part first runs the step for that long, then the W warm-up steps.
    t_pre = time.perf_counter()
    n_pre = 0
    while (time.perf_counter() - t_pre) < 0.05 and n_pre < 2000:
        step(out_buf)
        torch.cuda.synchronize()
        n_pre += 1
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
    t_w = time.perf_counter()
    while time.perf_counter() - t_w < 0.02:          # clocks, see above
        fx.sparse_conv_fwd(km, d_feat, d_w, out=out_buf)
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        fx.sparse_conv_fwd(km, d_feat, d_w, out=out_buf)
    e1.record()
    torch.cuda.synchronize()
    t_conv_b2b = e0.elapsed_time(e1) / 20

    # ---- backward pass on the same map (not part of `value`): warm, back to back
    d_gy = torch.randn(out_buf.shape, device="cuda").to(tdt).contiguous()

    def b2b(fn, reps=10):
        t_w = time.perf_counter()             # at least 20 ms of the same work first (clocks, see above), then timed
        for _ in range(200):
            fn()
            torch.cuda.synchronize()
            if time.perf_counter() - t_w > 0.02:
                break
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    # (outputs preallocated like the forward's: a fresh 100 MB tensor per call alternates between two blocks of
    # torch's allocator and the gradient then writes cold memory every time -- 0.52 instead of 0.43 ms at config 5)
    gin_buf = torch.empty((n_in, w.c_in), dtype=tdt, device="cuda")
    gw_buf = torch.empty((w.k3, w.c_in, w.c_out), dtype=tdt, device="cuda")
    t_dgrad = b2b(lambda: fx.sparse_conv_bwd_data(km, d_gy, d_w, out=gin_buf))
    t_wgrad = b2b(lambda: fx.sparse_conv_bwd_weight(km, d_feat, d_gy, out=gw_buf))
    del gin_buf, gw_buf

    # ---- the other operators of an encoder-decoder network on the same grid (not part of `value`):
    # factor-2 max pooling, nearest upsampling and the 2x2x2 stride-2 transposed convolution
    # (2*C -> C channels), warm, back to back, on the (2,2) kernel map of the input grid
    km2 = km if (w.kernel_size, w.stride) == (2, 2) else fx.build_kernel_map(g, 2, 2)
    n_c, c = km2.n_out, w.c_in
    d_fine = d_feat
    pooled = fx.pool2(km2, d_fine, "max")
    t_pool = b2b(lambda: fx.pool2(km2, d_fine, "max"))
    t_up = b2b(lambda: fx.upsample2(km2, pooled))
    move_bytes = (n_in + n_c) * c * elem + n_c * 8 * 4            # both sides' rows once + the dense (2,2) map
    ops = {"n_coarse": n_c, "channels": c,
           "max_pool_ms": t_pool, "max_pool_GBs": move_bytes / (t_pool * 1e-3) / 1e9,
           "upsample_ms": t_up, "upsample_GBs": move_bytes / (t_up * 1e-3) / 1e9,
           "algorithmic_bytes": move_bytes, "hbm_peak_GBs": HBM_PEAK_GBS}
    g_coarse = torch.randn(pooled.shape, device="cuda").to(tdt).contiguous()
    t_pool_b = b2b(lambda: fx.pool2_bwd(km2, g_coarse, "max", d_fine))
    t_up_b = b2b(lambda: fx.upsample2_bwd(km2, d_fine))
    ops["max_pool_bwd_ms"] = t_pool_b                      # reads the fine input and the coarse gradient, writes the fine gradient
    ops["max_pool_bwd_GBs"] = (move_bytes + n_in * c * elem) / (t_pool_b * 1e-3) / 1e9
    ops["upsample_bwd_ms"] = t_up_b
    ops["upsample_bwd_GBs"] = move_bytes / (t_up_b * 1e-3) / 1e9
    ops["max_pool_frac"] = ops["max_pool_GBs"] / HBM_PEAK_GBS
    ops["upsample_frac"] = ops["upsample_GBs"] / HBM_PEAK_GBS
    if w.dtype != "f32":
        d_coarse = torch.randn((n_c, 2 * c), device="cuda").to(tdt).contiguous()
        d_wt = (torch.randn((8, 2 * c, c), device="cuda") * (1.0 / (8 * 2 * c)) ** 0.5).to(tdt).contiguous()
        t_tc = b2b(lambda: fx.sparse_conv_transpose_fwd(km2, d_coarse, d_wt))
        ops["conv_transpose_ms"] = t_tc
        ops["conv_transpose_effective_TFLOPs"] = 2.0 * n_in * 2 * c * c / (t_tc * 1e-3) / 1e12
        tc_bytes = (n_c * 2 * c + n_in * c) * elem
        ops["conv_transpose_GBs"] = tc_bytes / (t_tc * 1e-3) / 1e9
    # the grids of the two directions, made from the input grid's leaves: the coarse grid of pooling / strided
    # convolution and the subdivided grid of upsampling (8 children per voxel)
    ops["grid_coarsen_ms"] = b2b(lambda: g.coarsen2(), reps=5)
    if 8 * n_in <= 2 ** 31 - 1:
        g_fine = g.subdivide2()
        ops["grid_subdivide_ms"] = b2b(lambda: g.subdivide2(), reps=5)
        ops["n_fine"] = g_fine.num_voxels
        del g_fine
    del pooled

    # ---- the low-depth operator (Sec. 3.5 scenario 1) on the volumetric class of Sec. 4.1.3 (leaf occupancy
    # above 40 %), 8 -> 16 channels at fp32, straight from the grid; next to it the same convolution through
    # the kernel map (not part of `value`)
    low_depth = None
    if not args.no_low_depth:
        wv = G.workload("volume1m")
        v_ijk, v_jo = wv.jagged_ijk()
        gv = fx.build_index_grid(torch.from_numpy(v_ijk).cuda(), v_jo)
        nv = gv.num_voxels
        v_feat = torch.randn((nv, wv.c_in), device="cuda")
        v_w = torch.randn((27, wv.c_in, wv.c_out), device="cuda") * (1.0 / (27 * wv.c_in)) ** 0.5
        t_leaf = b2b(lambda: fx.sparse_conv_leaf_fwd(gv, v_feat, v_w))
        kmv = fx.build_kernel_map(gv, 3, 1)
        v_pairs = kmv.info()[0]
        t_kmv = b2b(lambda: fx.build_kernel_map(gv, 3, 1), reps=5)
        fx.set_option("leaf_dispatch", 0)        # the comparison figures are the kernel-map kernels'
        t_cv = b2b(lambda: fx.sparse_conv_fwd(kmv, v_feat, v_w), reps=5)
        v_flops = 2.0 * v_pairs * wv.c_in * wv.c_out
        v_bytes = nv * (wv.c_in + wv.c_out) * 4 + 27 * wv.c_in * wv.c_out * 4 + 96 * gv.counts()[0]
        low_depth = {"workload": "volume1m: solid balls and thick shells in 224^3, 3x3x3 submanifold, 8->16 fp32",
                     "n_voxels": nv, "n_leaves": gv.counts()[0], "active_pairs": v_pairs,
                     "leaf_conv_ms": t_leaf, "leaf_conv_effective_TFLOPs": v_flops / (t_leaf * 1e-3) / 1e12,
                     "frac_of_fp32_mfma_peak": v_flops / (t_leaf * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS["f32"],
                     "algorithmic_bytes": v_bytes, "GBs": v_bytes / (t_leaf * 1e-3) / 1e9,
                     "frac_of_hbm_peak": v_bytes / (t_leaf * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "kernel_map_path_ms": {"kernel_map": t_kmv, "conv": t_cv}}
        # its weight gradient from the same window, against the scalar kernel over the kernel map
        v_gy = torch.randn((nv, wv.c_out), device="cuda")
        t_lw = b2b(lambda: fx.sparse_conv_leaf_bwd_weight(gv, v_feat, v_gy))
        t_sw = b2b(lambda: fx.sparse_conv_bwd_weight(kmv, v_feat, v_gy), reps=3)      # dispatch is off here: the scalar kernel
        low_depth["leaf_bwd_weight_ms"] = t_lw
        low_depth["leaf_bwd_weight_effective_TFLOPs"] = v_flops / (t_lw * 1e-3) / 1e12
        low_depth["kernel_map_path_ms"]["bwd_weight_scalar"] = t_sw
        # the same grid at 64 -> 64 bf16: the leaf-window kernel for 16-bit types against the kernel-map path
        h_feat = torch.randn((nv, 64), device="cuda").to(torch.bfloat16)
        h_w = (torch.randn((27, 64, 64), device="cuda") * (1.0 / (27 * 64)) ** 0.5).to(torch.bfloat16)
        t_l16 = b2b(lambda: fx.sparse_conv_leaf_fwd(gv, h_feat, h_w), reps=5)
        t_c16 = b2b(lambda: fx.sparse_conv_fwd(kmv, h_feat, h_w), reps=5)
        h_gy = torch.randn((nv, 64), device="cuda").to(torch.bfloat16)
        t_lw16 = b2b(lambda: fx.sparse_conv_leaf_bwd_weight(gv, h_feat, h_gy), reps=5)
        t_tw16 = b2b(lambda: fx.sparse_conv_bwd_weight(kmv, h_feat, h_gy), reps=3)      # dispatch is off: the tile kernel
        fx.set_option("leaf_dispatch", -1)
        h_flops = 2.0 * v_pairs * 64 * 64
        low_depth["leaf_window_bf16_64"] = {
            "leaf_conv_ms": t_l16, "leaf_conv_effective_TFLOPs": h_flops / (t_l16 * 1e-3) / 1e12,
            "frac_of_bf16_mfma_peak": h_flops / (t_l16 * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS["bf16"],
            "leaf_bwd_weight_ms": t_lw16, "leaf_bwd_weight_effective_TFLOPs": h_flops / (t_lw16 * 1e-3) / 1e12,
            "kernel_map_path_ms": {"kernel_map": t_kmv, "conv": t_c16, "bwd_weight_tiles": t_tw16}}
        del kmv, gv, v_feat, h_feat, h_gy

    # ---- per-leaf dispatch (the paper's future-work item; Sec. 3.5's scenarios are its regimes) on a grid that mixes
    # the sparsity classes: the same convolution through the tile kernel alone, the leaf-window kernel alone, and
    # split per leaf inside one call (not part of `value`)
    per_leaf = None
    if not args.no_low_depth:
        wm = G.workload("mixed1m")
        m_ijk, m_jo = wm.jagged_ijk()
        gm = fx.build_index_grid(torch.from_numpy(m_ijk).cuda(), m_jo)
        kmm = fx.build_kernel_map(gm, 3, 1)
        m_pairs = kmm.info()[0]
        m_feat = torch.randn((gm.num_voxels, 64), device="cuda").to(torch.bfloat16)
        m_w = (torch.randn((27, 64, 64), device="cuda") * (1.0 / (27 * 64)) ** 0.5).to(torch.bfloat16)
        m_out = torch.empty((gm.num_voxels, 64), dtype=torch.bfloat16, device="cuda")
        per_leaf = {"workload": WORKLOAD_DESC["mixed1m"], "n_voxels": gm.num_voxels, "n_leaves": gm.counts()[0], "active_pairs": m_pairs}
        for sw, key in ((0, "tile_kernel_only_ms"), (1, "leaf_window_kernel_only_ms"), (-1, "automatic_per_leaf_dispatch_ms")):
            fx.set_option("leaf_dispatch", sw)
            per_leaf[key] = b2b(lambda: fx.sparse_conv_fwd(kmm, m_feat, m_w, out=m_out), reps=5)
        fx.set_option("leaf_dispatch", -1)
        per_leaf["automatic_effective_TFLOPs"] = 2.0 * m_pairs * 64 * 64 / (per_leaf["automatic_per_leaf_dispatch_ms"] * 1e-3) / 1e12
        del kmm, gm, m_feat, m_out

    # ---- grid build from xyz points (Sec. 4.1.1's benchmark input: normally distributed points), 10 M points,
    # sigma = 100 voxels (not part of `value`)
    points_build = None
    if not args.no_low_depth:
        n_pts = 10_000_000
        d_xyz = torch.from_numpy(G.gaussian_point_cloud(7000, n_pts, 1.0)).cuda()
        pjo = np.array([[0, n_pts]], dtype=np.int64)
        gp = fx.build_index_grid_from_points(d_xyz, pjo, (0.0, 0.0, 0.0), (0.01, 0.01, 0.01))
        t_pts = b2b(lambda: fx.build_index_grid_from_points(d_xyz, pjo, (0.0, 0.0, 0.0), (0.01, 0.01, 0.01)), reps=5)
        points_build = {"n_points": n_pts, "n_voxels": gp.num_voxels, "n_leaves": gp.counts()[0], "ms": t_pts,
                        "Mpoints_per_s": n_pts / (t_pts * 1e-3) / 1e6,
                        "algorithmic_bytes": 12 * n_pts + 96 * gp.counts()[0],
                        "GBs": (12 * n_pts + 96 * gp.counts()[0]) / (t_pts * 1e-3) / 1e9}
        points_build["frac_of_hbm_peak"] = points_build["GBs"] / HBM_PEAK_GBS
        del gp, d_xyz

    # ---- convolution onto the padded grid (Sec. 3.6.2: a grid made by padding; the output set of a 3x3x3 convolution
    # that is not restricted to the input's voxels): grid padding, the map onto it, forward and both gradients at
    # the workload's channels (not part of `value`)
    padded_output = None
    if not args.no_low_depth and (w.kernel_size, w.stride) == (3, 1):
        gpad = g.pad(1)
        t_pad = b2b(lambda: g.pad(1), reps=3)
        kmp = fx.build_kernel_map_onto(g, gpad, 3)
        t_kmp = b2b(lambda: fx.build_kernel_map_onto(g, gpad, 3), reps=3)
        p_pairs = kmp.info()[0]
        d_gyp = torch.randn((gpad.num_voxels, w.c_out), device="cuda").to(tdt).contiguous()
        t_pf = b2b(lambda: fx.sparse_conv_fwd(kmp, d_feat, d_w), reps=5)
        t_pd = b2b(lambda: fx.sparse_conv_bwd_data(kmp, d_gyp, d_w), reps=5)
        t_pw = b2b(lambda: fx.sparse_conv_bwd_weight(kmp, d_feat, d_gyp), reps=5)
        p_flops = 2.0 * p_pairs * w.c_in * w.c_out
        padded_output = {"n_voxels_padded": gpad.num_voxels, "n_leaves_padded": gpad.counts()[0], "active_pairs": p_pairs,
                         "grid_pad_ms": t_pad, "kernel_map_onto_ms": t_kmp, "conv_ms": t_pf,
                         "conv_effective_TFLOPs": p_flops / (t_pf * 1e-3) / 1e12,
                         "bwd_data_ms": t_pd, "bwd_weight_ms": t_pw}
        del kmp, gpad, d_gyp

    # ---- the paper's timing protocol (Sec. 4.1: one warm-up, five timed runs, mean of the best
    # four), cold = a 768 MiB scratch buffer is overwritten before every run so that neither the
    # L2s nor the 256 MB last-level cache hold the operands, warm = no flush
    def protocol(fn, flush):
        scratch = torch.empty(768 << 20, dtype=torch.uint8, device="cuda") if flush else None
        ts = []
        for r in range(6):
            if flush:
                scratch.fill_(r)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        return float(np.sort(ts[1:])[:4].mean())

    conv_fn = lambda: fx.sparse_conv_fwd(km, d_feat, d_w, out=out_buf)
    kmap_fn = lambda: fx.build_kernel_map(g, w.kernel_size, w.stride)
    grid_fn = lambda: fx.build_index_grid(d_ijk, joffsets)
    paper_protocol = {
        "conv_cold_ms": protocol(conv_fn, True), "conv_warm_ms": protocol(conv_fn, False),
        "kernel_map_cold_ms": protocol(kmap_fn, True), "kernel_map_warm_ms": protocol(kmap_fn, False),
        "grid_build_cold_ms": protocol(grid_fn, True), "grid_build_warm_ms": protocol(grid_fn, False),
    }
    paper_protocol["conv_cold_effective_TFLOPs"] = flops / (paper_protocol["conv_cold_ms"] * 1e-3) / 1e12

    dom = next(k for k in ("k_conv_mfma", "k_conv_gather", "k_conv_leaf", "k_conv_scalar") if k in kern_ms)
    dom_ms = kern_ms[dom]
    # Both roofs of the dominant kernel.  Algorithmic bytes of one launch: every input row and every output row once,
    # the weights once, and the kernel map in the form the kernel reads (the tiled map's bytes).  The binding roof is
    # min(matrix peak, intensity x HBM peak); `bound` names it and `frac_of_binding_roof` is measured against it.
    peak = MFMA_PEAK_TFLOPS[w.dtype] if dom != "k_conv_scalar" else FP32_VALU_PEAK_TFLOPS
    achieved = flops / (dom_ms * 1e-3) / 1e12
    conv_bytes_with_map = conv_bytes + (tiled_bytes if dom in ("k_conv_mfma", "k_conv_gather") else (kmap_bytes if dom == "k_conv_scalar" else 0))
    intensity = flops / conv_bytes_with_map
    hbm_roof_tflops = intensity * HBM_PEAK_GBS / 1e3
    binding = min(peak, hbm_roof_tflops)
    roof = {"kernel": dom, "bound": ("hbm" if hbm_roof_tflops < peak else ("mfma" if dom != "k_conv_scalar" else "alu")),
            "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
            "intensity_flop_per_byte": intensity, "hbm_roof_TFLOPs": hbm_roof_tflops,
            "binding_roof_TFLOPs": binding, "frac_of_binding_roof": achieved / binding}
    roof["traffic"], roof["traffic_source"] = committed_traffic(dom, args.workload)
    roof["avg_launch_ms"] = dom_ms
    roof["hbm_view"] = {"algorithmic_bytes": conv_bytes_with_map, "of_which_kernel_map": conv_bytes_with_map - conv_bytes,
                        "GB/s": conv_bytes_with_map / (dom_ms * 1e-3) / 1e9,
                        "frac_of_8TBs": conv_bytes_with_map / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    # map build: bytes of the tiled map actually written + the 96-byte leaf records read once
    bt_ms = kern_ms.get("k_build_tiles")
    kmap_roof = None
    if bt_ms:
        bt_bytes = tiled_bytes + 96 * n_leaf_out
        kmap_roof = {"kernel": "k_build_tiles", "bound": "hbm", "achieved": bt_bytes / (bt_ms * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "avg_launch_ms": bt_ms, "algorithmic_bytes": bt_bytes,
                     "dense_map_equivalent_GBs": kmap_bytes / (bt_ms * 1e-3) / 1e9,
                     "traffic": committed_traffic("k_build_tiles", args.workload)[0],
                     "traffic_source": committed_traffic("k_build_tiles", args.workload)[1]}
        kmap_roof["frac"] = kmap_roof["achieved"] / HBM_PEAK_GBS
        # What binds this kernel is the issue of vector-ALU instructions (integer work: bit tests, popcounts, a
        # sort, address arithmetic), not memory: the instructions it executes per launch (counter summary under
        # profiles/) against the chip's vector issue rate, 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-operations/s.
        valu, valu_src = committed_valu_instructions("k_build_tiles", args.workload)
        if valu:
            lane_ops = valu * 64
            kmap_roof["alu_view"] = {"bound": "alu", "unit": "Tlane-op/s", "peak": VALU_PEAK_TLANEOPS,
                                     "valu_wave_instructions_per_launch": valu, "source": valu_src,
                                     "achieved": lane_ops / (bt_ms * 1e-3) / 1e12,
                                     "frac": lane_ops / (bt_ms * 1e-3) / 1e12 / VALU_PEAK_TLANEOPS}
        else:
            kmap_roof["alu_view"] = {"bound": "alu", "source": valu_src}

    # grid build: the rows read once plus the leaf table written (Sec. 3.3; no sort passes here)
    n_leaf_in = g.counts()[0]
    gb_bytes = grid_bytes + 96 * n_leaf_in
    grid_roof = {"stage": "build_index_grid", "bound": "hbm", "achieved": gb_bytes / (t_grid * 1e-3) / 1e9,
                 "peak": HBM_PEAK_GBS, "unit": "GB/s", "stage_ms": float(t_grid), "algorithmic_bytes": gb_bytes}
    grid_roof["frac"] = grid_roof["achieved"] / HBM_PEAK_GBS

    result = {
        "metric": "sparse conv effective TFLOP/s (active pairs), whole hot path: grid build + kernel map + conv",
        "value": flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "pre_warm_steps": n_pre, "ms_per_step": ms_per_step,
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
        "backward": {"bwd_data_ms": t_dgrad, "bwd_weight_ms": t_wgrad,
                     "bwd_data_effective_TFLOPs": flops / (t_dgrad * 1e-3) / 1e12,
                     "bwd_weight_effective_TFLOPs": flops / (t_wgrad * 1e-3) / 1e12},
        "encoder_decoder_ops": ops,
        "low_depth": low_depth,
        "grid_from_points": points_build,
        "padded_output": padded_output,
        "per_leaf_dispatch": per_leaf,
        "kernels_ms_per_launch": kern_ms,
        "kernels_ms_per_step": per_step_ms,
        "clocks": gpu_clocks(),
        "roofline": roof,
        "roofline_kernel_map": kmap_roof,
        "roofline_grid_build": grid_roof,
        "paper_protocol": paper_protocol,
    }

    # ---- CPU oracle on this machine's host cores: the oracle as it stands, on a bounded sample.  One thread first
    # (the headline of this leg), then the convolution again with its output rows cut over all host cores (the same
    # C routine on disjoint row ranges, one host thread per range).
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
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
        cores = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
        t = time.perf_counter()
        O.conv(og, ogo, w.kernel_size, w.stride, f64, w64, 0, rows, threads=cores)
        t_o3_mt = time.perf_counter() - t
        result["cpu_baseline"] = {
            "value": flops / (t_o1 + t_o2 + t_o3_full) / 1e12, "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
            "sample": f"grid build and kernel map on the full input ({t_o1:.2f} s, {t_o2:.2f} s); convolution "
                      f"on the first {rows} of {n_out} output rows ({t_o3:.2f} s), scaled by active pairs",
            "conv_only_TFLOPs": 2.0 * sample_pairs * w.c_in * w.c_out / t_o3 / 1e12,
            "all_cores": {"cores": cores, "conv_only_TFLOPs": 2.0 * sample_pairs * w.c_in * w.c_out / t_o3_mt / 1e12,
                          "conv_seconds": t_o3_mt,
                          "note": "the same oracle routine on disjoint ranges of output rows, one host thread per range"},
            "host_cpus": os.cpu_count(),
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
