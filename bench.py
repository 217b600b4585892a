#!/usr/bin/env python3
"""Benchmark of the statically batched MoE expert GEMM on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: build the task
map from the routing (histogram, scans, token index arrays) and run the grouped GEMM kernel.
Inputs are resident in HBM before the timed region.  The headline workload is the
Mixtral-8x7B-shaped fused gate+up projection at T=4096 (E=8, top-2, K=4096, N=28672, bf16);
`--points all` also times the other synthetic configurations and reports them in "points".

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2501_16103_amd import binding as mb  # noqa: E402
from paper_2501_16103_amd import workloads as wk  # noqa: E402

# Published MI355X peaks the fractions are taken against.
PEAK_BF16_TFLOPS = 2516.6   # dense bf16 MFMA (256 CUs x 2.4 GHz x 4096 FLOP/clk/CU)
PEAK_FP8_TFLOPS = 5033.2    # dense fp8 MFMA
PEAK_HBM_GBS = 8000.0

# HBM bytes per GEMM launch as measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE; each scaled by what the same
# counter reads for a plain copy of known size) are not something this run can measure itself: they are read from
# a small tracked file that names the command and the source revision they came from.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def measured_traffic(workload: str):
    """(bytes per launch, provenance) recorded for `workload` in profiles/hbm_traffic.json, or (None, None)."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f).get(workload)
    except (OSError, ValueError):
        return None, None
    if not rec:
        return None, None
    return rec.get("bytes_per_launch"), {k: rec.get(k) for k in ("source", "commit", "command")}


def algorithmic_bytes(wl: wk.Workload, ids: torch.Tensor, swiglu: bool = False) -> int:
    """Weights of every touched expert once + X once + Y once + the map."""
    es = 1 if wl.dtype == "fp8" else 2
    touched = int(torch.unique(ids).numel())
    b = touched * wl.K * wl.N * es + wl.T * wl.K * es + wl.R * (wl.N // 2 if swiglu else wl.N) * 2 + 4 * (wl.R + 3 * wl.E)
    if wl.dtype == "fp8":
        b += 4 * (wl.T + wl.E)
    return b


class Point:
    """Device buffers of one workload (optionally several weight copies to defeat the caches)."""

    def __init__(self, wl: wk.Workload, copies: int = 1, dev="cuda:0", order: int = 0, small=(0, 0), swiglu: bool = False,
                 w_nk: bool = False, launch_mode: int = 0, tail_split: bool = False):
        self.wl = wl
        self.w_nk = w_nk      # weights pre-packed as [E][N][K] (a labelled extra, never the headline)
        self.swiglu = swiglu  # fused gated activation: Y is [R, N/2]
        self.order = order
        self.small = small  # (tile_m_small, small_max_rows) of the second tiling strategy, or (0, 0)
        self.slack = 0 if small[0] else wl.tile_m_slack  # no kernel combines the two
        if w_nk and self.slack == 32:
            self.slack = 64   # the pre-packed layout has the 64-row slack kernel only
        self.dev = dev
        self.ids_cpu = wk.make_routing(wl)
        self.ids = self.ids_cpu.to(dev)
        self.xs = self.ws = None
        if wl.dtype == "fp8":
            X, xs = wk.make_x(wl, dev)
            W, ws = wk.make_w(wl, dev)
            self.X, self.xs, self.ws = X, xs, ws
        else:
            self.X = wk.make_x(wl, dev)
            W = wk.make_w(wl, dev)
        if w_nk:
            Wt = torch.empty((wl.E, wl.N, wl.K), dtype=W.dtype, device=dev)
            for e in range(wl.E):   # expert by expert: no second full-size temporary
                Wt[e].copy_(W[e].t())
            W = Wt
        self.W = [W] + [W.clone() for _ in range(copies - 1)]
        self.Y = torch.empty((wl.R, wl.N // 2 if swiglu else wl.N), dtype=torch.bfloat16, device=dev)
        self.tmap = mb.alloc_task_map(wl.T, wl.k, wl.E, wl.tile_m, wl.tile_n, wl.N, dev)
        dt = mb.MOE_DTYPE_FP8_E4M3 if wl.dtype == "fp8" else mb.MOE_DTYPE_BF16
        self.desc = mb.GemmDesc(dt, wl.T, wl.k, wl.E, wl.K, wl.N, wl.tile_m, wl.tile_n, self.xs, self.ws, *small, self.slack,
                                mb.MOE_EPILOGUE_SWIGLU if swiglu else mb.MOE_EPILOGUE_NONE,
                                mb.MOE_W_LAYOUT_NK if w_nk else mb.MOE_W_LAYOUT_KN, launch_mode)
        self.launch_mode = launch_mode
        # the tiles of a partly filled last round split along K (moe_grouped_gemm_tail_split; 64 MiB workspace)
        self.tail_ws = (torch.empty(mb.moe_tail_split_workspace_bytes(wl.tile_m, wl.tile_n) // 4, dtype=torch.float32, device=dev)
                        if tail_split else None)
        self.tiling = mb.Tiling(wl.tile_m, wl.tile_n, order, small[0], small[1], self.slack)

    def build_map(self):
        wl = self.wl
        mb.moe_build_task_map_ex(self.ids, wl.T, wl.k, wl.E, wl.N, self.tiling, self.tmap)

    def gemm(self, i: int = 0):
        if self.tail_ws is not None:
            mb.moe_grouped_gemm_tail_split(self.X, self.W[i % len(self.W)], self.tmap, self.Y, self.desc, self.tail_ws)
        else:
            mb.moe_grouped_gemm(self.X, self.W[i % len(self.W)], self.ids, self.tmap, self.Y, self.desc)

    def time(self, steps: int, warmup: int):
        """Returns (wall ms per step, mean GEMM-kernel ms, mean map-build ms) over `steps` steps.

        Wall time brackets exactly `steps` steps with device synchronisation.  Kernel durations come from
        HIP events on the launch stream in a second pass of the same steps, enqueued behind a short device
        spin so that host launch latency (comparable to the decode kernels) does not show up as GPU idle
        time between two events."""
        for i in range(warmup):
            self.build_map()
            self.gemm(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.build_map()
            self.gemm(i)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        torch.cuda._sleep(int(4e6))
        for i in range(steps):
            ev[i][0].record()
            self.build_map()
            ev[i][1].record()
            self.gemm(i)
            ev[i][2].record()
        torch.cuda.synchronize()
        g = [e[1].elapsed_time(e[2]) for e in ev]
        gemm_ms = float(np.mean(g))
        map_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
        self.gemm_ms_median, self.gemm_ms_min = float(np.median(g)), float(np.min(g))
        # the same launches back to back (one map, no event between them): what rocprofv3's per-kernel durations
        # correspond to, since an event pair around a single short launch also sees its dispatch latency
        b = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        torch.cuda._sleep(int(4e6))
        b[0].record()
        for i in range(steps):
            self.gemm(i)
        b[1].record()
        torch.cuda.synchronize()
        self.gemm_ms_b2b = b[0].elapsed_time(b[1]) / steps
        return wall_ms, gemm_ms, map_ms

    def time_graph(self, steps: int) -> float:
        """Wall ms per step when map build + GEMM are captured once in a HIP graph and replayed: what a serving
        loop pays in the launch-bound regime (the eager figure includes two to four host launches per step)."""
        self.build_map()
        self.gemm(0)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                per_graph = max(8, len(self.W))   # several steps per graph: replays rotate the weight copies too
                for i in range(per_graph):
                    self.build_map()
                    self.gemm(i)
        torch.cuda.synchronize()
        reps = max(1, steps // per_graph)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / (reps * per_graph)

    def report(self, steps: int, warmup: int) -> dict:
        wl = self.wl
        wall_ms, gemm_ms, map_ms = self.time(steps, warmup)
        peak_t = PEAK_FP8_TFLOPS if wl.dtype == "fp8" else PEAK_BF16_TFLOPS
        abytes = algorithmic_bytes(wl, self.ids_cpu, self.swiglu)
        tf_step = wl.flops / (wall_ms * 1e-3) / 1e12
        tf_gemm = wl.flops / (gemm_ms * 1e-3) / 1e12
        gbs = abytes / (gemm_ms * 1e-3) / 1e9
        ideal_mfma = wl.flops / (peak_t * 1e12)
        ideal_hbm = abytes / (PEAK_HBM_GBS * 1e9)
        bound = "mfma" if ideal_mfma >= ideal_hbm else "hbm"
        return dict(workload=f"{wl.name}_T{wl.T}" + ("_swiglu" if self.swiglu else "") + ("_wNK" if self.w_nk else ""), dtype=wl.dtype, T=wl.T, E=wl.E, k=wl.k, K=wl.K, N=wl.N,
                    tile=[wl.tile_m, wl.tile_n], sigma_order=("ascending", "spread", "interleave")[self.order], small_strategy=list(self.small), tile_m_slack=self.slack, ms_per_step=round(wall_ms, 4),
                    ms_per_step_graph=(round(self.time_graph(steps), 4) if wall_ms < 0.5 else None), gemm_ms=round(gemm_ms, 4),
                    gemm_ms_median=round(self.gemm_ms_median, 4), gemm_ms_min=round(self.gemm_ms_min, 4),
                    gemm_ms_back_to_back=round(self.gemm_ms_b2b, 4),
                    frac_hbm_back_to_back=round(abytes / (self.gemm_ms_b2b * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                    map_ms=round(map_ms, 4), tflops_step=round(tf_step, 2), tflops_gemm=round(tf_gemm, 2),
                    frac_mfma=round(tf_gemm / peak_t, 4), gbs_gemm=round(gbs, 1),
                    frac_hbm=round(gbs / PEAK_HBM_GBS, 4), bound=bound, alg_bytes=abytes, flops=wl.flops,
                    launch_mode=self.launch_mode, tail_split=self.tail_ws is not None,
                    kernel="moe_gemm_pipe_kernel")


def cpu_baseline(pt: Point, target_s: float = 30.0) -> dict:
    """Time the CPU oracle (as it stands) on a bounded sample of complete routed rows of the same
    workload, and check the GPU output on those rows against it."""
    import oracle
    from tests import helpers as H
    wl = pt.wl
    rng = np.random.default_rng(0)
    Xh = wk.bits(pt.X)
    ids_h = pt.ids_cpu.numpy()
    # the oracle reads one expert's weights per row: copy to the host only the experts sampled
    n_probe = 8
    rows = rng.choice(wl.R, size=min(wl.R, 4096), replace=False).astype(np.int32)
    experts = sorted(set(int(ids_h.reshape(-1)[r]) for r in rows))
    remap = {e: i for i, e in enumerate(experts)}
    Wh = np.stack([wk.bits(pt.W[0][e]) for e in experts])
    ids_local = np.full(wl.R, 0, dtype=np.int32)
    for r in rows:
        ids_local[r] = remap[int(ids_h.reshape(-1)[r])]
    ids_local = ids_local.reshape(wl.T, wl.k)

    def run(rsel):
        t0 = time.perf_counter()
        if wl.dtype == "fp8":
            res = oracle.grouped_gemm_fp8(Xh, Wh, pt.xs.cpu().numpy(), pt.ws.cpu().numpy()[experts], ids_local, rows=rsel)
        else:
            res = oracle.grouped_gemm_bf16(Xh, Wh, ids_local, rows=rsel)
        return res, time.perf_counter() - t0

    res, dt = run(rows[:n_probe])
    per_row = dt / n_probe
    n = int(max(n_probe, min(len(rows), target_s / max(per_row, 1e-9))))
    res, dt = run(rows[:n])
    flops = 2.0 * n * wl.K * wl.N
    # parity of the GPU result on the same rows
    got = H.y_bits(pt.Y[torch.from_numpy(rows[:n].astype(np.int64)).to(pt.dev)])
    ulp = H.ulp_distance(got, res.Ybf)
    err = np.abs(H.bf16_bits_to_f64(got) - res.Y64)
    return dict(value=round(flops / dt / 1e12, 6), unit="TFLOP/s", cores=oracle.num_threads(), kind="oracle",
                sample=f"{n} complete routed rows of {wl.name}_T{wl.T} ({flops / 1e9:.1f} GFLOP, {dt:.1f} s)",
                gpu_vs_oracle=dict(rows=n, max_abs_err=float(err.max()), frac_bit_equal=float((ulp == 0).mean())))


HEADLINE = "mixtral_up_T4096"


def weight_copies(w: wk.Workload) -> int:
    """fp8 decode points: the touched weights (35-354 MB) are comparable to the 256 MB last-level cache, so the
    launches rotate over enough full copies that none finds its experts cached by an earlier one."""
    if w.dtype != "fp8":
        return 1
    touched = int(torch.unique(wk.make_routing(w)).numel()) * w.K * w.N
    return min(16, max(4, -(-int(1.2e9) // touched)))


def decode_hbm_points(steps: int, warmup: int, with_cpu: bool) -> list:
    """The second half of the metric: the fp8 decode configuration (E=64, top-6, K=2048, N=2816) at T = 1, 8, 32,
    priced against the HBM peak.  `achieved` = algorithmic bytes / duration of one GEMM launch, the launches of one
    map timed back to back with HIP events on the launch stream (what a kernel trace's per-kernel durations
    correspond to).  Beside each: the CPU oracle on the WHOLE problem (seconds, threads) and the GPU result
    checked against it."""
    out = []
    for T in (1, 8, 32):
        w = wk.decode_fp8(T)
        p = Point(w, weight_copies(w))
        wall_ms, gemm_ms, map_ms = p.time(steps, warmup)
        abytes = algorithmic_bytes(w, p.ids_cpu)
        ms = p.gemm_ms_b2b
        gbs = abytes / (ms * 1e-3) / 1e9
        rec = {"workload": f"{w.name}_T{T}", "bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS,
               "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4), "kernel_ms": round(ms, 5),
               "kernel_ms_single_launch_events": round(gemm_ms, 5), "map_ms": round(map_ms, 5),
               "ms_per_step": round(wall_ms, 5), "alg_bytes": abytes, "tile": [w.tile_m, w.tile_n],
               "weight_copies": len(p.W), "tflops": round(w.flops / (ms * 1e-3) / 1e12, 2)}
        if with_cpu:
            import oracle
            from tests import helpers as H
            p.build_map()
            p.gemm(0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            res = oracle.grouped_gemm_fp8(wk.bits(p.X), wk.bits(p.W[0]), p.xs.cpu().numpy(), p.ws.cpu().numpy(),
                                          p.ids_cpu.numpy())
            dt = time.perf_counter() - t0
            got = H.y_bits(p.Y)
            err = np.abs(H.bf16_bits_to_f64(got) - res.Y64)
            rec["cpu_oracle"] = {"seconds": round(dt, 4), "cores": oracle.num_threads(), "sample": "the whole problem",
                                 "gb_per_s": round(abytes / dt / 1e9, 2),
                                 "gpu_vs_oracle": {"max_abs_err": float(err.max()),
                                                   "frac_bit_equal": float((H.ulp_distance(got, res.Ybf) == 0).mean())}}
        out.append(rec)
        del p
        torch.cuda.empty_cache()
    return out


def combine_point(T: int, k: int, N: int, steps: int, warmup: int, dev="cuda:0") -> dict:
    """The sum over a token's experts on a [T, k, N] bf16 product: pure streaming, priced against HBM."""
    g = torch.Generator(device=dev).manual_seed(wk.BASE_SEED + T + k)
    Y = torch.randn((T * k, N), generator=g, device=dev).to(torch.bfloat16)
    w = torch.rand((T, k), generator=g, device=dev, dtype=torch.float32)
    out = torch.empty((T, N), dtype=torch.bfloat16, device=dev)
    for _ in range(warmup):
        mb.moe_combine(Y, w, T, k, N, out)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    torch.cuda._sleep(int(4e6))
    for i in range(steps):
        ev[i][0].record()
        mb.moe_combine(Y, w, T, k, N, out)
        ev[i][1].record()
    torch.cuda.synchronize()
    ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    nbytes = T * k * N * 2 + T * N * 2 + T * k * 4
    gbs = nbytes / (ms * 1e-3) / 1e9
    return dict(workload=f"combine_T{T}_k{k}_N{N}", dtype="bf16", T=T, k=k, N=N, kernel_ms=round(ms, 4),
                gbs=round(gbs, 1), frac_hbm=round(gbs / PEAK_HBM_GBS, 4), bound="hbm", alg_bytes=nbytes)


def batched_point(wl: wk.Workload, rT: int, rk: int, rN: int, steps: int, warmup: int, dev="cuda:0") -> dict:
    """Heterogeneous batching (Sec. 3.2): the GEMM of `wl` with a reduction task (the weighted sum over [rT, rk, rN]
    finished products of an earlier call) in the same launch, against the two separate calls back to back."""
    p = Point(wl)
    g = torch.Generator(device=dev).manual_seed(wk.BASE_SEED + rT)
    Yin = torch.randn((rT * rk, rN), generator=g, device=dev).to(torch.bfloat16)
    w = torch.rand((rT, rk), generator=g, device=dev, dtype=torch.float32)
    out = torch.empty((rT, rN), dtype=torch.bfloat16, device=dev)
    p.build_map()

    def both():
        mb.moe_grouped_gemm(p.X, p.W[0], p.ids, p.tmap, p.Y, p.desc)
        mb.moe_combine(Yin, w, rT, rk, rN, out)

    def batched():
        mb.moe_grouped_gemm_batched(p.X, p.W[0], p.tmap, p.Y, p.desc, Yin, w, rT, rk, rN, out)

    res = {}
    for name, fn in (("separate", both), ("batched", batched), ("separate_again", both), ("batched_again", batched)):
        for _ in range(warmup):
            fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        torch.cuda._sleep(int(4e6))
        ev[0].record()
        for _ in range(steps):
            fn()
        ev[1].record()
        torch.cuda.synchronize()
        res[name] = ev[0].elapsed_time(ev[1]) / steps
    sep, bat = min(res["separate"], res["separate_again"]), min(res["batched"], res["batched_again"])
    return dict(workload=f"{wl.name}_T{wl.T}_batched_with_combine_T{rT}_k{rk}_N{rN}", dtype="bf16",
                separate_ms=round(sep, 4), batched_ms=round(bat, 4), reduce_tiles=mb.moe_reduce_task_tiles(rT, rN),
                tflops_batched=round(wl.flops / (bat * 1e-3) / 1e12, 2), tflops_separate=round(wl.flops / (sep * 1e-3) / 1e12, 2))


def layer_point(T: int, steps: int, warmup: int, dev="cuda:0") -> dict:
    """One whole bf16 feed-forward layer at the Mixtral-8x7B sizes (Sec. 2.2): two task maps, the gate+up product
    with the fused gated activation, the down product and the weighted sum, five library calls per step."""
    up = wk.mixtral_up(T)
    k, E, hidden, inter = up.k, up.E, up.K, up.N // 2
    ids = wk.make_routing(up).to(dev)
    g = torch.Generator(device=dev).manual_seed(wk.BASE_SEED + 31 * T)
    X = torch.randn((T, hidden), generator=g, device=dev).to(torch.bfloat16)
    W1 = torch.empty((E, hidden, 2 * inter), dtype=torch.bfloat16, device=dev)
    W2 = torch.empty((E, inter, hidden), dtype=torch.bfloat16, device=dev)
    for e in range(E):
        W1[e] = (torch.randn((hidden, 2 * inter), generator=g, device=dev) * hidden ** -0.5).to(torch.bfloat16)
        W2[e] = (torch.randn((inter, hidden), generator=g, device=dev) * inter ** -0.5).to(torch.bfloat16)
    wts = torch.softmax(torch.randn((T, k), generator=g, device=dev), dim=1)
    plan = mb.MoeLayerPlan(T, k, E, hidden, inter, dev)
    for _ in range(warmup):
        plan.forward(X, W1, W2, ids, wts)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    torch.cuda._sleep(int(4e6))
    for i in range(steps):
        ev[i][0].record()
        plan.forward(X, W1, W2, ids, wts)
        ev[i][1].record()
    torch.cuda.synchronize()
    ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    flops = 6 * T * k * hidden * inter
    return dict(workload=f"mixtral_layer_T{T}", dtype="bf16", T=T, k=k, E=E, hidden=hidden, inter=inter,
                layer_ms=round(ms, 4), tflops=round(flops / (ms * 1e-3) / 1e12, 2),
                tokens_per_s=round(T / (ms * 1e-3), 1),
                tilings={"gate_up": [plan.g1.tile_m, plan.g1.tile_n, plan.g1.tile_m_slack],
                         "down": [plan.g2.tile_m, plan.g2.tile_n, plan.g2.tile_m_slack], "down_k_parts": plan.k_parts})


def all_points():
    pts = [wk.tiny(64)]
    pts += [wk.mixtral_up(T) for T in (16, 256, 4096)]
    pts += [wk.mixtral_down_zipf(T) for T in (256, 4096)]
    pts += [wk.fine_grained(T) for T in (128, 2048, 8192)]
    pts += [wk.decode_fp8(T) for T in (1, 8, 32)]
    pts += [wk.paper_eval(s) for s in ("balanced", "best", "worst")]
    return pts


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--points", default="none", help="'all', 'none', or a comma list of workload names")
    ap.add_argument("--tile", default="", help="override tile_m,tile_n of the headline workload")
    ap.add_argument("--order", default="ascending", choices=["ascending", "spread", "interleave", "both", "all"],
                    help="expert order in sigma for the extra points (the headline always uses ascending)")
    ap.add_argument("--small", default="0,0",
                    help="tile_m_small,small_max_rows: second tiling strategy for the extra points with 256x256 tiles")
    ap.add_argument("--slack", type=int, default=-1, help="override tile_m_slack of every workload (0 = plain ceil tiling)")
    ap.add_argument("--launch-mode", type=int, default=-1,
                    help="moe_gemm_desc.launch_mode of every point: 0 the library's choice, 1 one workgroup per tile, "
                         "2 resident workgroups where a kernel exists, >= 8 resident with at most that many workgroups "
                         "(default: each point's own default)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-decode", action="store_true", help="skip the fp8 decode points (roofline_hbm)")
    ap.add_argument("--operand-fill", default="", choices=["", "zeros", "ones"],
                    help="measurement aid: ALSO time the headline launch with X and W overwritten by a constant (the "
                         "kernel's duration depends on the operand values through the chip's power management); "
                         "reported under 'operand_fill', never as the headline")
    ap.add_argument("--dense-reference", action="store_true",
                    help="also time the tensor library's dense bf16 matmul of the same size and weight layout "
                         "([T*k, K] x [K, N]) on random data; reported under 'dense_reference'")
    ap.add_argument("--mfma-probe", action="store_true",
                    help="also time the library's pure-MFMA probe (no memory traffic) with 16x16x32 and 32x32x16 blocks "
                         "on random and on constant operands: the sustained ceiling under the chip's power limit; "
                         "reported under 'mfma_probe'")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (a kernel of known traffic to scale profiler byte counters by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); no multi-GPU path exists.", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    mb.lib()
    torch.cuda.set_device(0)

    wl = wk.mixtral_up(4096)
    if args.tile:
        tm, tn = (int(v) for v in args.tile.split(","))
        wl = wl.with_T(wl.T, tile_m=tm, tile_n=tn, tile_m_slack=0)
    if args.slack >= 0:
        wl = wl.with_T(wl.T, tile_m_slack=args.slack)
    lm = max(0, args.launch_mode)
    pt = Point(wl, launch_mode=lm)
    head = pt.report(args.steps, args.warmup)
    traffic, traffic_from = measured_traffic(HEADLINE) if wl == wk.mixtral_up(4096) else (None, None)
    out = {
        "metric": "expert-GEMM TFLOP/s (useful FLOPs 2*T*k*K*N, task-map build + grouped GEMM per step)",
        "value": head["tflops_step"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": HEADLINE, "T": wl.T, "E": wl.E, "top_k": wl.k, "K": wl.K, "N": wl.N,
                   "tile_m": wl.tile_m, "tile_n": wl.tile_n, "tile_m_slack": wl.tile_m_slack, "routing": wl.routing,
                   "launch_mode": lm},
        "roofline": {"bound": "mfma", "achieved": head["tflops_gemm"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(head["tflops_gemm"] / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic, "traffic_source": traffic_from,
                     "kernel": head["kernel"],
                     "kernel_ms": head["gemm_ms"], "kernel_ms_median": head["gemm_ms_median"], "kernel_ms_min": head["gemm_ms_min"],
                     "map_ms": head["map_ms"], "alg_bytes": head["alg_bytes"]},
    }
    # what the runtime reports for this device, beside the published peak the fractions are taken against
    prop = torch.cuda.get_device_properties(0)
    out["device"] = {"name": prop.name, "compute_units": prop.multi_processor_count,
                     "gcn_arch": getattr(prop, "gcnArchName", None), "hbm_gib": round(prop.total_memory / 2 ** 30, 1)}
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(pt)
    if args.operand_fill:
        # same map, same launch, constant operands: separates what the instruction stream costs from what the data costs
        v = 0.0 if args.operand_fill == "zeros" else 1.0
        keep = (pt.X.clone(), pt.W[0].clone())
        pt.X.fill_(v)
        pt.W[0].fill_(v)
        _, g_ms, _ = pt.time(args.steps, args.warmup)
        pt.X.copy_(keep[0])
        pt.W[0].copy_(keep[1])
        del keep
        out["operand_fill"] = {"fill": args.operand_fill, "kernel_ms": round(g_ms, 4),
                               "tflops": round(wl.flops / (g_ms * 1e-3) / 1e12, 2),
                               "random_kernel_ms": head["gemm_ms"]}
    if args.mfma_probe:
        from paper_2501_16103_amd import probe
        sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")
        iters = 100000
        flops = 256 * 8 * iters * 524288
        res = []
        for block in (32, 16):
            for rnd in (False, True):
                probe.moe_probe_mfma(block, rnd, 1000, sink)
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                torch.cuda.synchronize()
                ev[0].record()
                probe.moe_probe_mfma(block, rnd, iters, sink)
                ev[1].record()
                torch.cuda.synchronize()
                ms = ev[0].elapsed_time(ev[1])
                res.append({"block": f"{block}x{block}x{512 // block}", "operands": "random" if rnd else "constant",
                            "ms": round(ms, 3), "tflops": round(flops / (ms * 1e-3) / 1e12, 1)})
        # the 256x256x64 tile's loop, one ingredient at a time (LDS reads, barrier, DMA from cache, half of it from HBM)
        # ... and the same ingredients in the schedule of the large tile's k loop (the two wavefronts of a SIMD alternate);
        # with --operand-fill zeros a second time on all-zero fragments (no switching power: what the schedule alone costs)
        src = (torch.randn((513 << 20) // 2, device="cuda:0") * 0.5).to(torch.bfloat16)
        for fill in ("random", "zeros") if args.operand_fill == "zeros" else ("random",):
            if fill == "zeros":
                src.zero_()
            for mode, what in ((1, "MFMA + LDS fragment reads"), (2, "+ barrier per k-tile"), (3, "+ DMA from cache"),
                               (4, "+ half of the DMA bytes from HBM"),
                               (10, "alternating roles: MFMA + LDS fragment reads + 4 barriers per k-tile"),
                               (11, "alternating roles: + DMA from cache"), (12, "alternating roles: + half of the DMA bytes from HBM")):
                probe.moe_probe_pipeline(mode, 1000, src, sink)
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                torch.cuda.synchronize()
                ev[0].record()
                probe.moe_probe_pipeline(mode, iters, src, sink)
                ev[1].record()
                torch.cuda.synchronize()
                ms = ev[0].elapsed_time(ev[1])
                res.append({"block": "16x16x32", "operands": fill, "loop": what,
                            "ms": round(ms, 3), "tflops": round(flops / (ms * 1e-3) / 1e12, 1)})
        # the LDS pipe alone: bytes per wavefront and k-step of each mode, reported per CU and nanosecond
        for mode, what, nbytes in ((5, "16-byte fragment reads only", 8192), (6, "transposing 8-byte reads only", 4096),
                                   (7, "both kinds of reads", 12288), (8, "DMA writes only", 4096)):
            probe.moe_probe_pipeline(mode, 1000, src, sink)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            torch.cuda.synchronize()
            ev[0].record()
            probe.moe_probe_pipeline(mode, iters, src, sink)
            ev[1].record()
            torch.cuda.synchronize()
            ms = ev[0].elapsed_time(ev[1])
            res.append({"lds_only": what, "ms": round(ms, 3), "lds_bytes_per_ns_per_cu": round(8 * iters * nbytes / (ms * 1e6), 1),
                        "ns_per_k_step": round(ms * 1e6 / iters, 1)})
        del src
        out["mfma_probe"] = res
    if args.dense_reference:
        # the tensor library's dense GEMM of the same size: with the weight stored as here ([K, N], N contiguous) and
        # with a K-contiguous weight ([N, K], the layout linear layers are usually stored in)
        A = torch.randn((wl.R, wl.K), device="cuda:0").to(torch.bfloat16)
        ref = []
        for layout in ("KN", "NK"):
            B = torch.randn((wl.K, wl.N) if layout == "KN" else (wl.N, wl.K), device="cuda:0").to(torch.bfloat16)
            Bm = B if layout == "KN" else B.t()
            for _ in range(3):
                C = A @ Bm
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            torch.cuda.synchronize()
            ev[0].record()
            for _ in range(10):
                C = A @ Bm
            ev[1].record()
            torch.cuda.synchronize()
            d_ms = ev[0].elapsed_time(ev[1]) / 10
            ref.append({"what": f"torch.matmul bf16 [{wl.R},{wl.K}] x weight stored [{'K,N' if layout == 'KN' else 'N,K'}], random data",
                        "ms": round(d_ms, 4), "tflops": round(wl.flops / (d_ms * 1e-3) / 1e12, 2)})
            del B, Bm, C
        del A
        out["dense_reference"] = ref
    del pt
    torch.cuda.empty_cache()
    if not args.no_decode:
        out["roofline_hbm"] = decode_hbm_points(max(20, args.steps), max(5, args.warmup), not args.no_cpu)

    if args.points != "none":
        want = None if args.points == "all" else set(args.points.split(","))
        points = []
        for w in all_points():
            name = f"{w.name}_T{w.T}"
            if want is not None and name not in want and w.name not in want:
                continue
            if args.slack >= 0:
                w = w.with_T(w.T, tile_m_slack=args.slack)
            if name == HEADLINE and not args.tile:
                points.append(head)
                continue
            copies = weight_copies(w)
            small = tuple(int(v) for v in args.small.split(","))
            if small[0] and not (w.dtype == "bf16" and mb.moe_tile_pair_supported(mb.MOE_DTYPE_BF16, w.tile_m, w.tile_n, small[0])):
                small = (0, 0)
            for order in {"both": [0, 1], "all": [0, 1, 2], "spread": [1], "interleave": [2]}.get(args.order, [0]):
                p = Point(w, copies, order=order, small=small, launch_mode=lm)
                points.append(p.report(max(10, args.steps // 2), max(3, args.warmup // 2)))
                del p
                torch.cuda.empty_cache()
                # tilings that have a tail-split launch (it pays when the tile count is not a whole number of rounds)
                if (w.dtype == "bf16" and w.tile_m in (64, 128, 256) and w.tile_n == 256 and not small[0]
                        and (w.tile_m_slack == 0 or (w.tile_m == 256 and w.tile_m_slack == 32 and args.slack < 0))
                        and w.K % 64 == 0 and w.N % 256 == 0):
                    p = Point(w, copies, order=order, launch_mode=lm, tail_split=True)
                    r = p.report(max(10, args.steps // 2), max(3, args.warmup // 2))
                    r["workload"] += "_tail_split"
                    points.append(r)
                    del p
                    torch.cuda.empty_cache()
        if want is None or "neighbours" in want:
            # the fused gated activation on the headline shape, and the sum over a token's experts
            p = Point(wl, swiglu=True)
            points.append(p.report(max(10, args.steps // 2), max(3, args.warmup // 2)))
            del p
            torch.cuda.empty_cache()
            # labelled extra: the fp8 layer of the decode points at a prefill size (256-row fp8 tiles)
            p = Point(wk.decode_fp8(4096))
            points.append(p.report(max(10, args.steps // 2), max(3, args.warmup // 2)))
            del p
            torch.cuda.empty_cache()
            # labelled extra: the same products with the weights pre-packed as [E][N][K]
            for w in (wl, wk.mixtral_up(256), wk.mixtral_up(16), wk.decode_fp8(32), wk.decode_fp8(8)):
                p = Point(w, weight_copies(w), w_nk=True)
                points.append(p.report(max(10, args.steps // 2), max(3, args.warmup // 2)))
                del p
                torch.cuda.empty_cache()
            for (T, k, N) in ((4096, 2, 4096), (8192, 8, 4096), (32, 6, 2816)):
                points.append(combine_point(T, k, N, max(10, args.steps // 2), max(3, args.warmup // 2)))
                torch.cuda.empty_cache()
        if want is None or "batched" in want or "neighbours" in want:
            # heterogeneous batch: the headline product with the previous layer's weighted sum in the same launch
            for (rT, rk, rN) in ((4096, 2, 4096), (8192, 8, 4096)):
                points.append(batched_point(wl, rT, rk, rN, max(10, args.steps // 2), max(3, args.warmup // 2)))
                torch.cuda.empty_cache()
        if want is None or "layer" in want:
            # labelled extra: the whole feed-forward layer composed from the library's calls
            for T in (4096, 512, 256, 16):
                points.append(layer_point(T, max(10, args.steps // 2), max(3, args.warmup // 2)))
                torch.cuda.empty_cache()
        out["points"] = points
    print(json.dumps(out))


if __name__ == "__main__":
    main()
