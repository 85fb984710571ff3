#!/usr/bin/env python3
"""Benchmark of the tiled SDPA forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4] [--tile TM,TN]

A step is one forward pass (one kernel launch: the whole hot path) over one seeded synthetic
batch that is already resident in HBM.  Policy follows the paper's harness (Section 4.2.3):
W warm-up calls, synchronise, events around every timed call, median and p95 over the K calls.
Prints ONE JSON line.  TFLOP/s = 4*B*H*S^2*D / t (the two matrix products, true S).
"""
from __future__ import annotations

import argparse
import json
import os
import platform
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = 2500.0      # MI355X dense FP16/BF16 MFMA, published
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published

PROFILES = os.path.join(ROOT, "profiles")


def profiled_traffic(workload, dtype, D, tm, tn):
    """HBM bytes per launch of a workload's kernel as the committed rocprofv3 summary states them
    (FETCH_SIZE + WRITE_SIZE per dispatch, scaled by the copy-kernel calibration): the "total" row of
    profiles/sdpa_fwd_<workload>_<dtype>[_tile_<T_M>x<T_N>].md whose `Kernel:` line names this very
    instantiation.  Returns (bytes or None, source file or the reason there is none)."""
    import re
    nw = tm // 32
    want = re.compile(r"sdpa_fwd_kernelI(DF16_|DF16b)Li%dELi%dELi%dELi\dELi0E" % (D, nw, tn))
    elem = "DF16_" if dtype == "f16" else "DF16b"
    for name in (f"sdpa_fwd_{workload}_{dtype}_tile_{tm}x{tn}.md", f"sdpa_fwd_{workload}_{dtype}.md"):
        path = os.path.join(PROFILES, name)
        if not os.path.exists(path):
            continue
        text = open(path).read()
        m = want.search(text)
        if m is None or m.group(1) != elem:
            continue
        t = re.search(r"^\|\s*total\s*\|[^|]*\|\s*([0-9.]+)\s*MB\s*\|", text, re.M)
        if t:
            return float(t.group(1)) * 1e6, "profiles/" + name
    return None, f"no committed counter run of sdpa_fwd_kernel<{dtype},D={D},T_M={tm},T_N={tn}> on {workload}"


# The paper's own figures, other hardware (NVIDIA DGX GB10): context only, never a target.
PAPER_CONTEXT = {
    "hardware": "NVIDIA DGX GB10",
    "fp16_noncausal_D128_S4096_tflops": 73.62,
    "fp16_noncausal_D128_S8192_tflops": 73.38,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C4", help="C1..C5 (default C4: B2 H32 S8192 D128 BF16)")
    ap.add_argument("--dtype", default=None, help="f16 / bf16 (default: the workload's first dtype)")
    ap.add_argument("--shape", default=None, help="B,H,S,D: a custom shape (seeded N(0,1) inputs) instead of --workload")
    ap.add_argument("--compare-tiles", default=None,
                    help="T_MxT_N,T_MxT_N,...: time these tiles on the workload in one process, taking turns in alternating "
                         "order over seven rounds (a tile measured after another finds the clocks warmed up: sequential "
                         "timings favour whatever runs later); one JSON line with the median of each")
    ap.add_argument("--kv", default=None,
                    help="B,H,Sq,Skv,D: time the Sq x Skv / split-KV entry point (decoding shapes) instead of a workload")
    ap.add_argument("--splits", type=int, default=0, help="with --kv: splits along the key axis (0 = heuristic)")
    ap.add_argument("--kv-fill", type=float, default=0.0,
                    help="with --kv: treat Skv as the capacity of a cache filled to this fraction in every batch entry "
                         "(tiled_sdpa_fwd_kvcache with a length per entry); 0 = a full cache without lengths")
    ap.add_argument("--kv-block", type=int, default=0,
                    help="with --kv: store the cache in pages of this many rows, scattered over the pool in a seeded "
                         "random order (tiled_sdpa_fwd_paged); Skv must be a multiple of it")
    ap.add_argument("--kv-heads", type=int, default=0,
                    help="with --kv: key/value heads (grouped heads: H query heads share H/kv-heads of them; 0 = H)")
    ap.add_argument("--bwd", action="store_true",
                    help="time the backward pass (tiled_sdpa_bwd: statistics, dV, dK and dQ kernels) of the workload")
    ap.add_argument("--tile", default=None, help="TM,TN to pin the schedule (default: heuristic)")
    ap.add_argument("--qk-std", type=float, default=None,
                    help="standard deviation of the Q and K entries (default: the workload's own; C5 uses sqrt(2))")
    ap.add_argument("--linear-grid", action="store_true", help="disable the per-XCD workgroup regrouping")
    ap.add_argument("--exact-max", action="store_true", help="raise the softmax reference on every new maximum")
    ap.add_argument("--causal", action="store_true",
                    help="causal mask (Section 4.1.3); flops are then counted as half of the non-causal figure")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the baseline sample")
    ap.add_argument("--no-all-workloads", dest="all_workloads", action="store_false",
                    help="skip the per-configuration summary (C1..C5: back-to-back, HIP-graph and cache-cold launch "
                         "times, each against its own roofline, and the error against the CPU oracle)")
    ap.add_argument("--csv", default=None,
                    help="also write the tile sweep and the per-configuration summary as CSV rows with status and "
                         "status_detail columns (unsupported cells are recorded, not dropped: Section 5 of the paper)")
    ap.add_argument("--no-tune", dest="tune", action="store_false",
                    help="take the library's heuristic tile; by default the tile is picked with tiled_sdpa_tune_tile "
                         "(the paper's per-shape schedule search, Table 1 and Sections 5.5-5.6) before and outside the timed region")
    ap.add_argument("--no-sweep-tiles", dest="sweep_tiles", action="store_false",
                    help="skip the sweep over every (T_M, T_N) of the workload (the schedule knobs of the paper's Table 1)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the MFMA-only ceiling measurement")
    ap.add_argument("--input-fill", default="normal", choices=["normal", "zeros", "ones"],
                    help="normal = the seeded workload; zeros / ones = same shapes with constant data "
                         "(clock experiment: the same instruction stream at lower switching activity)")
    ap.add_argument("--grid", default=None, metavar="B,H",
                    help="time the paper's workload grid (Section 4.3: S in 512..8192 x D in 64,96,128,160 x FP16/BF16 x "
                         "causal/non-causal, 80 points) at this batch and head count (the paper's profiled shape is 1,8) "
                         "instead of a workload; one JSON line, and CSV rows with --csv")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a device-to-device copy of --copy-mib MiB (reference for the HBM byte counters)")
    ap.add_argument("--copy-mib", type=int, default=1024)
    return ap.parse_args()


_DEVICE_TENSORS = {}


def device_workload(torch, name, dtype=None, fill="normal", shape=None, qk_std=None):
    """(workload, dtype, q, k, v) with the seeded tensors on the GPU; one copy per configuration is kept
    for the whole run (every leg of the bench then times and checks the same tensors)."""
    import dataclasses
    from paper_2603_01960_amd.workloads import WORKLOADS, Workload, make_qkv
    key = (name, dtype, fill, shape, qk_std)
    if key not in _DEVICE_TENSORS:
        if shape is not None:
            B, H, S, D = shape
            dt = dtype or "bf16"
            w = Workload("custom", B, H, S, D, (dt,), 4242)
        else:
            w = WORKLOADS[name]
            if qk_std is not None:
                w = dataclasses.replace(w, qk_std=float(qk_std))
            dt = dtype or w.dtypes[0]
        q, k, v = make_qkv(w.B, w.H, w.S, w.D, dt, w.seed, w.qk_std, w.v_std)
        if fill != "normal":
            q, k, v = (torch.zeros_like(t) if fill == "zeros" else torch.ones_like(t) for t in (q, k, v))
        _DEVICE_TENSORS[key] = (w, dt, q.cuda(), k.cuda(), v.cuda())
    return _DEVICE_TENSORS[key]


def time_workload(pkg, torch, name, dtype, steps, warmup, tile=None, flags=0, fill="normal", shape=None, qk_std=None):
    w, dtype, qd, kd, vd = device_workload(torch, name, dtype, fill, shape, qk_std)
    o = torch.empty_like(qd)
    run = lambda: pkg.sdpa(qd, kd, vd, out=o, tile=tile, flags=flags)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    # events go to the same (current) stream the kernel is enqueued on.  marks[i] precedes launch i and
    # marks[steps] follows the last one: the region average is (last - first) / steps, and consecutive
    # marks give the per-launch spread (for kernels of tens of microseconds each of those intervals
    # also holds the launch gap, so the median / p95 are an upper bound there).
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    for i in range(steps):
        marks[i].record()
        run()
    marks[steps].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_launch_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    region_ms = marks[0].elapsed_time(marks[steps])
    assert torch.isfinite(o.float()).all().item(), "non-finite output"
    return {
        "workload": w, "dtype": dtype, "wall_s": wall,
        "ms_per_step": 1e3 * wall / steps,
        "kernel_ms_avg": region_ms / steps,
        "kernel_ms_median": statistics.median(per_launch_ms),
        "kernel_ms_p95": per_launch_ms[min(steps - 1, int(0.95 * steps))],
        "tensors": (qd, kd, vd), "o": o,
    }


def time_batched(pkg, torch, name, dtype, n, warmup, rotate=1):
    """Per-launch time with the launches issued back to back between ONE pair of events: for kernels
    of a few tens of microseconds the event pair of time_workload() mostly measures launch latency.
    rotate > 1 cycles the launches over that many copies of (Q, K, V, O) in distinct memory, so that a
    launch finds none of its tensors in the L2 or in the 256 MB memory-side cache (a cache-cold figure
    for the workloads whose tensors would otherwise stay resident between launches)."""
    w, _, q, k, v = device_workload(torch, name, dtype)
    sets = [(q, k, v, torch.empty_like(q))]
    for _ in range(rotate - 1):
        qd, kd, vd = q.clone(), k.clone(), v.clone()
        sets.append((qd, kd, vd, torch.empty_like(qd)))
    for i in range(max(warmup, rotate)):
        qd, kd, vd, o = sets[i % rotate]
        pkg.sdpa(qd, kd, vd, out=o)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for i in range(n):
        qd, kd, vd, o = sets[i % rotate]
        pkg.sdpa(qd, kd, vd, out=o)
    b.record()
    torch.cuda.synchronize()
    return w, a.elapsed_time(b) / n, sets[0][3]


def time_graph_replay(pkg, torch, name, dtype, per_graph=20, replays=20):
    """Per-launch time of `per_graph` launches recorded once into a HIP graph and replayed: the rate of
    the kernel itself where the eager loop is bound by host time per call (C1)."""
    w, _, qd, kd, vd = device_workload(torch, name, dtype)
    o = torch.empty_like(qd)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(3):
            pkg.sdpa(qd, kd, vd, out=o)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(per_graph):
            pkg.sdpa(qd, kd, vd, out=o)
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(replays):
        graph.replay()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / (replays * per_graph)


def hbm_copy_ceiling(torch, mib=1024, steps=10):
    """GB/s (read + write) of a plain device-to-device copy too large for any cache: what a pure
    stream sustains on this GPU right now, next to the published 8 TB/s."""
    n = mib * (1 << 20)
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(3)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    return round(2 * n / (a.elapsed_time(b) / steps) / 1e6, 1)


def hbm_read_ceiling(pkg, torch, mib=2048, steps=10):
    """GB/s of a read-only stream over a buffer too large for any cache (tiled_sdpa_probe_hbm_read): what
    reading a K/V cache once can be compared with on this GPU right now, next to the published 8 TB/s."""
    src = torch.empty(mib * (1 << 20), dtype=torch.uint8, device="cuda").fill_(5)
    sink = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(2):
        done = pkg.probe_hbm_read(src.data_ptr(), src.numel(), sink.data_ptr(), stream)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        pkg.probe_hbm_read(src.data_ptr(), src.numel(), sink.data_ptr(), stream)
    b.record()
    torch.cuda.synchronize()
    return round(done / (a.elapsed_time(b) / steps) / 1e6, 1)


def mfma_ceilings(pkg, torch, dtype, iters=4000):
    """What a register-resident MFMA stream sustains on this GPU right now (TFLOP/s), with random and
    with constant operand data; the gap is the clock the chip gives up to its power limit."""
    sink = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    code = pkg.F16 if dtype == "f16" else pkg.BF16
    out = {}
    for label, rnd in (("random_operands", 1), ("constant_operands", 0), ("random_operands_plus_loop_mix", 2)):
        for _ in range(2):
            pkg.probe_mfma(code, rnd, iters, sink.data_ptr(), stream)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        flops = sum(pkg.probe_mfma(code, rnd, iters, sink.data_ptr(), stream) for _ in range(3))
        b.record()
        torch.cuda.synchronize()
        out[label] = round(flops / (a.elapsed_time(b) * 1e-3) / 1e12, 1)
    return out


def copy_calibration(torch, mib, steps):
    """Plain copy of known size: what FETCH_SIZE / WRITE_SIZE read for it scales those counters."""
    n = mib * (1 << 20)
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(3)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / steps
    print(json.dumps({"copy_bytes": n, "copies": steps, "ms_per_copy": round(ms, 4),
                      "GBs_read_plus_write": round(2 * n / ms / 1e6, 1)}), flush=True)


def bench_kv(pkg, torch, args, tile, flags):
    """One JSON line for tiled_sdpa_fwd_kv on a seeded B,H,Sq,Skv,D problem (both of its kernels timed
    as one step; output and workspace are allocated once, outside the timed region)."""
    from paper_2603_01960_amd.workloads import make_qkv
    B, H, Sq, Skv, D = (int(x) for x in args.kv.split(","))
    dtype = args.dtype or "bf16"
    code = pkg.F16 if dtype == "f16" else pkg.BF16
    Hkv = args.kv_heads or H
    G = H // Hkv
    q = make_qkv(B, H, Sq, D, dtype, seed=4242)[0].cuda()
    _, k, v = (t.cuda() for t in make_qkv(B, Hkv, Skv, D, dtype, seed=4243))
    # grouped heads run as Hkv heads of G*Sq query rows each (see binding.sdpa_kv)
    splits = args.splits or pkg.kv_default_splits(B, Hkv, G * Sq, Skv, D, code, flags if G == 1 else flags & ~pkg.binding.FLAG_CAUSAL)
    ws = torch.empty(max(16, pkg.kv_workspace_bytes(B, Hkv, G * Sq, D, splits)), dtype=torch.uint8, device="cuda")
    o = torch.empty_like(q)
    cap, lens = Skv, None
    if args.kv_fill > 0:
        Skv = max(1, int(round(cap * min(1.0, args.kv_fill))))          # valid rows per entry: what is read and computed
        lens = torch.full((B,), Skv, dtype=torch.int32, device="cuda")
    run = lambda: pkg.sdpa_kv(q, k, v, splits=splits, out=o, workspace=ws, tile=tile, flags=flags, kv_lens=lens)
    if args.kv_block:
        R = args.kv_block
        nb = cap // R
        assert nb * R == cap, "--kv-block must divide Skv"
        if lens is None:
            lens = torch.full((B,), cap, dtype=torch.int32, device="cuda")
        perm = torch.randperm(B * nb, generator=torch.Generator().manual_seed(4244)).to(torch.int32)
        table = perm.view(B, nb).contiguous().cuda()
        def paged(t):       # [B, Hkv, cap, D] -> pages [B*nb, Hkv, R, D], block (b, i) stored at page table[b][i]
            blocks = t.view(B, Hkv, nb, R, D).permute(0, 2, 1, 3, 4).reshape(B * nb, Hkv, R, D)
            out = torch.empty(blocks.shape, dtype=blocks.dtype, device=blocks.device)
            out[perm.long().cuda()] = blocks
            return out
        kp, vp = paged(k), paged(v)
        del k, v
        run = lambda: pkg.sdpa_paged(q, kp, vp, lens, table, splits=splits, out=o, workspace=ws, tile=tile, flags=flags)
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    a.record()
    for _ in range(args.steps):
        run()
    b.record()
    torch.cuda.synchronize()
    wall_ms = 1e3 * (time.perf_counter() - t0) / args.steps
    ms = a.elapsed_time(b) / args.steps
    assert torch.isfinite(o.float()).all().item(), "non-finite output"
    causal = bool(flags & pkg.binding.FLAG_CAUSAL)
    pairs = Sq * Skv - (Sq * (Sq - 1) // 2 if causal else 0)        # (query, key) pairs that contribute
    flops = 4.0 * B * H * pairs * D
    comp_bytes = 2.0 * B * D * (2 * Hkv * Skv + 2 * H * Sq)
    ridge = PEAK_MFMA_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    if flops / comp_bytes >= ridge:
        tf = flops / (ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(tf, 2), "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(tf / PEAK_MFMA_TFLOPS, 4)}
    else:
        gbs = comp_bytes / (ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(gbs / PEAK_HBM_GBS, 4)}
    if roofline["bound"] == "hbm" and not args.no_ceilings:
        roofline["hbm_read_ceiling_GBs"] = hbm_read_ceiling(pkg, torch)
        roofline["frac_of_hbm_read_ceiling"] = round(roofline["achieved"] / roofline["hbm_read_ceiling_GBs"], 4)
    roofline.update({"traffic": None, "kernel": "sdpa_fwd_kernel<KV> + sdpa_merge_kernel" if splits > 1 else "sdpa_fwd_kernel<KV>",
                     "ms_avg_both_kernels": round(ms, 5), "algorithmic_flops_per_launch": flops,
                     "compulsory_hbm_bytes_per_launch": comp_bytes})
    print(json.dumps({
        "metric": "SDPA forward TFLOP/s (4*B*H*pairs*D / t)", "value": round(flops / (wall_ms * 1e-3) / 1e12, 3),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"KV: SDPA fwd {'causal' if causal else 'non-causal'} B={B} H={H}{'' if G == 1 else f' (kv heads {Hkv})'} Sq={Sq} Skv={Skv} D={D} {dtype}",
                   "cache_capacity": cap, "page_rows": args.kv_block or None, "splits": splits, "tile": list(tile) if tile else "heuristic",
                   "cache_tokens_per_s": round(B * Hkv * Skv / (ms * 1e-3), 1)},
        "roofline": roofline}), flush=True)


def bench_bwd(pkg, torch, args, flags):
    """One JSON line for tiled_sdpa_bwd on a workload (its three kernels timed as one step; the forward
    pass that provides o and lse, the gradients and the workspace are set up outside the timed region)."""
    from paper_2603_01960_amd.workloads import WORKLOADS, Workload, make_qkv, make_workload
    if args.shape:
        B, H, S, D = (int(x) for x in args.shape.split(","))
        dtype = args.dtype or "bf16"
        w = Workload("custom", B, H, S, D, (dtype,), 4242, 1.0)
        q, k, v = make_qkv(B, H, S, D, dtype, seed=w.seed)
    else:
        w, q, k, v = make_workload(args.workload, args.dtype)
        dtype = args.dtype or w.dtypes[0]
    causal = bool(flags & pkg.binding.FLAG_CAUSAL)
    Hkv = args.kv_heads or w.H
    if Hkv != w.H:          # grouped heads: the first Hkv heads of the seeded K and V serve as the key/value heads
        k, v = k[:, :Hkv].contiguous(), v[:, :Hkv].contiguous()
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    g = torch.Generator(device="cpu").manual_seed(w.seed + 50)
    dout = torch.randn(*q.shape, dtype=torch.float32, generator=g).to(q.dtype).cuda()
    o, lse = pkg.sdpa_kv(qd, kd, vd, causal=causal, return_lse=True) if Hkv != w.H else pkg.sdpa(qd, kd, vd, causal=causal, return_lse=True)
    grads = (torch.empty_like(qd), torch.empty_like(kd), torch.empty_like(kd))
    ws = torch.empty(pkg.bwd_workspace_bytes(w.B, w.H, w.S), dtype=torch.uint8, device="cuda")
    run = lambda: pkg.sdpa_backward(qd, kd, vd, o, dout, lse, causal=causal, workspace=ws, grads=grads)
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    a.record()
    for _ in range(args.steps):
        run()
    b.record()
    torch.cuda.synchronize()
    wall_ms = 1e3 * (time.perf_counter() - t0) / args.steps
    ms = a.elapsed_time(b) / args.steps
    assert all(torch.isfinite(t.float()).all().item() for t in grads), "non-finite gradient"
    # five S x S x D products (scores, dP, dV, dK, dQ) of 2*B*H*S^2*D flops each; half under the causal mask
    flops = 2.5 * w.flops * (0.5 if causal else 1.0)
    tf = flops / (ms * 1e-3) / 1e12
    print(json.dumps({
        "metric": "SDPA backward TFLOP/s (10*B*H*S^2*D / t)", "value": round(flops / (wall_ms * 1e-3) / 1e12, 2),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: SDPA bwd {'causal' if causal else 'non-causal'} B={w.B} H={w.H}"
                               f"{'' if Hkv == w.H else f' (kv heads {Hkv})'} S={w.S} D={w.D} {dtype}"},
        "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tf / PEAK_MFMA_TFLOPS, 4),
                     # all four kernels of a call, FETCH_SIZE + WRITE_SIZE scaled (profiles/sdpa_bwd_C4_C2.md)
                     "traffic": 2515.7e6 if (w.name == "C4" and dtype == "bf16" and not causal and Hkv == w.H) else None,
                     "kernel": ("sdpa_bwd_prepare_kernel + sdpa_bwd_kernel<dK+dV> + sdpa_bwd_kernel<dQ>" if w.D == 64 else
                                "sdpa_bwd_prepare_kernel + sdpa_bwd_kernel<dV> + sdpa_bwd_kernel<dK> + sdpa_bwd_kernel<dQ>"),
                     "ms_avg_all_kernels": round(ms, 5), "algorithmic_flops_per_launch": flops,
                     # scores and dP are recomputed per pass: 7 products with the fused dK + dV pass of D = 64, else 8
                     "executed_mfma_flops_per_launch": flops * (7.0 if w.D == 64 else 8.0) / 5.0}}), flush=True)


TOL = {"f16": 2e-3, "bf16": 1.6e-2}     # max-abs error against the float64 oracle (the task's stated tolerances)


def oracle_rows(w, q, k, v, rows):
    """(seconds, float64 reference [B, H, len(rows), D]) of the unmodified CPU oracle on the given query
    rows of every head (rows = None: the whole configuration)."""
    from oracle import sdpa_oracle
    qn, kn, vn = (x.float().cpu().numpy() for x in (q, k, v))
    t = time.perf_counter()
    ref = sdpa_oracle.sdpa(qn, kn, vn, rows=rows)
    return time.perf_counter() - t, ref


def max_abs_err(torch, o, ref, rows):
    """max |float64(o) - ref| over the compared rows; o is the device output of a timed launch."""
    import numpy as np
    got = o if rows is None else o[:, :, torch.tensor(rows, device=o.device)]
    return float(np.abs(got.double().cpu().numpy() - ref).max())


def cpu_baseline(torch, w, dtype, q, k, v, o, target_seconds, causal=False):
    """Time the unmodified float64 CPU oracle on a bounded sample of the same workload, and hold the
    output of the timed launches against what it computed (the harness's correctness check, Section 4.2.3)."""
    from oracle import sdpa_oracle
    qn, kn, vn = (x.float().cpu().numpy() for x in (q, k, v))
    # calibrate on a few rows, then size the sample for ~target_seconds
    probe = list(range(0, w.S, max(1, w.S // 8)))[:8]
    t = time.perf_counter()
    sdpa_oracle.sdpa(qn, kn, vn, rows=probe, causal=causal)
    dt = max(time.perf_counter() - t, 1e-4)
    nrows = int(min(w.S, max(len(probe), len(probe) * target_seconds / dt)))
    rows = sorted({(i * w.S) // nrows for i in range(nrows)})      # evenly spread over the sequence
    t = time.perf_counter()
    ref = sdpa_oracle.sdpa(qn, kn, vn, rows=rows, causal=causal)
    dt = time.perf_counter() - t
    flops = 4.0 * w.BH * w.D * (sum(r + 1 for r in rows) if causal else len(rows) * w.S)
    base = {
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": sdpa_oracle.num_threads(),
        "kind": "oracle", "seconds": round(dt, 3),
        "sample": f"{w.name}: all {w.BH} heads x {len(rows)} of {w.S} query rows (evenly spaced) "
                  f"against {'the keys up to its own position' if causal else f'all {w.S} keys'}, float64",
    }
    check = {"max_abs_err": max_abs_err(torch, o, ref, rows), "tol": TOL[dtype],
             "rows_checked": len(rows) * w.BH, "rows_per_head": len(rows), "heads": w.BH,
             "against": "the cpu_baseline sample (float64 oracle), output of the last timed launch"}
    return base, check


def roofline_of(w, ms, flops=None):
    """The roof that bounds a configuration (arithmetic intensity on compulsory bytes against the ridge
    point) and the fraction of it a launch of `ms` milliseconds reaches.  C1 (two or four workgroups)
    is bound by the launch itself: no fraction is meaningful there."""
    flops = w.flops if flops is None else flops
    comp = w.compulsory_bytes(2)
    if w.BH * ((w.S + 127) // 128) < 64:
        return {"bound": "latency", "achieved": round(ms * 1e3, 3), "unit": "us per launch", "peak": None, "frac": None}
    if flops / comp >= PEAK_MFMA_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        tf = flops / (ms * 1e-3) / 1e12
        return {"bound": "mfma", "achieved": round(tf, 2), "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": round(tf / PEAK_MFMA_TFLOPS, 4)}
    gbs = comp / (ms * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": round(gbs / PEAK_HBM_GBS, 4)}


def summarise_workloads(pkg, torch, args, headline_check):
    """Every configuration of the metric (C1..C5) in the heuristic schedule: launch time back to back,
    replayed from a HIP graph (short kernels), cache-cold (tensors in rotation), each against the roof
    that bounds it; the CPU oracle's wall time on the whole of C1..C3; the error of a launch's output
    against the oracle (whole configuration for C1..C3, every query-tile boundary row for C5; C4's is
    the headline's check)."""
    from paper_2603_01960_amd.workloads import sample_rows
    out = {}
    for name, dts in (("C1", ["f16"]), ("C2", ["f16", "bf16"]), ("C3", ["bf16"]), ("C4", ["bf16"]), ("C5", ["f16"])):
        for dt in dts:
            ww, ms, o = time_batched(pkg, torch, name, dt, max(20, args.steps), args.warmup)
            code = pkg.F16 if dt == "f16" else pkg.BF16
            tm, tn = pkg.binding.default_tile(ww.B, ww.H, ww.S, ww.D, code, 0)
            e = {"shape": f"B={ww.B} H={ww.H} S={ww.S} D={ww.D} {dt}", "tile": [tm, tn],
                 "ms_per_launch_back_to_back": round(ms, 5),
                 "tflops": round(ww.flops / (ms * 1e-3) / 1e12, 2),
                 "compulsory_GBs": round(ww.compulsory_bytes(2) / (ms * 1e-3) / 1e9, 1),
                 "roofline": roofline_of(ww, ms), "status": "ok", "status_detail": ""}
            if ms < 0.1:
                gms = time_graph_replay(pkg, torch, name, dt)
                e["hip_graph_replay"] = {
                    "ms_per_launch": round(gms, 5), "tflops": round(ww.flops / (gms * 1e-3) / 1e12, 2),
                    "compulsory_GBs": round(ww.compulsory_bytes(2) / (gms * 1e-3) / 1e9, 1),
                    "roofline": roofline_of(ww, gms)}
            sets = -(-(1 << 30) // int(ww.compulsory_bytes(2)))      # >= 1 GiB of distinct tensors in rotation
            if 1 < sets <= 64:
                _, cms, _ = time_batched(pkg, torch, name, dt, max(4 * sets, args.steps), args.warmup, rotate=sets)
                e["cache_cold"] = {
                    "buffer_sets_in_rotation": sets, "ms_per_launch": round(cms, 5),
                    "tflops": round(ww.flops / (cms * 1e-3) / 1e12, 2),
                    "compulsory_GBs": round(ww.compulsory_bytes(2) / (cms * 1e-3) / 1e9, 1),
                    "roofline": roofline_of(ww, cms)}
            if not args.no_cpu_baseline:
                _, _, q, k, v = device_workload(torch, name, dt)
                if name == "C4":
                    e["check"] = headline_check      # the same tensors, checked on the headline's sample
                else:
                    rows = None if name in ("C1", "C2", "C3") else sample_rows(ww.S)
                    secs, ref = oracle_rows(ww, q, k, v, rows)
                    n = ww.S if rows is None else len(rows)
                    e["check"] = {"max_abs_err": max_abs_err(torch, o, ref, rows), "tol": TOL[dt],
                                  "rows_checked": n * ww.BH, "rows_per_head": n, "heads": ww.BH}
                    if rows is None:
                        e["cpu_oracle_seconds_whole_configuration"] = round(secs, 4)
                if e.get("check") and not (e["check"]["max_abs_err"] <= e["check"]["tol"]):
                    e["status"], e["status_detail"] = "error", "output outside the tolerance"
            out[f"{name}_{dt}"] = e
    return out


def sweep_tiles(pkg, torch, args, w, flops, flags, shape):
    """Every (T_M, T_N) of the paper's Table 1 grid {64,128} x {32,64,128} on the headline workload, and the
    library's own 256-row query tile.  A cell the library does not offer is recorded with its status, not
    dropped (Section 5)."""
    sweep = {}
    for tm_, tn_ in pkg.binding.TILE_ORDER:
        key = f"{tm_}x{tn_}"
        try:
            rr = time_workload(pkg, torch, args.workload, args.dtype, max(10, args.steps // 2), 3, (tm_, tn_), flags,
                               args.input_fill, shape, args.qk_std)
        except pkg.binding.TiledSdpaError as exc:
            sweep[key] = {"status": "unsupported", "status_detail": str(exc), "kernel_ms_avg": None,
                          "tflops": None, "frac_of_mfma_peak": None}
            continue
        tf = flops / (rr["kernel_ms_avg"] * 1e-3) / 1e12
        sweep[key] = {"status": "ok", "status_detail": "", "kernel_ms_avg": round(rr["kernel_ms_avg"], 5),
                      "tflops": round(tf, 2), "frac_of_mfma_peak": round(tf / PEAK_MFMA_TFLOPS, 4)}
    return sweep


def compare_tiles(pkg, torch, args, flags, shape):
    """Tiles of the same workload against each other without the bias of measuring one after the other: every
    round times each tile once (launches back to back between one pair of events), the order reverses from round
    to round, and the median over the rounds is reported."""
    tiles = [tuple(int(x) for x in t.lower().split("x")) for t in args.compare_tiles.split(",")]
    w, dtype, qd, kd, vd = device_workload(torch, args.workload, args.dtype, args.input_fill, shape, args.qk_std)
    o = torch.empty_like(qd)
    flops = w.flops * (0.5 if args.causal else 1.0)
    n = max(8, min(500, int(20e-3 / (flops / 1000e12 + 6e-6))))
    for t in tiles:
        for _ in range(5):
            pkg.sdpa(qd, kd, vd, out=o, tile=t, flags=flags)
    torch.cuda.synchronize()
    legs = {t: [] for t in tiles}
    rounds = 7
    for r in range(rounds):
        for t in (tiles if r % 2 == 0 else tiles[::-1]):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(n):
                pkg.sdpa(qd, kd, vd, out=o, tile=t, flags=flags)
            b.record()
            torch.cuda.synchronize()
            legs[t].append(a.elapsed_time(b) / n)
    med = {t: statistics.median(x) for t, x in legs.items()}
    print(json.dumps({
        "metric": "SDPA forward, tiles compared in alternating order", "unit": "ms per launch (median over rounds)",
        "config": {"workload": f"{w.name}: SDPA fwd {'causal' if args.causal else 'non-causal'} B={w.B} H={w.H} S={w.S} D={w.D} {dtype}",
                   "launches_per_leg": n, "rounds": rounds},
        "tiles": {f"{tm}x{tn}": {"ms": round(med[(tm, tn)], 5), "tflops": round(flops / (med[(tm, tn)] * 1e-3) / 1e12, 2),
                               "min_ms": round(min(legs[(tm, tn)]), 5), "max_ms": round(max(legs[(tm, tn)]), 5)}
                  for tm, tn in tiles},
        "data": "synthetic", "n_gpus": 1}))


# the paper's benchmark grid (Section 4.3): 4 head dims x 5 lengths x 2 dtypes x causal / non-causal = 80 points
GRID_HEAD_DIMS = (64, 96, 128, 160)
GRID_SEQ_LENS = (512, 1024, 2048, 4096, 8192)
GRID_DTYPES = ("f16", "bf16")


def bench_grid(pkg, torch, args):
    """The 80 points of the paper's grid (Section 4.3) on seeded N(0,1) tensors: the plain entry point
    (heuristic tile), and the Sq x Skv entry point with its heuristic key split, which is what fills the
    GPU when B*H*ceil(S/128) is small.  Launches back to back between one pair of events."""
    from paper_2603_01960_amd.workloads import make_qkv
    B, H = (int(x) for x in args.grid.split(","))
    rows = []
    for D in GRID_HEAD_DIMS:
        for S in GRID_SEQ_LENS:
            for dt in GRID_DTYPES:
                q, k, v = (t.cuda() for t in make_qkv(B, H, S, D, dt, seed=7000 + S + D))
                o = torch.empty_like(q)
                code = pkg.F16 if dt == "f16" else pkg.BF16
                for causal in (False, True):
                    flags = pkg.binding.FLAG_CAUSAL if causal else 0
                    flops = 4.0 * B * H * S * S * D * (0.5 if causal else 1.0)
                    n = max(5, min(200, int(2e-3 / (flops / 800e12 + 8e-6))))
                    splits = pkg.kv_default_splits(B, H, S, S, D, code, flags)
                    ws = torch.empty(max(16, pkg.kv_workspace_bytes(B, H, S, D, splits)), dtype=torch.uint8, device="cuda")
                    runs = {"fwd": lambda: pkg.sdpa(q, k, v, causal=causal, out=o),
                            "fwd_kv": lambda: pkg.sdpa_kv(q, k, v, causal=causal, out=o, splits=splits, workspace=ws)}
                    res, times = {}, {label: [] for label in runs}
                    for label, run in runs.items():
                        try:
                            for _ in range(3):
                                run()
                        except pkg.binding.TiledSdpaError as exc:
                            res[label] = {"status": "unsupported", "status_detail": str(exc), "ms": None, "tflops": None}
                    torch.cuda.synchronize()
                    # the two entry points alternate over three rounds (a short measurement taken right after a
                    # pause reads slow: the clocks ramp up), the median of each is kept
                    for _ in range(3):
                        for label, run in runs.items():
                            if label in res:
                                continue
                            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                            a.record()
                            for _ in range(n):
                                run()
                            b.record()
                            torch.cuda.synchronize()
                            times[label].append(a.elapsed_time(b) / n)
                    for label in runs:
                        if label not in res:
                            ms = statistics.median(times[label])
                            res[label] = {"status": "ok", "status_detail": "", "ms": round(ms, 5),
                                          "tflops": round(flops / (ms * 1e-3) / 1e12, 2)}
                    tm, tn = pkg.binding.default_tile(B, H, S, D, code, flags)
                    rows.append({"S": S, "D": D, "dtype": dt, "causal": causal, "tile": [tm, tn], "kv_splits": splits, **res})
    best = max((r["fwd"]["tflops"] or 0.0) for r in rows)
    out = {"metric": "SDPA forward TFLOP/s over the paper's workload grid (4*B*H*S^2*D / t, half under the causal mask)",
           "value": best, "unit": "TFLOP/s (best point, plain entry point)", "n_gpus": 1, "higher_is_better": True,
           "data": "synthetic", "config": {"workload": f"grid: B={B} H={H}, S in 512..8192, D in 64..160, f16/bf16, causal/non-causal"},
           "paper_context": PAPER_CONTEXT, "grid": rows}
    if args.csv:
        import csv
        with open(args.csv, "w", newline="") as f:
            wr = csv.writer(f)
            wr.writerow(["B", "H", "S", "D", "dtype", "causal", "tile_m", "tile_n", "entry", "kv_splits", "ms", "tflops", "status", "status_detail"])
            for r in rows:
                for entry in ("fwd", "fwd_kv"):
                    e = r[entry]
                    wr.writerow([B, H, r["S"], r["D"], r["dtype"], int(r["causal"]), r["tile"][0], r["tile"][1], entry,
                                 r["kv_splits"] if entry == "fwd_kv" else 1, "nan" if e["ms"] is None else e["ms"],
                                 "nan" if e["tflops"] is None else e["tflops"], e["status"], e["status_detail"]])
    print(json.dumps(out), flush=True)


def write_csv(path, out):
    """The sweep cells and the per-configuration rows as CSV, one row each, with status columns."""
    import csv
    with open(path, "w", newline="") as f:
        wr = csv.writer(f)
        wr.writerow(["kind", "name", "tile_m", "tile_n", "ms_per_launch", "tflops", "compulsory_GBs", "bound",
                     "frac_of_roof", "max_abs_err", "tol", "status", "status_detail"])
        for key, e in (out.get("tile_sweep") or {}).items():
            tm, tn = key.split("x")
            wr.writerow(["tile_sweep", out["config"]["workload"], tm, tn,
                         "nan" if e["kernel_ms_avg"] is None else e["kernel_ms_avg"],
                         "nan" if e["tflops"] is None else e["tflops"], "", "mfma",
                         "nan" if e["frac_of_mfma_peak"] is None else e["frac_of_mfma_peak"], "", "",
                         e["status"], e["status_detail"]])
        for key, e in (out.get("all_workloads") or {}).items():
            c = e.get("check") or {}
            wr.writerow(["workload", key, e["tile"][0], e["tile"][1], e["ms_per_launch_back_to_back"], e["tflops"],
                         e["compulsory_GBs"], e["roofline"]["bound"], e["roofline"]["frac"],
                         c.get("max_abs_err", ""), c.get("tol", ""), e["status"], e["status_detail"]])


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (heads are independent, so more GPUs would each run "
              "this same kernel on a slice of B*H); --gpus > 1 is not supported.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2603_01960_amd as pkg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    pkg.load_library()      # no fallback: raises if the HIP library is not built
    torch.cuda.set_device(0)
    if args.copy_calibration:
        copy_calibration(torch, args.copy_mib, args.steps)
        return
    tile = tuple(int(x) for x in args.tile.split(",")) if args.tile else None
    flags = (pkg.binding.FLAG_LINEAR_GRID if args.linear_grid else 0) \
        | (pkg.binding.FLAG_EXACT_MAX if args.exact_max else 0) \
        | (pkg.binding.FLAG_CAUSAL if args.causal else 0)

    if args.grid:
        bench_grid(pkg, torch, args)
        return
    if args.kv:
        bench_kv(pkg, torch, args, tile, flags)
        return
    if args.bwd:
        bench_bwd(pkg, torch, args, flags)
        return
    shape = tuple(int(x) for x in args.shape.split(",")) if args.shape else None
    if args.compare_tiles:
        compare_tiles(pkg, torch, args, flags, shape)
        return
    plain = shape is None and args.input_fill == "normal" and args.qk_std is None and not args.causal
    tuned = None
    if args.tune and tile is None:
        # schedule search on the workload's own tensors, before and outside the timed region
        _, _, tq, tk, tv = device_workload(torch, args.workload, args.dtype, args.input_fill, shape, args.qk_std)
        tile, times = pkg.tune_tile(tq, tk, tv, causal=args.causal, launches=20, flags=flags)
        tuned = {f"{a}x{b}": round(t, 5) for (a, b), t in times.items()}
    r = time_workload(pkg, torch, args.workload, args.dtype, args.steps, args.warmup, tile, flags, args.input_fill, shape, args.qk_std)
    w, dtype = r["workload"], r["dtype"]
    flops = w.flops * (0.5 if args.causal else 1.0)     # causal: 2*B*H*S^2*D, the usual convention
    tflops = flops / (r["ms_per_step"] * 1e-3) / 1e12
    kern_tflops = flops / (r["kernel_ms_avg"] * 1e-3) / 1e12
    tm, tn = tile if tile else pkg.binding.default_tile(w.B, w.H, w.S, w.D, pkg.F16 if dtype == "f16" else pkg.BF16, flags)

    # which roof bounds the kernel: arithmetic intensity on compulsory bytes vs the ridge point
    comp_bytes = w.compulsory_bytes(2)
    roofline = roofline_of(w, r["kernel_ms_avg"], flops)
    # counters are committed per instantiation: one tile's traffic says nothing about another's
    if plain and not args.linear_grid and not args.exact_max:
        roofline["traffic"], roofline["traffic_source"] = profiled_traffic(w.name, dtype, w.D, tm, tn)
    else:
        roofline["traffic"], roofline["traffic_source"] = None, "not the profiled configuration (flags, inputs or shape differ)"
    roofline["kernel"] = f"sdpa_fwd_kernel<{dtype},D={w.D},T_M={tm},T_N={tn}>"
    roofline["kernel_ms_avg"] = round(r["kernel_ms_avg"], 5)
    roofline["kernel_ms_median"] = round(r["kernel_ms_median"], 5)
    roofline["kernel_ms_p95"] = round(r["kernel_ms_p95"], 5)
    roofline["algorithmic_flops_per_launch"] = flops
    roofline["compulsory_hbm_bytes_per_launch"] = comp_bytes

    out = {
        "metric": "SDPA forward TFLOP/s (4*B*H*S^2*D / t)", "value": round(tflops, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(r["ms_per_step"], 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype,
        "data": "synthetic" if args.input_fill == "normal" else f"constant {args.input_fill} (clock experiment)",
        "config": {"workload": f"{w.name}: SDPA fwd {'causal' if args.causal else 'non-causal'} "
                               f"B={w.B} H={w.H} S={w.S} D={w.D} {dtype}",
                   "tile_m": tm, "tile_n": tn, "seed": w.seed, "qk_std": round(w.qk_std, 6),
                   "tokens_per_s": round(w.BH * w.S / (r["ms_per_step"] * 1e-3), 1)},
        "roofline": roofline,
        "frac_of_mfma_peak": round(tflops / PEAK_MFMA_TFLOPS, 4),
        "paper_context": PAPER_CONTEXT,
        "env": {"torch": torch.__version__, "hip": torch.version.hip, "device": torch.cuda.get_device_name(0),
                "library_version": pkg.version(), "host": platform.processor() or platform.machine()},
    }

    if tuned is not None:
        out["config"]["tile_chosen_by"] = "tiled_sdpa_tune_tile (20 launches per candidate)"
        out["config"]["tune_ms_per_launch"] = tuned
    if not args.no_ceilings:
        ceil = mfma_ceilings(pkg, torch, dtype)
        out["mfma_only_ceiling_tflops"] = ceil
        out["frac_of_mfma_only_ceiling_random_operands"] = round(kern_tflops / ceil["random_operands"], 4)
        out["frac_of_loop_mix_ceiling"] = round(kern_tflops / ceil["random_operands_plus_loop_mix"], 4)
        out["hbm_copy_ceiling_GBs"] = hbm_copy_ceiling(torch)
        if roofline["bound"] == "hbm" or (plain and args.all_workloads):
            out["hbm_read_ceiling_GBs"] = hbm_read_ceiling(pkg, torch)
        if roofline["bound"] == "hbm":
            out["frac_of_hbm_read_ceiling"] = round(roofline["achieved"] / out["hbm_read_ceiling_GBs"], 4)

    if args.sweep_tiles:
        out["tile_sweep"] = sweep_tiles(pkg, torch, args, w, flops, flags, shape)

    check = None
    if not args.no_cpu_baseline:
        q, k, v = r["tensors"]
        out["cpu_baseline"], check = cpu_baseline(torch, w, dtype, q, k, v, r["o"], args.cpu_seconds, args.causal)
        out["max_abs_err"], out["tol"], out["rows_checked"] = check["max_abs_err"], check["tol"], check["rows_checked"]
        out["correctness"] = check

    if args.all_workloads and plain:
        out["all_workloads"] = summarise_workloads(pkg, torch, args, check if w.name == "C4" and dtype == "bf16" else None)
        rd = out.get("hbm_read_ceiling_GBs")
        for e in out["all_workloads"].values():
            if rd and e["roofline"]["bound"] == "hbm":
                for leg in (e, e.get("hip_graph_replay"), e.get("cache_cold")):
                    if leg:
                        leg["roofline"]["frac_of_hbm_read_ceiling"] = round(leg["roofline"]["achieved"] / rd, 4)

    if args.csv:
        write_csv(args.csv, out)
    print(json.dumps(out), flush=True)
    if check is not None and not (check["max_abs_err"] <= check["tol"]):
        print(f"bench.py: output error {check['max_abs_err']} exceeds the tolerance {check['tol']}", file=sys.stderr)
        sys.exit(4)


if __name__ == "__main__":
    main()
