#!/usr/bin/env python3
"""Benchmark of the MotionDeltaCNN hot path on one MI355X.

One step = one frame of the whole per-frame path (camera shift + dynamic
initialisation, delta/truncation/mask, compaction, padded sparse convolutions,
residual adds, readout) on the headline workload: the ResNet-18-style 512x512
fp16 network on the seeded 60-frame moving-camera sequence, all frames resident
in HBM before the timed region starts.  The sequence is replayed cyclically (the
jump back to its start is one more camera shift, which the buffer manager
answers with a full reset).  The video goes through `mdcnn_frames`, in calls of as
many frames as the sequence has, which keeps up to --frames-in-flight consecutive frames
in flight (same launches, same results bit for bit as one `mdcnn_frame` call per
frame; that rate is reported next to it as "frame_at_a_time" and is the headline
with --frames-in-flight 1 and for networks of fewer than 16 launches per frame;
--crops uses mdcnn_frames_crop, --front-end mdcnn_frames_masked).

Prints ONE JSON line.  `value` is the median over --reps repetitions of the timed
region of --steps frames.  Besides the throughput the line carries
  roofline       -- the dominant kernel class, timed with HIP events recorded by
                    the library around every launch of a second, instrumented pass
                    over the same frames (algorithmic flops / bytes from device-side
                    counters of that pass);
  per_layer      -- the same per layer: the convolution launches into every site and
                    the delta launch of every site, with their own bound
                    max(bytes / HBM peak, flops / matrix peak);
  measured_peaks -- what a plain copy kernel and a loop of matrix-core instructions
                    reach on this machine, and the fractions against those;
  frame_at_a_time-- one mdcnn_frame call per frame (the latency of a frame), with the
                    rate over the frames that are neither the first nor a reset;
  dense_mode     -- the same library with threshold 0 and every pixel forced;
  cpu_baseline   -- the NumPy oracle timed on the host cores on the first frames
                    of the same sequence.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_F16_TFLOPS = 2500.0
PEAK_MFMA_F32_TFLOPS = 157.3      # fp32 networks: their layers run on v_mfma_f32_32x32x2_f32
PEAK_FP32_VALU_TFLOPS = 157.3


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=180)
    ap.add_argument("--warmup", type=int, default=60)
    ap.add_argument("--config", type=int, default=3, help="benchmark workload 1..5 (3 = headline)")
    ap.add_argument("--density", type=float, default=0.2, help="config 5 only")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the oracle baseline; 0 disables it")
    ap.add_argument("--reps", type=int, default=5, help="repetitions of the timed region; the median is reported")
    ap.add_argument("--dense", action="store_true", help="library dense mode: threshold 0 and all pixels forced")
    ap.add_argument("--no-dense-leg", action="store_true", help="skip the dense-mode leg of the default run")
    ap.add_argument("--f32-storage", action="store_true",
                    help="the same network and frames with fp32 storage instead of fp16 (what the storage type costs or buys; "
                         "its wide layers have no matrix-core kernel and run as plain FMA)")
    ap.add_argument("--truncation-free", action="store_true",
                    help="sites after a 1x1 convolution keep no pending ring and never truncate (config 5: one of its three inner sites)")
    ap.add_argument("--pool-stem", action="store_true",
                    help="config 3 with the usual ResNet stem: 3x3 stride-2 max pooling after the stem convolution (total stride 16)")
    ap.add_argument("--crops", action="store_true",
                    help="every frame covers a bounding box of about 2/3 x 2/3 of the view that wanders over it "
                         "(mdcnn_frame_crop; one stream only)")
    ap.add_argument("--front-end", action="store_true",
                    help="the input update mask of every frame comes from mdcnn_input_mask (isolated updates suppressed, "
                         "dilation by 2 pixels) and is forced; one stream only")
    ap.add_argument("--frames-in-flight", type=int, default=0,
                    help="streams on which mdcnn_frames keeps consecutive frames of the video in flight (1..4); 1: one mdcnn_frame "
                         "call per frame; 0 (default): the library's own rule, 4 if a frame has at least 16 launches, else 1")
    ap.add_argument("--streams", type=int, default=8,
                    help="after the headline run, the same workload as a batch of this many independent streams "
                         "(mdcnn_frame_batch; reported under \"batched\"); 0 disables it")
    ap.add_argument("--opt", action="append", default=[], metavar="ID=VALUE",
                    help="library tuning option (mdcnn_set_option), e.g. --opt 6=0 switches the halo-staged kernel off")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a kernel of known traffic, to scale rocprofv3 byte counters)")
    return ap.parse_args()


def site_bytes_per_pixel(g, i):
    return g.shape[i][2] * g.esize


def algorithmic_bytes(g, spec, before, after, frames, fused_skips=True):
    """Algorithmic HBM bytes of the memory-bound passes over `frames` frames,
    from the device-side counters (differences of the running sums).  With fused
    residual skips the delta kernel of the source also reads and writes the
    pending row of the skip's destination for every updated pixel."""
    d = {k: after["per_site"][k] - before["per_site"][k] for k in after["per_site"]}
    step1 = 0
    if fused_skips:
        seen = set()
        for e in spec.edges:
            if e.k == 0 and e.src not in seen:        # one fused skip per source site
                seen.add(e.src)
                step1 += int(d["updated"][e.src]) * 2 * site_bytes_per_pixel(g, e.src)
    for i, s in enumerate(spec.sites):
        if s.kind == "output":
            continue
        H, W, _ = g.shape[i]
        cb = site_bytes_per_pixel(g, i)
        # flags read+write per pixel; candidates read A and (X or P); updated write A, delta (and P)
        writes = 2 if s.kind == "input" else 3
        step1 += frames * H * W * 2 + int(d["candidates"][i]) * 2 * cb + int(d["updated"][i]) * writes * cb
    # convolutions: every updated source row once, read-modify-write of the pending
    # row of every compute-list entry, the weights once per launch
    conv = 0
    skip_entries = [0] * len(spec.sites)
    for e in spec.edges:
        if e.k == 0 and not fused_skips:              # fused skips add nothing to the compute statistics
            skip_entries[e.dst] += int(d["updated"][e.src])
    pool = 0
    pooled = set()
    for e in spec.edges:
        if getattr(e, "pool", False):
            # per computed output: stride^2 source rows (each source pixel once), previous output
            # read + written, pending row read + written
            pooled.add(e.dst)
            pool += int(d["compute"][e.dst]) * (e.stride * e.stride + 4) * site_bytes_per_pixel(g, e.dst)
    for e in spec.edges:
        if e.k == 0 or getattr(e, "pool", False):
            continue
        conv += int(d["updated"][e.src]) * site_bytes_per_pixel(g, e.src) + frames * e.w.size * g.esize
    for i, s in enumerate(spec.sites):
        if s.kind != "input" and i not in pooled:
            conv += max(int(d["compute"][i]) - skip_entries[i], 0) * 2 * site_bytes_per_pixel(g, i)
    return dict(step1=step1, conv=conv, pool=pool)


def measured_traffic(cfg, cls):
    """HBM bytes per launch from the committed rocprofv3 byte-counter summary, if any."""
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            return json.load(f)[f"config{cfg}"][cls]["hbm_bytes_per_launch"]
    except Exception:
        return None


def rooflines(prof, flops_mfma, flops_plain, ab, cfg, with_traffic=True, mfma_peak=PEAK_MFMA_F16_TFLOPS):
    """Per-class kernel times (from the library's HIP events) and the roofline entries."""
    tr = (lambda c: measured_traffic(cfg, c)) if with_traffic else (lambda c: None)
    classes = {}
    for k, (ms, cnt) in prof.items():
        if cnt:
            classes[k] = {"ms_total": round(ms, 3), "launches": int(cnt), "avg_us": round(1e3 * ms / cnt, 2)}
    kernel_ms = sum(v[0] for v in prof.values())
    dominant = max(prof, key=lambda k: prof[k][0])
    rl_all = {}
    if prof["conv_mfma"][1]:
        ms, cnt = prof["conv_mfma"]
        ach = flops_mfma / (ms * 1e-3) / 1e12
        rl_all["conv_mfma"] = {"bound": "mfma", "achieved": round(ach, 2), "peak": mfma_peak, "unit": "TFLOP/s",
                               "frac": round(ach / mfma_peak, 4), "traffic": tr("conv_mfma"),
                               "flop_per_launch": round(flops_mfma / cnt), "avg_us": round(1e3 * ms / cnt, 2), "launches": int(cnt),
                               "algorithmic_bytes_per_launch": round(ab["conv"] / (cnt + prof["conv_plain"][1])),
                               "hbm_bound_us": round(ab["conv"] / (cnt + prof["conv_plain"][1]) / PEAK_HBM_GBS / 1e3, 2),
                               "mfma_bound_us": round(flops_mfma / cnt / mfma_peak / 1e6, 2)}
    if prof["conv_plain"][1]:
        ms, cnt = prof["conv_plain"]
        ach = flops_plain / (ms * 1e-3) / 1e12
        rl_all["conv_plain"] = {"bound": "alu", "achieved": round(ach, 3), "peak": PEAK_FP32_VALU_TFLOPS, "unit": "TFLOP/s",
                                "frac": round(ach / PEAK_FP32_VALU_TFLOPS, 5), "traffic": tr("conv_plain"),
                                "flop_per_launch": round(flops_plain / cnt), "avg_us": round(1e3 * ms / cnt, 2), "launches": int(cnt)}
    if prof["step1"][1]:
        ms, cnt = prof["step1"]
        ach = ab["step1"] / (ms * 1e-3) / 1e9
        rl_all["step1"] = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": tr("step1"),
                           "bytes_per_launch": round(ab["step1"] / cnt), "avg_us": round(1e3 * ms / cnt, 2), "launches": int(cnt)}
    if prof.get("pool", (0, 0))[1]:
        ms, cnt = prof["pool"]
        ach = ab["pool"] / (ms * 1e-3) / 1e9
        rl_all["pool"] = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                          "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": None,
                          "bytes_per_launch": round(ab["pool"] / cnt), "avg_us": round(1e3 * ms / cnt, 2), "launches": int(cnt)}
    roofline = dict(rl_all.get(dominant, next(iter(rl_all.values()))))
    roofline["kernel"] = dominant if dominant in rl_all else next(iter(rl_all))
    return classes, kernel_ms, rl_all, roofline


def sum_totals(ts):
    """Adds up GpuNet.totals() of several streams."""
    out = {k: sum(t[k] for t in ts) for k in ts[0] if k != "per_site"}
    out["per_site"] = {k: sum(t["per_site"][k] for t in ts) for k in ts[0]["per_site"]}
    return out


def run_batched(a, cfg, net, T, frames, shifts, forced, fused):
    """The same workload as a.streams independent streams in shared launches: stream b
    plays the sequence cyclically from frame b * T / streams on."""
    import torch
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuBatch
    n = a.streams
    # with many videos of the ResNet-18-style network to a launch whole-segment convolution tiles are the faster choice (the
    # default follows one video); the small maps of the other networks are better off with the default
    whole_tiles = cfg == 3 and not any(o.startswith("7=") for o in a.opt)
    if whole_tiles:
        B.mdcnn_set_option(B.MDCNN_OPT_CONV_HALO_SUB, 1)
    gb = GpuBatch(net, n)
    phase = [(b * T) // n for b in range(n)]
    state = {"t": 0}

    def step():
        ts = [(state["t"] + p) % T for p in phase]
        first = state["t"] == 0
        gb.frame([frames[t] for t in ts], [0 if first else int(shifts[t][0]) for t in ts],
                 [0 if first else int(shifts[t][1]) for t in ts],
                 None if forced is None else [forced[t] for t in ts])
        state["t"] += 1

    steps = max(10, a.steps // n * 2)
    for _ in range(max(4, a.warmup // n)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    before = sum_totals([g.totals() for g in gb.streams])
    B.mdcnn_set_option(B.MDCNN_OPT_PROFILE, 1)
    B.mdcnn_profile_read()
    n_prof = min(steps, T)
    for _ in range(n_prof):
        step()
    launches = B.mdcnn_profile_read_launches()
    prof = {k: (0.0, 0) for k in B.KERNEL_CLASSES}
    for cls, _, _, us in launches:
        prof[cls] = (prof[cls][0] + us * 1e-3, prof[cls][1] + 1)
    B.mdcnn_set_option(B.MDCNN_OPT_PROFILE, 0)
    after = sum_totals([g.totals() for g in gb.streams])
    ab = algorithmic_bytes(gb.streams[0], net, before, after, n_prof * n, fused_skips=fused)
    classes, kernel_ms, rl_all, _ = rooflines(prof, 2.0 * (after["macs_mfma"] - before["macs_mfma"]),
                                              2.0 * (after["macs_plain"] - before["macs_plain"]), ab, cfg, with_traffic=False,
                                              mfma_peak=PEAK_MFMA_F32_TFLOPS if net.dtype == "f32" else PEAK_MFMA_F16_TFLOPS)
    peak = PEAK_MFMA_F32_TFLOPS if net.dtype == "f32" else PEAK_MFMA_F16_TFLOPS
    pf_mfma = 2.0 * (after["macs_mfma"] - before["macs_mfma"]) / (n_prof * n)
    pf_bytes = sum(ab.values()) / (n_prof * n)
    whole = lambda rate: {"mfma_tflops": round(pf_mfma * rate / 1e12, 2), "mfma_frac": round(pf_mfma * rate / 1e12 / peak, 4),
                          "algorithmic_gbs": round(pf_bytes * rate / 1e9, 1), "hbm_frac": round(pf_bytes * rate / 1e9 / PEAK_HBM_GBS, 4)}
    layers = per_layer_rows(launches, gb.streams[0], net, before, after, n_prof * n, peak, fused) if n <= 16 else None
    res = {"streams": n, "value": round(n * steps / dt, 2), "unit": "frames/s", "batch_steps": steps, "whole_path": whole(n * steps / dt),
           "per_layer": layers, "per_layer_note": "us, flops and bytes per frame of one video (a launch carries one frame of every video)",
           "ms_per_batch_step": round(1e3 * dt / steps, 4), "roofline_all": rl_all, "kernel_classes": classes,
           "kernel_ms_per_batch_step": round(kernel_ms / n_prof, 4)}
    # the same batch with frames of every video in flight (mdcnn_frames_batch): calls of T frames per video
    if a.frames_in_flight != 1 and T >= 8:
        outs = [[torch.empty_like(gb.streams[0].out) for _ in range(n)] for _ in range(T)]

        def call(depth):
            ts = [[(state["t"] + f + p) % T for p in phase] for f in range(T)]
            gb.frames([[frames[t] for t in row] for row in ts], [[int(shifts[t][0]) for t in row] for row in ts],
                      [[int(shifts[t][1]) for t in row] for row in ts],
                      None if forced is None else [[forced[t] for t in row] for row in ts], outs=outs, depth=depth)
            state["t"] += T

        flight = {}
        for depth in (2, 4):
            call(depth)
            torch.cuda.synchronize()
            rates = []
            for _ in range(3):
                t0 = time.perf_counter()
                call(depth)
                torch.cuda.synchronize()
                rates.append(n * T / (time.perf_counter() - t0))
            flight[f"depth_{depth}"] = round(sorted(rates)[1], 2)
        best = max(flight.values())
        res["in_flight"] = {"entry_point": "mdcnn_frames_batch, calls of %d frames x %d videos" % (T, n), "unit": "frames/s", **flight,
                            "value": best, "whole_path": whole(best)}
    gb.close()
    if whole_tiles:
        B.mdcnn_set_option(B.MDCNN_OPT_CONV_HALO_SUB, 0)
        res["options"] = "MDCNN_OPT_CONV_HALO_SUB = 1 (whole-segment convolution tiles)"
    return res


def measured_peaks(torch, B):
    """What this machine reaches on a plain copy kernel (1 GiB) and on a loop of independent matrix-core
    instructions: the achievable peaks to set beside the published ones."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    B.mdcnn_bench_copy(src.data_ptr(), dst.data_ptr(), n, st)
    ev[0].record()
    for _ in range(3):
        B.mdcnn_bench_copy(src.data_ptr(), dst.data_ptr(), n, st)
    ev[1].record()
    blocks, iters = 2048, 4000
    flops = B.mdcnn_bench_mfma(iters, blocks, sink.data_ptr(), st)
    ev[2].record()
    flops = B.mdcnn_bench_mfma(iters, blocks, sink.data_ptr(), st)
    ev[3].record()
    torch.cuda.synchronize()
    copy_gbs = 3 * 2.0 * n / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9          # bytes read + bytes written
    mfma_tflops = flops / (ev[2].elapsed_time(ev[3]) * 1e-3) / 1e12
    del src, dst
    return {"stream_copy_gbs": round(copy_gbs, 1), "stream_copy": "1 GiB device-to-device, own kernel, read + write counted",
            "mfma_f16_tflops": round(mfma_tflops, 1), "mfma_loop": f"{blocks} blocks x 4 waves x {iters} x 4 v_mfma_f32_32x32x16_f16, operands in registers"}


def per_layer_rows(launches, g, net, before, after, n_prof, mfma_peak, fused_skips):
    """One row per layer from the tagged launches of the instrumented pass: all convolution / pooling launches into
    a site together (their summed mean duration per frame against the site's algorithmic flops and bytes), and the
    delta launch of every site.  bound_us = max(bytes / HBM peak, flops / matrix peak); frac = bound_us / us."""
    d = {k: after["per_site"][k] - before["per_site"][k] for k in after["per_site"]}
    cb = lambda i: g.shape[i][2] * g.esize
    t_edge, t_step1, k_edge = {}, {}, {}
    for cls, site, edge, us in launches:
        if cls == "step1" and site >= 0:
            t_step1[site] = t_step1.get(site, 0.0) + us
        elif edge >= 0 and cls in ("conv_mfma", "conv_plain", "pool", "identity"):
            t_edge[edge] = t_edge.get(edge, 0.0) + us
            k_edge[edge] = cls
    rows = []
    skip_src = set()
    if fused_skips:
        seen = set()
        for e in net.edges:
            if e.k == 0 and e.src not in seen:
                seen.add(e.src)
                skip_src.add(e.src)
    for i, sp in enumerate(net.sites):
        if i in t_step1:
            writes = 2 if sp.kind == "input" else 3
            H, W, _ = g.shape[i]
            by = n_prof * H * W * 2 + int(d["candidates"][i]) * 2 * cb(i) + int(d["updated"][i]) * (writes + (2 if i in skip_src else 0)) * cb(i)
            us = t_step1[i] / n_prof
            bound = by / n_prof / PEAK_HBM_GBS / 1e3
            rows.append({"site": i, "name": sp.name, "kernel": "step1", "us": round(us, 2), "bytes": round(by / n_prof),
                         "bound_us": round(bound, 2), "frac": round(bound / us, 4) if us else None})
        mine = [k for k, e in enumerate(net.edges) if e.dst == i and k in t_edge]
        if not mine:
            continue
        us = sum(t_edge[k] for k in mine) / n_prof
        flops = 2.0 * (int(d["macs_mfma"][i]) + int(d["macs_plain"][i])) / n_prof
        by = int(d["compute"][i]) * 2 * cb(i)
        for k in mine:
            e = net.edges[k]
            by += int(d["updated"][e.src]) * cb(e.src) + (n_prof * e.w.size * g.esize if e.w is not None else 0)
        by /= n_prof
        bound = max(by / PEAK_HBM_GBS / 1e3, flops / mfma_peak / 1e6)
        rows.append({"site": i, "name": sp.name, "kernel": "+".join(sorted({k_edge[k] for k in mine})),
                     "edges": [f"{net.edges[k].src}->{i} {net.edges[k].k}x{net.edges[k].k}" + (f"/s{net.edges[k].stride}" if net.edges[k].stride > 1 else "") for k in mine],
                     "us": round(us, 2), "flops": round(flops), "bytes": round(by), "bound_us": round(bound, 2),
                     "bound": "mfma" if flops / mfma_peak / 1e6 > by / PEAK_HBM_GBS / 1e3 else "hbm", "frac": round(bound / us, 4) if us else None})
    return rows


class Workload:
    """One network on the GPU plus the two ways a video is pushed through it."""

    def __init__(self, a, net, seq, forced_all_ones=False):
        import numpy as np
        import torch
        from paper_2210_09887_amd import binding as B
        from paper_2210_09887_amd.runtime import GpuNet
        self.a, self.net, self.seq, self.B, self.torch = a, net, seq, B, torch
        self.T = T = len(seq.frames)
        shifts = seq.shifts.astype(np.int64).copy()
        shifts[0] = -shifts[1:].sum(axis=0)            # closing the cycle: jump back to the start
        self.shifts = shifts
        self.frames = torch.from_numpy(seq.frames).cuda()
        self.forced = None
        if forced_all_ones:
            self.forced = torch.ones((T, net.H, net.W), dtype=torch.uint8, device="cuda")
        elif seq.forced is not None:
            self.forced = torch.from_numpy(seq.forced).cuda()
        self.g = g = GpuNet(net, crops=a.crops)
        self.crops = None
        if a.crops:
            # a box of about 2/3 x 2/3 of the view, moving by one tile every fourth frame (seeded walk)
            rng = np.random.default_rng(2210)
            Ts = net.total_stride
            Ht, Wt = net.H // Ts, net.W // Ts
            th, tw = max(1, round(2 * Ht / 3)), max(1, round(2 * Wt / 3))
            y, x = (Ht - th) // 2, (Wt - tw) // 2
            crops = []
            for t in range(T):
                if t % 4 == 0 and t:
                    y = int(np.clip(y + rng.integers(-1, 2), 0, Ht - th))
                    x = int(np.clip(x + rng.integers(-1, 2), 0, Wt - tw))
                crops.append((y, x, th, tw))
            crops[0] = (0, 0, Ht, Wt)                  # the cycle starts from a frame that covers the whole view
            cut = lambda v, c: v[c[0] * Ts:(c[0] + c[2]) * Ts, c[1] * Ts:(c[1] + c[3]) * Ts].contiguous()
            self.crops = crops
            self.frames_c = [cut(self.frames[t], crops[t]) for t in range(T)]
            self.forced_c = None if self.forced is None else [cut(self.forced[t], crops[t]) for t in range(T)]
        self.FE = dict(suppress=True, dilate=2)
        self.state = {"t": 0, "resets": 0}
        self.in_flight = a.frames_in_flight or (4 if len(B.mdcnn_frame_plan(g.net, 1)[0]) >= 16 else 1)
        self.outs_pool = [torch.empty_like(g.out) for _ in range(min(T, max(a.steps, a.warmup)))] if self.in_flight > 1 else []
        self.masks_pool = [torch.empty((net.H, net.W), dtype=torch.uint8, device="cuda") for _ in self.outs_pool] if a.front_end else []
        self.step = self._make_step()

    def _make_step(self):
        """One frame through one call (closure over locals: at 20 us per frame the host's own overhead counts)."""
        a, g, net, B, st, T = self.a, self.g, self.net, self.B, self.state, self.T
        frames, forced, shifts, crops, FE = self.frames, self.forced, self.shifts, self.crops, self.FE
        frame_call = g.frame
        sh = [(int(v[0]), int(v[1])) for v in shifts]

        def step():
            n = st["t"]
            t = n % T
            dy, dx = sh[t] if n else (0, 0)
            if a.front_end:
                # the mask needs the shifted buffers: shift, mask, then the forward calls of mdcnn_frame one by one
                r = g.shift_camera(dy, dx)
                fm = g.input_mask(frames[t], **FE)
                for i, sp in enumerate(net.sites):
                    if sp.kind != "output":
                        g.layer_forward(i, frames[t] if i == 0 else None, fm if i == 0 else None)
                for i in g.terminals:
                    B.mdcnn_read_view(g.bufs[i], B.MDCNN_VIEW_OUT, g.out.data_ptr(), g.out.numel() * g.esize, g._stream())
            elif crops is not None:
                _, r = g.frame_crop(self.frames_c[t], dy, dx, crops[t], None if forced is None else self.forced_c[t])
            else:
                _, r = frame_call(frames[t], dy, dx, None if forced is None else forced[t])
            st["t"] = n + 1
            st["resets"] += r
            return r
        return step

    def one_by_one(self, n):
        step = self.step
        for _ in range(n):
            step()

    def run_frames(self, n):
        """n frames of the video through mdcnn_frames, in calls of as many frames as the sequence has."""
        a, g, st, T, frames, forced, shifts = self.a, self.g, self.state, self.T, self.frames, self.forced, self.shifts
        done = 0
        while done < n:
            t0_ = st["t"]
            m = min(n - done, len(self.outs_pool))
            idx = [(t0_ + k) % T for k in range(m)]
            sh = [(0, 0) if t0_ + k == 0 else (int(shifts[i][0]), int(shifts[i][1])) for k, i in enumerate(idx)]
            if a.front_end:
                _, _, rs = g.frames_masked([frames[i] for i in idx], [v[0] for v in sh], [v[1] for v in sh], outs=self.outs_pool[:m],
                                           masks=self.masks_pool[:m], depth=self.in_flight, **self.FE)
            elif self.crops is not None:
                _, rs = g.frames_crop([self.frames_c[i] for i in idx], [v[0] for v in sh], [v[1] for v in sh], [self.crops[i] for i in idx],
                                      None if forced is None else [self.forced_c[i] for i in idx], outs=self.outs_pool[:m], depth=self.in_flight)
            else:
                _, rs = g.frames([frames[i] for i in idx], [v[0] for v in sh], [v[1] for v in sh],
                                 None if forced is None else [forced[i] for i in idx], outs=self.outs_pool[:m], depth=self.in_flight)
            st["t"] += m
            st["resets"] += sum(int(r) for r in rs)
            done += m

    def timed(self, run, reps):
        """`reps` repetitions of the timed region (a.steps frames each, device synchronised on both sides) after
        a.warmup frames; returns the list of (seconds, resets)."""
        torch = self.torch
        run(self.a.warmup)
        out = []
        for _ in range(reps):
            torch.cuda.synchronize()
            self.state["resets"] = 0
            t0 = time.perf_counter()
            run(self.a.steps)
            torch.cuda.synchronize()
            out.append((time.perf_counter() - t0, self.state["resets"]))
        return out


def median_of(runs):
    """The repetition with the median time (the lower one of two): (seconds, resets)."""
    return sorted(runs)[(len(runs) - 1) // 2]


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from inputs import build_net, build_sequence
    from inputs.nets import truncation_free
    from paper_2210_09887_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)

    cfg = a.config
    net_kw = {"pool_stem": True} if a.pool_stem and cfg == 3 else {}
    net = build_net(cfg, **net_kw)
    if a.truncation_free:
        truncation_free(net)
    seq = build_sequence(cfg, **({"density": a.density} if cfg == 5 else {"tile": 16} if a.pool_stem and cfg == 3 else {}))
    if a.f32_storage and net.dtype == "f16":
        net.dtype = "f32"
        for e in net.edges:
            if e.w is not None:
                e.w = e.w.astype(np.float32)
        seq.frames = seq.frames.astype(np.float32)
    if a.dense:
        for s in net.sites:
            s.theta = 0.0
    for kv in a.opt:
        k, v = kv.split("=")
        B.mdcnn_set_option(int(k), int(v))
    if a.crops or a.front_end:
        a.streams = 0
    if a.front_end:
        assert not a.crops and not a.dense and seq.forced is None, "--front-end excludes --crops, --dense and config 5"

    peaks = measured_peaks(torch, B)
    wl = Workload(a, net, seq, forced_all_ones=a.dense)
    g, T, in_flight, crops, frames = wl.g, wl.T, wl.in_flight, wl.crops, wl.frames
    reps = max(1, a.reps)

    each_runs = None
    if in_flight > 1:
        runs = wl.timed(wl.run_frames, reps)
        each_runs = wl.timed(wl.one_by_one, reps)
    else:
        runs = wl.timed(wl.one_by_one, reps)
    dt, resets_timed = median_of(runs)
    dt_each = median_of(each_runs)[0] if each_runs else None

    # ---- one frame per call with a pair of events around every call: what a reset frame costs, and the rate
    #      over the frames that are neither the first of the cycle nor a reset
    n_kind = min(2 * T, max(a.steps, 2))
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_kind)]
    kinds = []
    torch.cuda.synchronize()
    for k in range(n_kind):
        first_of_cycle = wl.state["t"] % T == 0
        evs[k][0].record()
        r = wl.step()
        evs[k][1].record()
        kinds.append("reset" if r or first_of_cycle else "sparse")
    # what a pair of events costs by itself (nothing between them) is taken off every interval
    cal = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(50)]
    for e0, e1 in cal:
        e0.record()
        e1.record()
    torch.cuda.synchronize()
    ev_ms = sorted(e0.elapsed_time(e1) for e0, e1 in cal)[len(cal) // 2]
    ms_kind = {"reset": [], "sparse": []}
    for k in range(n_kind):
        ms_kind[kinds[k]].append(max(evs[k][0].elapsed_time(evs[k][1]) - ev_ms, 0.0))

    # ---- instrumented pass: per-launch kernel time (HIP events around every launch)
    before = g.totals()
    B.mdcnn_set_option(B.MDCNN_OPT_PROFILE, 1)
    B.mdcnn_profile_read()
    n_prof = min(a.steps, 2 * T)
    t1 = time.perf_counter()
    for _ in range(n_prof):
        wl.step()
    launches = B.mdcnn_profile_read_launches()
    dt_prof = time.perf_counter() - t1
    B.mdcnn_set_option(B.MDCNN_OPT_PROFILE, 0)
    after = g.totals()
    prof = {k: (0.0, 0) for k in B.KERNEL_CLASSES}
    for cls, _, _, us in launches:
        prof[cls] = (prof[cls][0] + us * 1e-3, prof[cls][1] + 1)

    fused = "8=0" not in a.opt
    flops_mfma = 2.0 * (after["macs_mfma"] - before["macs_mfma"])
    flops_plain = 2.0 * (after["macs_plain"] - before["macs_plain"])
    ab = algorithmic_bytes(g, net, before, after, n_prof, fused_skips=fused)
    mfma_peak = PEAK_MFMA_F32_TFLOPS if net.dtype == "f32" else PEAK_MFMA_F16_TFLOPS
    classes, kernel_ms, rl_all, roofline = rooflines(prof, flops_mfma, flops_plain, ab, cfg, mfma_peak=mfma_peak)
    layers = per_layer_rows(launches, g, net, before, after, n_prof, mfma_peak, fused)
    # fractions against what this machine reaches (the matrix-core loop is fp16: fp32 networks keep the published peak only)
    for k, v in rl_all.items():
        if v["bound"] == "hbm":
            v["frac_of_measured_copy"] = round(v["achieved"] / peaks["stream_copy_gbs"], 4)
        elif v["bound"] == "mfma" and net.dtype == "f16":
            v["frac_of_measured_mfma"] = round(v["achieved"] / peaks["mfma_f16_tflops"], 4)
    roofline = dict(rl_all.get(roofline["kernel"], roofline), kernel=roofline["kernel"])

    # ---- CPU baseline: the oracle as it stands, on the first frames of the same sequence
    cpu = None
    if a.cpu_seconds > 0:
        from oracle.mdcnn_oracle import OracleNet
        o = OracleNet(net, crops=a.crops)
        Ts = net.total_stride
        ncut = lambda v, c: np.ascontiguousarray(v[c[0] * Ts:(c[0] + c[2]) * Ts, c[1] * Ts:(c[1] + c[3]) * Ts])
        tc = time.perf_counter()
        n_cpu = 0
        while n_cpu < T and (n_cpu < 2 or time.perf_counter() - tc < a.cpu_seconds):
            dy, dx = (0, 0) if n_cpu == 0 else (int(seq.shifts[n_cpu][0]), int(seq.shifts[n_cpu][1]))
            fm = None
            if a.dense:
                fm = np.ones((net.H, net.W), np.uint8)
            elif seq.forced is not None:
                fm = seq.forced[n_cpu]
            if a.front_end:
                o.shift_camera(dy, dx)
                fmo = o.input_mask(seq.frames[n_cpu], **wl.FE)
                for i, sp in enumerate(net.sites):
                    if sp.kind != "output":
                        o.layer_forward(i, seq.frames[n_cpu] if i == 0 else None, fmo if i == 0 else None)
                [o.readout(i) for i in net.terminal_sites()]
            elif crops is not None:
                c = crops[n_cpu]
                o.frame(ncut(seq.frames[n_cpu], c), dy, dx, None if fm is None else ncut(fm, c), crop=c)
            else:
                o.frame(seq.frames[n_cpu], dy, dx, fm)
            n_cpu += 1
        dtc = time.perf_counter() - tc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        cpu = {"value": round(n_cpu / dtc, 4), "unit": "frames/s", "cores": int(cores), "kind": "oracle",
               "sample": f"first {n_cpu} frames of the same sequence ({o.n_resets} dense/reset frames), {dtc:.1f} s"}

    upd = after["per_site"]["updated"] - before["per_site"]["updated"]
    dens = [float(upd[i]) / (n_prof * g.shape[i][0] * g.shape[i][1]) for i, s in enumerate(net.sites) if s.kind != "output"]
    entry = (("mdcnn_frames_masked" if a.front_end else "mdcnn_frames_crop" if crops is not None else "mdcnn_frames") + f", calls of {len(wl.outs_pool)} frames" if in_flight > 1 else
             "mdcnn_frame_crop" if crops is not None else "mdcnn_shift_camera + mdcnn_input_mask + mdcnn_layer_forward" if a.front_end else "mdcnn_frame")
    entry_each = "mdcnn_shift_camera + mdcnn_input_mask + mdcnn_layer_forward" if a.front_end else "mdcnn_frame_crop" if crops is not None else "mdcnn_frame"
    out = {
        "metric": "frames/s (ResNet-18-style 512x512, 1 GPU)" if cfg == 3 else f"frames/s (config {cfg}, 1 GPU)",
        "value": round(a.steps / dt, 2), "unit": "frames/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(1e3 * dt / a.steps, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": net.dtype, "data": "synthetic",
        "config": {"workload": f"config {cfg}: {net.name}, {T}-frame seeded moving-camera sequence replayed cyclically"
                               + (", max-pooling stem" if a.pool_stem and cfg == 3 else "")
                               + (f", frames cropped to a wandering box of {crops[1][2]}x{crops[1][3]} of {net.H // net.total_stride}x{net.W // net.total_stride} tiles" if crops is not None else "")
                               + (", library dense mode" if a.dense else "")
                               + (", fp32 storage" if a.f32_storage else "")
                               + (", truncation-free sites: " + ",".join(s.name for s in net.sites if s.trunc_free) if a.truncation_free else "")
                               + (f", density {a.density}" if cfg == 5 else ""),
                   "input": [net.H, net.W, net.sites[0].C], "sites": len(net.sites), "edges": len(net.edges),
                   "launches_per_frame": len(B.mdcnn_frame_plan(g.net, 1)[0]) + 2,
                   "state_bytes": int(sum(m.numel() for m in g.mem)),
                   "resets_in_timed_steps": resets_timed, "mean_update_density": round(float(np.mean(dens)), 4),
                   "input_update_density": round(dens[0], 4), "frames_in_flight": in_flight, "entry_point": entry},
        "repetitions": {"n": reps, "value": "median", "values": [round(a.steps / r[0], 1) for r in runs]},
        "roofline": roofline,
        "roofline_all": rl_all,
        "measured_peaks": peaks,
        "kernel_classes": classes,
        "kernel_ms_per_step": round(kernel_ms / n_prof, 4),
        "instrumented_ms_per_step": round(1e3 * dt_prof / n_prof, 4),
        "per_layer": layers,
        "cpu_baseline": cpu,
    }
    # the whole path against the chip: algorithmic flops and bytes of a frame (instrumented pass) at the frame rate
    per_frame_flops = (flops_mfma + flops_plain) / n_prof
    per_frame_bytes = sum(ab.values()) / n_prof
    out["whole_path"] = {"tflops": round(per_frame_flops * out["value"] / 1e12, 2),
                         "mfma_frac": round(flops_mfma / n_prof * out["value"] / 1e12 / mfma_peak, 4),
                         "algorithmic_gbs": round(per_frame_bytes * out["value"] / 1e9, 1),
                         "hbm_frac": round(per_frame_bytes * out["value"] / 1e9 / PEAK_HBM_GBS, 4),
                         "gflop_per_frame": round(per_frame_flops / 1e9, 2), "mbytes_per_frame": round(per_frame_bytes / 1e6, 2)}
    # one frame per call: the latency of a frame (frames in flight raise the rate, not this), and the rate without the
    # first frame of the cycle and the reset frames, from the per-call events
    mean = lambda v: sum(v) / len(v) if v else None
    each_ms = 1e3 * (dt_each if dt_each is not None else dt) / a.steps
    fa = {"value": round(1e3 / each_ms, 2), "unit": "frames/s", "ms_per_step": round(each_ms, 4), "entry_point": entry_each,
          "latency_ms_per_frame": round(each_ms, 4),
          "reset_frames": {"n": len(ms_kind["reset"]), "ms": round(mean(ms_kind["reset"]), 4) if ms_kind["reset"] else None},
          "other_frames": {"n": len(ms_kind["sparse"]), "ms": round(mean(ms_kind["sparse"]), 4) if ms_kind["sparse"] else None},
          "value_no_resets": round(1e3 / mean(ms_kind["sparse"]), 2) if ms_kind["sparse"] and mean(ms_kind["sparse"]) > 0 else None,
          "event_pair_ms": round(ev_ms, 4)}
    if each_runs:
        fa["repetitions"] = [round(a.steps / r[0], 1) for r in each_runs]
    out["frame_at_a_time"] = fa
    out["latency_ms_per_frame"] = fa["latency_ms_per_frame"]
    out["value_no_resets"] = fa["value_no_resets"] if in_flight == 1 else None
    if in_flight > 1:
        out["in_flight_note"] = ("value is the rate of a clip that is already in HBM with up to %d frames in flight; a frame then takes about "
                                 "%.3f ms from its first to its last launch (frames_in_flight x ms_per_step), against latency_ms_per_frame alone; "
                                 "frames overlap, so the rate without reset frames is given for one call per frame only "
                                 "(frame_at_a_time.value_no_resets)" % (in_flight, in_flight * 1e3 * dt / a.steps))
    if a.front_end:
        # the mask kernel alone, HIP events on the stream it is launched on (torch's current stream)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps_fe = 200
        g.input_mask(frames[0], **wl.FE)
        ev0.record()
        for k in range(reps_fe):
            g.input_mask(frames[k % T], **wl.FE)
        ev1.record()
        torch.cuda.synchronize()
        us = 1e3 * ev0.elapsed_time(ev1) / reps_fe
        by = net.H * net.W * (2 * net.sites[0].C * g.esize + 1)       # frame + accumulated input read once, mask written
        out["front_end"] = {"kernel": "k_input_mask", "params": wl.FE, "avg_us": round(us, 2), "algorithmic_bytes_per_launch": by,
                            "roofline": {"bound": "hbm", "achieved": round(by / us / 1e3, 2), "peak": 8000.0, "unit": "GB/s",
                                         "frac": round(by / us / 1e3 / 8000.0, 5), "traffic": None}}
        out["config"]["workload"] += ", input masks from mdcnn_input_mask (suppress, dilate 2), one call per layer"
    g.close()
    del wl
    # ---- the library's own dense mode on the same frames: threshold 0, every pixel forced
    if not a.dense and not a.no_dense_leg and not a.crops and not a.front_end:
        dnet = build_net(cfg, **net_kw)
        for s in dnet.sites:
            s.theta = 0.0
        if a.f32_storage and dnet.dtype == "f16":
            dnet.dtype = "f32"
            for e in dnet.edges:
                if e.w is not None:
                    e.w = e.w.astype(np.float32)
        dw = Workload(a, dnet, seq, forced_all_ones=True)
        r1 = dw.timed(dw.run_frames if dw.in_flight > 1 else dw.one_by_one, 1)
        dm = {"value": round(a.steps / r1[0][0], 2), "unit": "frames/s", "frames_in_flight": dw.in_flight,
              "what": "threshold 0 and every pixel forced at the input: every frame is inferred densely"}
        if dw.in_flight > 1:
            r2 = dw.timed(dw.one_by_one, 1)
            dm["frame_at_a_time"] = round(a.steps / r2[0][0], 2)
        out["dense_mode"] = dm
        dw.g.close()
        del dw
    if a.streams > 1 and not a.copy_calibration:
        frames_d = torch.from_numpy(seq.frames).cuda()
        shifts = seq.shifts.astype(np.int64).copy()
        shifts[0] = -shifts[1:].sum(axis=0)
        forced = torch.ones((T, net.H, net.W), dtype=torch.uint8, device="cuda") if a.dense else \
            torch.from_numpy(seq.forced).cuda() if seq.forced is not None else None
        out["batched"] = run_batched(a, cfg, net, T, frames_d, shifts, forced, fused)
    if a.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration_bytes"] = 1 << 30
    print(json.dumps(out))


if __name__ == "__main__":
    main()
