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

Prints ONE JSON line.  Besides the throughput it carries
  roofline     -- the dominant kernel class, timed with HIP events recorded by
                  the library around every launch of a second, instrumented pass
                  over the same frames (algorithmic flops / bytes from device-side
                  counters of that pass);
  cpu_baseline -- the NumPy oracle timed on the host cores on the first frames
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
    ap.add_argument("--dense", action="store_true", help="library dense mode: threshold 0 and all pixels forced")
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
    prof = B.mdcnn_profile_read()
    B.mdcnn_set_option(B.MDCNN_OPT_PROFILE, 0)
    after = sum_totals([g.totals() for g in gb.streams])
    ab = algorithmic_bytes(gb.streams[0], net, before, after, n_prof * n, fused_skips=fused)
    classes, kernel_ms, rl_all, _ = rooflines(prof, 2.0 * (after["macs_mfma"] - before["macs_mfma"]),
                                              2.0 * (after["macs_plain"] - before["macs_plain"]), ab, cfg, with_traffic=False,
                                              mfma_peak=PEAK_MFMA_F32_TFLOPS if net.dtype == "f32" else PEAK_MFMA_F16_TFLOPS)
    gb.close()
    return {"streams": n, "value": round(n * steps / dt, 2), "unit": "frames/s", "batch_steps": steps,
            "ms_per_batch_step": round(1e3 * dt / steps, 4), "roofline_all": rl_all, "kernel_classes": classes,
            "kernel_ms_per_batch_step": round(kernel_ms / n_prof, 4)}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from inputs import build_net, build_sequence
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)

    cfg = a.config
    net = build_net(cfg, **({"pool_stem": True} if a.pool_stem and cfg == 3 else {}))
    seq = build_sequence(cfg, **({"density": a.density} if cfg == 5 else {"tile": 16} if a.pool_stem and cfg == 3 else {}))
    if a.dense:
        for s in net.sites:
            s.theta = 0.0
    T = len(seq.frames)
    shifts = seq.shifts.astype(np.int64).copy()
    shifts[0] = -shifts[1:].sum(axis=0)            # closing the cycle: jump back to the start
    frames = torch.from_numpy(seq.frames).cuda()
    forced = None
    if a.dense:
        forced = torch.ones((T, net.H, net.W), dtype=torch.uint8, device="cuda")
    elif seq.forced is not None:
        forced = torch.from_numpy(seq.forced).cuda()
    for kv in a.opt:
        k, v = kv.split("=")
        B.mdcnn_set_option(int(k), int(v))
    g = GpuNet(net, crops=a.crops)

    crops = None
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
        frames_c = [cut(frames[t], crops[t]) for t in range(T)]
        forced_c = None if forced is None else [cut(forced[t], crops[t]) for t in range(T)]
        a.streams = 0

    FE = dict(suppress=True, dilate=2)
    if a.front_end:
        assert crops is None and forced is None, "--front-end excludes --crops, --dense and config 5"
        a.streams = 0

    state = {"t": 0, "resets": 0}

    def step():
        t = state["t"] % T
        dy, dx = (0, 0) if state["t"] == 0 else (int(shifts[t][0]), int(shifts[t][1]))
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
            _, r = g.frame_crop(frames_c[t], dy, dx, crops[t], None if forced is None else forced_c[t])
        else:
            _, r = g.frame(frames[t], dy, dx, None if forced is None else forced[t])
        state["t"] += 1
        state["resets"] += int(r)

    in_flight = a.frames_in_flight or (4 if len(B.mdcnn_frame_plan(g.net, 1)[0]) >= 16 else 1)
    outs_pool = [torch.empty_like(g.out) for _ in range(min(T, max(a.steps, a.warmup)))] if in_flight > 1 else []
    masks_pool = [torch.empty((net.H, net.W), dtype=torch.uint8, device="cuda") for _ in outs_pool] if a.front_end else []

    def run_frames(n):
        """n frames of the video through mdcnn_frames, in calls of as many frames as the sequence has."""
        done = 0
        while done < n:
            t0_ = state["t"]
            m = min(n - done, len(outs_pool))
            idx = [(t0_ + k) % T for k in range(m)]
            sh = [(0, 0) if t0_ + k == 0 else (int(shifts[i][0]), int(shifts[i][1])) for k, i in enumerate(idx)]
            if a.front_end:
                _, _, rs = g.frames_masked([frames[i] for i in idx], [v[0] for v in sh], [v[1] for v in sh], outs=outs_pool[:m],
                                           masks=masks_pool[:m], depth=in_flight, **FE)
            elif crops is not None:
                _, rs = g.frames_crop([frames_c[i] for i in idx], [v[0] for v in sh], [v[1] for v in sh], [crops[i] for i in idx],
                                      None if forced is None else [forced_c[i] for i in idx], outs=outs_pool[:m], depth=in_flight)
            else:
                _, rs = g.frames([frames[i] for i in idx], [v[0] for v in sh], [v[1] for v in sh],
                                 None if forced is None else [forced[i] for i in idx], outs=outs_pool[:m], depth=in_flight)
            state["t"] += m
            state["resets"] += sum(int(r) for r in rs)
            done += m

    def timed_region(run):
        run(a.warmup)
        torch.cuda.synchronize()
        state["resets"] = 0
        t0 = time.perf_counter()
        run(a.steps)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    one_by_one = lambda n: [step() for _ in range(n)]
    dt_each = None
    if in_flight > 1:
        dt = timed_region(run_frames)
        resets_timed = state["resets"]
        dt_each = timed_region(one_by_one)
    else:
        dt = timed_region(one_by_one)
        resets_timed = state["resets"]

    # ---- instrumented pass: per-class kernel time (HIP events around every launch)
    before = g.totals()
    B.mdcnn_set_option(B.MDCNN_OPT_PROFILE, 1)
    B.mdcnn_profile_read()
    n_prof = min(a.steps, 2 * T)
    t1 = time.perf_counter()
    for _ in range(n_prof):
        step()
    prof = B.mdcnn_profile_read()
    dt_prof = time.perf_counter() - t1
    B.mdcnn_set_option(B.MDCNN_OPT_PROFILE, 0)
    after = g.totals()

    flops_mfma = 2.0 * (after["macs_mfma"] - before["macs_mfma"])
    flops_plain = 2.0 * (after["macs_plain"] - before["macs_plain"])
    ab = algorithmic_bytes(g, net, before, after, n_prof, fused_skips="8=0" not in a.opt)
    mfma_peak = PEAK_MFMA_F32_TFLOPS if net.dtype == "f32" else PEAK_MFMA_F16_TFLOPS
    classes, kernel_ms, rl_all, roofline = rooflines(prof, flops_mfma, flops_plain, ab, cfg, mfma_peak=mfma_peak)

    # ---- CPU baseline: the oracle as it stands, on the first frames of the same sequence
    cpu = None
    if a.cpu_seconds > 0:
        from oracle.mdcnn_oracle import OracleNet
        o = OracleNet(net, crops=a.crops)
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
                fmo = o.input_mask(seq.frames[n_cpu], **FE)
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
    out = {
        "metric": "frames/s (ResNet-18-style 512x512, 1 GPU)" if cfg == 3 else f"frames/s (config {cfg}, 1 GPU)",
        "value": round(a.steps / dt, 2), "unit": "frames/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(1e3 * dt / a.steps, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": net.dtype, "data": "synthetic",
        "config": {"workload": f"config {cfg}: {net.name}, {T}-frame seeded moving-camera sequence replayed cyclically"
                               + (", max-pooling stem" if a.pool_stem and cfg == 3 else "")
                               + (f", frames cropped to a wandering box of {crops[1][2]}x{crops[1][3]} of {net.H // net.total_stride}x{net.W // net.total_stride} tiles" if crops is not None else "")
                               + (", library dense mode" if a.dense else "")
                               + (f", density {a.density}" if cfg == 5 else ""),
                   "input": [net.H, net.W, net.sites[0].C], "sites": len(net.sites), "edges": len(net.edges),
                   "resets_in_timed_steps": resets_timed, "mean_update_density": round(float(np.mean(dens)), 4),
                   "input_update_density": round(dens[0], 4), "frames_in_flight": in_flight,
                   "entry_point": ("mdcnn_frames_masked" if a.front_end else "mdcnn_frames_crop" if crops is not None else "mdcnn_frames") + f", calls of {len(outs_pool)} frames" if in_flight > 1 else
                                  "mdcnn_frame_crop" if crops is not None else "mdcnn_shift_camera + mdcnn_input_mask + mdcnn_layer_forward" if a.front_end else "mdcnn_frame"},
        "roofline": roofline,
        "roofline_all": rl_all,
        "kernel_classes": classes,
        "kernel_ms_per_step": round(kernel_ms / n_prof, 4),
        "instrumented_ms_per_step": round(1e3 * dt_prof / n_prof, 4),
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
    if dt_each is not None:
        out["frame_at_a_time"] = {"value": round(a.steps / dt_each, 2), "unit": "frames/s", "ms_per_step": round(1e3 * dt_each / a.steps, 4),
                                  "entry_point": "mdcnn_shift_camera + mdcnn_input_mask + mdcnn_layer_forward" if a.front_end else "mdcnn_frame_crop" if crops is not None else "mdcnn_frame"}
    if a.front_end:
        # the mask kernel alone, HIP events on the stream it is launched on (torch's current stream)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 200
        g.input_mask(frames[0], **FE)
        ev0.record()
        for k in range(reps):
            g.input_mask(frames[k % T], **FE)
        ev1.record()
        torch.cuda.synchronize()
        us = 1e3 * ev0.elapsed_time(ev1) / reps
        by = net.H * net.W * (2 * net.sites[0].C * g.esize + 1)       # frame + accumulated input read once, mask written
        out["front_end"] = {"kernel": "k_input_mask", "params": FE, "avg_us": round(us, 2), "algorithmic_bytes_per_launch": by,
                            "roofline": {"bound": "hbm", "achieved": round(by / us / 1e3, 2), "peak": 8000.0, "unit": "GB/s",
                                         "frac": round(by / us / 1e3 / 8000.0, 5), "traffic": None}}
        out["config"]["workload"] += ", input masks from mdcnn_input_mask (suppress, dilate 2), one call per layer"
    g.close()
    if a.streams > 1 and not a.copy_calibration:
        out["batched"] = run_batched(a, cfg, net, T, frames, shifts, forced, "8=0" not in a.opt)
    if a.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration_bytes"] = 1 << 30
    print(json.dumps(out))


if __name__ == "__main__":
    main()
