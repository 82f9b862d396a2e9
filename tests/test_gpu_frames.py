"""mdcnn_frames runs consecutive frames of one video with several of them in flight.
A frame touches a site only after the frame before has finished with it, so outputs
and every piece of state must be the same, bit for bit, as with one mdcnn_frame call
per frame - for every number of streams, both ways of using them (runs of layers on
streams, whole frames on streams), every group size of the pipeline and every way of
cutting the video into calls."""
import numpy as np
import pytest
import torch

from inputs import build_net, build_sequence
from inputs.nets import random_dag_net

pytestmark = pytest.mark.gpu

CASES = {
    "c1_single_conv": (1, {}, {}),
    "c2_cnn5_96": (2, dict(H=96, W=96), dict(n_frames=7, H=96, W=96)),
    "c3_resnet_96": (3, dict(H=96, W=96, widths=(32, 64, 64, 128)), dict(n_frames=9, H=96, W=96)),
    "c3_resnet_poolstem_128": (3, dict(H=128, W=128, widths=(32, 64, 64, 128), pool_stem=True), dict(n_frames=6, H=128, W=128, tile=16)),
    "c4_hrnet_128x96": (4, dict(H=128, W=96, widths=(32, 64, 64, 128), blocks=2), dict(n_frames=8, H=128, W=96)),
    "c5_bottleneck_40": (5, dict(H=40, W=40, C=128, Cm=32), dict(n_frames=8, H=40, W=40, C=128, density=0.2, shift_every=3, shift=8)),
}


def state_of(g, net, statistics=True):
    """All state views; statistics=False leaves out the counters and the compute list of the last producer, which
    depend on whether a residual skip had a launch of its own."""
    from paper_2210_09887_amd import binding as B
    state = []
    for i, s in enumerate(net.sites):
        views = [B.MDCNN_VIEW_A, B.MDCNN_VIEW_DELTA, B.MDCNN_VIEW_FLAGS, B.MDCNN_VIEW_LIST] if s.kind != "output" else []
        views += [B.MDCNN_VIEW_STATS] if s.kind != "output" and statistics else []
        views += [B.MDCNN_VIEW_P] if s.kind != "input" else []
        views += [B.MDCNN_VIEW_CLIST] if s.kind != "input" and statistics else []
        state += [g.read(i, v) for v in views]
    return state


def one_by_one(net, seq):
    import gpu_harness as H
    from paper_2210_09887_amd.runtime import GpuNet
    g = GpuNet(net)
    try:
        outs, resets = [], []
        for t, X in enumerate(seq.frames):
            fd = H.dev(seq.forced[t]) if seq.forced is not None else None
            o, r = g.frame(H.dev(X), int(seq.shifts[t][0]), int(seq.shifts[t][1]), fd)
            torch.cuda.synchronize()
            outs.append(o.clone())
            resets.append(r)
        return outs, resets, state_of(g, net)
    finally:
        g.close()


def in_flight(net, seq, depth, group, cuts, mode=1):
    """The video in calls of cuts[0], cuts[1], ... frames (the last call takes the rest)."""
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    B.mdcnn_set_option(B.MDCNN_OPT_PIPE_GROUP, group)
    B.mdcnn_set_option(B.MDCNN_OPT_PIPE_MODE, mode)
    g = GpuNet(net)
    try:
        Xs = [H.dev(X) for X in seq.frames]
        Fs = None if seq.forced is None else [H.dev(f) for f in seq.forced]
        outs, resets, t = [], [], 0
        cuts = list(cuts)
        while t < len(Xs):
            n = min(cuts.pop(0), len(Xs) - t) if cuts else len(Xs) - t
            o, r = g.frames(Xs[t:t + n], [int(s[0]) for s in seq.shifts[t:t + n]], [int(s[1]) for s in seq.shifts[t:t + n]],
                            None if Fs is None else Fs[t:t + n], depth=depth)
            outs += o
            resets += r
            t += n
        torch.cuda.synchronize()
        return outs, resets, state_of(g, net)
    finally:
        B.mdcnn_set_option(B.MDCNN_OPT_PIPE_GROUP, 0)
        B.mdcnn_set_option(B.MDCNN_OPT_PIPE_MODE, 1)
        g.close()


def same(a, b, what):
    (oa, ra, sa), (ob, rb, sb) = a, b
    assert ra == rb, f"{what}: reset decisions differ"
    assert len(oa) == len(ob) and len(sa) == len(sb)
    for t, (x, y) in enumerate(zip(oa, ob)):
        assert torch.equal(x, y), f"{what}: output of frame {t} differs"
    for k, (u, v) in enumerate(zip(sa, sb)):
        assert np.array_equal(u, v), f"{what}: state view {k} differs"


@pytest.mark.parametrize("name", [k for k in CASES if k != "c3_full_512"])
def test_frames_in_flight_do_not_change_a_bit(name):
    cfg, kn, ks = CASES[name]
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
    ref = one_by_one(net, seq)
    for depth, group, cuts in [(1, 2, ()), (2, 1, ()), (2, 2, (3,)), (3, 2, ()), (3, 1, (1, 2)), (4, 1, ()), (4, 3, (4,)), (0, 2, ()), (4, 64, ())]:
        for mode in (0, 1):
            print(f"{name}: depth {depth}, groups of {group}, calls {cuts or 'one'}, mode {mode}", flush=True)
            same(ref, in_flight(net, seq, depth, group, cuts, mode), f"depth {depth}, groups of {group}, cuts {cuts}, mode {mode}")


@pytest.mark.parametrize("seed", range(6))
def test_frames_in_flight_random_networks(seed):
    dtype = "f16" if seed % 2 else "f32"
    net = random_dag_net(seed, dtype)
    rng = np.random.default_rng(100 + seed)

    class Seq:
        forced = None
    seq = Seq()
    x = rng.normal(0, 1, (net.H, net.W, net.sites[0].C)).astype(np.float32)
    seq.frames = []
    for _ in range(7):
        x = x.copy()
        x[rng.random((net.H, net.W)) < 0.15] += rng.normal(0, 0.7, net.sites[0].C).astype(np.float32)
        seq.frames.append(x.astype(net.np_dtype))
    seq.shifts = [(0, 0), (1, 0), (0, -1), (0, 0), (-1, 0), (0, 1), (0, 1)]       # frame 4 reverses: full reset
    ref = one_by_one(net, seq)
    for depth, group, mode in [(2, 1, 0), (4, 1, 0), (4, 1, 1), (3, 2, 0), (3, 2, 1), (4, 4, 0)]:
        print(f"dag {seed}: depth {depth}, groups of {group}, mode {mode}", flush=True)
        same(ref, in_flight(net, seq, depth, group, (3,), mode), f"depth {depth}, groups of {group}, mode {mode}")


def test_frames_argument_checks():
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    cfg, kn, ks = CASES["c2_cnn5_96"]
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
    g = GpuNet(net)
    try:
        Xs = [H.dev(X) for X in seq.frames[:3]]
        nb = g.out.numel() * g.esize
        outs = [torch.empty_like(g.out) for _ in Xs]
        ptr = lambda ts: [t.data_ptr() for t in ts]
        with pytest.raises(B.MdcnnError) as e:
            B.mdcnn_frames(g.net, ptr(Xs), None, [0] * 3, [0] * 3, ptr([outs[0], outs[1], outs[0]]), nb)
        assert e.value.status == 6          # ERR_STATE: two outputs share memory
        with pytest.raises(B.MdcnnError) as e:
            B.mdcnn_frames(g.net, ptr(Xs), None, [0] * 3, [0] * 3, ptr(outs), nb, depth=5)
        assert e.value.status == 5          # ERR_SIZE
        with pytest.raises(B.MdcnnError) as e:
            B.mdcnn_frames(g.net, ptr(Xs), None, [0] * 3, [0] * 3, ptr(outs), nb - 2)
        assert e.value.status == 5
        with pytest.raises(B.MdcnnError) as e:
            B.mdcnn_frames(g.net, [Xs[0].data_ptr(), None, Xs[2].data_ptr()], None, [0] * 3, [0] * 3, ptr(outs), nb)
        assert e.value.status == 1          # ERR_NULL
        # a refused call has changed nothing: the first frame is still the first
        o, r = g.frames(Xs, [0] * 3, [0] * 3)
        assert r == [True, False, False]
    finally:
        g.close()


def crops_of(net, n):
    Ht, Wt = net.H // net.total_stride, net.W // net.total_stride
    return [(0, 0, Ht, Wt) if t == 0 else (t % 2, (t + 1) % 2, Ht - 1 - t % 2, Wt - 1 - (t // 2) % 2) for t in range(n)]


CASES["c3_full_512"] = (3, {}, dict(n_frames=8))


@pytest.mark.parametrize("name", ["c3_resnet_96", "c3_resnet_poolstem_128", "c4_hrnet_128x96", "c3_full_512"])
def test_cropped_frames_in_flight(name):
    """mdcnn_frames_crop against one mdcnn_frame_crop call per frame: outputs, reset decisions, all state incl. the
    per-pixel crop state."""
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    cfg, kn, ks = CASES[name]
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
    n = len(seq.frames)
    crops = crops_of(net, n)
    Xs = [H.dev(H.cut(net, X, c)) for X, c in zip(seq.frames, crops)]
    dys, dxs = [int(s[0]) for s in seq.shifts], [int(s[1]) for s in seq.shifts]

    def state(g):
        return state_of(g, net) + [g.read(i, B.MDCNN_VIEW_PENDING) for i, s in enumerate(net.sites) if s.kind != "output"]

    g = GpuNet(net, crops=True)
    try:
        ref_o, ref_r = [], []
        for t in range(n):
            o, r = g.frame_crop(Xs[t], dys[t], dxs[t], crops[t])
            torch.cuda.synchronize()
            ref_o.append([x.clone() for x in o])
            ref_r.append(r)
        ref_s = state(g)
    finally:
        g.close()
    for depth, group, mode, cut in [(4, 1, 1, n), (3, 2, 1, 3), (4, 1, 0, n), (2, 3, 0, 2), (1, 1, 1, n)]:
        print(f"{name}: depth {depth}, groups of {group}, mode {mode}, calls of {cut}", flush=True)
        B.mdcnn_set_option(B.MDCNN_OPT_PIPE_GROUP, group)
        B.mdcnn_set_option(B.MDCNN_OPT_PIPE_MODE, mode)
        g = GpuNet(net, crops=True)
        try:
            got_o, got_r = [], []
            for t0 in range(0, n, cut):
                sl = slice(t0, min(t0 + cut, n))
                o, r = g.frames_crop(Xs[sl], dys[sl], dxs[sl], crops[sl], depth=depth)
                got_o += o
                got_r += r
            torch.cuda.synchronize()
            assert got_r == ref_r
            for t in range(n):
                for a, b in zip(ref_o[t], got_o[t]):
                    assert torch.equal(a, b), f"frame {t}: cropped outputs differ"
            for k, (u, v) in enumerate(zip(ref_s, state(g))):
                assert np.array_equal(u, v), f"state view {k} differs"
        finally:
            B.mdcnn_set_option(B.MDCNN_OPT_PIPE_GROUP, 0)
            B.mdcnn_set_option(B.MDCNN_OPT_PIPE_MODE, 1)
            g.close()


@pytest.mark.parametrize("name", ["c2_cnn5_96", "c3_resnet_96", "c4_hrnet_128x96"])
def test_masked_frames_in_flight(name):
    """mdcnn_frames_masked against shift, mdcnn_input_mask, the forward calls and the readout frame by frame: masks,
    outputs, reset decisions and all state, with and without a sensitivity map."""
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    cfg, kn, ks = CASES[name]
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
    n = len(seq.frames)
    Xs = [H.dev(X) for X in seq.frames]
    dys, dxs = [int(s[0]) for s in seq.shifts], [int(s[1]) for s in seq.shifts]
    rng = np.random.default_rng(7)
    # the forward calls of the reference give every residual skip a launch of its own; mdcnn_frames_masked lets the delta
    # kernel add it (same values, other statistics) unless told otherwise: compare everything with the option off, and
    # everything but the statistics with the default
    for fe, with_roi, fuse in [(dict(suppress=True, dilate=2), False, 0), (dict(pool=2, dilate=1, base=0.4, gain=0.6), True, 0),
                               (dict(suppress=True, dilate=2), False, 1)]:
        rois = [torch.from_numpy(rng.random((net.H, net.W), dtype=np.float32)).cuda() if with_roi and t % 2 else None for t in range(n)] if with_roi else None
        g = GpuNet(net)
        try:
            ref_o, ref_m, ref_r = [], [], []
            for t in range(n):
                r = g.shift_camera(dys[t], dxs[t])
                fm = g.input_mask(Xs[t], roi=None if rois is None else rois[t], **fe)
                for i, sp in enumerate(net.sites):
                    if sp.kind != "output":
                        g.layer_forward(i, Xs[t] if i == 0 else None, fm if i == 0 else None)
                o = torch.empty_like(g.out)
                off = 0
                for i in g.terminals:
                    m = int(np.prod(g.shape[i]))
                    B.mdcnn_read_view(g.bufs[i], B.MDCNN_VIEW_OUT, o[off:off + m].data_ptr(), m * g.esize, g._stream())
                    off += m
                torch.cuda.synchronize()
                ref_o.append(o)
                ref_m.append(fm.clone())
                ref_r.append(r)
            ref_s = state_of(g, net, statistics=not fuse)
        finally:
            g.close()
        for depth, mode, cut in [(4, 1, n), (3, 0, 3), (1, 1, n)]:
            print(f"{name}: front end {fe}, depth {depth}, mode {mode}, calls of {cut}, fused skips {fuse}", flush=True)
            B.mdcnn_set_option(B.MDCNN_OPT_PIPE_MODE, mode)
            B.mdcnn_set_option(B.MDCNN_OPT_FUSE_SKIP, fuse)
            g = GpuNet(net)
            try:
                got_o, got_m, got_r = [], [], []
                for t0 in range(0, n, cut):
                    sl = slice(t0, min(t0 + cut, n))
                    o, m, r = g.frames_masked(Xs[sl], dys[sl], dxs[sl], None if rois is None else rois[sl], depth=depth, **fe)
                    got_o += o
                    got_m += m
                    got_r += r
                torch.cuda.synchronize()
                assert got_r == ref_r
                for t in range(n):
                    assert torch.equal(ref_m[t], got_m[t]), f"frame {t}: masks differ"
                    assert torch.equal(ref_o[t], got_o[t]), f"frame {t}: outputs differ"
                for k, (u, v) in enumerate(zip(ref_s, state_of(g, net, statistics=not fuse))):
                    assert np.array_equal(u, v), f"state view {k} differs"
            finally:
                B.mdcnn_set_option(B.MDCNN_OPT_PIPE_MODE, 1)
                B.mdcnn_set_option(B.MDCNN_OPT_FUSE_SKIP, 1)
                g.close()


@pytest.mark.parametrize("name,n", [("c3_resnet_96", 40), ("c4_hrnet_128x96", 26), ("c2_cnn5_96", 33)])
def test_long_runs_issued_by_one_thread_per_stream(name, n):
    """Runs of at least 4 x depth frames are issued by one host thread per stream (a frame is issued only after the
    events it waits for have been recorded by the thread of the frame before).  Same bits as one call per frame and
    as the single-threaded issue; several calls in a row, so that threads start and end more than once."""
    from paper_2210_09887_amd import binding as B
    cfg, kn, ks = CASES[name]
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **dict(ks, n_frames=n))
    ref = one_by_one(net, seq)
    assert sum(ref[1]) >= 1
    try:
        for threads in (1, 0):
            B.mdcnn_set_option(B.MDCNN_OPT_PIPE_THREADS, threads)
            for depth, cuts in [(4, ()), (2, (n // 2,)), (3, (12, 12))]:
                print(f"{name}: {n} frames, depth {depth}, calls {cuts or 'one'}, threads {threads}", flush=True)
                same(ref, in_flight(net, seq, depth, 1, cuts), f"depth {depth}, cuts {cuts}, threads {threads}")
    finally:
        B.mdcnn_set_option(B.MDCNN_OPT_PIPE_THREADS, 1)
