"""Batch of independent streams (mdcnn_frame_batch): every stream must give, bit for
bit, what mdcnn_frame gives on it alone -- outputs, reset decisions and counters --
although all streams share their launches; and every stream is checked against an
oracle of its own."""
import numpy as np
import pytest
import torch

from test_gpu_parity import load_case

pytestmark = pytest.mark.gpu


def stream_inputs(seq, b):
    """Stream b plays the sequence from frame b on (its own camera path and resets)."""
    forced = None if seq.forced is None else seq.forced[b:]
    return seq.frames[b:], seq.shifts[b:], forced


@pytest.mark.parametrize("name,n_streams", [("c1_single_conv", 2), ("c3_resnet_96", 3), ("c4_hrnet_128x96", 4),
                                            ("c5_bottleneck_40", 3), ("c3_resnet_plain_80x112", 2)])
def test_batch_equals_single_streams(name, n_streams):
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuBatch, GpuNet
    net, seq = load_case(name)
    T = len(seq.frames) - n_streams + 1
    # reference: every stream alone
    want, want_resets, want_stats = [], [], []
    for b in range(n_streams):
        fr, sh, fo = stream_inputs(seq, b)
        g = GpuNet(net)
        outs, resets = [], []
        try:
            for t in range(T):
                o, r = g.frame(H.dev(fr[t]), int(sh[t][0]), int(sh[t][1]), None if fo is None else H.dev(fo[t]))
                outs.append(o.cpu().numpy().copy())
                resets.append(r)
            want_stats.append([g.read(i, B.MDCNN_VIEW_STATS).copy() for i in range(len(net.sites))])
        finally:
            g.close()
        want.append(outs)
        want_resets.append(resets)
    gb = GpuBatch(net, n_streams)
    try:
        for t in range(T):
            ins = [stream_inputs(seq, b) for b in range(n_streams)]
            frames = [H.dev(fr[t]) for fr, _, _ in ins]
            forced = None if seq.forced is None else [H.dev(fo[t]) for _, _, fo in ins]
            outs, resets = gb.frame(frames, [int(sh[t][0]) for _, sh, _ in ins], [int(sh[t][1]) for _, sh, _ in ins], forced)
            torch.cuda.synchronize()
            for b in range(n_streams):
                assert resets[b] == want_resets[b][t], f"frame {t} stream {b}: reset decision"
                assert np.array_equal(outs[b].cpu().numpy(), want[b][t]), f"frame {t} stream {b}: output differs"
        for b, g in enumerate(gb.streams):
            for i in range(len(net.sites)):
                assert np.array_equal(g.read(i, B.MDCNN_VIEW_STATS), want_stats[b][i]), f"stream {b} site {i}: counters"
    finally:
        gb.close()


def different_paths(net, seq, n_streams):
    """n streams over the frames of one sequence, each with a camera path of its own: stream b takes the frames
    from b on; streams 1.. get other steps, and one of them a reversal, i.e. a reset in the middle."""
    T = len(seq.frames) - n_streams + 1
    seqs = []
    for b in range(n_streams):
        fr, sh, fo = stream_inputs(seq, b)
        sh = [tuple(int(v) for v in x) for x in sh[:T]]
        if b == 1:
            sh = [(0, 0), (1, 0), (1, 0), (-1, 0)] + [(0, 1)] * T          # the fourth frame steps back: reset
        if b == 2:
            sh = [(0, 0), (0, -1), (0, 0), (0, -1), (0, 1)] + [(0, 0)] * T  # the fifth frame steps back: reset
        seqs.append((fr[:T], sh[:T], None if fo is None else fo[:T]))
    return seqs


@pytest.mark.parametrize("name", ["c3_resnet_96", "c5_bottleneck_40", "c2_cnn5_88x72"])
def test_batch_against_per_stream_oracles(name):
    """mdcnn_frame_batch against the oracle, not against the library: three streams with different camera paths and
    resets; every stream's decisions within the guard band of an oracle that follows its masks, its reset
    decisions and input-site lists bit for bit, its outputs at the tight tolerance."""
    import gpu_harness as H
    net, seq = load_case(name)
    seqs = different_paths(net, seq, 3)
    assert len(seqs[0][0]) >= 4
    res = H.followed_batch(net, seqs, log=print)
    for b, r in enumerate(res):
        print(f"[batch vs oracle] {name} stream {b}: {r}", flush=True)
        assert r["flips"] <= 0.02 * r["decisions"] and r["worst_margin"] < H.TOL[net.dtype] / 4     # seen: below 1e-3


def test_batch_of_more_streams_than_one_launch_carries():
    """37 streams (the paper's batches go to 66): the library splits them into groups that share launches; every stream
    still equals its single run bit for bit, with its own frames, camera path and resets."""
    import gpu_harness as H
    from paper_2210_09887_amd.runtime import GpuBatch, GpuNet
    net, seq = load_case("c3_resnet_plain_80x112")
    n, T = 37, 4
    rng = np.random.default_rng(5)
    start = [int(rng.integers(0, len(seq.frames) - T + 1)) for _ in range(n)]
    path = [[(0, 0)] + [(int(rng.integers(-1, 2)), int(rng.integers(-1, 2))) for _ in range(T - 1)] for _ in range(n)]
    want = {}
    for b in range(0, n, 6):                                # every sixth stream is checked against its single run
        g = GpuNet(net)
        try:
            want[b] = [(lambda o, r: (o.cpu().numpy().copy(), r))(*g.frame(H.dev(seq.frames[start[b] + t]), *path[b][t])) for t in range(T)]
        finally:
            g.close()
    gb = GpuBatch(net, n)
    try:
        for t in range(T):
            outs, rs = gb.frame([H.dev(seq.frames[start[b] + t]) for b in range(n)], [path[b][t][0] for b in range(n)],
                                [path[b][t][1] for b in range(n)])
            torch.cuda.synchronize()
            for b in want:
                assert rs[b] == want[b][t][1] and np.array_equal(outs[b].cpu().numpy(), want[b][t][0]), f"frame {t} stream {b}"
    finally:
        gb.close()


def test_batch_with_max_pooling():
    """The pooling kernel in a batch: streams with different camera paths equal their single runs."""
    import gpu_harness as H
    from test_gpu_parity import pool_cases, pool_sequence
    from paper_2210_09887_amd.runtime import GpuBatch, GpuNet
    net, tile = pool_cases()["resnet_poolstem_128"]
    seqs = [pool_sequence(net, tile, n=6, seed=b) for b in range(3)]
    want = []
    for fr, sh in seqs:
        g = GpuNet(net)
        try:
            want.append([g.frame(H.dev(fr[t]), int(sh[t][0]), int(sh[t][1]))[0].cpu().numpy().copy() for t in range(len(fr))])
        finally:
            g.close()
    gb = GpuBatch(net, 3)
    try:
        for t in range(6):
            outs, _ = gb.frame([H.dev(fr[t]) for fr, _ in seqs], [int(sh[t][0]) for _, sh in seqs], [int(sh[t][1]) for _, sh in seqs])
            torch.cuda.synchronize()
            for b in range(3):
                assert np.array_equal(outs[b].cpu().numpy(), want[b][t]), f"frame {t} stream {b}"
    finally:
        gb.close()


def test_batch_argument_checks():
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuBatch, GpuNet
    net, seq = load_case("c1_single_conv")
    gb = GpuBatch(net, 2)
    other_net, _ = load_case("c5_bottleneck_40")
    other = GpuNet(other_net)
    try:
        X = torch.zeros((net.H, net.W, net.sites[0].C), dtype=gb.streams[0].tdtype, device="cuda")
        nets = [g.net for g in gb.streams]
        outs = [g.out.data_ptr() for g in gb.streams]
        nbytes = gb.streams[0].out.numel() * gb.streams[0].esize
        with pytest.raises(B.MdcnnError):              # the same stream twice
            B.mdcnn_frame_batch([nets[0], nets[0]], [X.data_ptr()] * 2, None, [0, 0], [0, 0], outs, nbytes)
        with pytest.raises(B.MdcnnError):              # different networks
            B.mdcnn_frame_batch([nets[0], other.net], [X.data_ptr()] * 2, None, [0, 0], [0, 0], outs, nbytes)
        with pytest.raises(B.MdcnnError):              # too many streams
            B.mdcnn_frame_batch(nets * 65, [X.data_ptr()] * 130, None, [0] * 130, [0] * 130, outs * 65, nbytes)
    finally:
        other.close()
        gb.close()


@pytest.mark.parametrize("name,n_streams", [("c3_resnet_96", 3), ("c4_hrnet_128x96", 2), ("c5_bottleneck_40", 3), ("c2_cnn5_88x72", 2)])
def test_frames_of_a_batch_in_flight(name, n_streams):
    """mdcnn_frames_batch: several videos, each with frames in flight.  First the videos go frame by frame through
    mdcnn_frame_batch with an oracle following every one of them (decisions within the guard band, outputs at the tight
    tolerance); then the same videos go through mdcnn_frames_batch at several depths and cuts into calls, and every output
    of every frame and all state at the end must be the same bits."""
    import gpu_harness as H
    from test_gpu_frames import state_of
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuBatch
    net, seq = load_case(name)
    seqs = different_paths(net, seq, n_streams)
    T = len(seqs[0][0])
    assert T >= 4
    fs = [H.Follower(net) for _ in range(n_streams)]
    want_o, want_r = [], []
    gb = GpuBatch(net, n_streams)
    try:
        for t in range(T):
            Xs = [sq[0][t] for sq in seqs]
            dys, dxs = [sq[1][t][0] for sq in seqs], [sq[1][t][1] for sq in seqs]
            fms = [None if sq[2] is None else sq[2][t] for sq in seqs]
            outs, rs = gb.frame([H.dev(X) for X in Xs], dys, dxs, None if fms[0] is None else [H.dev(m) for m in fms])
            torch.cuda.synchronize()
            for b, g in enumerate(gb.streams):
                got = [x.cpu().numpy() for x in g.split_outputs(outs[b])]
                fs[b].check(t, Xs[b], dys[b], dxs[b], fms[b], got, bool(rs[b]), H.gpu_masks(g, fs[b].inner), g.read(0, B.MDCNN_VIEW_LIST),
                            tag=f"stream {b} ")
            want_o.append([o.clone() for o in outs])
            want_r.append([bool(r) for r in rs])
        want_s = [state_of(g, net) for g in gb.streams]
    finally:
        gb.close()
    for b, f in enumerate(fs):
        r = f.result()
        print(f"[batch in flight, reference run vs oracle] {name} stream {b}: {r}", flush=True)
        assert r["flips"] <= 0.02 * r["decisions"] and r["worst_margin"] < H.TOL[net.dtype] / 4
    assert any(any(r) for r in want_r[1:]), "a reset after the first frame belongs to the case"
    dev_frames = [[H.dev(sq[0][t]) for sq in seqs] for t in range(T)]
    dev_forced = None if seqs[0][2] is None else [[H.dev(sq[2][t]) for sq in seqs] for t in range(T)]
    dty = [[sq[1][t][0] for sq in seqs] for t in range(T)]
    dtx = [[sq[1][t][1] for sq in seqs] for t in range(T)]
    for depth, cut in [(4, T), (2, 3), (1, T), (0, 2)]:
        print(f"{name}: {n_streams} videos, depth {depth}, calls of {cut} frames", flush=True)
        gb = GpuBatch(net, n_streams)
        try:
            got_o, got_r = [], []
            for t0 in range(0, T, cut):
                sl = slice(t0, min(t0 + cut, T))
                o, r = gb.frames(dev_frames[sl], dty[sl], dtx[sl], None if dev_forced is None else dev_forced[sl], depth=depth)
                got_o += o
                got_r += r
            torch.cuda.synchronize()
            assert got_r == want_r
            for t in range(T):
                for b in range(n_streams):
                    assert torch.equal(got_o[t][b], want_o[t][b]), f"depth {depth}: frame {t}, video {b}: output differs"
            for b, g in enumerate(gb.streams):
                for k, (u, v) in enumerate(zip(want_s[b], state_of(g, net))):
                    assert np.array_equal(u, v), f"depth {depth}: video {b}: state view {k} differs"
        finally:
            gb.close()


def test_frames_batch_of_more_videos_than_one_launch_carries_and_argument_checks():
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuBatch, GpuNet
    net, seq = load_case("c3_resnet_plain_80x112")
    n, T = 19, 5
    rng = np.random.default_rng(11)
    start = [int(rng.integers(0, len(seq.frames) - T + 1)) for _ in range(n)]
    path = [[(0, 0)] + [(int(rng.integers(-1, 2)), int(rng.integers(-1, 2))) for _ in range(T - 1)] for _ in range(n)]
    want = {}
    for b in (0, 7, 15, 16, 18):                             # videos of both groups against their single runs
        g = GpuNet(net)
        try:
            want[b] = [(lambda o, r: (o.cpu().numpy().copy(), r))(*g.frame(H.dev(seq.frames[start[b] + t]), *path[b][t])) for t in range(T)]
        finally:
            g.close()
    gb = GpuBatch(net, n)
    try:
        frames = [[H.dev(seq.frames[start[b] + t]) for b in range(n)] for t in range(T)]
        dty = [[path[b][t][0] for b in range(n)] for t in range(T)]
        dtx = [[path[b][t][1] for b in range(n)] for t in range(T)]
        outs, rs = gb.frames(frames, dty, dtx, depth=3)
        torch.cuda.synchronize()
        for b in want:
            for t in range(T):
                assert rs[t][b] == want[b][t][1] and np.array_equal(outs[t][b].cpu().numpy(), want[b][t][0]), f"frame {t} video {b}"
        g0 = gb.streams[0]
        nets = [g.net for g in gb.streams]
        nbytes = g0.out.numel() * g0.esize
        X = frames[0][0].data_ptr()
        o2 = [torch.empty_like(g0.out) for _ in range(4)]
        with pytest.raises(B.MdcnnError):                    # the same video twice
            B.mdcnn_frames_batch([nets[0], nets[0]], [[X, X]] * 2, None, [[0, 0]] * 2, [[0, 0]] * 2, [[o2[0].data_ptr(), o2[1].data_ptr()], [o2[2].data_ptr(), o2[3].data_ptr()]], nbytes)
        with pytest.raises(B.MdcnnError):                    # two frames write the same output
            B.mdcnn_frames_batch(nets[:2], [[X, X]] * 2, None, [[0, 0]] * 2, [[0, 0]] * 2, [[o2[0].data_ptr(), o2[1].data_ptr()], [o2[0].data_ptr(), o2[3].data_ptr()]], nbytes)
        with pytest.raises(B.MdcnnError):                    # wrong output size
            B.mdcnn_frames_batch(nets[:2], [[X, X]], None, [[0, 0]], [[0, 0]], [[o2[0].data_ptr(), o2[1].data_ptr()]], nbytes - 16)
        with pytest.raises(B.MdcnnError):                    # depth out of range
            B.mdcnn_frames_batch(nets[:2], [[X, X]], None, [[0, 0]], [[0, 0]], [[o2[0].data_ptr(), o2[1].data_ptr()]], nbytes, depth=5)
    finally:
        gb.close()
