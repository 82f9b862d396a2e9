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
