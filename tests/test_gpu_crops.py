"""GPU parity for cropped frames (a frame that covers a tile-aligned part of the
view): the HIP path through the C ABI against the oracle, to the same bars as
the uncropped path (integers bit-exact, fp32 1e-4, fp16 2e-2)."""
import numpy as np
import pytest
import torch

from inputs import build_net, build_sequence
from inputs.nets import pool_net

pytestmark = pytest.mark.gpu


def log(msg):
    print(msg, flush=True)


def rand_crops(net, n, seed, full_first=True, full_last=True):
    rng = np.random.default_rng(seed)
    Ht, Wt = net.H // net.total_stride, net.W // net.total_stride
    out = []
    for t in range(n):
        if (t == 0 and full_first) or (t == n - 1 and full_last):
            out.append((0, 0, Ht, Wt))
            continue
        th, tw = int(rng.integers(1, Ht + 1)), int(rng.integers(1, Wt + 1))
        out.append((int(rng.integers(0, Ht - th + 1)), int(rng.integers(0, Wt - tw + 1)), th, tw))
    return out


def crop_cases():
    return {
        # name: (config, net overrides, sequence overrides, first frame covers everything)
        "c2_cnn5_88x72": (2, dict(H=88, W=72), dict(n_frames=7, H=88, W=72), True),
        "c3_resnet_96": (3, dict(H=96, W=96, widths=(32, 64, 64, 128)), dict(n_frames=8, H=96, W=96), True),
        "c3_resnet_96_partial_start": (3, dict(H=96, W=96, widths=(32, 64, 64, 128)), dict(n_frames=8, H=96, W=96), False),
        "c3_resnet_plain_80x112": (3, dict(H=80, W=112, widths=(8, 16, 24, 40)), dict(n_frames=6, H=80, W=112), False),
        "c3_resnet_poolstem_128": (3, dict(H=128, W=128, widths=(32, 64, 64, 128), pool_stem=True), dict(n_frames=7, H=128, W=128, tile=16), True),
        "c4_hrnet_128x96": (4, dict(H=128, W=96, widths=(32, 64, 64, 128), blocks=1), dict(n_frames=8, H=128, W=96), True),
    }


@pytest.mark.parametrize("name", list(crop_cases()))
def test_teacher_forced_with_crops(name):
    """Moving camera and a different crop every frame (the sequences contain a reset)."""
    import gpu_harness as H
    cfg, kn, ks, full_first = crop_cases()[name]
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
    crops = rand_crops(net, len(seq.frames), 7, full_first=full_first)
    log(f"[crops teacher-forced] {name}: {len(net.sites)} sites, crops {crops}")
    worst = H.teacher_forced(net, seq.frames, seq.shifts, seq.forced, log=log, crops=crops)
    log(f"[crops teacher-forced] {name}: worst fp error {worst:.3e}")


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_teacher_forced_pooling_with_crops(dtype):
    import gpu_harness as H
    net = pool_net(dtype, 32, 48, (8, 16, 8), 3, 2, 1, theta=0.15, seed=2)
    rng = np.random.default_rng(3)
    x = rng.normal(0, 1, (net.H, net.W, 8)).astype(np.float32)
    frames, shifts = [], []
    for t in range(7):
        chg = rng.random((net.H, net.W)) < 0.15
        x = x.copy()
        x[chg] += rng.normal(0, 0.5, (int(chg.sum()), 8)).astype(np.float32)
        frames.append(x.astype(net.np_dtype))
        shifts.append((0, 0) if t in (0, 3) else (1, 0) if t < 5 else (-1, 1))    # frame 5 reverses: reset
    crops = rand_crops(net, 7, 11)
    worst = H.teacher_forced(net, frames, shifts, None, log=log, crops=crops)
    log(f"[crops pooling {dtype}] worst fp error {worst:.3e}")


@pytest.mark.parametrize("name", ["c3_resnet_96", "c4_hrnet_128x96", "c3_resnet_poolstem_128"])
def test_whole_view_crop_is_the_uncropped_path_bit_for_bit(name):
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    cfg, kn, ks, _ = crop_cases()[name]
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
    Ht, Wt = net.H // net.total_stride, net.W // net.total_stride
    a, b = GpuNet(net), GpuNet(net, crops=True)
    try:
        for t, X in enumerate(seq.frames):
            dy, dx = (int(v) for v in seq.shifts[t])
            fd = H.dev(seq.forced[t]) if seq.forced is not None else None
            oa, ra = a.frame(H.dev(X), dy, dx, fd)
            ob, rb = (b.frame(H.dev(X), dy, dx, fd) if t % 2 else b.frame_crop(H.dev(X), dy, dx, (0, 0, Ht, Wt), fd))
            torch.cuda.synchronize()
            assert ra == rb
            ob = ob if t % 2 else torch.cat([o.reshape(-1) for o in ob])
            assert torch.equal(oa, ob), f"frame {t}: outputs differ"
        for i, s in enumerate(net.sites):
            views = [B.MDCNN_VIEW_A, B.MDCNN_VIEW_DELTA, B.MDCNN_VIEW_FLAGS, B.MDCNN_VIEW_LIST] if s.kind != "output" else []
            views += [B.MDCNN_VIEW_P] if s.kind != "input" else []
            for v in views:
                assert np.array_equal(a.read(i, v), b.read(i, v)), f"site {i} view {v}"
            if s.kind != "output":
                assert not b.read(i, B.MDCNN_VIEW_PENDING).any()
    finally:
        a.close()
        b.close()


@pytest.mark.parametrize("name", ["c2_cnn5_88x72", "c3_resnet_plain_80x112"])
def test_free_running_crops_at_threshold_zero(name):
    """mdcnn_frame_crop end to end at threshold 0 in fp32: no mask depends on a rounding, so the
    outputs follow the oracle to the fp32 tolerance and the input-site list is exact."""
    import gpu_harness as H
    from oracle.mdcnn_oracle import OracleNet
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    cfg, kn, ks, _ = crop_cases()[name]
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
    net.dtype = "f32"
    for e in net.edges:
        if e.w is not None:
            e.w = e.w.astype(np.float32)
    for s in net.sites:
        s.theta = 0.0
    crops = rand_crops(net, len(seq.frames), 5)
    g, o = GpuNet(net, crops=True), OracleNet(net, crops=True)
    try:
        for t, X in enumerate(seq.frames):
            dy, dx = (int(v) for v in seq.shifts[t])
            Xc = H.cut(net, X.astype(np.float32), crops[t])
            want, r_o = o.frame(Xc, dy, dx, crop=crops[t])
            got, r_g = g.frame_crop(H.dev(Xc), dy, dx, crops[t])
            torch.cuda.synchronize()
            assert r_g == r_o
            for a, b in zip(got, want):
                assert a.shape == b.shape
                assert H.maxerr(a.cpu().numpy(), b) < 1e-4, f"frame {t}"
            assert np.array_equal(g.read(0, B.MDCNN_VIEW_LIST), o.sites[0].L)
            for i, s in enumerate(o.sites):
                if s.spec.kind != "output":
                    assert np.array_equal(g.read(i, B.MDCNN_VIEW_PENDING) & B.STATE_UNSEEN, H.oracle_pending(s) & B.STATE_UNSEEN)
    finally:
        g.close()


def test_crop_argument_checks():
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    net = build_net(2, H=64, W=64)
    seq = build_sequence(2, n_frames=2, H=64, W=64)
    plain, g = GpuNet(net), GpuNet(net, crops=True)
    try:
        X = H.dev(seq.frames[0])
        with pytest.raises(B.MdcnnError) as ei:
            plain.frame_crop(X, 0, 0, (0, 0, 1, 1))
        assert ei.value.status == 6
        with pytest.raises(B.MdcnnError) as ei:
            plain.set_crop(0, 0, 1, 1)
        assert ei.value.status == 6
        Ht = net.H // net.total_stride
        for bad in [(0, 0, Ht + 1, 1), (-1, 0, 1, 1), (0, 0, 0, 1), (Ht, 0, 1, 1), (1, 1, Ht, Ht)]:
            with pytest.raises(B.MdcnnError) as ei:
                B.mdcnn_frame_crop(g.net, X.data_ptr(), None, 0, 0, bad, g.out.data_ptr(), g.out.numel() * g.esize)
            assert ei.value.status == 2, bad
        g.frame_crop(X, 0, 0, (0, 0, Ht, Ht))
        half = H.dev(H.cut(net, seq.frames[1], (0, 0, Ht // 2, Ht)))
        g.frame_crop(half, 0, 0, (0, 0, Ht // 2, Ht))
        with pytest.raises(B.MdcnnError) as ei:          # the plain frame call needs the whole view
            g.frame(X, 0, 0)
        assert ei.value.status == 6
        with pytest.raises(B.MdcnnError) as ei:          # wrong output size for the crop
            B.mdcnn_frame_crop(g.net, half.data_ptr(), None, 0, 0, (0, 0, Ht // 2, Ht), g.out.data_ptr(), g.out.numel() * g.esize)
        assert ei.value.status == 5
        torch.cuda.synchronize()
    finally:
        plain.close()
        g.close()


def random_chain_cases(n=10, seed=909):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        k = int(rng.choice([1, 3, 5]))
        stride = int(rng.choice([1, 2, 3]))
        C = tuple(int(rng.choice([3, 5, 8, 16, 32, 40])) for _ in range(3))
        T = stride * stride
        cases.append(("f16" if i % 2 else "f32", C, T * int(rng.integers(3, 9)), T * int(rng.integers(3, 9)), k, stride))
    return cases


@pytest.mark.parametrize("case", random_chain_cases(), ids=lambda c: "{}_{}_{}x{}_k{}s{}".format(c[0], "-".join(map(str, c[1])), *c[2:]))
def test_random_chains_with_crops(case):
    """Seeded two-convolution chains (odd channels, 5x5, stride 3) with a different crop every frame."""
    import gpu_harness as H
    from inputs.nets import tiny_net
    dtype, C, Hh, Ww, k, stride = case
    net = tiny_net(dtype, Hh, Ww, C, k=k, stride=stride, theta=0.05, seed=sum(C))
    rng = np.random.default_rng(Hh * 31 + Ww)
    x = rng.normal(0, 1, (Hh, Ww, C[0])).astype(np.float32)
    frames = []
    for _ in range(6):
        x = x.copy()
        x[rng.random((Hh, Ww)) < 0.2] += rng.normal(0, 1, C[0]).astype(np.float32)
        frames.append(x.astype(net.np_dtype))
    shifts = [(0, 0), (0, 1), (1, 0), (0, 0), (-1, 0), (0, 0)]        # frame 4 reverses: full reset
    worst = H.teacher_forced(net, frames, shifts, crops=rand_crops(net, 6, sum(C) + k, full_first=bool(k % 2 == 1 and stride < 3)))
    log(f"[random chains with crops] {case}: worst {worst:.3e}")


@pytest.mark.parametrize("name", ["c2_cnn5_88x72", "c3_resnet_plain_80x112"])
def test_batch_of_cropped_streams_against_per_stream_oracles(name):
    """mdcnn_frame_batch_crop at threshold 0 in fp32 (no mask depends on a rounding): three streams with crops and camera
    paths of their own share their launches; every stream follows an oracle of its own - outputs to the fp32 tolerance,
    reset decisions, input-site lists and crop state exact."""
    import gpu_harness as H
    from oracle.mdcnn_oracle import OracleNet
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuBatch
    cfg, kn, ks, _ = crop_cases()[name]
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
    net.dtype = "f32"
    for e in net.edges:
        if e.w is not None:
            e.w = e.w.astype(np.float32)
    for s in net.sites:
        s.theta = 0.0
    n, T = 3, len(seq.frames) - 2
    crops = [rand_crops(net, T, 5 + b, full_first=b != 1) for b in range(n)]      # stream 1 starts with a partial frame
    paths = [[(int(v[0]), int(v[1])) for v in seq.shifts[b:b + T]] for b in range(n)]
    paths[2] = [(0, 0), (0, 1), (0, 1), (0, -1)] + [(1, 0)] * T                    # the fourth frame of stream 2 steps back: reset
    gb, os_ = GpuBatch(net, n, crops=True), [OracleNet(net, crops=True) for _ in range(n)]
    try:
        resets = 0
        for t in range(T):
            cs = [crops[b][t] for b in range(n)]
            Xs = [H.cut(net, seq.frames[b + t].astype(np.float32), cs[b]) for b in range(n)]
            dys, dxs = [paths[b][t][0] for b in range(n)], [paths[b][t][1] for b in range(n)]
            got, rs = gb.frame_crop([H.dev(X) for X in Xs], dys, dxs, cs)
            torch.cuda.synchronize()
            for b in range(n):
                want, r_o = os_[b].frame(Xs[b], dys[b], dxs[b], crop=cs[b])
                assert bool(rs[b]) == bool(r_o), f"frame {t} stream {b}: reset decision"
                resets += bool(r_o) and t > 0
                for a, w in zip(got[b], want):
                    assert a.shape == w.shape
                    assert H.maxerr(a.cpu().numpy(), w) < 1e-4, f"frame {t} stream {b}"
                g = gb.streams[b]
                assert np.array_equal(g.read(0, B.MDCNN_VIEW_LIST), os_[b].sites[0].L), f"frame {t} stream {b}: input list"
                for i, s in enumerate(os_[b].sites):
                    if s.spec.kind != "output":
                        assert np.array_equal(g.read(i, B.MDCNN_VIEW_PENDING) & B.STATE_UNSEEN, H.oracle_pending(s) & B.STATE_UNSEEN)
        assert resets >= 1
    finally:
        gb.close()


@pytest.mark.parametrize("name", ["c3_resnet_96", "c4_hrnet_128x96", "c3_resnet_poolstem_128"])
def test_batch_of_cropped_streams_equals_single_streams(name):
    """Every stream of mdcnn_frame_batch_crop gives the bits mdcnn_frame_crop gives on it alone (which the teacher-forced
    tests above hold against the oracle): outputs, reset decisions and all state at the end; 18 streams, so that the
    library has to split them into two groups of launches."""
    import gpu_harness as H
    from test_gpu_frames import state_of
    from paper_2210_09887_amd.runtime import GpuBatch, GpuNet
    cfg, kn, ks, _ = crop_cases()[name]
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
    n, T = 18, 5
    rng = np.random.default_rng(3)
    start = [int(rng.integers(0, len(seq.frames) - T + 1)) for _ in range(n)]
    crops = [rand_crops(net, T, 40 + b, full_first=b % 3 != 1, full_last=False) for b in range(n)]
    paths = [[(0, 0)] + [(int(rng.integers(-1, 2)), int(rng.integers(-1, 2))) for _ in range(T - 1)] for _ in range(n)]
    check = (0, 1, 7, 15, 16, 17)
    want = {}
    for b in check:
        g = GpuNet(net, crops=True)
        try:
            per = []
            for t in range(T):
                X = H.cut(net, seq.frames[start[b] + t], crops[b][t])
                o, r = g.frame_crop(H.dev(X), paths[b][t][0], paths[b][t][1], crops[b][t], None if seq.forced is None else H.dev(H.cut(net, seq.forced[start[b] + t], crops[b][t])))
                torch.cuda.synchronize()
                per.append(([x.cpu().numpy().copy() for x in o], r))
            want[b] = (per, state_of(g, net))
        finally:
            g.close()
    gb = GpuBatch(net, n, crops=True)
    try:
        for t in range(T):
            cs = [crops[b][t] for b in range(n)]
            Xs = [H.dev(H.cut(net, seq.frames[start[b] + t], cs[b])) for b in range(n)]
            Fs = None if seq.forced is None else [H.dev(H.cut(net, seq.forced[start[b] + t], cs[b])) for b in range(n)]
            got, rs = gb.frame_crop(Xs, [paths[b][t][0] for b in range(n)], [paths[b][t][1] for b in range(n)], cs, Fs)
            torch.cuda.synchronize()
            for b in check:
                assert bool(rs[b]) == bool(want[b][0][t][1]), f"frame {t} stream {b}: reset decision"
                for a, w in zip(got[b], want[b][0][t][0]):
                    assert np.array_equal(a.cpu().numpy(), w), f"frame {t} stream {b}: output differs"
        for b in check:
            for k, (u, v) in enumerate(zip(want[b][1], state_of(gb.streams[b], net))):
                assert np.array_equal(u, v), f"stream {b}: state view {k} differs"
    finally:
        gb.close()
