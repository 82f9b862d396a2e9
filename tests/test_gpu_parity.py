"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Integer outputs (update masks, lists L, compute lists, counters, reset
decisions) must be bit-exact; floating-point state within max-abs 1e-4 (fp32)
or 2e-2 (fp16 storage, fp32 accumulate).
"""
import numpy as np
import pytest
import torch

from inputs import build_net, build_sequence

pytestmark = pytest.mark.gpu


def log(msg):
    print(msg, flush=True)


def set_theta(net, th):
    for s in net.sites:
        s.theta = th
    return net


CASES = {
    # name: (config, net overrides, sequence overrides)
    "c1_single_conv": (1, {}, {}),
    "c2_cnn5_88x72": (2, dict(H=88, W=72), dict(n_frames=6, H=88, W=72)),
    "c3_resnet_96": (3, dict(H=96, W=96, widths=(32, 64, 64, 128)), dict(n_frames=8, H=96, W=96)),
    "c3_resnet_plain_80x112": (3, dict(H=80, W=112, widths=(8, 16, 24, 40)), dict(n_frames=6, H=80, W=112)),
    "c4_hrnet_128x96": (4, dict(H=128, W=96, widths=(32, 64, 64, 128), blocks=1), dict(n_frames=10, H=128, W=96)),
    "c5_bottleneck_40": (5, dict(H=40, W=40, C=128, Cm=32), dict(n_frames=12, H=40, W=40, C=128, density=0.2, shift_every=4, shift=8)),
}


def load_case(name):
    cfg, kn, ks = CASES[name]
    net = build_net(cfg, **kn)
    seq = build_sequence(cfg, **ks)
    return net, seq


@pytest.mark.parametrize("name", list(CASES))
def test_teacher_forced(name):
    import gpu_harness as H
    net, seq = load_case(name)
    log(f"[teacher-forced] {name}: {len(net.sites)} sites, {len(seq.frames)} frames")
    worst = H.teacher_forced(net, seq.frames, seq.shifts, seq.forced, log=log)
    log(f"[teacher-forced] {name}: worst fp error {worst:.3e}")


@pytest.mark.parametrize("name", list(CASES))
def test_mask_forced(name):
    import gpu_harness as H
    net, seq = load_case(name)
    log(f"[mask-forced] {name}")
    worst = H.mask_forced(net, seq.frames, seq.shifts, seq.forced, log=log)
    log(f"[mask-forced] {name}: worst fp error {worst:.3e}")


@pytest.mark.parametrize("name", list(CASES))
def test_free_running(name):
    import gpu_harness as H
    net, seq = load_case(name)
    log(f"[free-running] {name}")
    r = H.free_running(net, seq.frames, seq.shifts, seq.forced, log=log)
    th = max(s.theta for s in net.sites)
    log(f"[free-running] {name}: out_err={r['out_err']:.3e} mask mismatch={r['mask_mismatch']:.2e} resets={sum(r['resets'])}")
    assert r["mask_mismatch"] < 0.02
    assert r["out_err"] < 10 * th + 4 * H.TOL[net.dtype]


@pytest.mark.parametrize("name", list(CASES))
def test_free_running_within_the_guard_band(name):
    """Free-running with an oracle that follows the GPU's masks: a decision may differ from the oracle's only where
    the oracle's magnitude is within 4 x tolerance of the threshold; the count is reported and capped at 2 %."""
    import gpu_harness as H
    net, seq = load_case(name)
    r = H.followed(net, seq.frames, seq.shifts, seq.forced, log=log)
    log(f"[guard band] {name}: {r['flips']} of {r['decisions']} decisions off the oracle's, worst margin {r['worst_margin']:.2e}, out_err {r['out_err']:.2e}")
    assert r["flips"] <= 0.02 * r["decisions"] and r["worst_margin"] < H.TOL[net.dtype] / 4     # seen: below 1e-3


@pytest.mark.parametrize("name", ["c1_single_conv", "c3_resnet_96", "c4_hrnet_128x96"])
def test_theta0_free_running_matches_oracle(name):
    """Threshold 0: nothing is truncated, so the free-running GPU result must
    agree with the oracle (and hence with the dense canvas result) within tolerance."""
    import gpu_harness as H
    net, seq = load_case(name)
    set_theta(net, 0.0)
    r = H.free_running(net, seq.frames, seq.shifts, seq.forced, log=log)
    log(f"[theta 0] {name}: out_err={r['out_err']:.3e}")
    assert r["out_err"] < 2 * H.TOL[net.dtype]


def test_theta0_static_equals_library_dense_conv():
    """Threshold 0, no camera motion: output == dense CNN of the current frame
    computed with torch's CPU convolution (not the oracle)."""
    import gpu_harness as H
    import refs
    net, seq = load_case("c2_cnn5_88x72")
    set_theta(net, 0.0)
    from paper_2210_09887_amd.runtime import GpuNet
    g = GpuNet(net)
    try:
        for t, X in enumerate(seq.frames):
            out, _ = g.frame(H.dev(X), 0, 0)
            got = g.split_outputs(out)[0].cpu().numpy()
            want = refs.dense_cnn(net, X)[0]
            assert H.maxerr(got, want) < 1e-4
    finally:
        g.close()


@pytest.mark.parametrize("name", ["c1_single_conv", "c3_resnet_96"])
def test_origin_rotation_is_invisible(name):
    """Any physical ring origin gives bit-identical view-ordered results."""
    import gpu_harness as H
    net, seq = load_case(name)
    rng = np.random.default_rng(11)
    origins = [(int(rng.integers(0, 1000)), int(rng.integers(-1000, 0))) for _ in net.sites]
    a = H.free_running(net, seq.frames, seq.shifts, seq.forced)
    b = H.free_running(net, seq.frames, seq.shifts, seq.forced, origins=origins)
    for fa, fb in zip(a["outputs"], b["outputs"]):
        for x, y in zip(fa, fb):
            assert np.array_equal(x, y)


@pytest.mark.parametrize("path", [1, 2, 3])
def test_fallback_conv_paths_on_f16(path):
    """The fallback kernels (plain FMA; MFMA without LDS tiling; the tiled MFMA kernel
    where the halo-staged one would run) agree with the oracle too."""
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    net, seq = load_case("c3_resnet_96")
    B.mdcnn_set_option(B.MDCNN_OPT_CONV_PATH, path)
    try:
        H.teacher_forced(net, seq.frames[:3], seq.shifts[:3], log=log)
    finally:
        B.mdcnn_set_option(B.MDCNN_OPT_CONV_PATH, 0)


def _fp32_shapes_net():
    """fp32 network over the layer shapes of the matrix-core kernels that the benchmark networks lack: a 96-cout stem
    (three cout tiles), 16-cout and 16-cin layers (half-used cout tile), a strided 64 -> 128 layer, a 1x1 with 64 inputs."""
    from inputs.nets import NetSpec, _Builder
    net = NetSpec("fp32_shapes", "f32", 64, 48, 4)
    b = _Builder(net, np.random.default_rng(77), bias_amp=0.1)
    th = 0.02
    x = b.site("in", 3, 1, "input", False, th)
    s1 = b.site("stem", 96, 1, theta=th)
    s2 = b.site("a", 64, 1, theta=th)
    s3 = b.site("b", 16, 1, theta=th)
    s4 = b.site("c", 64, 2, theta=th)
    s5 = b.site("d", 128, 4, theta=th)
    y = b.site("out", 16, 4, "output", False, 0.0)
    b.conv(x, s1, 3, 1)
    b.conv(s1, s2, 1, 1, pad=0)          # 96 inputs: stays on the FMA kernel
    b.conv(s2, s3, 3, 1)                 # 64 -> 16
    b.conv(s3, s4, 3, 2)                 # 16 -> 64, stride 2
    b.conv(s4, s5, 3, 2)                 # 64 -> 128, stride 2
    b.conv(s5, y, 1, 1, pad=0)           # 128 inputs: FMA kernel
    return net


@pytest.mark.parametrize("waves_per_tile", [0, 1, 2, 4])
def test_fp32_matrix_core_kernels_other_shapes(waves_per_tile):
    """Teacher-forced parity of the fp32 matrix-core kernels on shapes the benchmark networks do not have, with the
    taps of a tile on one, two or four waves (0: the library's choice)."""
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    net = _fp32_shapes_net()
    seq = build_sequence(2, n_frames=5, H=64, W=48)
    B.mdcnn_set_option(B.MDCNN_OPT_CONV_TILE, waves_per_tile)
    try:
        worst = H.teacher_forced(net, seq.frames, seq.shifts, log=log)
        log(f"[fp32 shapes, {waves_per_tile} waves per tile] worst fp error {worst:.3e}")
    finally:
        B.mdcnn_set_option(B.MDCNN_OPT_CONV_TILE, 0)


def test_fp32_layers_on_the_plain_fma_kernels():
    """fp32 layers with 32 or 64 input channels run on the matrix cores by default; with
    that switched off the plain FMA kernels take them and agree with the oracle too."""
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    net, seq = load_case("c2_cnn5_88x72")
    B.mdcnn_set_option(B.MDCNN_OPT_CONV_F32_MFMA, 0)
    try:
        H.teacher_forced(net, seq.frames, seq.shifts, log=log)
        H.mask_forced(net, seq.frames, seq.shifts, seq.forced, log=log)
    finally:
        B.mdcnn_set_option(B.MDCNN_OPT_CONV_F32_MFMA, 1)


@pytest.mark.parametrize("name", ["c3_resnet_96", "c3_resnet_plain_80x112", "c4_hrnet_128x96", "c5_bottleneck_40"])
def test_fused_skip_equals_separate_launch(name):
    """mdcnn_frame adds residual skips inside the delta kernel of their source; the
    outputs must equal, bit for bit, those of one launch per edge."""
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    net, seq = load_case(name)
    a = H.free_running(net, seq.frames, seq.shifts, seq.forced)
    B.mdcnn_set_option(B.MDCNN_OPT_FUSE_SKIP, 0)
    try:
        b = H.free_running(net, seq.frames, seq.shifts, seq.forced)
    finally:
        B.mdcnn_set_option(B.MDCNN_OPT_FUSE_SKIP, 1)
    for fa, fb in zip(a["outputs"], b["outputs"]):
        for x, y in zip(fa, fb):
            assert np.array_equal(x, y)
    assert a["resets"] == b["resets"]


def pool_cases():
    from inputs.nets import pool_front_net, pool_net
    return {
        "pool_f32_k3s2": (pool_net("f32", 40, 56, (3, 8, 5), 3, 2, 1, theta=0.05, seed=1), 2),
        "pool_f16_k3s2": (pool_net("f16", 48, 64, (3, 16, 8), 3, 2, 1, theta=0.05, seed=2), 2),
        "pool_f16_k2s2_odd_channels": (pool_net("f16", 32, 48, (3, 12, 6), 2, 2, 0, theta=0.05, seed=3), 2),
        "pool_f32_k3s1": (pool_net("f32", 24, 40, (2, 6, 4), 3, 1, 1, theta=0.05, seed=4), 1),
        "pool_front": (pool_front_net("f16", 32, 48, (8, 8), 3, 2, 1, theta=0.05, seed=5), 2),
        "resnet_poolstem_128": (build_net(3, H=128, W=128, widths=(32, 64, 64, 128), pool_stem=True), 16),
    }


def pool_sequence(net, tile, n=7, seed=0):
    """Frames of a seeded blob panorama under a camera that moves by whole tiles and reverses once."""
    rng = np.random.default_rng(seed)
    C = net.sites[0].C
    pano = rng.normal(0, 1, (net.H + 8 * tile, net.W + 8 * tile, C)).astype(np.float32)
    from scipy.ndimage import gaussian_filter
    pano = gaussian_filter(pano, (3, 3, 0)) * 4
    pos = [(2 * tile, 2 * tile)]
    steps = [(1, 0), (1, 1), (0, 1), (0, 0), (-1, 0), (1, 1)]
    for k in range(n - 1):
        dy, dx = steps[k % len(steps)]
        pos.append((pos[-1][0] + dy * tile, pos[-1][1] + dx * tile))
    frames, shifts = [], []
    for k, (y, x) in enumerate(pos):
        f = pano[y:y + net.H, x:x + net.W] + rng.normal(0, 0.01, (net.H, net.W, C)).astype(np.float32)
        frames.append(f.astype(net.np_dtype))
        shifts.append((0, 0) if k == 0 else ((y - pos[k - 1][0]) // tile, (x - pos[k - 1][1]) // tile))
    return np.stack(frames), np.array(shifts, np.int32)


@pytest.mark.parametrize("name", ["pool_f32_k3s2", "pool_f16_k3s2", "pool_f16_k2s2_odd_channels", "pool_f32_k3s1",
                                  "pool_front", "resnet_poolstem_128"])
def test_max_pooling(name):
    """Max pooling in delta form (previous-output buffer, zero reference for newly
    unveiled pixels): all three protocols against the oracle, moving camera with a reset."""
    import gpu_harness as H
    net, tile = pool_cases()[name]
    frames, shifts = pool_sequence(net, tile)
    H.teacher_forced(net, frames, shifts, log=log)
    H.mask_forced(net, frames, shifts)
    r = H.free_running(net, frames, shifts)
    log(f"{name}: free-running out_err {r['out_err']:.2e} mask mismatch {r['mask_mismatch']:.2e} resets {r['resets']}")
    assert sum(r["resets"]) >= 2
    assert r["mask_mismatch"] < 0.02 and r["out_err"] < 10 * 0.05 + 4 * H.TOL[net.dtype]


def test_degenerate_frames():
    """Identical consecutive frames produce empty lists and leave the state untouched;
    a shift of a whole view resets; calls in the wrong order are refused."""
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    net, seq = load_case("c2_cnn5_88x72")
    g = GpuNet(net)
    try:
        with pytest.raises(B.MdcnnError) as ei:
            g.layer_forward(0, H.dev(seq.frames[0]))
        assert ei.value.status == 6
        X = H.dev(seq.frames[0])
        out0, r0 = g.frame(X, 0, 0)
        out0 = out0.clone()
        assert r0
        out1, r1 = g.frame(X, 0, 0)
        torch.cuda.synchronize()
        assert not r1
        for i, s in enumerate(net.sites):
            if s.kind != "output":
                assert len(g.read(i, B.MDCNN_VIEW_LIST)) == 0
                assert g.read(i, B.MDCNN_VIEW_STATS)[0] == 0
        assert torch.equal(out0, out1)
        _, r2 = g.frame(X, 0, net.W // net.total_stride)      # a whole view to the right
        assert r2
        _, r3 = g.frame(X, 0, 1)
        _, r4 = g.frame(X, 0, -1)                              # back over a restricted side
        assert (r3, r4) == (False, True)
        torch.cuda.synchronize()
    finally:
        g.close()


@pytest.mark.parametrize("cin,cout,H,W,k,stride", [
    (64, 256, 128, 128, 3, 1),     # 128 x 128 tile
    (64, 128, 160, 160, 3, 1),     # 64 x 128 tile
    (64, 64, 240, 240, 3, 1),      # 256 x 64 tile
    (128, 64, 184, 176, 3, 1),     # 128 x 64 tile
    (32, 64, 96, 80, 3, 2),        # 64 x 64 tile, 32-channel K step, stride 2
    (96, 32, 72, 72, 1, 1),        # 128 x 32 tile, 1x1
    (16, 32, 40, 40, 3, 1),        # MFMA without LDS tiling (Cin % 32 != 0)
    (3, 64, 64, 64, 3, 2),         # plain kernel with LDS weights (3-channel stem)
])
def test_conv_kernel_shapes(cin, cout, H, W, k, stride):
    """Every convolution kernel variant / tile shape against the oracle: a dense
    frame, a sparse frame and a frame after a camera shift."""
    import gpu_harness as H_
    from inputs.nets import tiny_net
    net = tiny_net("f16", H, W, (cin, cout), k=k, stride=stride, theta=0.05, seed=cin + cout, total_stride=8)
    rng = np.random.default_rng(cin * 1000 + cout)
    x = rng.normal(0, 1, (H, W, cin)).astype(np.float32)
    frames = [x.astype(np.float16)]
    for _ in range(2):
        x = x.copy()
        y0, x0 = int(rng.integers(0, H - 24)), int(rng.integers(0, W - 24))
        x[y0:y0 + 24, x0:x0 + 17] += rng.normal(0, 1, (24, 17, cin)).astype(np.float32)
        x[rng.random((H, W)) < 0.02] += 0.5
        frames.append(x.astype(np.float16))
    worst = H_.teacher_forced(net, frames, [(0, 0), (0, 0), (1, -1)], log=log)
    log(f"[conv shapes] {cin}->{cout} {H}x{W} k{k} s{stride}: worst {worst:.3e}")


@pytest.mark.parametrize("cin,cout,H,W,sub", [
    (64, 64, 40, 56, 1),           # whole-segment rectangles, no K split, 64-channel chunk; ragged last tiles in both directions
    (32, 32, 24, 88, 1),           # the same with a 32-channel chunk and 32-cout tiles
    (128, 64, 40, 40, 2),          # half-segment rectangles, K split two ways, two chunks
    (96, 64, 33, 47, 2),           # 32-channel chunks (three of them), odd window
    (256, 128, 16, 24, 4),         # quarter-segment rectangles, K split four ways, four chunks, two cout tiles
    (32, 32, 9, 70, 4),            # quarter segments with 32-channel chunks; a window lower than a tile is high
    (64, 64, 72, 96, 0),           # the library's own choice on a window of more than 4096 pixels
])
def test_halo_kernel_on_rectangular_tiles(cin, cout, H, W, sub):
    """The halo-staged kernel with rectangular tiles in each of its configurations, forced for windows the library would
    give index-range tiles: a dense frame, a sparse frame and a frame after a camera shift, teacher-forced against the
    oracle (masks, lists and compute lists bit for bit), and the same frames with index-range tiles: the same bits in
    every output (both walk the chunks and taps of an entry in the same order)."""
    import gpu_harness as H_
    from inputs.nets import tiny_net
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    net = tiny_net("f16", H, W, (cin, cout), k=3, stride=1, theta=0.05, seed=cin + cout + H, total_stride=1)
    rng = np.random.default_rng(cin * 1000 + cout + W)
    x = rng.normal(0, 1, (H, W, cin)).astype(np.float32)
    frames = [x.astype(np.float16)]
    for _ in range(2):
        x = x.copy()
        y0, x0 = int(rng.integers(0, max(1, H - 8))), int(rng.integers(0, max(1, W - 17)))
        x[y0:y0 + 8, x0:x0 + 17] += rng.normal(0, 1, x[y0:y0 + 8, x0:x0 + 17].shape).astype(np.float32)
        x[rng.random((H, W)) < 0.02] += 0.5
        frames.append(x.astype(np.float16))
    shifts = [(0, 0), (0, 0), (1, -1)]

    def outputs():
        g = GpuNet(net)
        try:
            return [g.frame(H_.dev(f), dy, dx)[0].cpu().numpy().copy() for f, (dy, dx) in zip(frames, shifts)]
        finally:
            g.close()

    try:
        B.mdcnn_set_option(B.MDCNN_OPT_CONV_HALO, 4)
        B.mdcnn_set_option(B.MDCNN_OPT_CONV_HALO_SUB, sub)
        worst = H_.teacher_forced(net, frames, shifts, log=log)
        rect = outputs()
        B.mdcnn_set_option(B.MDCNN_OPT_CONV_HALO, 3)
        ranges = outputs()
    finally:
        B.mdcnn_set_option(B.MDCNN_OPT_CONV_HALO, 1)
        B.mdcnn_set_option(B.MDCNN_OPT_CONV_HALO_SUB, 0)
    log(f"[rectangular tiles] {cin}->{cout} {H}x{W} split {sub}: worst {worst:.3e}")
    if sub in (2, 4):  # (whole-segment tiles: the rectangles do not split K, the index ranges do - other sums; left to
                       # themselves the two may also choose different splits)
        for t, (a, b) in enumerate(zip(rect, ranges)):
            assert np.array_equal(a, b), f"frame {t}: rectangular and index-range tiles differ"


def random_conv_cases(n=28, seed=2210):
    """Seeded single-convolution networks over the corners no named workload reaches: odd channel
    counts, 5x5 kernels, strides 3 and 4, 1x1 strided, both storage types."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        k = int(rng.choice([1, 3, 5]))
        stride = int(rng.choice([1, 2, 3, 4]))
        cin = int(rng.choice([1, 3, 5, 8, 12, 16, 24, 32, 40, 64]))
        cout = int(rng.choice([1, 4, 7, 8, 16, 24, 32, 48, 64, 96]))
        dtype = "f16" if i % 2 else "f32"
        H = stride * int(rng.integers(6, 22))
        W = stride * int(rng.integers(6, 22))
        cases.append((dtype, cin, cout, H, W, k, stride))
    return cases


@pytest.mark.parametrize("case", random_conv_cases(), ids=lambda c: "{}_{}to{}_{}x{}_k{}s{}".format(*c))
def test_random_single_convs(case):
    import gpu_harness as H_
    from inputs.nets import tiny_net
    dtype, cin, cout, H, W, k, stride = case
    net = tiny_net(dtype, H, W, (cin, cout), k=k, stride=stride, theta=0.05, seed=cin * 7 + cout, total_stride=stride)
    rng = np.random.default_rng(cin * 131 + cout * 17 + H)
    x = rng.normal(0, 1, (H, W, cin)).astype(np.float32)
    frames = [x.astype(net.np_dtype)]
    for _ in range(3):
        x = x.copy()
        x[rng.random((H, W)) < 0.15] += rng.normal(0, 1, cin).astype(np.float32)
        frames.append(x.astype(net.np_dtype))
    worst = H_.teacher_forced(net, frames, [(0, 0), (0, 0), (1, -1), (-1, 0)])
    log(f"[random conv] {case}: worst {worst:.3e}")


@pytest.mark.parametrize("seed", range(12))
def test_random_networks(seed):
    """Seeded random networks (several producers per site, skips, upsampling, pooling, two outputs) under a
    moving camera with a reset: teacher-forced against the oracle, then mdcnn_frame on 1 and 4 streams bit for bit."""
    import gpu_harness as H_
    from inputs.nets import random_dag_net
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    net = random_dag_net(seed, "f16" if seed % 2 else "f32")
    rng = np.random.default_rng(seed)
    x = rng.normal(0, 1, (net.H, net.W, net.sites[0].C)).astype(np.float32)
    frames = []
    for _ in range(6):
        x = x.copy()
        x[rng.random((net.H, net.W)) < 0.15] += rng.normal(0, 0.7, net.sites[0].C).astype(np.float32)
        frames.append(x.astype(net.np_dtype))
    shifts = [(0, 0), (1, 0), (0, -1), (0, 0), (-1, 0), (0, 1)]        # frame 4 reverses: full reset
    worst = H_.teacher_forced(net, frames, shifts)
    log(f"[random network {seed}] {len(net.sites)} sites, {len(net.edges)} edges: worst {worst:.3e}")
    outs = {}
    for ns in (1, 4):
        B.mdcnn_set_option(B.MDCNN_OPT_STREAMS, ns)
        g = GpuNet(net)
        try:
            res = []
            for X, (dy, dx) in zip(frames, shifts):
                o, _ = g.frame(H_.dev(X), dy, dx)
                torch.cuda.synchronize()
                res.append(o.clone())
            outs[ns] = res
        finally:
            B.mdcnn_set_option(B.MDCNN_OPT_STREAMS, 0)
            g.close()
    for a, b in zip(outs[1], outs[4]):
        assert torch.equal(a, b)
