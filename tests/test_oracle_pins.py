"""Pins for the CPU oracle: it is checked against things other than itself --
a library convolution, a global-canvas dense reference, an independently
written static-camera delta reference, brute force on tiny inputs, set
morphology from scipy, invariants of the method and constants the paper prints.
CPU only."""
import os

import numpy as np
import pytest
import scipy.ndimage as ndi

import refs
from inputs import build_net, build_sequence
from inputs.nets import tiny_net
from oracle.mdcnn_oracle import OracleNet, conv_border

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")


def golden():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def set_theta(net, th):
    for s in net.sites:
        s.theta = th
    return net


def as_f32(net):
    net.dtype = "f32"
    for e in net.edges:
        if e.w is not None:
            e.w = e.w.astype(np.float32)
    return net


def small_nets():
    return {
        "single": build_net(1),
        "cnn5": build_net(2, H=64, W=64),
        "resnet": build_net(3, H=64, W=64, widths=(4, 8, 8, 16)),
        "hrnet": build_net(4, H=128, W=96, widths=(2, 4, 4, 8), blocks=1),
        "bottleneck": build_net(5, H=16, W=16, C=8, Cm=4),
    }


def rand_frames(net, n, seed, walk=0.2):
    """Frames with temporal coherence: a base image plus sparse changes."""
    rng = np.random.default_rng(seed)
    C = net.sites[0].C
    x = rng.normal(0, 1, (net.H, net.W, C)).astype(np.float32)
    out = []
    for _ in range(n):
        chg = rng.random((net.H, net.W)) < walk
        x = x.copy()
        x[chg] += rng.normal(0, 0.5, (int(chg.sum()), C)).astype(np.float32)
        out.append(x.astype(net.np_dtype))
    return out


def monotone_shifts(n, seed, max_step=2):
    rng = np.random.default_rng(seed)
    sy, sx = rng.choice([-1, 1]), rng.choice([-1, 1])
    sh = [(0, 0)]
    for _ in range(n - 1):
        sh.append((int(sy * rng.integers(0, max_step + 1)), int(sx * rng.integers(0, max_step + 1))))
    return sh


TOL = {"f32": 1e-4, "f16": 6e-2}   # oracle-vs-float64 dense reference (storage rounding accumulates)


# ---- I1: threshold 0, static camera == dense CNN of the current frame (linearity)
@pytest.mark.parametrize("name", ["single", "cnn5", "resnet", "hrnet", "bottleneck"])
def test_theta0_static_equals_dense(name):
    net = set_theta(small_nets()[name], 0.0)
    o = OracleNet(net)
    for X in rand_frames(net, 4, 1):
        outs, _ = o.frame(X, 0, 0)
        ref = refs.dense_cnn(net, X)
        for a, b in zip(outs, ref):
            assert np.abs(a.astype(np.float64) - b).max() < TOL[net.dtype]


# ---- I2: threshold 0, monotone camera path == dense inference on the fused canvas
@pytest.mark.parametrize("name", ["single", "cnn5", "resnet", "hrnet", "bottleneck"])
@pytest.mark.parametrize("seed", [0, 1])
def test_canvas_invariant(name, seed):
    net = set_theta(as_f32(small_nets()[name]), 0.0)
    o = OracleNet(net)
    cv = refs.CanvasReference(net, 16)
    frames = rand_frames(net, 6, seed + 10)
    for X, (dy, dx) in zip(frames, monotone_shifts(6, seed)):
        outs, r = o.frame(X, dy, dx)
        ref = cv.frame(X, dy, dx, r)
        assert np.abs(outs[0].astype(np.float64) - ref[0]).max() < 1e-4


def test_canvas_differs_from_dense_only_near_trailing_edges():
    """Corollary: away from the view edges by the receptive-field radius the canvas
    result is the dense result of the current frame (Discussion, Receptive Field)."""
    net = set_theta(build_net(1), 0.0)
    seq = build_sequence(1)
    o = OracleNet(net)
    for t in range(3):
        outs, _ = o.frame(seq.frames[t], *seq.shifts[t])
        d = refs.dense_cnn(net, seq.frames[t])[0]
        err = np.abs(outs[0] - d)
        assert err[1:-1, 1:-1].max() < 1e-4
        if t > 0:
            assert err.max() > 1e-2       # the trailing edge really differs


# ---- I3: zero shift, threshold > 0 == independently written static-camera delta inference
@pytest.mark.parametrize("name", ["single", "cnn5", "resnet", "bottleneck", "hrnet"])
def test_static_camera_matches_delta_reference(name):
    net = small_nets()[name]
    if name == "bottleneck":
        set_theta(net, 0.05)
    o = OracleNet(net)
    ref = refs.StaticDeltaRef(net)
    for X in rand_frames(net, 5, 3, walk=0.05):
        outs, _ = o.frame(X, 0, 0)
        routs, rmasks = ref.frame(X)
        k = 0
        for i, s in enumerate(net.sites):
            if s.kind == "output":
                continue
            assert np.array_equal(o.sites[i].M, rmasks[k]), f"mask differs at site {i}"
            k += 1
        for a, b in zip(outs, routs):
            assert np.array_equal(a, b)
    # at least one inner site was actually sparse
    assert any(0 < o.sites[i].M.mean() < 1 for i in range(1, len(net.sites) - 1)) or len(net.sites) == 2


# ---- I4: physical ring origin does not matter
@pytest.mark.parametrize("name", ["single", "resnet", "hrnet"])
def test_origin_rotation_invariance(name):
    net = small_nets()[name]
    rng = np.random.default_rng(5)
    origins = [(int(rng.integers(0, 50)), int(rng.integers(0, 50))) for _ in net.sites]
    a, b = OracleNet(net), OracleNet(net, origins)
    frames = rand_frames(net, 5, 4, walk=0.05)
    for X, (dy, dx) in zip(frames, monotone_shifts(5, 2)):
        oa, ra = a.frame(X, dy, dx)
        ob, rb = b.frame(X, dy, dx)
        assert ra == rb
        assert all(np.array_equal(x, y) for x, y in zip(oa, ob))
        for sa, sb in zip(a.sites, b.sites):
            assert np.array_equal(sa.M, sb.M) and np.array_equal(sa.L, sb.L)
            assert np.array_equal(sa.get_A(), sb.get_A()) and np.array_equal(sa.get_P(), sb.get_P())


# ---- I5: brute force on tiny inputs
def brute_conv(x, w, b, k, stride, pad):
    """Pure-Python zero-padded correlation, x [H, W, Cin], w [k*k, Cout, Cin]."""
    H, W, Cin = x.shape
    Cout = w.shape[1]
    oh, ow = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    y = np.zeros((oh, ow, Cout))
    for oy in range(oh):
        for ox in range(ow):
            for co in range(Cout):
                acc = float(b[co])
                for jy in range(k):
                    for jx in range(k):
                        iy, ix = oy * stride - pad + jy, ox * stride - pad + jx
                        if 0 <= iy < H and 0 <= ix < W:
                            for ci in range(Cin):
                                acc += float(x[iy, ix, ci]) * float(w[jy * k + jx, co, ci])
                y[oy, ox, co] = acc
    return y


@pytest.mark.parametrize("k,stride", [(3, 1), (3, 2), (1, 1)])
def test_brute_force_tiny(k, stride):
    n = 8 if stride == 2 else 6
    net = tiny_net("f32", n, n, (2, 3, 2), k=k, stride=stride, theta=0.0, seed=k + stride)
    o = OracleNet(net)
    rng = np.random.default_rng(0)
    for t in range(3):
        X = rng.normal(0, 1, (n, n, 2)).astype(np.float32)
        outs, _ = o.frame(X, 0, 0)
        e0, e1 = net.edges
        h = np.maximum(brute_conv(X, e0.w, e0.b, k, stride, k // 2), 0)
        y = brute_conv(h, e1.w, e1.b, k, stride, k // 2)
        assert np.abs(outs[0] - y).max() < 1e-5


# ---- max pooling (Supplementary, Maximum Pooling)
def pool_cases():
    from inputs.nets import pool_net
    return {"k3s2": pool_net("f32", 16, 16, (2, 4, 3), 3, 2, 1, seed=1), "k2s2": pool_net("f32", 16, 16, (2, 4, 3), 2, 2, 0, seed=2),
            "k3s1": pool_net("f32", 12, 12, (2, 3, 2), 3, 1, 1, seed=3), "f16": pool_net("f16", 16, 16, (2, 8, 3), 3, 2, 1, seed=4),
            "resnet_poolstem": build_net(3, H=64, W=64, widths=(8, 8, 16, 16), pool_stem=True)}


@pytest.mark.parametrize("name", ["k3s2", "k2s2", "k3s1", "f16", "resnet_poolstem"])
def test_pool_theta0_static_equals_dense(name):
    """Threshold 0, static camera: delta inference through a max pooling equals dense
    inference with a library pooling routine, frame after frame."""
    net = set_theta(pool_cases()[name], 0.0)
    o = OracleNet(net)
    for X in rand_frames(net, 4, 7):
        outs, _ = o.frame(X, 0, 0)
        ref = refs.dense_cnn(net, X)
        for a, b in zip(outs, ref):
            assert np.abs(a.astype(np.float64) - b).max() < TOL[net.dtype]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_pool_on_moving_frames_equals_library_pooling(seed):
    """Pooling straight on the frames, threshold 0, moving camera, every pixel changing every
    frame: what the pooled site has accumulated is exactly the library max pooling of the
    current frame -- newly unveiled pixels included (their delta is taken against zero, not
    against the previous output of the pixel that left their ring slot)."""  # noqa
    from inputs.nets import pool_front_net
    net = pool_front_net("f32", 16, 24, (3, 2), 3, 2, 1, seed=seed)
    rng = np.random.default_rng(seed)
    origins = [(int(rng.integers(0, 30)), int(rng.integers(0, 30))) for _ in net.sites]
    o = OracleNet(net, origins)
    frames = rand_frames(net, 7, seed + 20, walk=1.0)
    for X, (dy, dx) in zip(frames, monotone_shifts(7, seed)):
        o.frame(X, dy, dx)
        p = o.sites[1]
        want = refs.maxpool64(X, 3, 2, 1)
        assert np.abs(p.get_A().astype(np.float64) - want).max() < 1e-5      # sums of fp32 deltas: a few ulp
        assert np.array_equal(p.get_Y().astype(np.float64), want)             # the stored previous output is exact


def test_pool_conservation_under_truncation():
    """Threshold > 0, static camera: accumulated + pending of the pooled site always equals the
    library pooling of the source's accumulated activations (nothing is lost, only deferred)."""
    from inputs.nets import pool_net
    net = pool_net("f32", 16, 16, (2, 4, 3), 3, 2, 1, theta=0.3, seed=5)
    o = OracleNet(net)
    sparse = False
    for X in rand_frames(net, 6, 9, walk=0.1):
        o.frame(X, 0, 0)
        a, p = o.sites[1], o.sites[2]
        want = refs.maxpool64(np.maximum(a.get_A(), 0), 3, 2, 1)
        got = p.get_A().astype(np.float64) + p.view_of_window(p.get_P())
        assert np.abs(got - want).max() < 1e-5
        sparse |= 0 < p.M.mean() < 1
    assert sparse


def test_pool_brute_force_tiny():
    from inputs.nets import pool_front_net
    net = pool_front_net("f32", 6, 8, (2, 2), 3, 2, 1, seed=3)
    o = OracleNet(net)
    rng = np.random.default_rng(1)
    for t in range(3):
        X = rng.normal(0, 1, (6, 8, 2)).astype(np.float32)
        o.frame(X, 0, 0)
        got = o.sites[1].get_A()
        for oy in range(3):
            for ox in range(4):
                for c in range(2):
                    m = max(float(X[iy, ix, c]) for iy in range(2 * oy - 1, 2 * oy + 2) for ix in range(2 * ox - 1, 2 * ox + 2)
                            if 0 <= iy < 6 and 0 <= ix < 8)
                    assert abs(float(got[oy, ox, c]) - m) < 1e-5


def test_pins_catch_a_pool_delta_against_the_stale_output(monkeypatch):
    """Planted mistake: the previous output is used also for pixels reset this frame."""
    from inputs.nets import pool_front_net
    net = pool_front_net("f32", 16, 24, (3, 2), 3, 2, 1, seed=0)
    o = OracleNet(net)
    frames = rand_frames(net, 5, 20, walk=1.0)
    bad = False
    for X, (dy, dx) in zip(frames, [(0, 0), (1, 1), (1, 0), (0, 1), (1, 1)]):
        o.shift_camera(dy, dx)
        o.sites[1].N[:] = False                      # the mistake: nobody is "newly unveiled" for the pooling
        for i in (0, 1):
            o.layer_forward(i, X if i == 0 else None)
        bad |= np.abs(o.sites[1].get_A().astype(np.float64) - refs.maxpool64(X, 3, 2, 1)).max() > 1e-3
    assert bad


def test_impulse_footprint_and_padded_extent():
    g = golden()
    # a 64x64 input under a 3x3 kernel produces 66x66 outputs
    b0, b1 = conv_border(3, 1, 1, 64, 64)
    assert 64 + b0 + b1 == g["padded_out_of_64_k3"]
    net = build_net(1)
    o = OracleNet(net)
    assert (o.sites[1].Hp, o.sites[1].Wp) == (66, 66)
    o.frame(np.zeros((64, 64, 16), np.float32), 0, 0)
    # one changed pixel -> compute list is exactly its 3x3 footprint (padded-window coords)
    for (py, px) in [(10, 20), (0, 0), (63, 63), (0, 63)]:
        X = np.zeros((64, 64, 16), np.float32)
        X[py, px, 3] = 1.0
        o2 = OracleNet(net)
        o2.frame(np.zeros((64, 64, 16), np.float32), 0, 0)
        lists = None
        o2.shift_camera(0, 0)
        lists = o2.layer_forward(0, X)
        want = sorted((py + 1 + a) * 66 + (px + 1 + b) for a in (-1, 0, 1) for b in (-1, 0, 1))
        assert lists[0].tolist() == want
        assert o2.sites[0].L.tolist() == [py * 64 + px]


# ---- I6 / I7: truncation bound and conservation
@pytest.mark.parametrize("name", ["cnn5", "resnet"])
def test_truncation_bound_and_conservation(name):
    net = as_f32(small_nets()[name])
    o = OracleNet(net)
    sums = [np.zeros(s.A.shape, np.float64) for s in o.sites]
    frames = rand_frames(net, 6, 7, walk=0.05)
    for X in frames:
        o.shift_camera(0, 0)
        for i, s in enumerate(o.sites):
            if s.spec.kind == "output":
                continue
            o.layer_forward(i, X if i == 0 else None)
            sums[i] += s.delta.astype(np.float64)
        for i, s in enumerate(o.sites):
            if s.spec.kind != "preact":
                continue
            a = s.get_A().astype(np.float32)
            t = s.view_of_window(s.get_P()).astype(np.float32)
            f = (lambda v: np.maximum(v, 0)) if s.spec.relu else (lambda v: v)
            resid = np.abs(f(a + t) - f(a)).max(axis=2)
            assert resid.max() <= np.float32(s.spec.theta)            # nothing above threshold is left pending
            assert np.abs(sums[i] - f(a)).max() < 1e-4                # emitted deltas sum to f(A)
    # A + P at every inner site equals the dense pre-activation of the accumulated inputs
    vals = [s.get_A().astype(np.float64) for s in o.sites]
    for i, s in enumerate(o.sites):
        if s.spec.kind == "input":
            continue
        want = np.zeros(s.A.shape) + refs.site_bias(net, i)
        for e in net.edges:
            if e.dst == i:
                src = o.sites[e.src]
                fa = vals[e.src] if not src.spec.relu else np.maximum(vals[e.src], 0)
                want = want + (fa if e.k == 0 else refs._conv64(fa, e))
        got = s.view_of_window(s.get_P()).astype(np.float64)
        if s.spec.kind == "preact":
            got = got + s.get_A().astype(np.float64)
        assert np.abs(got - want).max() < 1e-4


# ---- I8: the conv compute list is the morphological dilation of the update mask
@pytest.mark.parametrize("k,stride,pad", [(3, 1, 1), (3, 2, 1), (1, 1, 0), (1, 2, 0)])
def test_compute_list_is_dilation(k, stride, pad):
    rng = np.random.default_rng(k * 10 + stride)
    H = W = 16
    net = tiny_net("f32", H, W, (1, 1), k=k, stride=stride, theta=0.0)
    net.edges[0].pad = pad
    net.sites[1].stride = stride
    o = OracleNet(net)
    o.frame(np.zeros((H, W, 1), np.float32), 0, 0)
    m = rng.random((H, W)) < 0.1
    m[0, 0] = m[H - 1, W - 1] = True
    X = m[:, :, None].astype(np.float32)
    o.shift_camera(0, 0)
    lst = o.layer_forward(0, X)[0]
    d = o.sites[1]
    got = np.zeros(d.Hp * d.Wp, bool)
    got[lst] = True
    got = got.reshape(d.Hp, d.Wp)
    by0, by1, bx0, bx1 = d.border
    want = np.zeros((d.Hp, d.Wp), bool)
    if stride == 1:
        full = np.zeros((H + by0 + by1, W + bx0 + bx1), bool)
        full[by0:by0 + H, bx0:bx0 + W] = m
        want = ndi.binary_dilation(full, structure=np.ones((k, k), bool))
    else:
        for wy in range(d.Hp):
            for wx in range(d.Wp):
                oy, ox = wy - by0, wx - bx0
                for jy in range(k):
                    for jx in range(k):
                        iy, ix = oy * stride - pad + jy, ox * stride - pad + jx
                        if 0 <= iy < H and 0 <= ix < W and m[iy, ix]:
                            want[wy, wx] = True
    assert np.array_equal(got, want)
    assert np.all(np.diff(lst) > 0)


# ---- I9: first frame and every post-reset frame are dense for any threshold
@pytest.mark.parametrize("name", ["cnn5", "resnet"])
def test_reset_frames_are_dense(name):
    net = as_f32(small_nets()[name])
    set_theta(net, 0.5)
    o = OracleNet(net)
    frames = rand_frames(net, 4, 9)
    shifts = [(0, 0), (1, 0), (-1, 0), (0, 0)]          # frame 2 reverses -> reset
    resets = []
    for X, (dy, dx) in zip(frames, shifts):
        outs, r = o.frame(X, dy, dx)
        resets.append(r)
        if r:
            for s in o.sites:
                if s.spec.kind != "output":
                    assert s.M.all()
            assert np.abs(outs[0] - refs.dense_cnn(net, X)[0]).max() < 1e-4
    assert resets == [True, False, True, False]


# ---- I10: resets are a pure function of the camera path
def test_reset_count_matches_independent_rule():
    for cfg, kw in [(3, dict(n_frames=60, H=64, W=64)), (4, dict(n_frames=40, H=128, W=96)), (2, dict(n_frames=30, H=64, W=64))]:
        seq = build_sequence(cfg, **kw)
        net = {3: build_net(3, H=64, W=64, widths=(2, 2, 2, 2)), 4: build_net(4, H=128, W=96, widths=(1, 1, 1, 1), blocks=1),
               2: build_net(2, H=64, W=64)}[cfg]
        o = OracleNet(net)
        got = [t for t, (dy, dx) in enumerate(seq.shifts) if o.shift_camera(dy, dx)]
        want = refs.reset_frames(seq.shifts.tolist(), (net.H // net.total_stride, net.W // net.total_stride))
        assert got == want
    # without dynamic initialisation every camera motion would be a reset (ablation)
    seq = build_sequence(2, n_frames=30, H=64, W=64)
    assert sum(1 for d in seq.shifts[1:] if d.any()) == 29 and len(got) == 1


def test_a_step_of_a_whole_view_resets_and_clears_the_restrictions():
    """Buffer management: a step of a whole view extent (or more) leaves nothing to keep, so it is a full reset --
    and like every reset it lifts the restrictions: the step AFTER it may go back without another reset.  The
    sequences take such steps on either axis, in both directions, after growth in the other direction, and are
    checked against the independent rule; the frames of the resets must be dense, the steps that follow them not."""
    net = as_f32(small_nets()["cnn5"])                      # 24 x 24 pixels, total stride 4: a view of 6 x 6 tiles
    Ht, Wt = net.H // net.total_stride, net.W // net.total_stride
    paths = [
        [(0, 0), (1, 0), (Ht, 0), (-1, 0), (0, 1)],         # grow down, whole view down (reset), back up: no reset
        [(0, 0), (0, -1), (0, -Wt), (0, 1), (0, 1), (0, -1)],
        [(0, 0), (0, 1), (-(Ht + 2), 0), (1, 0), (0, -1)],  # more than a view; the x restriction is lifted too
        [(0, 0), (Ht - 1, 0), (-1, 0)],                     # one tile short of a view is growth; then a reversal
        [(0, 0), (1, 1), (0, Wt), (-1, -1)],
    ]
    for path in paths:
        o = OracleNet(net)
        frames = rand_frames(net, len(path), 5)
        want = refs.reset_frames(path, (Ht, Wt))
        got = []
        for t, (X, (dy, dx)) in enumerate(zip(frames, path)):
            outs, r = o.frame(X, dy, dx)
            if r:
                got.append(t)
                assert all(s.M.all() for s in o.sites if s.spec.kind != "output")       # inferred densely
                assert np.abs(outs[0] - refs.dense_cnn(net, X)[0]).max() < 1e-4
        assert got == want, (path, got, want)
    # the rule itself on a hand-made case: the whole-view step is frame 2, and frame 3 does not reset
    assert refs.reset_frames(paths[0], (Ht, Wt)) == [0, 2]
    assert refs.reset_frames(paths[3], (Ht, Wt)) == [0, 2]


# ---- I11: constants printed in the paper
def test_paper_constants():
    g = golden()
    assert g["hrnet_full_res"] / g["hrnet_low_res"] == g["hrnet_tile"]
    net = build_net(4)
    assert net.total_stride == g["hrnet_tile"]
    o_tiles = sorted({net.total_stride // s.stride for s in net.sites})
    assert o_tiles[0] == 1 and o_tiles[-1] == 32         # 32x32 px at full resolution ... 1x1 at the lowest
    assert g["offset_alloc_px"] - g["offset_px"] == g["offset_zero_right"]
    assert round(1 - (1 - g["buffer_shrink_per_axis"]) ** 2, 2) == g["buffer_memory_saved"]
    assert 2 * g["mask_dilation_px"] + 1 == g["mask_dilation_extent"]


# ---- planted mistakes must be caught (the pins are sharp enough)
def test_pins_catch_a_dropped_border(monkeypatch):
    """If the dilated border were not kept, the canvas invariant must fail."""
    import oracle.mdcnn_oracle as om
    monkeypatch.setattr(om, "conv_border", lambda *a: (0, 0))
    net = set_theta(build_net(1), 0.0)
    o = om.OracleNet(net)
    cv = refs.CanvasReference(net, 8)
    seq = build_sequence(1)
    worst = 0.0
    for t in range(3):
        # without a border the compute list must be clipped to the view
        try:
            outs, r = o.frame(seq.frames[t], *seq.shifts[t])
        except IndexError:
            return
        worst = max(worst, np.abs(outs[0] - cv.frame(seq.frames[t], *seq.shifts[t], r)[0]).max())
    assert worst > 1e-2


# ---- random networks: threshold 0 on a static camera equals the dense network, every site
@pytest.mark.parametrize("seed", range(10))
def test_random_networks_theta0_static_equal_dense(seed):
    from inputs.nets import random_dag_net
    net = set_theta(random_dag_net(seed, "f32"), 0.0)
    o = OracleNet(net)
    for X in rand_frames(net, 4, seed + 50, walk=0.2):
        outs, _ = o.frame(X, 0, 0)
        vals = refs.dense_cnn(net, X, return_all=True)
        for a, i in zip(outs, net.terminal_sites()):
            assert np.abs(a.astype(np.float64) - vals[i]).max() < 1e-4
        for i, s in enumerate(o.sites):
            if s.spec.kind == "preact":
                fa = s.get_A().astype(np.float64)
                assert np.abs((np.maximum(fa, 0) if s.spec.relu else fa) - vals[i]).max() < 1e-4
