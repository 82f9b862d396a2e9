"""Pins for the oracle's cropped frames (a frame that covers a tile-aligned part
of the buffers only): they tie it to the uncropped oracle, to dense inference on
a canvas that is written inside the crops only, and to conservation, so that a
mistake in the crop bookkeeping (a lost pending update, work outside the crop, a
wrong scale of the crop at a strided site) fails one of them."""
import numpy as np
import pytest

import refs
from inputs import build_net
from inputs.nets import pool_net
from oracle.mdcnn_oracle import OracleNet
from test_oracle_pins import as_f32, monotone_shifts, rand_frames, set_theta, small_nets


def tiles_of(net):
    return net.H // net.total_stride, net.W // net.total_stride


def rand_crop(rng, Ht, Wt):
    th, tw = int(rng.integers(1, Ht + 1)), int(rng.integers(1, Wt + 1))
    return int(rng.integers(0, Ht - th + 1)), int(rng.integers(0, Wt - tw + 1)), th, tw


def cut(net, X, crop):
    T = net.total_stride
    ty0, tx0, th, tw = crop
    return np.ascontiguousarray(X[ty0 * T:(ty0 + th) * T, tx0 * T:(tx0 + tw) * T])


def state(o):
    out = []
    for s in o.sites:
        out += [s.get_A(), s.get_P(), s.delta.copy(), s.M.copy(), s.L.copy()]
        if s.pooled:
            out.append(s.get_Y())
    return out


# ---- a crop that covers the whole view is the uncropped method, bit for bit
@pytest.mark.parametrize("name", ["cnn5", "resnet", "hrnet", "bottleneck", "pool"])
def test_full_crop_equals_uncropped(name):
    net = pool_net("f16", 16, 16, (2, 4, 3), 3, 2, 1, theta=0.2, seed=3) if name == "pool" else small_nets()[name]
    a, b = OracleNet(net), OracleNet(net, crops=True)
    Ht, Wt = tiles_of(net)
    shifts = monotone_shifts(6, 4, max_step=1) + [(0, 0)]
    shifts[4] = (-shifts[1][0] - shifts[2][0] - shifts[3][0] or 1, 0)      # a reversal: full reset
    for X, (dy, dx) in zip(rand_frames(net, 7, 2, walk=0.1), shifts):
        oa, ra = a.frame(X, dy, dx)
        ob, rb = b.frame(X, dy, dx, crop=(0, 0, Ht, Wt))
        assert ra == rb
        for u, v in zip(oa + state(a), ob + state(b)):
            assert np.array_equal(u, v)


# ---- threshold 0: dense inference on canvases that are written inside the crops only
@pytest.mark.parametrize("name", ["single", "cnn5", "resnet", "hrnet", "bottleneck"])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_crop_canvas_invariant(name, seed):
    net = set_theta(as_f32(small_nets()[name]), 0.0)
    o = OracleNet(net, crops=True)
    cv = refs.CanvasReference(net, 16)
    rng = np.random.default_rng(100 + seed)
    Ht, Wt = tiles_of(net)
    frames = rand_frames(net, 8, seed + 20)
    shifts = monotone_shifts(8, seed, max_step=1) if seed else [(0, 0)] * 8
    partial = False
    for t, (X, (dy, dx)) in enumerate(zip(frames, shifts)):
        crop = (0, 0, Ht, Wt) if t == 7 else rand_crop(rng, Ht, Wt)
        partial |= crop[2] < Ht or crop[3] < Wt
        outs, r = o.frame(cut(net, X, crop), dy, dx, crop=crop)
        ref = cv.frame(cut(net, X, crop), dy, dx, r, crop=crop)
        assert outs[0].shape == ref[0].shape
        assert np.abs(outs[0].astype(np.float64) - ref[0]).max() < 1e-4
        # every inner site too, over its whole view: pixels outside the crop kept their values
        for i, s in enumerate(o.sites):
            if s.spec.kind != "preact":
                continue
            fa = s.get_A().astype(np.float64)
            fa = np.maximum(fa, 0) if s.spec.relu else fa
            assert np.abs(fa - cv.canvas[i][cv._view(i)]).max() < 1e-4
    assert partial


# ---- static camera, threshold 0: once a frame covers everything again, the result is the
# dense network of the image assembled from the crops (max pooling included)
@pytest.mark.parametrize("kind", ["resnet", "pool", "resnet_poolstem"])
def test_crops_then_full_frame_equals_dense_of_the_assembled_image(kind):
    if kind == "pool":
        net = pool_net("f32", 16, 16, (2, 4, 3), 3, 2, 1, theta=0.0, seed=1)
    elif kind == "resnet":
        net = set_theta(as_f32(small_nets()["resnet"]), 0.0)
    else:
        net = set_theta(as_f32(build_net(3, H=64, W=64, widths=(4, 8, 8, 16), pool_stem=True)), 0.0)
    o = OracleNet(net, crops=True)
    rng = np.random.default_rng(5)
    Ht, Wt = tiles_of(net)
    frames = rand_frames(net, 6, 11, walk=0.3)
    image = frames[0].copy()
    o.frame(frames[0], 0, 0, crop=(0, 0, Ht, Wt))
    T = net.total_stride
    for X in frames[1:]:
        ty0, tx0, th, tw = crop = rand_crop(rng, Ht, Wt)
        image[ty0 * T:(ty0 + th) * T, tx0 * T:(tx0 + tw) * T] = cut(net, X, crop)
        o.frame(cut(net, X, crop), 0, 0, crop=crop)
    outs, _ = o.frame(image, 0, 0, crop=(0, 0, Ht, Wt))          # nothing changes at the input
    for a, b in zip(outs, refs.dense_cnn(net, image)):
        assert np.abs(a.astype(np.float64) - b).max() < 1e-4


# ---- threshold > 0: nothing is lost, and nothing outside the crop is worked on
@pytest.mark.parametrize("name", ["cnn5", "resnet"])
def test_crop_conservation_and_locality(name):
    net = as_f32(small_nets()[name])
    o = OracleNet(net, crops=True)
    rng = np.random.default_rng(8)
    Ht, Wt = tiles_of(net)
    pending_outside = False
    for t, X in enumerate(rand_frames(net, 7, 3, walk=0.1)):
        crop = (0, 0, Ht, Wt) if t == 0 else rand_crop(rng, Ht, Wt)
        before = [s.get_A().copy() for s in o.sites]
        o.frame(cut(net, X, crop), 0, 0, crop=crop)
        vals = [s.get_A().astype(np.float64) for s in o.sites]
        for i, s in enumerate(o.sites):
            inside = s.in_crop()
            assert not s.M[~inside].any()
            assert np.array_equal(before[i][~inside], s.get_A()[~inside])
            if s.spec.kind != "input":
                assert np.array_equal(s.get_ring("dirty") & inside, np.zeros_like(inside))
                pending_outside |= bool(s.get_ring("dirty").any())
            if s.spec.kind == "input":
                assert s.n_candidates == inside.sum()
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
    assert pending_outside        # the case occurred: updates waited outside a crop


# ---- planted mistake: forgetting the updates that arrived outside the crop
def test_pins_catch_forgotten_updates_outside_the_crop():
    class Forgetful(OracleNet):
        def _truncate(self, i, frame, forced):
            s = self.sites[i]
            s.U = s.U & s.in_crop()
            super()._truncate(i, frame, forced)

    net = set_theta(as_f32(small_nets()["cnn5"]), 0.0)
    o = Forgetful(net, crops=True)
    Ht, Wt = tiles_of(net)
    rng = np.random.default_rng(5)
    frames = rand_frames(net, 5, 11, walk=0.3)
    image = frames[0].copy()
    o.frame(frames[0], 0, 0, crop=(0, 0, Ht, Wt))
    T = net.total_stride
    for X in frames[1:]:
        ty0, tx0, th, tw = crop = rand_crop(rng, Ht, Wt)
        image[ty0 * T:(ty0 + th) * T, tx0 * T:(tx0 + tw) * T] = cut(net, X, crop)
        o.frame(cut(net, X, crop), 0, 0, crop=crop)
    outs, _ = o.frame(image, 0, 0, crop=(0, 0, Ht, Wt))
    assert np.abs(outs[0].astype(np.float64) - refs.dense_cnn(net, image)[0]).max() > 1e-3


# ---- the same with max pooling (static camera: a pooled value is refreshed only when its window changes)
@pytest.mark.parametrize("kind", ["pool", "resnet_poolstem"])
def test_crop_canvas_invariant_with_max_pooling(kind):
    if kind == "pool":
        net = pool_net("f32", 32, 32, (2, 4, 3), 3, 2, 1, theta=0.0, seed=4)
    else:
        net = set_theta(as_f32(build_net(3, H=64, W=64, widths=(4, 8, 8, 16), pool_stem=True)), 0.0)
    o = OracleNet(net, crops=True)
    cv = refs.CanvasReference(net, 2)
    rng = np.random.default_rng(12)
    Ht, Wt = tiles_of(net)
    for t, X in enumerate(rand_frames(net, 8, 31, walk=0.3)):
        crop = (0, 0, Ht, Wt) if t == 0 else rand_crop(rng, Ht, Wt)
        outs, r = o.frame(cut(net, X, crop), 0, 0, crop=crop)
        ref = cv.frame(cut(net, X, crop), 0, 0, r, crop=crop)
        assert np.abs(outs[0].astype(np.float64) - ref[0]).max() < 1e-4
        for i, s in enumerate(o.sites):
            if s.spec.kind == "preact":
                fa = s.get_A().astype(np.float64)
                fa = np.maximum(fa, 0) if s.spec.relu else fa
                assert np.abs(fa - cv.canvas[i][cv._view(i)]).max() < 1e-4, (t, i)
