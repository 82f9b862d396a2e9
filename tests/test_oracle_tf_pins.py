"""Pins for the oracle's truncation-free activation sites (Supplementary, Optimizing memory consumption:
truncation is switched off at the activation layers that do not follow a 3x3 convolution; such a layer keeps
only its accumulated-values buffer and passes on every update it receives)."""
import copy

import numpy as np
import pytest

import refs
from inputs import build_net, build_sequence
from inputs.nets import NetSpec, _Builder, truncation_free
from oracle.mdcnn_oracle import OracleNet
from test_oracle_pins import as_f32, golden, monotone_shifts, rand_frames, set_theta


def pairs_net(dtype="f32", H=24, W=24, C=(3, 6, 8, 6, 8, 4), relu=True, theta=0.05, seed=0, stride1=1):
    """A DenseNet-like chain of (3x3, 1x1) pairs: in -3x3-> a -1x1-> b -3x3-> c -1x1-> d -3x3-> out.  The 1x1
    convolutions may be strided (stride1)."""
    rng = np.random.default_rng(seed)
    net = NetSpec("pairs", dtype, H, W, 4 * stride1 * stride1)
    b = _Builder(net, rng, 0.1)
    x = b.site("in", C[0], 1, "input", False, theta)
    s = 1
    a = b.site("a", C[1], s, theta=theta, relu=relu)
    b.conv(x, a, 3, 1)
    s *= stride1
    bb = b.site("b", C[2], s, theta=theta, relu=relu)
    b.conv(a, bb, 1, stride1, pad=0)
    c = b.site("c", C[3], s, theta=theta, relu=relu)
    b.conv(bb, c, 3, 1)
    s *= stride1
    d = b.site("d", C[4], s, theta=theta, relu=relu)
    b.conv(c, d, 1, stride1, pad=0)
    y = b.site("out", C[5], s, "output", False, 0.0)
    b.conv(d, y, 3, 1)
    return net


def moving_path(n):
    """Growth in both axes, then a reversal (a reset), then growth the other way."""
    return ([(0, 0), (1, 0), (0, 1), (1, 1), (-1, 0), (0, -1), (-1, -1), (0, 0)] * 2)[:n]


def test_marking_follows_the_paper():
    """Only the activation layers after a 1x1 convolution lose their truncation: in a chain of (3x3, 1x1) pairs that
    is every second one; and such a layer keeps half the state (the printed 50 %)."""
    net = truncation_free(pairs_net())
    assert [s.trunc_free for s in net.sites] == [False, False, True, False, True, False]
    for cfg, kw, want in [(5, dict(H=16, W=16, C=8, Cm=4), [1]), (3, dict(H=64, W=64, widths=(4, 8, 8, 16)), []),
                          (2, dict(H=64, W=64), [3])]:
        n2 = truncation_free(build_net(cfg, **kw))
        assert [i for i, s in enumerate(n2.sites) if s.trunc_free] == want
    std, tf = OracleNet(pairs_net()), OracleNet(net)
    for i in (2, 4):
        assert tf.sites[i].P is None
        saved = 1 - tf.sites[i].state_elements() / std.sites[i].state_elements()
        assert saved == golden()["truncation_free_layer_memory_saved"]
    assert tf.sites[1].state_elements() == std.sites[1].state_elements()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("stride1", [1, 2])
def test_equals_threshold_zero_at_those_sites(dtype, relu, stride1):
    """Not truncating is truncating with threshold 0: with the other sites truncating as before, the network with
    truncation-free sites gives the same update masks, lists, deltas, accumulated values and outputs, bit for bit,
    as the ordinary path with threshold 0 at those sites - under a moving camera with resets.  (With ReLU the two
    could part by a rounding where a pixel's pending value stays pending because the activation did not change;
    the sequences below are compared for that and must at least agree within the tolerance.)"""
    base = pairs_net(dtype, relu=relu, stride1=stride1, H=32, W=32, seed=3)
    ref_net = copy.deepcopy(base)
    tf_net = truncation_free(copy.deepcopy(base))
    for s_ref, s_tf in zip(ref_net.sites, tf_net.sites):
        if s_tf.trunc_free:
            s_ref.theta = 0.0
    ref, tf = OracleNet(ref_net), OracleNet(tf_net)
    frames = rand_frames(base, 12, 4, walk=0.1)
    exact = True
    for X, (dy, dx) in zip(frames, moving_path(12)):
        a, r1 = ref.frame(X, dy, dx)
        b, r2 = tf.frame(X, dy, dx)
        assert r1 == r2
        still_pending = any(np.abs(ref.sites[i].view_of_window(ref.sites[i].get_P()).astype(np.float32)).max() > 0
                            for i, s in enumerate(tf_net.sites) if s.trunc_free)
        if still_pending:
            assert relu                      # only an unchanged activation leaves a value pending at threshold 0
            exact = False
        for i, (sr, st) in enumerate(zip(ref.sites, tf.sites)):
            if sr.spec.kind == "output":
                continue
            if exact:
                assert np.array_equal(sr.M, st.M) and np.array_equal(sr.L, st.L), f"site {i}: masks"
                assert np.array_equal(sr.get_A(), st.get_A()) and np.array_equal(sr.delta, st.delta), f"site {i}: values"
        tol = 0.0 if exact else (1e-4 if dtype == "f32" else 2e-2)
        assert np.abs(a[0].astype(np.float64) - b[0].astype(np.float64)).max() <= tol
    if not relu:
        assert exact


@pytest.mark.parametrize("name", ["pairs", "pairs_s2", "bottleneck"])
def test_threshold_zero_everywhere_equals_dense_inference(name):
    """Linearity: with no truncation anywhere the output is the dense network of the current frame (static camera),
    and dense inference on the fused canvas under a moving camera - with truncation-free sites as without."""
    net = {"pairs": lambda: pairs_net(), "pairs_s2": lambda: pairs_net(stride1=2, H=32, W=32),
           "bottleneck": lambda: as_f32(build_net(5, H=16, W=16, C=8, Cm=4))}[name]()
    net = truncation_free(set_theta(net, 0.0))
    assert any(s.trunc_free for s in net.sites)
    o = OracleNet(net)
    for X in rand_frames(net, 4, 1):
        outs, _ = o.frame(X, 0, 0)
        vals = refs.dense_cnn(net, X, return_all=True)
        assert np.abs(outs[0].astype(np.float64) - vals[net.terminal_sites()[0]]).max() < 1e-4
        for i, s in enumerate(o.sites):
            if s.tf:       # the accumulated values ARE the dense pre-activations
                fa = s.get_A().astype(np.float64)
                assert np.abs((np.maximum(fa, 0) if s.spec.relu else fa) - vals[i]).max() < 1e-4
    o = OracleNet(net)
    cv = refs.CanvasReference(net, 16)
    for X, (dy, dx) in zip(rand_frames(net, 6, 11), monotone_shifts(6, 1)):
        outs, r = o.frame(X, dy, dx)
        assert np.abs(outs[0].astype(np.float64) - cv.frame(X, dy, dx, r)[0]).max() < 1e-4


def test_conservation_with_truncation_at_the_other_sites():
    """The other sites truncate (threshold 0.05): at a truncation-free site the accumulated values still equal bias +
    the producer's convolution of the source's activations, and the deltas it emitted sum to its activation."""
    net = truncation_free(pairs_net(theta=0.05))
    o = OracleNet(net)
    sums = {i: np.zeros(s.A.shape, np.float64) for i, s in enumerate(o.sites) if s.tf}
    for X in rand_frames(net, 8, 7, walk=0.05):
        o.shift_camera(0, 0)
        for i, s in enumerate(o.sites):
            if s.spec.kind == "output":
                continue
            o.layer_forward(i, X if i == 0 else None)
            if s.tf:
                sums[i] += s.delta.astype(np.float64)
        for i, s in enumerate(o.sites):
            if not s.tf:
                continue
            e = [e for e in net.edges if e.dst == i][0]
            src = o.sites[e.src]
            fa = src.get_A().astype(np.float64)
            fa = np.maximum(fa, 0) if src.spec.relu else fa
            want = refs.site_bias(net, i) + refs._conv64(fa, e)
            a = s.get_A().astype(np.float64)
            assert np.abs(a - want).max() < 1e-4
            assert np.abs(sums[i] - (np.maximum(a, 0) if s.spec.relu else a)).max() < 1e-4
            assert 0 < s.M.mean() < 1 or s.M.all()


@pytest.mark.parametrize("mistake", ["no_bias", "stale_previous"])
def test_planted_mistakes_are_caught(monkeypatch, mistake):
    """A newly unveiled pixel must start from its bias, and its previous activation must count as zero."""
    import oracle.mdcnn_oracle as om
    net = truncation_free(set_theta(pairs_net(relu=False), 0.0))
    if mistake == "no_bias":
        orig = om.OracleNet.__init__

        def init(self, *a, **k):
            orig(self, *a, **k)
            for s in self.sites:
                if s.tf:
                    s.beta = np.zeros_like(s.beta)
        monkeypatch.setattr(om.OracleNet, "__init__", init)
    else:
        orig_shift = om.OracleNet.shift_camera

        def shift(self, dty, dtx):
            r = orig_shift(self, dty, dtx)
            for s in self.sites:
                if s.tf:
                    s.N[:] = False           # new pixels are no longer told apart: delta against a stale value
            return r
        monkeypatch.setattr(om.OracleNet, "shift_camera", shift)
    o = om.OracleNet(net)
    cv = refs.CanvasReference(net, 16)
    worst = 0.0
    for X, (dy, dx) in zip(rand_frames(net, 6, 11), monotone_shifts(6, 1)):
        outs, r = o.frame(X, dy, dx)
        worst = max(worst, np.abs(outs[0].astype(np.float64) - cv.frame(X, dy, dx, r)[0]).max())
    assert worst > 1e-2
