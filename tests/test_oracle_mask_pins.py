"""Pins for the oracle's post-processing of the input update mask (ROI-focused
sensing, suppression of isolated updates on a downscaled delta, dilation): each
step against a library routine or a value the paper prints."""
import numpy as np
import pytest
import scipy.ndimage as ndi
import torch

from inputs import build_net
from oracle.mdcnn_oracle import OracleNet
from test_oracle_pins import golden, rand_frames


def fresh(H=64, W=64, theta=0.05):
    net = build_net(2, H=H, W=W)
    net.sites[0].theta = theta
    o = OracleNet(net)
    o.shift_camera(0, 0)
    return net, o


def magnitude(o, X):
    return np.abs(X.astype(np.float64) - o.sites[0].get_A().astype(np.float64)).max(axis=2)


def test_plain_mask_is_the_threshold_test_of_the_input_site():
    net, o = fresh()
    frames = rand_frames(net, 3, 0, walk=0.05)
    o.frame(frames[0], 0, 0)
    want = o.input_mask(frames[1])
    o.frame(frames[1], 0, 0)
    assert np.array_equal(want.astype(bool), o.sites[0].M)
    assert 0 < want.mean() < 1


def test_dilation_equals_library_binary_dilation_and_the_printed_extent():
    g = golden()
    net, o = fresh()
    X = np.zeros((64, 64, 3), np.float32)
    X[30, 40] = 1.0
    d = int(g["mask_dilation_px"])
    m = o.input_mask(X, dilate=d)
    assert m.sum() == g["mask_dilation_extent"] ** 2                     # one pixel -> 21 x 21
    ys, xs = np.nonzero(m)
    assert (ys.min(), ys.max(), xs.min(), xs.max()) == (30 - d, 30 + d, 40 - d, 40 + d)
    rng = np.random.default_rng(1)
    X = (rng.random((64, 64, 3)) < 0.01).astype(np.float32)
    for d in (1, 3, 7):
        base = o.input_mask(X).astype(bool)
        want = ndi.binary_dilation(base, structure=np.ones((2 * d + 1, 2 * d + 1), bool))
        assert np.array_equal(o.input_mask(X, dilate=d).astype(bool), want)      # clipped at the view edge


def test_roi_weighting_uses_the_printed_factors():
    net, o = fresh(theta=0.05)
    X = np.full((64, 64, 3), 0.1, np.float32)              # 0.1 * 0.4 < 0.05 < 0.1 * 1.0
    roi = np.zeros((64, 64), np.float32)
    roi[:, 32:] = 1.0
    m = o.input_mask(X, roi=roi)
    assert not m[:, :32].any() and m[:, 32:].all()
    roi[:] = 0.5                                           # 0.1 * 0.7 = 0.07 > 0.05
    assert o.input_mask(X, roi=roi).all()
    assert not o.input_mask(X, roi=roi, base=0.2, gain=0.4).any()     # 0.1 * 0.4


@pytest.mark.parametrize("q", [2, 4, 8])
def test_downscaling_equals_library_average_pooling(q):
    net, o = fresh()
    rng = np.random.default_rng(q)
    X = rng.normal(0, 0.05, (64, 64, 3)).astype(np.float32)
    e = magnitude(o, X)
    pooled = torch.nn.functional.avg_pool2d(torch.from_numpy(e)[None, None], q)[0, 0].numpy()
    theta = float(np.median(pooled))
    got = o.input_mask(X, theta=theta, pool=q).astype(bool)
    want = np.repeat(np.repeat(pooled > theta, q, 0), q, 1)
    clear = np.repeat(np.repeat(np.abs(pooled - theta) > 1e-6, q, 0), q, 1)
    assert np.array_equal(got[clear], want[clear]) and clear.mean() > 0.99
    assert 0.3 < got.mean() < 0.7


def test_suppression_keeps_what_a_3x3_average_pooling_above_one_ninth_keeps():
    net, o = fresh()
    rng = np.random.default_rng(3)
    X = (rng.random((64, 64, 3)) < 0.02).astype(np.float32)
    base = o.input_mask(X).astype(bool)
    avg = torch.nn.functional.avg_pool2d(torch.from_numpy(base.astype(np.float64))[None, None], 3, stride=1, padding=1,
                                         count_include_pad=True)[0, 0].numpy()
    want = base & (avg > 1 / 9 + 1e-9)
    got = o.input_mask(X, suppress=True).astype(bool)
    assert np.array_equal(got, want)
    assert 0 < got.sum() < base.sum()
    # by hand: a lone pixel goes, a pair (also a diagonal one) stays
    X = np.zeros((64, 64, 3), np.float32)
    X[5, 5] = X[20, 20] = X[20, 21] = X[40, 40] = X[41, 41] = X[0, 0] = 1
    got = o.input_mask(X, suppress=True)
    assert got.sum() == 4 and got[20, 20] and got[20, 21] and got[40, 40] and got[41, 41]


def test_all_steps_together_against_the_library_routines():
    net, o = fresh()
    rng = np.random.default_rng(9)
    frames = rand_frames(net, 2, 5, walk=0.03)
    o.frame(frames[0], 0, 0)
    roi = rng.random((64, 64)).astype(np.float32)
    q, d, theta = 2, 3, 0.05
    e = magnitude(o, frames[1]) * (0.4 + 0.6 * roi.astype(np.float64))
    pooled = e.reshape(32, q, 32, q).mean(axis=(1, 3))
    hit = pooled > theta
    cnt = ndi.convolve(hit.astype(int), np.ones((3, 3), int), mode="constant")
    keep = np.repeat(np.repeat(hit & (cnt >= 2), q, 0), q, 1)
    want = ndi.binary_dilation(keep, structure=np.ones((2 * d + 1, 2 * d + 1), bool))
    got = o.input_mask(frames[1], roi=roi, theta=theta, pool=q, suppress=True, dilate=d).astype(bool)
    assert np.abs(pooled - theta).min() > 1e-6
    assert np.array_equal(got, want)
    assert 0 < got.mean() < 1


def test_mask_follows_the_crop():
    net = build_net(2, H=64, W=64)
    o = OracleNet(net, crops=True)
    frames = rand_frames(net, 2, 1, walk=0.05)
    T = net.total_stride
    o.frame(frames[0], 0, 0, crop=(0, 0, 64 // T, 64 // T))
    full = o.input_mask(frames[1], dilate=2)
    o.set_crop(2, 4, 8, 6)
    part = o.input_mask(frames[1][2 * T:10 * T, 4 * T:10 * T], dilate=0)
    o.set_crop(0, 0, 64 // T, 64 // T)
    whole = o.input_mask(frames[1])
    assert np.array_equal(part, whole[2 * T:10 * T, 4 * T:10 * T])
    assert full.sum() > whole.sum()


def test_a_cell_mean_equal_to_the_threshold_is_not_an_update():
    """The downscaled delta is compared with the threshold by strict >, like every pixel delta (a delta that
    equals the threshold is truncated, so that threshold 0 skips exactly the unchanged pixels): cells whose
    mean is exactly theta, one ulp below and one ulp above it.  All values are exact in float32."""
    theta = np.float32(0.25)
    net, o = fresh(H=16, W=16, theta=float(theta))
    up = np.nextafter(theta, np.float32(1))
    dn = np.nextafter(theta, np.float32(0))
    X = np.zeros((16, 16, 3), np.float32)                  # A is zero after the reset: the magnitude is max_c |X|
    X[0:2, 0:2, 1] = theta                                 # cell (0, 0): four pixels at theta -> mean == theta
    X[0:2, 2:4, 0] = [[0.5, 0.0], [0.25, 0.25]]            # cell (0, 1): sum 1.0 -> mean == theta exactly
    X[2:4, 0:2, 2] = up                                    # cell (1, 0): just above
    X[2:4, 2:4, 0] = dn                                    # cell (1, 1): just below
    m = o.input_mask(X, pool=2)
    cells = m.reshape(8, 2, 8, 2).max(axis=(1, 3))
    assert cells[0, 0] == 0 and cells[0, 1] == 0 and cells[1, 1] == 0
    assert cells[1, 0] == 1 and cells.sum() == 1
    assert m[2:4, 0:2].all() and m.sum() == 4
    # per pixel (pool = 1) the same rule: only the pixels above theta
    m1 = o.input_mask(X)
    assert m1.sum() == 4 + 1 and m1[0, 2] == 1 and m1[2:4, 0:2].all()
