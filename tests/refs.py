"""Independent references used ONLY to pin the oracle (CPU tests).

None of them shares code with `oracle/`:
  dense_cnn       -- per-frame dense inference with a library convolution
                     (torch CPU conv2d, float64): what linearity says delta
                     inference must reproduce at threshold 0 with a static camera.
  CanvasReference -- dense inference on a global-coordinate canvas in which
                     out-of-view pixels stay frozen: the "fused input" result that
                     padded convolutions are stated to reproduce.
  StaticDeltaRef  -- static-camera delta inference (no ring, no border) written
                     from the DeltaCNN background section, dense-array formulation.
  reset_frames    -- which frames of a shift sequence force a full reset.
"""
from __future__ import annotations

import numpy as np
import torch
import torch.nn.functional as F


def _conv64(x_hwc, e):
    """x [H, W, Cin] float64 -> conv of edge e, [H', W', Cout] float64 (no bias)."""
    k = e.k
    w = torch.from_numpy(e.w.astype(np.float64))             # [k*k, Cout, Cin]
    w = w.reshape(k, k, w.shape[1], w.shape[2]).permute(2, 3, 0, 1).contiguous()
    x = torch.from_numpy(np.ascontiguousarray(x_hwc)).permute(2, 0, 1)[None]
    y = F.conv2d(x, w, None, stride=e.stride, padding=e.pad)[0].permute(1, 2, 0).numpy()
    if e.up:
        y = y.repeat(1 << e.up, axis=0).repeat(1 << e.up, axis=1)
    return y


def maxpool64(x_hwc, k, stride, pad):
    """Library max pooling (torch, padding counts as -inf), x [H, W, C] float64."""
    x = torch.from_numpy(np.ascontiguousarray(x_hwc.astype(np.float64))).permute(2, 0, 1)[None]
    return F.max_pool2d(x, k, stride, pad)[0].permute(1, 2, 0).numpy()


def site_bias(net, i):
    b = np.zeros(net.sites[i].C, np.float64)
    for e in net.edges:
        if e.dst == i and e.b is not None:
            b += e.b.astype(np.float64)
    return b


def dense_cnn(net, X, return_all=False):
    """Plain dense inference of one frame X [H, W, C]; float64 throughout."""
    val = [None] * len(net.sites)
    val[0] = X.astype(np.float64)
    for i in range(1, len(net.sites)):
        acc = np.zeros(net.site_hw(i) + (net.sites[i].C,), np.float64) + site_bias(net, i)
        for e in net.edges:
            if e.dst == i:
                if getattr(e, "pool", False):
                    acc = acc + maxpool64(val[e.src], e.k, e.stride, e.pad)
                else:
                    acc = acc + (val[e.src] if e.k == 0 else _conv64(val[e.src], e))
        val[i] = np.maximum(acc, 0) if net.sites[i].relu else acc
    if return_all:
        return val
    return [val[i] for i in net.terminal_sites()]


class CanvasReference:
    """Global canvases per site.  Each frame: paste the frame into canvas_0 over
    the view; for every later site recompute f(bias + conv(canvas_src)) over the
    whole canvas and copy it into the site's canvas only inside the site's current
    view.  Pixels outside the view keep their last value, pixels never seen are 0,
    and a full reset clears everything."""

    def __init__(self, net, extent_tiles):
        self.net = net
        self.ext = extent_tiles            # canvas spans tiles [-ext, ext) around the start, plus the view
        T = net.total_stride
        self.oy = extent_tiles * T         # input-pixel offset of global (0, 0) in the canvas
        self.ox = extent_tiles * T
        self.GH = net.H + 2 * extent_tiles * T
        self.GW = net.W + 2 * extent_tiles * T
        self.ty = 0
        self.tx = 0
        self.clear()

    def clear(self):
        self.canvas = []
        for s in self.net.sites:
            self.canvas.append(np.zeros((self.GH // s.stride, self.GW // s.stride, s.C), np.float64))

    def _view(self, i):
        s = self.net.sites[i]
        H, W = self.net.site_hw(i)
        y0 = (self.oy + self.ty * self.net.total_stride) // s.stride
        x0 = (self.ox + self.tx * self.net.total_stride) // s.stride
        return slice(y0, y0 + H), slice(x0, x0 + W)

    def _crop(self, i, crop):
        """The part of site i's view that a frame covering tiles `crop` =
        (ty0, tx0, th, tw) of the view works on."""
        vy, vx = self._view(i)
        if crop is None:
            return vy, vx
        t = self.net.total_stride // self.net.sites[i].stride
        ty0, tx0, th, tw = crop
        return (slice(vy.start + ty0 * t, vy.start + (ty0 + th) * t),
                slice(vx.start + tx0 * t, vx.start + (tx0 + tw) * t))

    def frame(self, X, dty, dtx, reset, crop=None):
        self.ty += int(dty)
        self.tx += int(dtx)
        assert abs(self.ty) <= self.ext and abs(self.tx) <= self.ext
        if reset:
            self.clear()
        if crop is not None:
            return self._frame_crop(X, crop)
        net = self.net
        self.canvas[0][self._view(0)] = X.astype(np.float64)
        for i in range(1, len(net.sites)):
            acc = np.zeros_like(self.canvas[i]) + site_bias(net, i)
            for e in net.edges:
                if e.dst == i:
                    src = self.canvas[e.src]
                    acc = acc + (src if e.k == 0 else _conv64(src, e))
            val = np.maximum(acc, 0) if net.sites[i].relu else acc
            v = self._view(i)
            self.canvas[i][v] = val[v]
        return [self.canvas[i][self._view(i)].copy() for i in net.terminal_sites()]

    def _pool(self, i, src, e):
        """Library max pooling of site i's canvas.  A pooling window takes the pixels of the source's
        current view only (what lies outside takes no part), so everything else is masked out; outputs
        whose window holds no view pixel are not used by the callers."""
        vy, vx = self._view(i)
        masked = np.full_like(src, -np.inf)
        masked[vy, vx] = src[vy, vx]
        out = maxpool64(masked, e.k, e.stride, e.pad)
        return np.where(np.isfinite(out), out, 0.0)

    def _frame_crop(self, X, crop):
        """Cropped frame: the same recomputation, but a site's canvas takes the new
        values inside the crop only (scaled to the site); everything else, inside or
        outside the view, keeps what it had."""
        net = self.net
        self.canvas[0][self._crop(0, crop)] = X.astype(np.float64)
        for i in range(1, len(net.sites)):
            acc = np.zeros_like(self.canvas[i]) + site_bias(net, i)
            for e in net.edges:
                if e.dst == i:
                    src = self.canvas[e.src]
                    if getattr(e, "pool", False):
                        acc = acc + self._pool(e.src, src, e)
                    else:
                        acc = acc + (src if e.k == 0 else _conv64(src, e))
            val = np.maximum(acc, 0) if net.sites[i].relu else acc
            v = self._crop(i, crop)
            self.canvas[i][v] = val[v]
        return [self.canvas[i][self._crop(i, crop)].copy() for i in net.terminal_sites()]

    def dense_valid_mask(self, i, radius_px):
        """[H, W] bool for site i: pixels further than radius_px (site pixels)
        from every view edge (where the canvas equals dense-of-current-frame)."""
        H, W = self.net.site_hw(i)
        m = np.zeros((H, W), bool)
        m[radius_px:H - radius_px, radius_px:W - radius_px] = True
        return m


class StaticDeltaRef:
    """Static-camera delta inference (DeltaCNN background): first frame dense,
    then per site d = f(acc + pending) - f(acc), truncated per pixel by max-abs
    over channels; truncated pixels keep their pending value.  Dense arrays, the
    convolution of the (zero-filled) delta map is taken over the whole map.
    Arithmetic mirrors the stated precision rules: float32 elementwise, float64
    convolution sums rounded once to float32, one rounding per stored value."""

    def __init__(self, net):
        self.net = net
        self.dt = net.np_dtype
        self.first = True
        self.acc, self.pend = [], []
        for i, s in enumerate(net.sites):
            H, W = net.site_hw(i)
            self.acc.append(np.zeros((H, W, s.C), self.dt))
            self.pend.append(np.zeros((H, W, s.C), self.dt) + site_bias(net, i).astype(np.float32).astype(self.dt))

    def _conv(self, d, e):
        """Dense zero-padded correlation by explicit shifted slices, float64."""
        H, W, _ = d.shape
        k, s, p = e.k, e.stride, e.pad
        oh, ow = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
        dp = np.zeros((H + 2 * p + s, W + 2 * p + s, d.shape[2]), np.float64)
        dp[p:p + H, p:p + W] = d
        y = np.zeros((oh, ow, e.w.shape[1]), np.float64)
        w = e.w.astype(np.float64)
        for jy in range(k):
            for jx in range(k):
                sl = dp[jy:jy + s * oh:s, jx:jx + s * ow:s]
                y += sl @ w[jy * k + jx].T
        if e.up:
            y = y.repeat(1 << e.up, axis=0).repeat(1 << e.up, axis=1)
        return y

    def frame(self, X):
        net, f32 = self.net, np.float32
        masks = []
        touched = [np.zeros(net.site_hw(i), bool) for i in range(len(net.sites))]
        for i, s in enumerate(net.sites):
            if s.kind == "output":
                continue
            a = self.acc[i].astype(f32)
            if s.kind == "input":
                out = X.astype(f32) - a
                new_acc = X
                cand = np.ones(net.site_hw(i), bool)
            else:
                t = self.pend[i].astype(f32)
                new = a + t
                out = (np.maximum(new, f32(0)) - np.maximum(a, f32(0))) if s.relu else (new - a)
                new_acc = new.astype(self.dt)
                cand = touched[i] | self.first
            m = cand & ((np.abs(out).max(axis=2) > f32(s.theta)) | self.first)
            self.acc[i][m] = new_acc[m]
            if s.kind != "input":
                self.pend[i][m] = 0
            d = np.where(m[:, :, None], out.astype(self.dt), self.dt(0))
            masks.append(m)
            for e in net.edges:
                if e.src != i:
                    continue
                if e.k == 0:
                    y = d.astype(f32)
                    hit = m
                else:
                    y = self._conv(d.astype(np.float64), e).astype(f32)
                    hit = self._conv(m[:, :, None].astype(np.float64),
                                     _ones_edge(e)).reshape(net.site_hw(e.dst)) > 0
                P = self.pend[e.dst]
                P[hit] = (P[hit].astype(f32) + y[hit]).astype(self.dt)
                touched[e.dst] |= hit
        self.first = False
        outs = []
        for i in net.terminal_sites():
            o = self.pend[i].copy()
            outs.append(np.maximum(o, self.dt(0)) if net.sites[i].relu else o)
        return outs, masks


class _OnesEdge:
    pass


def _ones_edge(e):
    o = _OnesEdge()
    o.k, o.stride, o.pad, o.up = e.k, e.stride, e.pad, e.up
    o.w = np.ones((e.k * e.k, 1, 1), np.float64)
    return o


def reset_frames(shifts, site_shapes_tiles):
    """Frames whose shift forces a full reset: the first frame, a step against a
    direction in which the view has grown since the last reset, or a step of a
    whole view extent or more.  `site_shapes_tiles` = (H, W) of the view in tiles."""
    Ht, Wt = site_shapes_tiles
    out = []
    moved = {"+y": False, "-y": False, "+x": False, "-x": False}
    for t, (dy, dx) in enumerate(shifts):
        r = t == 0 or abs(dy) >= Ht or abs(dx) >= Wt
        r |= (dy > 0 and moved["-y"]) or (dy < 0 and moved["+y"])
        r |= (dx > 0 and moved["-x"]) or (dx < 0 and moved["+x"])
        if r:
            moved = dict.fromkeys(moved, False)
            out.append(t)
        else:
            if dy:
                moved["+y" if dy > 0 else "-y"] = True
            if dx:
                moved["+x" if dx > 0 else "-x"] = True
    return out
