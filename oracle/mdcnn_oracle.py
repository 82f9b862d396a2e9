"""CPU oracle for the MotionDeltaCNN hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow NumPy statement of what the path computes, written from the
paper; it shares no code with the HIP library and must never be imported by
the product path (only by tests, the smoke check and the CPU-baseline leg of
the benchmark).

What is followed, and where the paper defines it:

* delta input, truncation to a per-pixel update mask, accumulated-values and
  truncated-values buffers, delta propagation through linear layers by
  linearity and through activations as f(acc + d) - f(acc)
  -- Background: DeltaCNN;
* spherical (2-D ring) buffers addressed with wrapped coordinates and a
  per-layer pixel offset = tile offset x layer tile size -- Spherical Buffers;
* newly unveiled pixels overwrite the pixels that left the ring, are reset and
  receive the biases -- Dynamic Initialization; the bias is placed into the
  truncated-values buffer of the reset pixels so the activation adds it
  -- Supplementary, Implicit bias application;
* every output that an in-view input can touch is computed; the outputs
  outside the view ("dilated" pixels) are accumulated in a slightly enlarged
  truncated-values buffer and attach when that region is unveiled
  -- Padded Convolutions (a 64x64 input under a 3x3 kernel yields 66x66);
* growing in one direction invalidates the stash of the opposite side, moving
  back over it resets all buffers and the frame is inferred densely
  -- Buffer management;
* max pooling keeps the previous output of every pixel in a buffer of its own:
  the delta of a pixel is taken against that previous output, or against zero
  if the pixel was reset in the current frame -- Supplementary, Maximum Pooling;
* a frame may cover only a tile-aligned part of the buffers (a crop, e.g. the
  bounding box of a region of interest); the tile offsets given with the frame
  place it in the buffers, every layer works on the crop scaled to its own
  tile size, and the rest of the buffers keeps what it holds -- Spherical
  Buffers (cropped inputs), Evaluation: Human Pose Estimation;
* the update mask of the input may be post-processed before it is used: the
  delta is weighted by a region-of-interest map, isolated updates are
  suppressed on a downscaled delta, and the mask is dilated by a few pixels
  -- Optimizations; Supplementary (ROI-focused sensing, first-layer dilation);
* truncation may be switched off at selected activation layers - those that do
  not follow a 3x3 convolution - which then need only their accumulated-values
  buffer, at the cost of passing on every update they receive
  -- Supplementary, Optimizing memory consumption.

Arithmetic: stored tensors (A, P, delta maps, weights, frames) are in the
network's storage dtype; every elementwise operation is done in float32 in the
written order with one rounding to the storage dtype per stored value; a
convolution output is summed in float64, rounded once to float32 and added to
the pending value in float32.

Naming: A = accumulated values, P = pending = truncated values incl. the
dilated border, N = newly unveiled this frame, U = touched by a producer this
frame, M = update mask, L = compacted list of updated pixels.
"""
from __future__ import annotations

import numpy as np

N_BIT, U_BIT, M_BIT = 1, 2, 4


def conv_border(k, stride, pad, w_in, w_out):
    """Dilated border (before, after) along one axis: the outputs outside
    [0, w_out) that still read at least one input in [0, w_in).
    Padded Convolutions: all outputs affected by the current input."""
    if k == 0:
        return 0, 0
    before = (k - 1 - pad) // stride
    after = (w_in - 1 + pad) // stride - (w_out - 1)
    return max(before, 0), max(after, 0)


class OracleSite:
    def __init__(self, spec, H, W, tile, dtype, origin=(0, 0)):
        self.spec = spec
        self.H, self.W, self.C = H, W, spec.C
        self.tile = tile
        self.dtype = dtype
        self.border = [0, 0, 0, 0]          # before_y, after_y, before_x, after_x
        self.beta = np.zeros(spec.C, np.float32)
        self.origin = origin                # physical rotation of the rings
        self.gy = 0                         # global pixel coordinate of view pixel (0, 0)
        self.gx = 0
        self.pooled = False                 # destination of a max-pooling edge
        self.tf = bool(getattr(spec, "trunc_free", False))   # truncation-free: accumulated values only, no P

    def allocate(self):
        by0, by1, bx0, bx1 = self.border
        self.Hp, self.Wp = self.H + by0 + by1, self.W + bx0 + bx1
        self.A = np.zeros((self.H, self.W, self.C), self.dtype)
        self.P = None if self.tf else np.zeros((self.Hp, self.Wp, self.C), self.dtype)
        self.N = np.zeros((self.H, self.W), bool)
        self.U = np.zeros((self.H, self.W), bool)
        self.M = np.zeros((self.H, self.W), bool)
        self.delta = np.zeros((self.H, self.W, self.C), self.dtype)
        self.L = np.zeros(0, np.int32)
        self.n_candidates = 0
        self.Y = np.zeros((self.H, self.W, self.C), self.dtype) if self.pooled else None   # previous pooling output (ring like A)
        # cropped frames: what a pixel of the ring still owes (rings like A)
        self.unseen = np.zeros((self.H, self.W), bool)   # allocated, not yet inside any frame
        self.dirty = np.zeros((self.H, self.W), bool)    # touched by a producer while outside the frame
        self.crop = (0, self.H, 0, self.W)               # rows y0:y1, columns x0:x1 of the view the frame covers

    # ring addressing: global pixel -> physical slot, wrapped (Spherical Buffers)
    def _a_index(self):
        r = (self.gy + np.arange(self.H) + self.origin[0]) % self.H
        c = (self.gx + np.arange(self.W) + self.origin[1]) % self.W
        return np.ix_(r, c)

    def _p_index(self):
        by0, _, bx0, _ = self.border
        r = (self.gy - by0 + np.arange(self.Hp) + self.origin[0]) % self.Hp
        c = (self.gx - bx0 + np.arange(self.Wp) + self.origin[1]) % self.Wp
        return np.ix_(r, c)

    def get_A(self):
        return self.A[self._a_index()]

    def set_A(self, v):
        self.A[self._a_index()] = v

    def get_Y(self):
        return self.Y[self._a_index()]

    def set_Y(self, v):
        self.Y[self._a_index()] = v

    def get_ring(self, name):
        return getattr(self, name)[self._a_index()]

    def set_ring(self, name, v):
        getattr(self, name)[self._a_index()] = v

    def in_crop(self):
        y0, y1, x0, x1 = self.crop
        m = np.zeros((self.H, self.W), bool)
        m[y0:y1, x0:x1] = True
        return m

    def get_P(self):
        """Pending values over the padded window (view plus dilated border)."""
        assert not self.tf, "a truncation-free site keeps no truncated-values buffer"
        return self.P[self._p_index()]

    def state_elements(self):
        """Elements of the buffers the site keeps from frame to frame."""
        return self.A.size + (0 if self.P is None else self.P.size) + (0 if self.Y is None else self.Y.size)

    def set_P(self, v):
        self.P[self._p_index()] = v

    def view_of_window(self, win):
        by0, _, bx0, _ = self.border
        return win[by0:by0 + self.H, bx0:bx0 + self.W]


class OracleNet:
    def __init__(self, net, origins=None, crops=False):
        """crops=True: frames may cover a part of the buffers only (set_crop)."""
        self.net = net
        self.crops = bool(crops)
        self.dtype = net.np_dtype
        self.sites = []
        for i, s in enumerate(net.sites):
            H, W = net.H // s.stride, net.W // s.stride
            org = (0, 0) if origins is None else origins[i]
            self.sites.append(OracleSite(s, H, W, net.total_stride // s.stride, self.dtype, org))
        for e in net.edges:
            src, dst = self.sites[e.src], self.sites[e.dst]
            if e.k == 0:
                assert (src.H, src.W, src.C) == (dst.H, dst.W, dst.C)
            elif getattr(e, "pool", False):
                oh = (src.H + 2 * e.pad - e.k) // e.stride + 1
                ow = (src.W + 2 * e.pad - e.k) // e.stride + 1
                assert (oh, ow, src.C) == (dst.H, dst.W, dst.C) and e.up == 0 and dst.spec.kind == "preact"
                dst.pooled = True               # pooling outputs exist inside the view only: no border
            else:
                oh = (src.H + 2 * e.pad - e.k) // e.stride + 1
                ow = (src.W + 2 * e.pad - e.k) // e.stride + 1
                if e.up:
                    assert e.k == 1 and e.stride == 1 and e.pad == 0
                assert (oh << e.up, ow << e.up) == (dst.H, dst.W), "edge shape mismatch"
                by = conv_border(e.k, e.stride, e.pad, src.H, oh)
                bx = conv_border(e.k, e.stride, e.pad, src.W, ow)
                b = [by[0], by[1], bx[0], bx[1]]
                dst.border = [max(p, q) for p, q in zip(dst.border, b)]
                if e.b is not None:
                    dst.beta = dst.beta + e.b.astype(np.float32)
        for i, s in enumerate(self.sites):
            if s.tf:
                # no truncation only where updates are not dilated: one producer, a 1x1 convolution
                prods = [e for e in net.edges if e.dst == i]
                assert s.spec.kind == "preact" and len(prods) == 1 and prods[0].k == 1 and prods[0].up == 0 and not prods[0].pad
                assert not getattr(prods[0], "pool", False) and s.border == [0, 0, 0, 0] and not self.crops
            s.allocate()
        self.fresh = True
        self.R = dict(up=False, down=False, left=False, right=False)
        self.n_resets = 0

    # ------------------------------------------------------------------ shift
    def shift_camera(self, dty, dtx):
        """Buffer management: move every site's view by (dty, dtx) tiles; reset
        the pixels that enter, or everything when growth is restricted."""
        dty, dtx = int(dty), int(dtx)
        R = self.R
        full = self.fresh
        full |= (dtx > 0 and R["right"]) or (dtx < 0 and R["left"])
        full |= (dty > 0 and R["down"]) or (dty < 0 and R["up"])
        for s in self.sites:
            full |= abs(dtx) * s.tile >= s.W or abs(dty) * s.tile >= s.H
        if full:
            for s in self.sites:
                s.gy += dty * s.tile
                s.gx += dtx * s.tile
                s.A[:] = 0
                if not s.tf:
                    s.P[:] = s.beta.astype(s.dtype)
                s.N[:] = True
                s.U[:] = False
                s.unseen[:] = True
                s.dirty[:] = False
                if self.crops and s.pooled:
                    s.Y[:] = 0
            self.R = dict(up=False, down=False, left=False, right=False)
            self.fresh = False
            self.n_resets += 1
            return True
        if dtx > 0:
            R["left"] = True
        if dtx < 0:
            R["right"] = True
        if dty > 0:
            R["up"] = True
        if dty < 0:
            R["down"] = True
        for s in self.sites:
            by0, _, bx0, _ = s.border
            oy, ox = s.gy, s.gx
            s.gy += dty * s.tile
            s.gx += dtx * s.tile
            # pixels of the new padded window that the old one did not hold
            Y = (s.gy - by0 + np.arange(s.Hp))[:, None]
            X = (s.gx - bx0 + np.arange(s.Wp))[None, :]
            held = (Y >= oy - by0) & (Y < oy - by0 + s.Hp) & (X >= ox - bx0) & (X < ox - bx0 + s.Wp)
            if not s.tf:
                Pw = s.get_P()
                Pw[~held] = s.beta.astype(s.dtype)
                s.set_P(Pw)
            # pixels of the new view that the old view did not hold
            Y = (s.gy + np.arange(s.H))[:, None]
            X = (s.gx + np.arange(s.W))[None, :]
            seen = (Y >= oy) & (Y < oy + s.H) & (X >= ox) & (X < ox + s.W)
            Av = s.get_A()
            Av[~seen] = 0
            s.set_A(Av)
            s.N = ~seen
            s.U[:] = False
            for name, fresh in (("unseen", True), ("dirty", False)):
                v = s.get_ring(name)
                v[~seen] = fresh
                s.set_ring(name, v)
            if self.crops and s.pooled:
                Yv = s.get_Y()
                Yv[~seen] = 0
                s.set_Y(Yv)
        return False

    def set_crop(self, ty0, tx0, th, tw):
        """The next frames cover tiles [ty0, ty0+th) x [tx0, tx0+tw) of the
        buffers' view (tile offsets relative to the view after the shift); every
        site works on that rectangle scaled by its own tile size
        (Spherical Buffers: tile offset x layer tile size)."""
        assert self.crops
        for s in self.sites:
            assert 0 <= ty0 and 0 < th and (ty0 + th) * s.tile <= s.H
            assert 0 <= tx0 and 0 < tw and (tx0 + tw) * s.tile <= s.W
            s.crop = (ty0 * s.tile, (ty0 + th) * s.tile, tx0 * s.tile, (tx0 + tw) * s.tile)

    # ------------------------------------------------------- step 1 of a site
    def _truncate(self, i, frame, forced):
        s = self.sites[i]
        f32 = np.float32
        if s.tf:
            # Nothing is truncated here: the update mask and the deltas of this frame were made when the
            # producer's output arrived (_edge); what is left is the compaction.
            assert forced is None, "the mask of a truncation-free site cannot be forced"
            s.L = np.flatnonzero(s.M.ravel()).astype(np.int32)
            s.n_candidates = int(s.touched.sum())
            s.N = np.zeros_like(s.N)
            return
        theta = f32(s.spec.theta)
        A = s.get_A()
        a = A.astype(f32)
        inside = np.ones((s.H, s.W), bool)
        if self.crops:
            # Only the pixels the frame covers are worked on.  Of those, the ones no frame
            # has covered since they were allocated are the newly unveiled ones, and the ones
            # a producer touched while they lay outside earlier frames count as touched.
            y0, y1, x0, x1 = s.crop
            inside = s.in_crop()
            unseen, dirty = s.get_ring("unseen"), s.get_ring("dirty")
            s.N = inside & unseen
            dirty |= s.U & ~inside                     # remembered until a frame covers the pixel
            s.U = inside & (s.U | dirty)
            unseen[inside] = False
            dirty[inside] = False
            s.set_ring("unseen", unseen)
            s.set_ring("dirty", dirty)
            if frame is not None:                      # the frame and the forced mask have the crop's shape
                assert frame.shape == (y1 - y0, x1 - x0, s.C)
                full = np.zeros((s.H, s.W, s.C), s.dtype)
                full[y0:y1, x0:x1] = frame
                frame = full
            if forced is not None:
                assert forced.shape == (y1 - y0, x1 - x0)
                full = np.zeros((s.H, s.W), bool)
                full[y0:y1, x0:x1] = forced.astype(bool)
                forced = full
        if s.spec.kind == "input":
            assert frame.shape == (s.H, s.W, s.C) and frame.dtype == s.dtype
            cand = inside.copy()
            out = frame.astype(f32) - a
            newA = frame
        else:
            Pw = s.get_P()
            t = s.view_of_window(Pw).astype(f32)
            cand = s.U | s.N
            if forced is not None:
                cand = inside.copy()
            acc = a + t
            if s.spec.relu:
                out = np.maximum(acc, f32(0)) - np.maximum(a, f32(0))
            else:
                out = acc - a
            newA = acc.astype(s.dtype)
        mag = np.abs(out).max(axis=2)
        # diagnostics for the comparison protocols (no effect on the state): the magnitude the
        # threshold test looks at, and the decision that test takes on the site's own candidates
        # -- also when a forced mask replaces it below
        s.mag = mag
        s.own = (inside if s.spec.kind == "input" else (s.U | s.N)) & (s.N | (mag > theta))
        if forced is not None:
            hit = forced.astype(bool)
        else:
            hit = mag > theta
        M = cand & (s.N | hit)
        A[M] = newA[M]
        s.set_A(A)
        s.delta[:] = 0
        s.delta[M] = out.astype(s.dtype)[M]
        if s.spec.kind != "input":
            Pv = s.view_of_window(Pw)
            Pv[M] = 0
            s.set_P(Pw)
        s.M = M
        s.L = np.flatnonzero(M.ravel()).astype(np.int32)   # ascending view-linear index
        s.n_candidates = int(cand.sum())
        s.N = np.zeros_like(s.N)
        s.U = np.zeros_like(s.U)

    # ------------------------------------------------------------- one edge
    def compute_list(self, e):
        """Outputs (padded-window linear index of the destination, ascending)
        whose footprint holds at least one updated in-view input pixel."""
        src, dst = self.sites[e.src], self.sites[e.dst]
        by0, _, bx0, _ = dst.border
        cover = np.zeros((dst.Hp, dst.Wp), bool)
        iy, ix = np.nonzero(src.M)
        if e.k == 0:
            cover[iy + by0, ix + bx0] = True
        elif e.up:
            f = 1 << e.up
            for a in range(f):
                for b in range(f):
                    cover[iy * f + a + by0, ix * f + b + bx0] = True
        else:
            for jy in range(e.k):
                for jx in range(e.k):
                    ny, nx = iy + e.pad - jy, ix + e.pad - jx
                    ok = (ny % e.stride == 0) & (nx % e.stride == 0)
                    oy, ox = ny[ok] // e.stride, nx[ok] // e.stride
                    if getattr(e, "pool", False):   # pooling outputs exist inside the view only
                        inv = (oy >= 0) & (oy < dst.H) & (ox >= 0) & (ox < dst.W)
                        oy, ox = oy[inv], ox[inv]
                    cover[oy + by0, ox + bx0] = True
        return np.flatnonzero(cover.ravel()).astype(np.int32)

    def _edge(self, e):
        src, dst = self.sites[e.src], self.sites[e.dst]
        f32 = np.float32
        by0, _, bx0, _ = dst.border
        lst = self.compute_list(e)
        wy, wx = lst // dst.Wp, lst % dst.Wp          # padded-window coordinates
        oy, ox = wy - by0, wx - bx0                   # view coordinates of the destination
        if getattr(e, "pool", False):
            # Maximum Pooling: the output is recomputed from the source's activations
            # (in-view pixels of the window only); its delta is taken against the pixel's
            # previous output, or against zero if the pixel was reset this frame.
            act = src.get_A().astype(f32)
            if src.spec.relu:
                act = np.maximum(act, f32(0))
            out = np.full((len(lst), dst.C), -np.inf, f32)
            for jy in range(e.k):
                for jx in range(e.k):
                    iy = oy * e.stride - e.pad + jy
                    ix = ox * e.stride - e.pad + jx
                    ok = (iy >= 0) & (iy < src.H) & (ix >= 0) & (ix < src.W)
                    out[ok] = np.maximum(out[ok], act[iy[ok], ix[ok]])
            Yv = dst.get_Y()
            if self.crops:
                # a reset pixel may be pooled in a later frame than the one that reset it:
                # the reset itself zeroes the previous output (shift_camera)
                prev = Yv[oy, ox].astype(f32)
            else:
                prev = np.where(dst.N[oy, ox][:, None], f32(0), Yv[oy, ox].astype(f32))
            y = out - prev
            Yv[oy, ox] = out.astype(dst.dtype)
            dst.set_Y(Yv)
        elif e.k == 0:
            y = src.delta[oy, ox].astype(f32)
        else:
            f = 1 << e.up
            cy, cx = oy // f, ox // f                 # conv output coordinates
            acc = np.zeros((len(lst), dst.C), np.float64)
            w = e.w.astype(np.float64)
            for jy in range(e.k):
                for jx in range(e.k):
                    iy = cy * e.stride - e.pad + jy
                    ix = cx * e.stride - e.pad + jx
                    ok = (iy >= 0) & (iy < src.H) & (ix >= 0) & (ix < src.W)
                    ok[ok] = src.M[iy[ok], ix[ok]]
                    rows = np.zeros((len(lst), src.C), np.float64)
                    rows[ok] = src.delta[iy[ok], ix[ok]]
                    acc += rows @ w[jy * e.k + jx].T
            y = acc.astype(f32)
        if dst.tf:
            # Optimizing memory consumption: no truncated-values buffer.  The output of the (1x1) producer is
            # accumulated at once and the change of the activation is passed on wherever it is not zero.
            # A newly unveiled pixel starts from its bias and its previous activation counts as zero.  The
            # roundings are those the path through a truncated-values buffer would take with threshold 0:
            # the arriving value is rounded to the storage type (on top of the bias for a new pixel), then
            # added to the accumulated value.
            new = dst.N[oy, ox]
            beta = dst.beta.astype(dst.dtype).astype(f32)
            pend = (np.where(new[:, None], beta[None, :], f32(0)) + y).astype(dst.dtype).astype(f32)
            A = dst.get_A()
            a = np.where(new[:, None], f32(0), A[oy, ox].astype(f32))
            acc = a + pend
            if dst.spec.relu:
                out = np.maximum(acc, f32(0)) - np.maximum(a, f32(0))
            else:
                out = acc - a
            A[oy, ox] = acc.astype(dst.dtype)
            dst.set_A(A)
            mag = np.abs(out).max(axis=1) if len(lst) else np.zeros(0, f32)
            dst.M = np.zeros((dst.H, dst.W), bool)
            dst.M[oy, ox] = new | (mag > f32(0))
            dst.mag = np.zeros((dst.H, dst.W), f32)
            dst.mag[oy, ox] = mag
            dst.own = dst.M.copy()
            dst.touched = np.zeros((dst.H, dst.W), bool)
            dst.touched[oy, ox] = True
            dst.delta[:] = 0
            upd = dst.M[oy, ox]
            dst.delta[oy[upd], ox[upd]] = out.astype(dst.dtype)[upd]
            return lst
        Pw = dst.get_P()
        Pw[wy, wx] = (Pw[wy, wx].astype(f32) + y).astype(dst.dtype)
        dst.set_P(Pw)
        inview = (oy >= 0) & (oy < dst.H) & (ox >= 0) & (ox < dst.W)
        dst.U[oy[inview], ox[inview]] = True
        return lst

    # ------------------------------------------------------------ public API
    def layer_forward(self, i, frame=None, forced=None):
        """Truncate site i (delta, threshold, mask, compaction) and push its
        delta through all of its outgoing edges into the destinations' P."""
        self._truncate(i, frame, forced)
        lists = []
        for e in self.net.out_edges(i):
            lists.append(self._edge(e))
        return lists

    def readout(self, i):
        s = self.sites[i]
        out = s.view_of_window(s.get_P()).copy()
        if s.spec.relu:
            out = np.maximum(out, s.dtype(0))
        if self.crops:
            y0, y1, x0, x1 = s.crop
            out = out[y0:y1, x0:x1].copy()
        return out

    def frame(self, X, dty=0, dtx=0, forced=None, forced_all=None, crop=None):
        """One frame: shift, every non-terminal site in order, readout.
        `forced` is an input-site mask; `forced_all` maps site index -> mask;
        `crop` = (ty0, tx0, th, tw): the tiles of the view that X covers."""
        did_reset = self.shift_camera(dty, dtx)
        if crop is not None:
            self.set_crop(*crop)
        for i, s in enumerate(self.sites):
            if s.spec.kind == "output":
                continue
            fm = None
            if forced_all is not None:
                fm = forced_all.get(i)
            elif i == 0:
                fm = forced
            self.layer_forward(i, X if s.spec.kind == "input" else None, fm)
        outs = [self.readout(i) for i in self.net.terminal_sites()]
        return outs, did_reset

    # ------------------------------------------------- mask post-processing
    def input_mask(self, X, roi=None, theta=None, base=0.4, gain=0.6, pool=1, suppress=False, dilate=0):
        """Update mask of the input site for frame X with the optional
        post-processing steps, to be used as the forced mask of that frame
        (newly unveiled pixels are updated in any case).  X, roi and the
        result cover the current crop (the whole view without crops).
          1. magnitude e = max over channels of |X - A|   (Background: DeltaCNN)
          2. ROI-focused sensing: e is scaled by base + gain * roi, roi in
             [0, 1] from the previous result (Supplementary: 0.4 + 0.6 m)
          3. downscaling: e is averaged over pool x pool cells and the cells
             are compared with the threshold, strict >        (Optimizations)
          4. a cell that exceeds the threshold alone among the 3 x 3 cells
             around it is dropped: the 3 x 3 average pooling of the binary
             map stays at 1/9 there                            (Optimizations)
          5. every remaining cell covers its pixels, and the mask is dilated
             by `dilate` pixels in all directions (d = 10 spreads one pixel
             over 21 x 21)                       (Supplementary, first layer)
        All floating-point steps in float32, the cell sum row by row."""
        s = self.sites[0]
        f32 = np.float32
        theta = f32(s.spec.theta if theta is None else theta)
        y0, y1, x0, x1 = s.crop if self.crops else (0, s.H, 0, s.W)
        Hc, Wc = y1 - y0, x1 - x0
        assert X.shape == (Hc, Wc, s.C) and Hc % pool == 0 and Wc % pool == 0
        A = s.get_A()[y0:y1, x0:x1].astype(f32)
        e = np.abs(X.astype(f32) - A).max(axis=2)
        if roi is not None:
            assert roi.shape == (Hc, Wc)
            e = e * (f32(base) + f32(gain) * roi.astype(f32))
        acc = np.zeros((Hc // pool, Wc // pool), f32)
        for dy in range(pool):
            for dx in range(pool):
                acc = acc + e[dy::pool, dx::pool]
        hit = acc / f32(pool * pool) > theta
        if suppress:
            cnt = np.zeros(hit.shape, np.int32)
            padded = np.pad(hit, 1).astype(np.int32)
            for dy in range(3):
                for dx in range(3):
                    cnt += padded[dy:dy + hit.shape[0], dx:dx + hit.shape[1]]
            hit = hit & (cnt >= 2)
        m = np.repeat(np.repeat(hit, pool, axis=0), pool, axis=1)
        if dilate:
            d = int(dilate)
            padded = np.pad(m, d)
            out = np.zeros_like(m)
            for dy in range(2 * d + 1):
                for dx in range(2 * d + 1):
                    out |= padded[dy:dy + Hc, dx:dx + Wc]
            m = out
        return m.astype(np.uint8)
