"""Marshalling helper: instantiate a network description on the GPU.

Allocates device memory through PyTorch (site buffers, weights, biases),
creates the library handles and forwards calls to the C ABI.  No step of the
method is computed here.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B

_KIND = {"input": B.MDCNN_SITE_INPUT, "preact": B.MDCNN_SITE_PREACT, "output": B.MDCNN_SITE_OUTPUT}


class GpuNet:
    """`spec` is any object with the fields of inputs.nets.NetSpec."""

    def __init__(self, spec, origins=None, device="cuda:0", share_weights=None, crops=False):
        """share_weights: another GpuNet of the same spec whose weight tensors are reused
        (streams of one batch share the model).  crops: frames may cover a part of the
        view only (set_crop / frame_crop)."""
        if not torch.cuda.is_available():
            raise RuntimeError("mdcnn needs a GPU: there is no CPU path")
        B.lib()
        self.spec = spec
        self.dev = torch.device(device)
        self.tdtype = torch.float16 if spec.dtype == "f16" else torch.float32
        self.ndtype = np.float16 if spec.dtype == "f16" else np.float32
        self.esize = 2 if spec.dtype == "f16" else 4
        dt = B.MDCNN_F16 if spec.dtype == "f16" else B.MDCNN_F32
        n = len(spec.sites)
        self.shape = [(spec.H // s.stride, spec.W // s.stride, s.C) for s in spec.sites]
        border = [[0, 0, 0, 0] for _ in range(n)]
        bias = [None] * n
        self.weights, self.edges, self.esrc, self.edst = [], [], [], []
        pooled = set()
        for e in spec.edges:
            Hs, Ws, _ = self.shape[e.src]
            cd = B.mdcnn_conv_desc(e.k, e.stride, e.pad, spec.sites[e.src].C, spec.sites[e.dst].C, e.up, None, None,
                                   1 if getattr(e, "pool", False) else 0)
            if getattr(e, "pool", False):
                pooled.add(e.dst)                    # max pooling: no weights, no border
            elif e.k:
                oh = (Hs + 2 * e.pad - e.k) // e.stride + 1
                ow = (Ws + 2 * e.pad - e.k) // e.stride + 1
                by = B.mdcnn_conv_border(e.k, e.stride, e.pad, Hs, oh)
                bx = B.mdcnn_conv_border(e.k, e.stride, e.pad, Ws, ow)
                border[e.dst] = [max(a, b) for a, b in zip(border[e.dst], [by[0], by[1], bx[0], bx[1]])]
                if share_weights is not None:
                    src = share_weights.edges[len(self.edges)]
                    cd.w_dev, cd.w_packed_dev = src.w_dev, src.w_packed_dev
                else:
                    w = torch.from_numpy(np.ascontiguousarray(e.w)).to(self.dev)
                    assert w.dtype == self.tdtype
                    self.weights.append(w)
                    cd.w_dev = w.data_ptr()
                    if dt == B.MDCNN_F16 and e.k == 3 and e.stride == 1 and not e.up and cd.Cin % 16 == 0 and cd.Cout % 32 == 0:
                        wp = torch.empty_like(w)             # second copy in matrix-core operand order
                        B.mdcnn_pack_weights(cd, dt, wp.data_ptr(), wp.numel() * 2)
                        self.weights.append(wp)
                        cd.w_packed_dev = wp.data_ptr()
                if e.b is not None:
                    bias[e.dst] = e.b.astype(np.float32) if bias[e.dst] is None else bias[e.dst] + e.b.astype(np.float32)
            self.edges.append(cd)
            self.esrc.append(e.src)
            self.edst.append(e.dst)
        self.bias = [None if b is None else torch.from_numpy(b).to(self.dev) for b in bias]
        self.mem, self.bufs, self.win = [], [], []
        for i, s in enumerate(spec.sites):
            H, W, Cc = self.shape[i]
            d = B.mdcnn_buffer_desc()
            d.H, d.W, d.C, d.dtype, d.kind = H, W, Cc, dt, _KIND[s.kind]
            for j in range(4):
                d.border[j] = border[i][j]
            d.tile = spec.total_stride // s.stride
            d.relu = int(s.relu)
            d.theta = float(s.theta)
            d.bias_dev = None if self.bias[i] is None else self.bias[i].data_ptr()
            d.origin_y, d.origin_x = (0, 0) if origins is None else origins[i]
            d.pool_prev = int(i in pooled)
            d.crops = int(bool(crops))
            d.truncation_free = int(bool(getattr(s, "trunc_free", False)))
            nbytes = B.mdcnn_buffer_bytes(d)
            mem = torch.empty(nbytes, dtype=torch.uint8, device=self.dev)
            self.mem.append(mem)
            self.bufs.append(B.mdcnn_create_buffer(d, mem.data_ptr(), nbytes))
            self.win.append((H + border[i][0] + border[i][1], W + border[i][2] + border[i][3]))
        self.border = border
        self.net = B.mdcnn_net_create(self.bufs, self.esrc, self.edst, self.edges)
        self.terminals = [i for i, s in enumerate(spec.sites) if s.kind == "output"]
        self.out_elems = sum(int(np.prod(self.shape[i])) for i in self.terminals)
        self.out = torch.empty(self.out_elems, dtype=self.tdtype, device=self.dev)
        self.tile = [spec.total_stride // s.stride for s in spec.sites]
        self.crop = None                     # (ty0, tx0, th, tw) once set

    def close(self):
        if self.net:
            B.mdcnn_net_destroy(self.net)
            self.net = None
        for b in self.bufs:
            B.mdcnn_destroy_buffer(b)
        self.bufs = []

    def keep_alive(self, other):
        self._shared = other                 # the owner of shared weights must outlive this net

    @staticmethod
    def _stream():
        return torch.cuda.current_stream().cuda_stream

    # -- the four calls of the boundary -------------------------------------------------
    def shift_camera(self, dty, dtx) -> bool:
        return B.mdcnn_shift_camera(self.bufs, dty, dtx, self._stream())

    def set_crop(self, ty0, tx0, th, tw):
        B.mdcnn_set_crop(self.bufs, ty0, tx0, th, tw)
        self.crop = (int(ty0), int(tx0), int(th), int(tw))

    def crop_shape(self, i):
        """Extent of the crop at site i."""
        if self.crop is None:
            return self.shape[i]
        return (self.crop[2] * self.tile[i], self.crop[3] * self.tile[i], self.shape[i][2])

    def frame_crop(self, X, dty, dtx, crop, forced=None):
        """X: device tensor covering the crop at the input site.  Returns (list of output tensors in crop
        order, did_reset)."""
        th, tw = int(crop[2]), int(crop[3])
        n = sum(th * self.tile[i] * tw * self.tile[i] * self.shape[i][2] for i in self.terminals)
        out = self.out[:n]
        r = B.mdcnn_frame_crop(self.net, X.data_ptr(), None if forced is None else forced.data_ptr(), dty, dtx, crop,
                               out.data_ptr(), n * self.esize, self._stream())
        self.crop = tuple(int(v) for v in crop)
        res, o = [], 0
        for i in self.terminals:
            shp = self.crop_shape(i)
            m = int(np.prod(shp))
            res.append(out[o:o + m].reshape(shp))
            o += m
        return res, r

    def frames_crop(self, Xs, dty, dtx, crops, forced=None, outs=None, depth=0):
        """Consecutive cropped frames of the video in one call.  Returns (per frame the list of output tensors in
        crop order, reset flags)."""
        ns = [sum(int(c[2]) * self.tile[i] * int(c[3]) * self.tile[i] * self.shape[i][2] for i in self.terminals) for c in crops]
        if outs is None:
            outs = [torch.empty_like(self.out) for _ in Xs]
        r = B.mdcnn_frames_crop(self.net, [x.data_ptr() for x in Xs],
                                None if forced is None else [None if f is None else f.data_ptr() for f in forced],
                                dty, dtx, crops, [o.data_ptr() for o in outs], [n * self.esize for n in ns], depth, self._stream())
        self.crop = tuple(int(v) for v in crops[-1])
        res = []
        for c, out in zip(crops, outs):
            per, o = [], 0
            for i in self.terminals:
                shp = (int(c[2]) * self.tile[i], int(c[3]) * self.tile[i], self.shape[i][2])
                m = int(np.prod(shp))
                per.append(out[o:o + m].reshape(shp))
                o += m
            res.append(per)
        return res, r

    def input_mask(self, X, roi=None, theta=None, base=0.4, gain=0.6, pool=1, suppress=False, dilate=0):
        """Post-processed update mask of the input site for frame X (device tensor over the crop): a uint8
        device tensor to pass as the forced mask of that frame."""
        prm = B.mdcnn_mask_params(float(self.spec.sites[0].theta if theta is None else theta), float(base), float(gain),
                                  int(pool), int(bool(suppress)), int(dilate))
        mask = torch.empty(X.shape[:2], dtype=torch.uint8, device=self.dev)
        B.mdcnn_input_mask(self.bufs[0], X.data_ptr(), None if roi is None else roi.data_ptr(), prm, mask.data_ptr(),
                           mask.numel(), self._stream())
        return mask

    def frames_masked(self, Xs, dty, dtx, rois=None, outs=None, masks=None, depth=0, theta=None, base=0.4, gain=0.6, pool=1,
                      suppress=False, dilate=0):
        """Consecutive frames with the input masks made by mdcnn_input_mask inside the call.  Returns (outputs, masks,
        reset flags)."""
        prm = B.mdcnn_mask_params(float(self.spec.sites[0].theta if theta is None else theta), float(base), float(gain),
                                  int(pool), int(bool(suppress)), int(dilate))
        if outs is None:
            outs = [torch.empty_like(self.out) for _ in Xs]
        if masks is None:
            masks = [torch.empty(x.shape[:2], dtype=torch.uint8, device=self.dev) for x in Xs]
        r = B.mdcnn_frames_masked(self.net, [x.data_ptr() for x in Xs],
                                  None if rois is None else [None if q is None else q.data_ptr() for q in rois], prm,
                                  [m.data_ptr() for m in masks], masks[0].numel(), dty, dtx, [o.data_ptr() for o in outs],
                                  self.out.numel() * self.esize, depth, self._stream())
        return outs, masks, r

    def layer_forward(self, i, frame=None, forced=None, noalloc=False):
        idx = [j for j, s in enumerate(self.esrc) if s == i]
        call = B.mdcnn_layer_forward_noalloc if noalloc else B.mdcnn_layer_forward
        call(self.bufs[i], None if frame is None else frame.data_ptr(),
                              None if forced is None else forced.data_ptr(),
                              [self.edges[j] for j in idx], [self.bufs[self.edst[j]] for j in idx], self._stream())

    def frame(self, X, dty=0, dtx=0, forced=None, out=None):
        """X: device tensor [H, W, C] storage dtype.  Returns (flat output tensor, did_reset)."""
        out = self.out if out is None else out
        r = B.mdcnn_frame(self.net, X.data_ptr(), None if forced is None else forced.data_ptr(), dty, dtx,
                          out.data_ptr(), out.numel() * self.esize, self._stream())
        return out, r

    def frames(self, Xs, dty, dtx, forced=None, outs=None, depth=0):
        """Xs: consecutive frames of the video (device tensors [H, W, C]).  Returns (list of flat outputs, reset flags)."""
        if outs is None:
            outs = [torch.empty_like(self.out) for _ in Xs]
        r = B.mdcnn_frames(self.net, [x.data_ptr() for x in Xs],
                           None if forced is None else [None if f is None else f.data_ptr() for f in forced],
                           dty, dtx, [o.data_ptr() for o in outs], self.out.numel() * self.esize, depth, self._stream())
        return outs, r

    def split_outputs(self, out):
        res, o = [], 0
        for i in self.terminals:
            n = int(np.prod(self.shape[i]))
            res.append(out[o:o + n].reshape(self.shape[i]))
            o += n
        return res

    # -- state access ---------------------------------------------------------------------
    def read(self, i, what) -> np.ndarray:
        H, W, Cc = self.shape[i]
        Hp, Wp = self.win[i]
        if what in (B.MDCNN_VIEW_A, B.MDCNN_VIEW_DELTA, B.MDCNN_VIEW_OUT, B.MDCNN_VIEW_POOL_PREV):
            t = torch.empty((H, W, Cc), dtype=self.tdtype, device=self.dev)
        elif what == B.MDCNN_VIEW_P:
            t = torch.empty((Hp, Wp, Cc), dtype=self.tdtype, device=self.dev)
        elif what == B.MDCNN_VIEW_CROP_OUT:
            t = torch.empty(self.crop_shape(i), dtype=self.tdtype, device=self.dev)
        elif what in (B.MDCNN_VIEW_FLAGS, B.MDCNN_VIEW_PENDING):
            t = torch.empty((H, W), dtype=torch.uint8, device=self.dev)
        elif what == B.MDCNN_VIEW_LIST:
            t = torch.empty(H * W + 1, dtype=torch.int32, device=self.dev)
        elif what == B.MDCNN_VIEW_CLIST:
            t = torch.empty(Hp * Wp + 1, dtype=torch.int32, device=self.dev)
        else:
            t = torch.empty(18, dtype=torch.int32, device=self.dev)
        B.mdcnn_read_view(self.bufs[i], what, t.data_ptr(), t.numel() * t.element_size(), self._stream())
        a = t.cpu().numpy()
        if what in (B.MDCNN_VIEW_LIST, B.MDCNN_VIEW_CLIST):
            return a[1:1 + a[0]].copy()
        return a

    def totals(self):
        """Sums since creation over all sites: dict of updated / candidates / macs_mfma /
        compute / macs_plain, plus per-site arrays of the same."""
        keys = ["updated", "candidates", "macs_mfma", "compute", "macs_plain"]
        per_site = np.stack([self.read(i, B.MDCNN_VIEW_STATS)[8:18].view(np.uint64) for i in range(len(self.bufs))])
        out = {k: int(per_site[:, j].sum()) for j, k in enumerate(keys)}
        out["per_site"] = {k: per_site[:, j].astype(np.int64) for j, k in enumerate(keys)}
        return out

    def write(self, i, what, arr: np.ndarray):
        t = torch.from_numpy(np.ascontiguousarray(arr)).to(self.dev)
        B.mdcnn_write_view(self.bufs[i], what, t.data_ptr(), t.numel() * t.element_size(), self._stream())
        torch.cuda.current_stream().synchronize()      # t must outlive the copy


class GpuBatch:
    """n independent streams of one network behind mdcnn_frame_batch: own buffers and
    camera paths, shared weights.  Marshalling only."""

    def __init__(self, spec, n_streams, device="cuda:0", crops=False):
        first = GpuNet(spec, device=device, crops=crops)
        self.streams = [first]
        for _ in range(n_streams - 1):
            g = GpuNet(spec, device=device, share_weights=first, crops=crops)
            g.keep_alive(first)
            self.streams.append(g)

    def frame(self, frames, dty, dtx, forced=None):
        """frames: one device tensor [H, W, C] per stream.  Returns (list of flat outputs, list of reset flags)."""
        g0 = self.streams[0]
        outs = [g.out for g in self.streams]
        r = B.mdcnn_frame_batch([g.net for g in self.streams], [x.data_ptr() for x in frames],
                                None if forced is None else [None if f is None else f.data_ptr() for f in forced],
                                dty, dtx, [o.data_ptr() for o in outs], g0.out.numel() * g0.esize, g0._stream())
        return outs, r

    def frame_crop(self, frames, dty, dtx, crops, forced=None):
        """frames[b]: device tensor covering crops[b] = (ty0, tx0, th, tw) at the input site of stream b.  Returns (per
        stream the list of output tensors in crop order, list of reset flags)."""
        ns = [sum(int(c[2]) * g.tile[i] * int(c[3]) * g.tile[i] * g.shape[i][2] for i in g.terminals) for g, c in zip(self.streams, crops)]
        outs = [g.out[:n] for g, n in zip(self.streams, ns)]
        g0 = self.streams[0]
        r = B.mdcnn_frame_batch_crop([g.net for g in self.streams], [x.data_ptr() for x in frames],
                                     None if forced is None else [None if f is None else f.data_ptr() for f in forced],
                                     dty, dtx, crops, [o.data_ptr() for o in outs], [n * g0.esize for n in ns], g0._stream())
        res = []
        for g, c, out in zip(self.streams, crops, outs):
            g.crop = tuple(int(v) for v in c)
            per, o = [], 0
            for i in g.terminals:
                shp = g.crop_shape(i)
                m = int(np.prod(shp))
                per.append(out[o:o + m].reshape(shp))
                o += m
            res.append(per)
        return res, r

    def frames(self, frames, dty, dtx, forced=None, outs=None, depth=0):
        """frames[f][b]: frame f of video b (device tensors), dty / dtx / forced alike.  Returns (outs[f][b], resets[f][b])."""
        g0 = self.streams[0]
        if outs is None:
            outs = [[torch.empty_like(g0.out) for _ in row] for row in frames]
        r = B.mdcnn_frames_batch([g.net for g in self.streams], [[x.data_ptr() for x in row] for row in frames],
                                 None if forced is None else [[None if f is None else f.data_ptr() for f in row] for row in forced],
                                 dty, dtx, [[o.data_ptr() for o in row] for row in outs], g0.out.numel() * g0.esize, depth, g0._stream())
        return outs, r

    def close(self):
        for g in reversed(self.streams):
            g.close()
