"""Lock-step drivers that run the HIP path (through the C ABI) beside the oracle.

Three comparison protocols, because masks come from float compares and
convolution sums differ in their last bits:
  teacher_forced -- before every mdcnn_layer_forward the GPU site (and the P of
                    its destinations) is loaded with the oracle's state bit for
                    bit: masks, lists, compute lists and U flags must then be
                    bit-exact, A / P / delta within the fp tolerance.
  mask_forced    -- whole sequence on the GPU with the oracle's masks forced at
                    every site: all floating-point outputs within tolerance.
  free_running   -- mdcnn_frame end to end: reset decisions and the input-site
                    list bit-exact, inner masks nearly equal, outputs close.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle.mdcnn_oracle import OracleNet
from paper_2210_09887_amd import binding as B
from paper_2210_09887_amd.runtime import GpuNet

TOL = {"f32": 1e-4, "f16": 2e-2}


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def maxerr(a, b):
    return float(np.abs(a.astype(np.float64) - b.astype(np.float64)).max()) if a.size else 0.0


def oracle_flags(s):
    return (s.N.astype(np.uint8) * B.FLAG_N) | (s.U.astype(np.uint8) * B.FLAG_U)


def oracle_pending(s):
    return (s.get_ring("unseen").astype(np.uint8) * B.STATE_UNSEEN) | (s.get_ring("dirty").astype(np.uint8) * B.STATE_DIRTY)


def cut(net, a, crop):
    """The part of an input-site array [H, W, ...] that a frame covering `crop` = (ty0, tx0, th, tw) tiles holds."""
    T = net.total_stride
    ty0, tx0, th, tw = crop
    return np.ascontiguousarray(a[ty0 * T:(ty0 + th) * T, tx0 * T:(tx0 + tw) * T])


def load_site(g: GpuNet, o: OracleNet, i: int):
    s = o.sites[i]
    if s.tf:                                  # accumulated values and the flags of the shift only: there is no P
        g.write(i, B.MDCNN_VIEW_A, s.get_A())
        g.write(i, B.MDCNN_VIEW_FLAGS, oracle_flags(s))
        return
    if o.crops and s.spec.kind != "output":
        g.write(i, B.MDCNN_VIEW_PENDING, oracle_pending(s))
    if s.spec.kind != "output":
        g.write(i, B.MDCNN_VIEW_A, s.get_A())
        g.write(i, B.MDCNN_VIEW_FLAGS, oracle_flags(s))
    if s.spec.kind != "input":
        g.write(i, B.MDCNN_VIEW_P, s.get_P())
    if s.pooled:
        g.write(i, B.MDCNN_VIEW_POOL_PREV, s.get_Y())


def teacher_forced(net, frames, shifts, forced=None, origins=None, log=None, crops=None):
    """Returns the worst fp error seen; raises AssertionError on any integer mismatch.
    crops: per frame the tiles (ty0, tx0, th, tw) of the view that the frame covers; frames
    and forced masks are given over the whole view and cut here."""
    tol = TOL[net.dtype]
    g, o = GpuNet(net, origins, crops=crops is not None), OracleNet(net, origins, crops=crops is not None)
    worst = 0.0
    try:
        for t, X in enumerate(frames):
            dy, dx = (int(v) for v in shifts[t])
            r_g = g.shift_camera(dy, dx)
            r_o = o.shift_camera(dy, dx)
            assert r_g == r_o, f"frame {t}: reset decision differs"
            if crops is not None:
                g.set_crop(*crops[t])
                o.set_crop(*crops[t])
                X = cut(net, X, crops[t])
                for i, s in enumerate(o.sites):
                    if s.spec.kind != "output":
                        assert np.array_equal(g.read(i, B.MDCNN_VIEW_PENDING), oracle_pending(s)), f"frame {t} site {i}: crop state after the shift"
                    if s.pooled:
                        assert np.array_equal(g.read(i, B.MDCNN_VIEW_POOL_PREV), s.get_Y()), f"frame {t} site {i}: previous pooling output after the shift"
            if t == 0 or r_o:
                # state after a (re)initialisation must already agree exactly
                for i, s in enumerate(o.sites):
                    if s.spec.kind != "input" and not s.tf:
                        assert np.array_equal(g.read(i, B.MDCNN_VIEW_P), s.get_P()), f"frame {t} site {i}: P after reset"
                    if s.spec.kind != "output":
                        assert np.array_equal(g.read(i, B.MDCNN_VIEW_A), s.get_A()), f"frame {t} site {i}: A after reset"
            for i, s in enumerate(o.sites):
                if s.spec.kind == "output":
                    continue
                if not s.tf:
                    # flags set by the GPU's own shift / producers must match the oracle's N, U
                    fl = g.read(i, B.MDCNN_VIEW_FLAGS)
                    assert np.array_equal(fl & (B.FLAG_N | B.FLAG_U), oracle_flags(s)), f"frame {t} site {i}: N/U flags"
                edges = net.out_edges(i)
                if not s.tf:                  # a truncation-free site keeps the mask and the deltas its producer's call made
                    load_site(g, o, i)
                for e in edges:
                    load_site(g, o, e.dst)
                fm = forced[t] if (forced is not None and i == 0) else None
                if fm is not None and crops is not None:
                    fm = cut(net, fm, crops[t])
                Xd = dev(X) if i == 0 else None
                fd = dev(fm) if fm is not None else None
                g.layer_forward(i, Xd, fd)
                lists = o.layer_forward(i, X if i == 0 else None, fm)
                torch.cuda.synchronize()
                where = f"frame {t} site {i} ({s.spec.name})"
                fl = g.read(i, B.MDCNN_VIEW_FLAGS)
                assert np.array_equal((fl & B.FLAG_M) != 0, s.M), where + ": update mask"
                if crops is not None:
                    assert np.array_equal(g.read(i, B.MDCNN_VIEW_PENDING), oracle_pending(s)), where + ": crop state"
                assert np.array_equal(g.read(i, B.MDCNN_VIEW_LIST), s.L), where + ": list L"
                st = g.read(i, B.MDCNN_VIEW_STATS)
                assert st[0] == len(s.L) and st[1] == s.n_candidates, where + ": counters"
                errs = [maxerr(g.read(i, B.MDCNN_VIEW_A), s.get_A()), maxerr(g.read(i, B.MDCNN_VIEW_DELTA), s.delta)]
                if s.spec.kind != "input" and not s.tf:
                    errs.append(maxerr(g.read(i, B.MDCNN_VIEW_P), s.get_P()))
                for e, lst in zip(edges, lists):
                    d = o.sites[e.dst]
                    w2 = where + f" -> site {e.dst}"
                    if d.tf:
                        # the call made the destination's mask and deltas: compared here, bit for bit / within tolerance
                        fl = g.read(e.dst, B.MDCNN_VIEW_FLAGS)
                        assert np.array_equal((fl & B.FLAG_M) != 0, d.M), w2 + ": update mask of the truncation-free site"
                        assert np.array_equal((fl & 8) != 0, d.touched), w2 + ": touched pixels of the truncation-free site"
                        errs += [maxerr(g.read(e.dst, B.MDCNN_VIEW_A), d.get_A()), maxerr(g.read(e.dst, B.MDCNN_VIEW_DELTA), d.delta)]
                        continue
                    errs.append(maxerr(g.read(e.dst, B.MDCNN_VIEW_P), d.get_P()))
                    if getattr(e, "pool", False):   # a maximum of stored values: exact
                        assert np.array_equal(g.read(e.dst, B.MDCNN_VIEW_POOL_PREV), d.get_Y()), w2 + ": previous pooling output"
                    if d.spec.kind != "output":
                        fl = g.read(e.dst, B.MDCNN_VIEW_FLAGS)
                        assert np.array_equal(fl & (B.FLAG_N | B.FLAG_U), oracle_flags(d)), w2 + ": U flags"
                # compute list: the last non-upsampling edge into each destination
                last = {}
                for e, lst in zip(edges, lists):
                    if not e.up:
                        last[e.dst] = lst
                for dst, lst in last.items():
                    assert np.array_equal(g.read(dst, B.MDCNN_VIEW_CLIST), lst), where + f": compute list into {dst}"
                worst = max(worst, max(errs))
                assert max(errs) < tol, where + f": fp error {max(errs):.3e} (A, delta, P, P_dst...) = {errs}"
            for i in net.terminal_sites():
                worst = max(worst, maxerr(g.read(i, B.MDCNN_VIEW_CROP_OUT if crops is not None else B.MDCNN_VIEW_OUT), o.readout(i)))
            if log:
                log(f"  teacher-forced frame {t}: reset={r_o} worst={worst:.2e}")
    finally:
        g.close()
    assert worst < tol
    return worst


def oracle_run(net, frames, shifts, forced=None, origins=None, crops=None):
    """Oracle alone; returns per-frame outputs, masks of every non-terminal site, resets."""
    o = OracleNet(net, origins, crops=crops is not None)
    outs, masks, resets = [], [], []
    for t, X in enumerate(frames):
        dy, dx = (int(v) for v in shifts[t])
        if crops is not None:
            fm = None if forced is None else cut(net, forced[t], crops[t])
            out, r = o.frame(cut(net, X, crops[t]), dy, dx, fm, crop=crops[t])
        else:
            out, r = o.frame(X, dy, dx, None if forced is None else forced[t])
        outs.append(out)
        resets.append(r)
        masks.append({i: s.M.copy() for i, s in enumerate(o.sites) if s.spec.kind != "output"})
    return o, outs, masks, resets


def mask_forced(net, frames, shifts, forced=None, log=None):
    tol = TOL[net.dtype]
    o, outs, masks, resets = oracle_run(net, frames, shifts, forced)
    g = GpuNet(net)
    worst = 0.0
    try:
        for t, X in enumerate(frames):
            dy, dx = (int(v) for v in shifts[t])
            assert g.shift_camera(dy, dx) == resets[t]
            keep = []
            for i, s in enumerate(net.sites):
                if s.kind == "output":
                    continue
                fm = None if getattr(s, "trunc_free", False) else dev(masks[t][i].astype(np.uint8))   # (such a mask cannot be forced)
                Xd = dev(X) if i == 0 else None
                keep += [fm, Xd]
                g.layer_forward(i, Xd, fm)
            torch.cuda.synchronize()
            for k, i in enumerate(net.terminal_sites()):
                e = maxerr(g.read(i, B.MDCNN_VIEW_OUT), outs[t][k])
                worst = max(worst, e)
                assert e < tol, f"frame {t}: output error {e:.3e}"
            for i, s in enumerate(net.sites):
                if s.kind != "output":
                    fl = g.read(i, B.MDCNN_VIEW_FLAGS)
                    assert np.array_equal((fl & B.FLAG_M) != 0, masks[t][i]), f"frame {t} site {i}: forced mask not honoured"
            if log:
                log(f"  mask-forced frame {t}: reset={resets[t]} worst={worst:.2e}")
        for i, s in enumerate(o.sites):
            if s.spec.kind != "output":
                worst = max(worst, maxerr(g.read(i, B.MDCNN_VIEW_A), s.get_A()))
            if s.spec.kind != "input" and not s.tf:
                worst = max(worst, maxerr(g.read(i, B.MDCNN_VIEW_P), s.get_P()))
    finally:
        g.close()
    assert worst < tol, f"final state error {worst:.3e}"
    return worst


def free_running(net, frames, shifts, forced=None, origins=None, log=None, crops=None):
    """mdcnn_frame (with crops: mdcnn_frame_crop) end to end.  Returns dict(out_err, mask_mismatch, resets, outputs)."""
    o, outs, masks, resets = oracle_run(net, frames, shifts, forced, origins, crops)
    g = GpuNet(net, origins, crops=crops is not None)
    out_err, mism, total = 0.0, 0, 0
    got_all = []
    try:
        for t, X in enumerate(frames):
            dy, dx = (int(v) for v in shifts[t])
            if crops is not None:
                fd = dev(cut(net, forced[t], crops[t])) if forced is not None else None
                parts, r = g.frame_crop(dev(cut(net, X, crops[t])), dy, dx, crops[t], fd)
            else:
                fd = dev(forced[t]) if forced is not None else None
                out, r = g.frame(dev(X), dy, dx, fd)
                parts = g.split_outputs(out)
            torch.cuda.synchronize()
            assert r == resets[t], f"frame {t}: reset decision differs"
            got = [x.cpu().numpy() for x in parts]
            got_all.append(got)
            for a, b in zip(got, outs[t]):
                out_err = max(out_err, maxerr(a, b))
            l0 = g.read(0, B.MDCNN_VIEW_LIST)
            assert np.array_equal(l0, np.flatnonzero(masks[t][0].ravel())), f"frame {t}: input-site list differs"
            for i in masks[t]:
                m = (g.read(i, B.MDCNN_VIEW_FLAGS) & B.FLAG_M) != 0
                mism += int((m != masks[t][i]).sum())
                total += m.size
            if log:
                log(f"  free-running frame {t}: reset={r} out_err={out_err:.2e} mask mismatches={mism}/{total}")
    finally:
        g.close()
    return dict(out_err=out_err, mask_mismatch=mism / max(total, 1), resets=resets, outputs=got_all, oracle_outputs=outs)


class Follower:
    """An oracle that follows a free-running GPU stream (protocol R with the guard band).  After every
    frame the GPU's update masks of all sites are forced on the oracle, whose state therefore stays
    within the fp tolerance of the GPU's, frame after frame.  check() asserts, per frame:
      * reset decisions, and the input-site mask and list, bit for bit;
      * every decision of the GPU against the decision this oracle takes by itself in that state
        (OracleSite.own): where they differ, the magnitude the oracle compares with theta must lie
        within 4 x tolerance of theta -- a wrong mask far from the threshold fails;
      * the outputs at the tight tolerance (the masks agree by construction)."""

    def __init__(self, net, origins=None, tol=None):
        """tol: the fp tolerance (default: the absolute one of the storage type)."""
        self.net, self.o = net, OracleNet(net, origins)
        self.tol = TOL[net.dtype] if tol is None else tol
        self.band = 4 * self.tol
        self.inner = [i for i, s in enumerate(net.sites) if s.kind != "output"]
        self.out_err, self.flips, self.decisions, self.worst = 0.0, 0, 0, 0.0

    def check(self, t, X, dy, dx, fm, got, reset, masks, l0, tag=""):
        o = self.o
        want, r_o = o.frame(X, dy, dx, forced_all={i: masks[i] for i in self.inner if not o.sites[i].tf})
        assert reset == r_o, f"{tag}frame {t}: reset decision differs"
        for i in self.inner:
            s = o.sites[i]
            if not s.tf:      # (the mask of a truncation-free site cannot be forced: it is compared like any decision)
                assert np.array_equal(s.M, masks[i]), f"{tag}frame {t} site {i}: a pixel that was no candidate was updated"
            if i == 0 and fm is not None:
                continue                          # the workload forces this mask: no threshold decision to compare
            diff = s.own != masks[i]
            self.decisions += masks[i].size
            if i == 0:
                assert not diff.any(), f"{tag}frame {t}: input-site mask differs"
                assert np.array_equal(l0, np.flatnonzero(s.own.ravel())), f"{tag}frame {t}: input-site list differs"
            if diff.any():
                margin = np.abs(s.mag[diff] - np.float32(s.spec.theta))
                self.flips += int(diff.sum())
                self.worst = max(self.worst, float(margin.max()))
                assert margin.max() < self.band, (
                    f"{tag}frame {t} site {i} ({s.spec.name}): {int((margin >= self.band).sum())} decisions differ from the oracle's "
                    f"outside the guard band (|magnitude - theta| up to {margin.max():.3e}, band {self.band:.1e})")
        for a, b in zip(got, want):
            e = maxerr(a, b)
            self.out_err = max(self.out_err, e)
            assert e < self.tol, f"{tag}frame {t}: output error {e:.3e} with the oracle following the GPU's masks"
        return r_o

    def result(self):
        return dict(out_err=self.out_err, flips=self.flips, decisions=self.decisions, worst_margin=self.worst)


def gpu_masks(g, inner):
    return {i: (g.read(i, B.MDCNN_VIEW_FLAGS) & B.FLAG_M) != 0 for i in inner}


def followed(net, frames, shifts, forced=None, origins=None, log=None, tol=None):
    """mdcnn_frame end to end with a Follower.  Returns dict(out_err, flips, decisions, worst_margin)."""
    f = Follower(net, origins, tol)
    g = GpuNet(net, origins)
    try:
        for t, X in enumerate(frames):
            dy, dx = (int(v) for v in shifts[t])
            fm = None if forced is None else forced[t]
            out, r = g.frame(dev(X), dy, dx, None if fm is None else dev(fm))
            torch.cuda.synchronize()
            got = [x.cpu().numpy() for x in g.split_outputs(out)]
            f.check(t, X, dy, dx, fm, got, r, gpu_masks(g, f.inner), g.read(0, B.MDCNN_VIEW_LIST))
            if log:
                log(f"  followed frame {t}: reset={r} out_err={f.out_err:.2e} decisions off the oracle's: {f.flips}/{f.decisions}, worst margin {f.worst:.2e}")
    finally:
        g.close()
    return f.result()


def followed_batch(net, seqs, log=None):
    """mdcnn_frame_batch: stream b runs seqs[b] = (frames, shifts, forced or None); every stream is checked
    against a Follower of its own.  All sequences have the same length."""
    from paper_2210_09887_amd.runtime import GpuBatch
    n = len(seqs)
    fs = [Follower(net) for _ in range(n)]
    gb = GpuBatch(net, n)
    try:
        for t in range(len(seqs[0][0])):
            Xs = [sq[0][t] for sq in seqs]
            dys = [int(sq[1][t][0]) for sq in seqs]
            dxs = [int(sq[1][t][1]) for sq in seqs]
            fms = [None if sq[2] is None else sq[2][t] for sq in seqs]
            keep = [None if m is None else dev(m) for m in fms]
            outs, rs = gb.frame([dev(X) for X in Xs], dys, dxs, keep if any(m is not None for m in fms) else None)
            torch.cuda.synchronize()
            for b, g in enumerate(gb.streams):
                got = [x.cpu().numpy() for x in g.split_outputs(outs[b])]
                fs[b].check(t, Xs[b], dys[b], dxs[b], fms[b], got, bool(rs[b]), gpu_masks(g, fs[b].inner), g.read(0, B.MDCNN_VIEW_LIST),
                            tag=f"stream {b} ")
            if log:
                log(f"  batch step {t}: resets={[bool(r) for r in rs]} out_err={[f'{f.out_err:.1e}' for f in fs]} flips={[f.flips for f in fs]}")
    finally:
        gb.close()
    return [f.result() for f in fs]
