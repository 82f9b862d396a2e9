"""GPU parity of the truncation-free activation sites (Supplementary, Optimizing memory consumption): sites after
a 1x1 convolution that keep only their accumulated values.  The producer's launch makes their update mask and
deltas; they get no delta launch and no pending ring."""
import copy

import numpy as np
import pytest
import torch

from inputs import build_net, build_sequence
from inputs.nets import truncation_free
from test_oracle_pins import rand_frames
from test_oracle_tf_pins import moving_path, pairs_net

pytestmark = pytest.mark.gpu


def log(msg):
    print(msg, flush=True)


def cases():
    return {
        "pairs_f32": truncation_free(pairs_net("f32", H=32, W=32)),
        "pairs_f32_strided_id": truncation_free(pairs_net("f32", H=32, W=32, relu=False, stride1=2, seed=2)),
        "pairs_f16_small": truncation_free(pairs_net("f16", H=32, W=32, seed=1)),                       # plain kernel (6 / 8 channels)
        "pairs_f16_mfma": truncation_free(pairs_net("f16", H=48, W=40, C=(3, 16, 32, 16, 64, 8), seed=4)),  # matrix cores
        "pairs_f16_mfma_s2": truncation_free(pairs_net("f16", H=64, W=48, C=(3, 32, 96, 16, 32, 8), stride1=2, seed=5)),
        "bottleneck": truncation_free(build_net(5, H=40, W=40, C=128, Cm=32)),
    }


def inputs_of(name, net):
    if name == "bottleneck":
        seq = build_sequence(5, n_frames=12, H=40, W=40, C=128, density=0.2, shift_every=4, shift=8)
        return seq.frames, seq.shifts, seq.forced
    n = 9
    return rand_frames(net, n, 6, walk=0.1), moving_path(n), None


@pytest.mark.parametrize("name", list(cases()))
def test_truncation_free_teacher_forced(name):
    import gpu_harness as H
    net = cases()[name]
    assert any(s.trunc_free for s in net.sites)
    frames, shifts, forced = inputs_of(name, net)
    worst = H.teacher_forced(net, frames, shifts, forced, log=log)
    log(f"[truncation-free, teacher-forced] {name}: worst fp error {worst:.2e}")


@pytest.mark.parametrize("name", list(cases()))
def test_truncation_free_mask_forced_and_followed(name):
    import gpu_harness as H
    net = cases()[name]
    frames, shifts, forced = inputs_of(name, net)
    worst = H.mask_forced(net, frames, shifts, forced)
    r = H.followed(net, frames, shifts, forced, log=log)
    log(f"[truncation-free] {name}: mask-forced worst {worst:.2e}; followed {r}")
    assert r["flips"] <= 0.02 * r["decisions"] and r["worst_margin"] < H.TOL[net.dtype] / 4


def test_truncation_free_state_is_half_and_launches_drop():
    """The site's memory shrinks by exactly its pending ring, and the frame has one launch less per such site."""
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    base = build_net(5, H=40, W=40, C=128, Cm=32)
    tf = truncation_free(copy.deepcopy(base))
    g0, g1 = GpuNet(base), GpuNet(tf)
    try:
        for i, s in enumerate(tf.sites):
            a, b = g0.mem[i].numel(), g1.mem[i].numel()
            if s.trunc_free:
                H_, W_, C_ = g0.shape[i]
                ring = (H_ * W_ * C_ * 2 + 255) // 256 * 256
                assert a - b == ring, (i, a, b, ring)
            else:
                assert a == b
        n0, n1 = len(B.mdcnn_frame_plan(g0.net, 1)[0]), len(B.mdcnn_frame_plan(g1.net, 1)[0])
        assert n0 - n1 == sum(s.trunc_free for s in tf.sites) == 1
    finally:
        g0.close()
        g1.close()


def test_truncation_free_argument_checks():
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    net = truncation_free(pairs_net("f32", H=32, W=32))
    g = GpuNet(net)
    try:
        d = B.mdcnn_buffer_desc()
        d.H, d.W, d.C, d.dtype, d.kind, d.tile, d.truncation_free = 8, 8, 4, B.MDCNN_F32, B.MDCNN_SITE_PREACT, 1, 1
        assert B.mdcnn_buffer_bytes(d) > 0
        d.border[0] = 1
        with pytest.raises(B.MdcnnError):                  # a border means a producer that dilates
            B.mdcnn_buffer_bytes(d)
        d.border[0] = 0
        d.kind = B.MDCNN_SITE_OUTPUT
        with pytest.raises(B.MdcnnError):
            B.mdcnn_buffer_bytes(d)
        g.shift_camera(0, 0)
        i = next(i for i, s in enumerate(net.sites) if s.trunc_free)
        mask = torch.ones(g.shape[i][:2], dtype=torch.uint8, device="cuda")
        with pytest.raises(B.MdcnnError):                  # its mask cannot be forced
            g.layer_forward(i, None, mask)
        with pytest.raises(B.MdcnnError):                  # it has no pending ring to read
            g.read(i, B.MDCNN_VIEW_P)
    finally:
        g.close()
    # two producers into such a site are refused when the network is made
    bad = copy.deepcopy(net)
    from inputs.nets import EdgeSpec
    i = next(i for i, s in enumerate(bad.sites) if s.trunc_free)
    src = [e for e in bad.edges if e.dst == i][0]
    bad.edges.append(EdgeSpec(src.src, i, 1, src.stride, 0, 0, src.w.copy(), None))
    bad.edges.sort(key=lambda e: e.src)
    with pytest.raises(B.MdcnnError):
        GpuNet(bad)


@pytest.mark.parametrize("name", ["pairs_f16_mfma", "bottleneck"])
def test_truncation_free_frames_in_flight_and_batch(name):
    """The same launches through mdcnn_frames (the initialisation that would ride on the missing delta launch gets a
    launch of its own) and through mdcnn_frame_batch: bit-identical to one mdcnn_frame call per frame."""
    import gpu_harness as H
    from paper_2210_09887_amd.runtime import GpuBatch, GpuNet
    net = cases()[name]
    frames, shifts, forced = inputs_of(name, net)
    Xs = [H.dev(x) for x in frames]
    Fs = None if forced is None else [H.dev(f) for f in forced]
    dys, dxs = [int(s[0]) for s in shifts], [int(s[1]) for s in shifts]
    g = GpuNet(net)
    want, resets = [], []
    try:
        for t in range(len(Xs)):
            o, r = g.frame(Xs[t], dys[t], dxs[t], None if Fs is None else Fs[t])
            want.append(o.clone())
            resets.append(r)
    finally:
        g.close()
    for depth in (1, 2, 4):
        g = GpuNet(net)
        try:
            outs, rs = g.frames(Xs, dys, dxs, Fs, depth=depth)
            torch.cuda.synchronize()
            assert rs == resets
            for t in range(len(Xs)):
                assert torch.equal(outs[t], want[t]), f"depth {depth} frame {t}"
        finally:
            g.close()
    gb = GpuBatch(net, 2)
    try:
        # stream 0 plays the sequence, stream 1 the same sequence: both must equal the single run
        for t in range(len(Xs)):
            outs, rs = gb.frame([Xs[t], Xs[t]], [dys[t]] * 2, [dxs[t]] * 2, None if Fs is None else [Fs[t], Fs[t]])
            torch.cuda.synchronize()
            for b in range(2):
                assert rs[b] == resets[t] and torch.equal(outs[b], want[t]), f"batch frame {t} stream {b}"
    finally:
        gb.close()


def test_config5_full_size_truncation_free():
    """The density workload at full size with its qualifying site (after the first 1x1 convolution) truncation-free."""
    import gpu_harness as H
    net = truncation_free(build_net(5))
    assert [s.trunc_free for s in net.sites] == [False, True, False, False]
    seq = build_sequence(5, density=0.2, n_frames=12)
    worst = H.teacher_forced(net, seq.frames, seq.shifts, seq.forced)
    r = H.followed(net, seq.frames, seq.shifts, seq.forced, log=log)
    log(f"config 5 truncation-free: teacher-forced worst {worst:.2e}; followed {r}")
    assert r["flips"] <= 0.02 * r["decisions"] and r["worst_margin"] < H.TOL["f16"] / 4
