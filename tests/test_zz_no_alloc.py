"""mdcnn_layer_forward_noalloc: the forward call for callers that cannot allocate.  The lists and per-segment counts
a forward call leaves behind go to a device array the library holds instead of the sites' memory; rings, delta maps,
flags, readout and the multiply-accumulate counters must be those of mdcnn_layer_forward, bit for bit - on calls in a
row that share the array, the later ones with smaller inputs, so that what an earlier call left there is seen to do no
harm."""
import numpy as np
import pytest
import torch

from inputs import build_net, build_sequence
from inputs.nets import truncation_free

pytestmark = pytest.mark.gpu

# larger first: every later video finds the array full of the lists of a larger site
CASES = [
    ("c3_resnet_160", 3, dict(H=160, W=160, widths=(32, 64, 64, 128)), dict(n_frames=5, H=160, W=160)),
    ("c4_hrnet_128x96", 4, dict(H=128, W=96, widths=(32, 64, 64, 128), blocks=2), dict(n_frames=5, H=128, W=96)),
    ("c2_cnn5_96", 2, dict(H=96, W=96), dict(n_frames=5, H=96, W=96)),
    ("c5_bottleneck_40", 5, dict(H=40, W=40, C=128, Cm=32), dict(n_frames=6, H=40, W=40, C=128, density=0.2, shift_every=3, shift=8)),
    ("c5_bottleneck_40_truncation_free", 5, dict(H=40, W=40, C=128, Cm=32), dict(n_frames=6, H=40, W=40, C=128, density=0.2, shift_every=3, shift=8)),
    ("c1_single_conv", 1, {}, {}),
]


def views_of(g, net):
    """Everything the two entry points have to agree on; per site the name of the view for the messages."""
    from paper_2210_09887_amd import binding as B
    out = []
    for i, s in enumerate(net.sites):
        if s.kind != "output":
            out += [(f"site {i} A", g.read(i, B.MDCNN_VIEW_A)), (f"site {i} delta", g.read(i, B.MDCNN_VIEW_DELTA)),
                    (f"site {i} flags", g.read(i, B.MDCNN_VIEW_FLAGS))]
            st = g.read(i, B.MDCNN_VIEW_STATS)[8:18].view(np.uint64)
            out += [(f"site {i} multiply-accumulates", st[[2, 4]].copy())]
        if s.kind != "input" and not getattr(s, "trunc_free", False):
            out += [(f"site {i} P", g.read(i, B.MDCNN_VIEW_P))]
        if s.kind == "output":
            out += [(f"site {i} readout", g.read(i, B.MDCNN_VIEW_OUT))]
    return out


def run_video(net, seq, noalloc):
    import gpu_harness as H
    from paper_2210_09887_amd.runtime import GpuNet
    g = GpuNet(net)
    try:
        per_frame = []
        for t, X in enumerate(seq.frames):
            g.shift_camera(int(seq.shifts[t][0]), int(seq.shifts[t][1]))
            Xd = H.dev(X)
            fd = H.dev(seq.forced[t]) if seq.forced is not None else None
            for i, sp in enumerate(net.sites):
                if sp.kind != "output":
                    g.layer_forward(i, Xd if i == 0 else None, fd if i == 0 else None, noalloc=noalloc)
            torch.cuda.synchronize()
            per_frame.append(views_of(g, net))
        return per_frame
    finally:
        g.close()


def test_noalloc_forward_matches_layer_forward_on_calls_in_a_row():
    for name, cfg, kn, ks in CASES:
        net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
        if name.endswith("truncation_free"):
            assert any(sp.trunc_free for sp in truncation_free(net).sites)
        print(f"no-alloc forward: {name}, {len(seq.frames)} frames, input {net.H}x{net.W}", flush=True)
        ref = run_video(net, seq, noalloc=False)
        got = run_video(net, seq, noalloc=True)
        assert len(ref) == len(got)
        for t, (a, b) in enumerate(zip(ref, got)):
            assert len(a) == len(b)
            for (what, u), (_, v) in zip(a, b):
                assert u.shape == v.shape and np.array_equal(u, v), f"{name}, frame {t}: {what} differs"


def test_noalloc_forward_interleaved_with_a_smaller_site():
    """Two sites of different size take turns, call by call, so every call finds the array as the other size left it."""
    import gpu_harness as H
    from paper_2210_09887_amd.runtime import GpuNet
    big_net, big_seq = build_net(2, H=128, W=128), build_sequence(2, n_frames=4, H=128, W=128)
    small_net, small_seq = build_net(2, H=48, W=48), build_sequence(2, n_frames=4, H=48, W=48)

    def run(noalloc):
        gb, gs = GpuNet(big_net), GpuNet(small_net)
        try:
            seen = []
            for t in range(4):
                for g, net, seq in ((gb, big_net, big_seq), (gs, small_net, small_seq)):
                    g.shift_camera(int(seq.shifts[t][0]), int(seq.shifts[t][1]))
                Xb, Xs = H.dev(big_seq.frames[t]), H.dev(small_seq.frames[t])
                for i, sp in enumerate(big_net.sites):       # same topology: layer i of the large, then of the small video
                    if sp.kind == "output":
                        continue
                    gb.layer_forward(i, Xb if i == 0 else None, None, noalloc=noalloc)
                    gs.layer_forward(i, Xs if i == 0 else None, None, noalloc=noalloc)
                torch.cuda.synchronize()
                seen.append(views_of(gb, big_net) + views_of(gs, small_net))
            return seen
        finally:
            gb.close()
            gs.close()

    ref, got = run(False), run(True)
    for t, (a, b) in enumerate(zip(ref, got)):
        for (what, u), (_, v) in zip(a, b):
            assert np.array_equal(u, v), f"frame {t}: {what} differs"


def test_noalloc_forward_leaves_the_lists_of_the_sites_alone_and_rejects_what_does_not_fit():
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    net, seq = build_net(1), build_sequence(1)
    g = GpuNet(net)
    try:
        g.shift_camera(0, 0)
        g.layer_forward(0, H.dev(seq.frames[0]))
        torch.cuda.synchronize()
        before = [g.read(0, B.MDCNN_VIEW_LIST), g.read(0, B.MDCNN_VIEW_STATS)[[0, 1]]]
        g.shift_camera(int(seq.shifts[1][0]), int(seq.shifts[1][1]))
        g.layer_forward(0, H.dev(seq.frames[1]), noalloc=True)
        torch.cuda.synchronize()
        after = [g.read(0, B.MDCNN_VIEW_LIST), g.read(0, B.MDCNN_VIEW_STATS)[[0, 1]]]
        for u, v in zip(before, after):
            assert np.array_equal(u, v)
    finally:
        g.close()
    # a 1024 x 1024 input: its list alone is 4 MiB, the library keeps 2
    big = build_net(2, H=1024, W=1024)
    g = GpuNet(big)
    try:
        g.shift_camera(0, 0)
        X = torch.zeros((1024, 1024, big.sites[0].C), dtype=g.tdtype, device="cuda")
        with pytest.raises(B.MdcnnError) as err:
            g.layer_forward(0, X, noalloc=True)
        assert err.value.status == 5                          # MDCNN_ERR_SIZE
        g.layer_forward(0, X)                                 # the site is as it was: the ordinary call goes through
        torch.cuda.synchronize()
    finally:
        g.close()
