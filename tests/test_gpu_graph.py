"""mdcnn_frame can replay a recorded HIP graph of the frame (MDCNN_OPT_GRAPH): the
launches then read ring origins, frame, mask and output pointers from the sites'
memory.  Every result must equal the ordinary launches bit for bit."""
import numpy as np
import pytest
import torch

from inputs import build_net, build_sequence

pytestmark = pytest.mark.gpu

CASES = {
    "c1_single_conv": (1, {}, {}),
    "c3_resnet_96": (3, dict(H=96, W=96, widths=(32, 64, 64, 128)), dict(n_frames=8, H=96, W=96)),
    "c3_resnet_poolstem_128": (3, dict(H=128, W=128, widths=(32, 64, 64, 128), pool_stem=True), dict(n_frames=6, H=128, W=128, tile=16)),
    "c4_hrnet_128x96": (4, dict(H=128, W=96, widths=(32, 64, 64, 128), blocks=2), dict(n_frames=10, H=128, W=96)),
    "c5_bottleneck_40": (5, dict(H=40, W=40, C=128, Cm=32), dict(n_frames=8, H=40, W=40, C=128, density=0.2, shift_every=4, shift=8)),
}


def run(net, seq, graph, stream):
    import gpu_harness as H
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    B.mdcnn_set_option(B.MDCNN_OPT_GRAPH, int(graph))
    outs, state = [], []
    g = None
    try:
        with torch.cuda.stream(stream):
            g = GpuNet(net)
            for t, X in enumerate(seq.frames):
                dy, dx = (int(v) for v in seq.shifts[t])
                # fresh tensors every frame: the recorded launches must follow the pointers of the call
                Xd = H.dev(X)
                fd = H.dev(seq.forced[t]) if seq.forced is not None and t % 3 != 2 else None
                out = torch.empty_like(g.out)
                o, r = g.frame(Xd, dy, dx, fd, out=out)
                stream.synchronize()
                outs.append((o.clone(), r))
            for i, s in enumerate(net.sites):
                views = [B.MDCNN_VIEW_A, B.MDCNN_VIEW_DELTA, B.MDCNN_VIEW_FLAGS, B.MDCNN_VIEW_LIST, B.MDCNN_VIEW_STATS] if s.kind != "output" else []
                views += [B.MDCNN_VIEW_P, B.MDCNN_VIEW_CLIST] if s.kind != "input" else []
                state += [g.read(i, v) for v in views]
    finally:
        B.mdcnn_set_option(B.MDCNN_OPT_GRAPH, 0)
        if g is not None:
            g.close()
    return outs, state


@pytest.mark.parametrize("name", list(CASES))
def test_recorded_frames_equal_ordinary_launches(name):
    cfg, kn, ks = CASES[name]
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
    stream = torch.cuda.Stream()                      # the legacy default stream cannot be captured
    ref = run(net, seq, False, stream)
    got = run(net, seq, True, stream)
    assert len(ref[0]) == len(got[0])
    for t, ((a, ra), (b, rb)) in enumerate(zip(ref[0], got[0])):
        assert ra == rb, f"frame {t}: reset decision"
        assert torch.equal(a, b), f"frame {t}: outputs differ"
    for k, (u, v) in enumerate(zip(ref[1], got[1])):
        assert np.array_equal(u, v), f"state view {k} differs"


def test_recording_is_skipped_on_the_default_stream():
    """On the legacy default stream the library falls back to ordinary launches; results are the same."""
    cfg, kn, ks = CASES["c3_resnet_96"]
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
    ref = run(net, seq, False, torch.cuda.default_stream())
    got = run(net, seq, True, torch.cuda.default_stream())
    for (a, ra), (b, rb) in zip(ref[0], got[0]):
        assert ra == rb and torch.equal(a, b)
