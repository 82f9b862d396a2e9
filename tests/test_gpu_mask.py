"""GPU parity of the post-processing of the input update mask (mdcnn_input_mask)
against the oracle: the masks are bytes decided by fp32 comparisons that both
sides evaluate in the same order, so they must agree bit for bit."""
import numpy as np
import pytest
import torch

from inputs import build_net, build_sequence

pytestmark = pytest.mark.gpu

PARAMS = [
    dict(),
    dict(dilate=10),
    dict(dilate=32),
    dict(suppress=True),
    dict(pool=2, suppress=True, dilate=3),
    dict(pool=4, dilate=5),
    dict(pool=8, suppress=True, dilate=1),
    dict(roi=True, base=0.4, gain=0.6, dilate=2),
    dict(roi=True, pool=2, suppress=True, dilate=10, theta=0.01),
]


@pytest.mark.parametrize("cfg,kn,ks", [
    (2, dict(H=88, W=72), dict(n_frames=5, H=88, W=72)),                                    # fp32, ragged tiles
    (3, dict(H=96, W=160, widths=(8, 16, 16, 32)), dict(n_frames=5, H=96, W=160)),          # fp16, moving camera with resets
])
def test_input_mask_equals_oracle(cfg, kn, ks):
    import gpu_harness as H
    from oracle.mdcnn_oracle import OracleNet
    from paper_2210_09887_amd.runtime import GpuNet
    net, seq = build_net(cfg, **kn), build_sequence(cfg, **ks)
    rng = np.random.default_rng(4)
    origins = [(int(rng.integers(0, 50)), int(rng.integers(0, 50))) for _ in net.sites]
    g, o = GpuNet(net, origins), OracleNet(net, origins)
    some = 0
    try:
        for t, X in enumerate(seq.frames):
            dy, dx = (int(v) for v in seq.shifts[t])
            # the mask is taken after the shift and before the frame is consumed
            assert g.shift_camera(dy, dx) == o.shift_camera(dy, dx)
            roi = rng.random((net.H, net.W)).astype(np.float32)
            Xd, rd = H.dev(X), H.dev(roi)
            for prm in PARAMS:
                kw = {k: v for k, v in prm.items() if k != "roi"}
                want = o.input_mask(X, roi if prm.get("roi") else None, **kw)
                got = g.input_mask(Xd, rd if prm.get("roi") else None, **kw).cpu().numpy()
                assert np.array_equal(got, want), f"frame {t} params {prm}: {int((got != want).sum())} pixels differ"
                some += int(0 < want.mean() < 1)
            # the frame itself, with one of the masks forced
            fm = o.input_mask(X, dilate=2)
            for i, s in enumerate(o.sites):
                if s.spec.kind == "output":
                    continue
                g.layer_forward(i, Xd if i == 0 else None, H.dev(fm) if i == 0 else None)
                o.layer_forward(i, X if i == 0 else None, fm if i == 0 else None)
            torch.cuda.synchronize()
            assert np.array_equal((g.read(0, 3) & 4) != 0, o.sites[0].M)
    finally:
        g.close()
    assert some > len(PARAMS)


def test_input_mask_with_crops_and_argument_checks():
    import gpu_harness as H
    from oracle.mdcnn_oracle import OracleNet
    from paper_2210_09887_amd import binding as B
    from paper_2210_09887_amd.runtime import GpuNet
    net, seq = build_net(2, H=96, W=64), build_sequence(2, n_frames=3, H=96, W=64)
    T = net.total_stride
    g, o = GpuNet(net, crops=True), OracleNet(net, crops=True)
    try:
        g.frame_crop(H.dev(seq.frames[0]), 0, 0, (0, 0, 96 // T, 64 // T))
        o.frame(seq.frames[0], 0, 0, crop=(0, 0, 96 // T, 64 // T))
        crop = (3, 2, 12, 9)
        g.shift_camera(*[int(v) for v in seq.shifts[1]])
        o.shift_camera(*[int(v) for v in seq.shifts[1]])
        g.set_crop(*crop)
        o.set_crop(*crop)
        Xc = H.cut(net, seq.frames[1], crop)
        for kw in [dict(), dict(pool=4, suppress=True, dilate=6)]:
            want = o.input_mask(Xc, **kw)
            got = g.input_mask(H.dev(Xc), **kw).cpu().numpy()
            assert got.shape == want.shape == (12 * T, 9 * T)
            assert np.array_equal(got, want)
        Xd = H.dev(Xc)
        for bad, status in [(dict(pool=3), 2), (dict(pool=16), 2), (dict(dilate=33), 2), (dict(dilate=-1), 2)]:
            with pytest.raises(B.MdcnnError) as ei:
                g.input_mask(Xd, **bad)
            assert ei.value.status == status
        prm = B.mdcnn_mask_params(0.1, 0.4, 0.6, 1, 0, 0)
        mask = torch.empty(Xd.shape[:2], dtype=torch.uint8, device="cuda")
        with pytest.raises(B.MdcnnError) as ei:
            B.mdcnn_input_mask(g.bufs[0], Xd.data_ptr(), None, prm, mask.data_ptr(), mask.numel() - 1)
        assert ei.value.status == 5
        with pytest.raises(B.MdcnnError) as ei:
            B.mdcnn_input_mask(g.bufs[1], Xd.data_ptr(), None, prm, mask.data_ptr(), mask.numel())
        assert ei.value.status == 2
        torch.cuda.synchronize()
    finally:
        g.close()
