"""Argument checks of mdcnn_frames, mdcnn_frames_crop and mdcnn_frames_masked.  Every check is made before
anything is launched or any state changes, so they run without a GPU (buffers wrap a fake address)."""
import ctypes as C

import pytest

from inputs import build_net
from paper_2210_09887_amd import binding as B
from test_plan_host import FAKE, host_net

ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_SIZE, ERR_STATE = 1, 2, 4, 5, 6


@pytest.fixture()
def net():
    spec = build_net(3, H=64, W=64, widths=(32, 64, 64, 128))
    handle, bufs = host_net(spec)
    out_bytes = sum((spec.H // s.stride) * (spec.W // s.stride) * s.C * 2 for s in spec.sites if s.kind == "output")
    yield spec, handle, out_bytes
    B.mdcnn_net_destroy(handle)
    for b in bufs:
        B.mdcnn_destroy_buffer(b)


def status_of(fn, *a, **kw):
    with pytest.raises(B.MdcnnError) as e:
        fn(*a, **kw)
    return e.value.status


def test_frames_refuses_bad_arguments(net):
    spec, h, nb = net
    X = [FAKE + 0x100000 * k for k in range(3)]
    O = [FAKE + 0x40000000 + 0x1000000 * k for k in range(3)]
    z = [0, 0, 0]
    assert status_of(B.mdcnn_frames, h, X, None, z, z, O, nb, depth=5) == ERR_SIZE
    assert status_of(B.mdcnn_frames, h, X, None, z, z, O, nb + 16) == ERR_SIZE
    assert status_of(B.mdcnn_frames, h, [X[0], None, X[2]], None, z, z, O, nb) == ERR_NULL
    assert status_of(B.mdcnn_frames, h, [X[0], X[1] + 2, X[2]], None, z, z, O, nb) == ERR_ALIGN
    assert status_of(B.mdcnn_frames, h, X, None, z, z, [O[0], O[1], O[0] + 64], nb) == ERR_STATE      # outputs overlap
    assert status_of(B.mdcnn_frames, None, X, None, z, z, O, nb) == ERR_NULL
    r = (C.c_int * 1)()
    assert B.lib().mdcnn_frames(h, 0, (C.c_void_p * 1)(X[0]), None, (C.c_int * 1)(0), (C.c_int * 1)(0), (C.c_void_p * 1)(O[0]), nb, 0, None, r) == ERR_SIZE
    assert "n_frames" in B.mdcnn_last_error()


def test_frames_crop_refuses_bad_arguments(net):
    spec, h, nb = net
    X = [FAKE + 0x100000 * k for k in range(2)]
    O = [FAKE + 0x40000000 + 0x1000000 * k for k in range(2)]
    z = [0, 0]
    whole = (0, 0, spec.H // spec.total_stride, spec.W // spec.total_stride)
    # the sites of this network were created without crops
    assert status_of(B.mdcnn_frames_crop, h, X, None, z, z, [whole, whole], O, [nb, nb]) == ERR_STATE
    assert B.lib().mdcnn_frames_crop(h, 2, (C.c_void_p * 2)(*X), None, (C.c_int * 2)(), (C.c_int * 2)(), None, (C.c_void_p * 2)(*O),
                                     (C.c_size_t * 2)(nb, nb), 0, None, None) == ERR_NULL


def test_frames_masked_refuses_bad_arguments(net):
    spec, h, nb = net
    X = [FAKE + 0x100000 * k for k in range(2)]
    O = [FAKE + 0x40000000 + 0x1000000 * k for k in range(2)]
    M = [FAKE + 0x60000000 + 0x100000 * k for k in range(2)]
    z = [0, 0]
    hw = spec.H * spec.W
    ok = B.mdcnn_mask_params(0.02, 0.4, 0.6, 1, 1, 2)
    assert status_of(B.mdcnn_frames_masked, h, X, None, B.mdcnn_mask_params(0.02, 0.4, 0.6, 3, 0, 0), M, hw, z, z, O, nb) == ERR_SHAPE     # pool
    assert status_of(B.mdcnn_frames_masked, h, X, None, B.mdcnn_mask_params(0.02, 0.4, 0.6, 1, 0, 33), M, hw, z, z, O, nb) == ERR_SHAPE    # dilate
    assert status_of(B.mdcnn_frames_masked, h, X, None, ok, M, hw - 1, z, z, O, nb) == ERR_SIZE
    assert status_of(B.mdcnn_frames_masked, h, X, None, ok, [M[0], M[0] + 16], hw, z, z, O, nb) == ERR_STATE                               # masks overlap
    assert status_of(B.mdcnn_frames_masked, h, X, None, ok, [M[0], None], hw, z, z, O, nb) == ERR_NULL
    assert status_of(B.mdcnn_frames_masked, h, X, [None, M[1] + 2], ok, M, hw, z, z, O, nb) == ERR_ALIGN                                   # roi


def test_options_accept_their_documented_values_only():
    """mdcnn_set_option is host-only: every option takes its documented range and refuses the next value."""
    ranges = {
        B.MDCNN_OPT_CONV_PATH: (0, 3), B.MDCNN_OPT_PROFILE: (0, 1), B.MDCNN_OPT_CONV_XCD: (0, 1),
        B.MDCNN_OPT_CONV_HALO: (0, 4), B.MDCNN_OPT_FUSE_SKIP: (0, 1), B.MDCNN_OPT_PIPE_MODE: (0, 1),
        B.MDCNN_OPT_PIPE_THREADS: (0, 1), B.MDCNN_OPT_CONV_F32_MFMA: (0, 1), B.MDCNN_OPT_PIPE_GROUP: (0, 64),
    }
    defaults = {B.MDCNN_OPT_CONV_XCD: 1, B.MDCNN_OPT_CONV_HALO: 1, B.MDCNN_OPT_FUSE_SKIP: 1, B.MDCNN_OPT_PIPE_MODE: 1,
                B.MDCNN_OPT_PIPE_THREADS: 1, B.MDCNN_OPT_CONV_F32_MFMA: 1}
    for opt, (lo, hi) in ranges.items():
        try:
            for v in (lo, hi):
                B.mdcnn_set_option(opt, v)
            assert status_of(B.mdcnn_set_option, opt, hi + 1) == ERR_SIZE
            assert status_of(B.mdcnn_set_option, opt, lo - 1) == ERR_SIZE
        finally:
            B.mdcnn_set_option(opt, defaults.get(opt, 0))
    assert status_of(B.mdcnn_set_option, 99, 0) == ERR_SIZE
