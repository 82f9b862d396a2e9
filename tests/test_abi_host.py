"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and validates its arguments."""
import ctypes as C
import os
import re

import pytest

from paper_2210_09887_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000000000          # an aligned address that is never dereferenced on the host


def desc(H=8, W=8, Cc=16, dtype=B.MDCNN_F32, kind=B.MDCNN_SITE_PREACT, border=(1, 1, 1, 1), tile=1):
    d = B.mdcnn_buffer_desc()
    d.H, d.W, d.C, d.dtype, d.kind, d.tile = H, W, Cc, dtype, kind, tile
    for i in range(4):
        d.border[i] = border[i]
    return d


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mdcnn.h")).read()
    declared = set(re.findall(r"\b(mdcnn_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert "gfx950" in B.mdcnn_version()


def test_conv_border_matches_the_paper_example_and_the_oracle():
    from oracle.mdcnn_oracle import conv_border
    assert B.mdcnn_conv_border(3, 1, 1, 64, 64) == (1, 1)        # 64 + 1 + 1 = 66
    for k, s, p, n in [(3, 1, 1, 64), (3, 2, 1, 64), (3, 2, 1, 63), (1, 1, 0, 17), (1, 2, 0, 16), (5, 1, 2, 9), (5, 2, 2, 12), (3, 1, 0, 8)]:
        out = (n + 2 * p - k) // s + 1
        assert B.mdcnn_conv_border(k, s, p, n, out) == conv_border(k, s, p, n, out)
    assert B.mdcnn_conv_border(0, 1, 0, 8, 8) == (0, 0)


def test_buffer_bytes_and_create():
    d = desc()
    n = B.mdcnn_buffer_bytes(d)
    assert n % 256 == 0
    # rings alone: A 8*8*16*4 + P 10*10*16*4
    assert n >= 8 * 8 * 16 * 4 + 10 * 10 * 16 * 4
    small = B.mdcnn_buffer_bytes(desc(kind=B.MDCNN_SITE_OUTPUT))
    assert small < n
    h = B.mdcnn_create_buffer(d, FAKE, n)
    assert h
    B.mdcnn_destroy_buffer(h)


@pytest.mark.parametrize("mutate,status", [
    (lambda d: setattr(d, "dtype", 7), 3),
    (lambda d: setattr(d, "H", 0), 2),
    (lambda d: setattr(d, "kind", 9), 2),
    (lambda d: setattr(d, "tile", 0), 2),
    (lambda d: setattr(d, "C", 5000), 5),
])
def test_bad_descriptors_are_refused(mutate, status):
    d = desc()
    mutate(d)
    with pytest.raises(B.MdcnnError) as e:
        B.mdcnn_buffer_bytes(d)
    assert e.value.status == status
    assert B.mdcnn_last_error()


def test_create_buffer_argument_checks():
    d = desc()
    n = B.mdcnn_buffer_bytes(d)
    with pytest.raises(B.MdcnnError) as e:
        B.mdcnn_create_buffer(d, FAKE + 8, n)
    assert e.value.status == 4
    with pytest.raises(B.MdcnnError) as e:
        B.mdcnn_create_buffer(d, FAKE, n - 1)
    assert e.value.status == 5
    with pytest.raises(B.MdcnnError) as e:
        B.mdcnn_create_buffer(d, None, n)
    assert e.value.status == 1
    bad = desc(kind=B.MDCNN_SITE_INPUT)
    with pytest.raises(B.MdcnnError) as e:
        B.mdcnn_buffer_bytes(bad)
    assert e.value.status == 2          # an input site has no border


def make(kind, H, W, Cc, border=(0, 0, 0, 0), dtype=B.MDCNN_F32):
    d = desc(H, W, Cc, dtype, kind, border)
    return B.mdcnn_create_buffer(d, FAKE, B.mdcnn_buffer_bytes(d))


def test_net_create_validates_edges():
    x = make(B.MDCNN_SITE_INPUT, 16, 16, 4)
    y = make(B.MDCNN_SITE_OUTPUT, 16, 16, 8, (1, 1, 1, 1))
    y_nob = make(B.MDCNN_SITE_OUTPUT, 16, 16, 8)
    y_half = make(B.MDCNN_SITE_OUTPUT, 8, 8, 8, (0, 1, 0, 1))
    y16 = make(B.MDCNN_SITE_OUTPUT, 16, 16, 8, (1, 1, 1, 1), B.MDCNN_F16)
    good = B.mdcnn_conv_desc(3, 1, 1, 4, 8, 0, FAKE)
    h = B.mdcnn_net_create([x, y], [0], [1], [good])
    B.mdcnn_net_destroy(h)
    h = B.mdcnn_net_create([x, y_half], [0], [1], [B.mdcnn_conv_desc(3, 2, 1, 4, 8, 0, FAKE)])
    B.mdcnn_net_destroy(h)
    cases = [
        ([x, y_nob], good, 2),                                        # border too small for a 3x3
        ([x, y], B.mdcnn_conv_desc(3, 1, 1, 5, 8, 0, FAKE), 2),       # Cin mismatch
        ([x, y], B.mdcnn_conv_desc(3, 2, 1, 4, 8, 0, FAKE), 2),       # output extent mismatch
        ([x, y], B.mdcnn_conv_desc(3, 1, 1, 4, 8, 0, None), 1),       # no weights
        ([x, y], B.mdcnn_conv_desc(3, 1, 1, 4, 8, 0, FAKE + 4), 4),   # misaligned weights
        ([x, y], B.mdcnn_conv_desc(3, 1, 1, 4, 8, 1, FAKE), 2),       # upsampling needs 1x1
        ([x, y], B.mdcnn_conv_desc(0, 1, 0, 4, 8, 0, None), 2),       # identity with Cin != Cout
        ([x, y16], good, 3),                                          # dtype mismatch
        ([y, x], good, 2),                                            # site 0 must be the input
    ]
    for sites, cd, status in cases:
        with pytest.raises(B.MdcnnError) as e:
            B.mdcnn_net_create(sites, [0], [1], [cd])
        assert e.value.status == status, B.mdcnn_last_error()
    # a forward before the first shift is a state error and launches nothing
    with pytest.raises(B.MdcnnError) as e:
        B.mdcnn_layer_forward(x, FAKE, None, [good], [y])
    assert e.value.status == 6
    for b in (x, y, y_nob, y_half, y16):
        B.mdcnn_destroy_buffer(b)


def test_multi_gpu_bench_is_refused():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)


def test_pack_weights_and_batch_argument_checks_need_no_gpu():
    """Both entry points validate before they touch the device."""
    from paper_2210_09887_amd import binding as B
    cd = B.mdcnn_conv_desc(3, 1, 1, 64, 64, 0, 4096, None)
    ok_bytes = 9 * 64 * 64 * 2
    for desc, dtype, dst, nbytes in [
        (B.mdcnn_conv_desc(3, 1, 1, 24, 64, 0, 4096, None), B.MDCNN_F16, 8192, 9 * 24 * 64 * 2),   # Cin % 16
        (B.mdcnn_conv_desc(3, 1, 1, 64, 48, 0, 4096, None), B.MDCNN_F16, 8192, 9 * 64 * 48 * 2),   # Cout % 32
        (cd, B.MDCNN_F32, 8192, ok_bytes),                                                          # dtype
        (cd, B.MDCNN_F16, 8200, ok_bytes),                                                          # alignment
        (cd, B.MDCNN_F16, 8192, ok_bytes - 2),                                                      # size
        (cd, B.MDCNN_F16, None, ok_bytes),                                                          # NULL
    ]:
        with pytest.raises(B.MdcnnError):
            B.mdcnn_pack_weights(desc, dtype, dst, nbytes)
    for n in (0, 129):                        # more streams than a call takes: refused before any handle is read
        with pytest.raises(B.MdcnnError):
            B.mdcnn_frame_batch([4096] * n, [4096] * n, None, [0] * n, [0] * n, [4096] * n, 16)
        with pytest.raises(B.MdcnnError):
            B.mdcnn_frame_batch_crop([4096] * n, [4096] * n, None, [0] * n, [0] * n, [(0, 0, 1, 1)] * n, [4096] * n, [16] * n)
        with pytest.raises(B.MdcnnError):
            B.mdcnn_frames_batch([4096] * n, [[4096] * n], None, [[0] * n], [[0] * n], [[4096] * n], 16)


def test_crop_argument_checks_need_no_gpu():
    d = desc(H=16, W=16, tile=4)
    n0 = B.mdcnn_buffer_bytes(d)
    d.crops = 1
    n1 = B.mdcnn_buffer_bytes(d)
    assert n1 == n0 + 256                      # one more byte per view pixel
    h = B.mdcnn_create_buffer(d, FAKE, n1)
    B.mdcnn_set_crop([h], 1, 2, 3, 2)          # host state only
    for bad in [(0, 0, 5, 1), (3, 0, 2, 1), (0, 0, 0, 1), (0, -1, 1, 1)]:
        with pytest.raises(B.MdcnnError) as ei:
            B.mdcnn_set_crop([h], *bad)
        assert ei.value.status == 2
    B.mdcnn_destroy_buffer(h)
    d.crops = 0
    h = B.mdcnn_create_buffer(d, FAKE, n0)
    with pytest.raises(B.MdcnnError) as ei:
        B.mdcnn_set_crop([h], 0, 0, 1, 1)
    assert ei.value.status == 6
    B.mdcnn_destroy_buffer(h)
    d.crops = 2
    with pytest.raises(B.MdcnnError) as ei:
        B.mdcnn_buffer_bytes(d)
    assert ei.value.status == 2


def test_input_mask_argument_checks_need_no_gpu():
    prm = B.mdcnn_mask_params(0.1, 0.4, 0.6, 1, 0, 0)
    d = desc(H=16, W=16, Cc=3, kind=B.MDCNN_SITE_INPUT, border=(0, 0, 0, 0))
    h = B.mdcnn_create_buffer(d, FAKE, B.mdcnn_buffer_bytes(d))
    with pytest.raises(B.MdcnnError) as ei:                 # never shifted
        B.mdcnn_input_mask(h, FAKE, None, prm, FAKE, 256)
    assert ei.value.status == 6
    with pytest.raises(B.MdcnnError) as ei:
        B.mdcnn_input_mask(h, None, None, prm, FAKE, 256)
    assert ei.value.status == 1
    B.mdcnn_destroy_buffer(h)
    p = desc()
    h = B.mdcnn_create_buffer(p, FAKE, B.mdcnn_buffer_bytes(p))
    with pytest.raises(B.MdcnnError) as ei:                 # not an INPUT site
        B.mdcnn_input_mask(h, FAKE, None, prm, FAKE, 64)
    assert ei.value.status == 2
    B.mdcnn_destroy_buffer(h)
