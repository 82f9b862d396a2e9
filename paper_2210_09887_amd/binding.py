"""ctypes binding of libmdcnn.so: the same names as the C ABI (include/mdcnn.h).

Argument marshalling only -- every step of the path runs in the HIP kernels.
PyTorch provides device memory (tensors whose data_ptr() is handed over) and
the stream.  Loading fails loudly when the library has not been built; there
is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmdcnn.so")

MDCNN_OK = 0
MDCNN_F32, MDCNN_F16 = 0, 1
MDCNN_SITE_INPUT, MDCNN_SITE_PREACT, MDCNN_SITE_OUTPUT = 0, 1, 2
(MDCNN_VIEW_A, MDCNN_VIEW_P, MDCNN_VIEW_DELTA, MDCNN_VIEW_FLAGS, MDCNN_VIEW_LIST,
 MDCNN_VIEW_CLIST, MDCNN_VIEW_STATS, MDCNN_VIEW_OUT, MDCNN_VIEW_POOL_PREV, MDCNN_VIEW_CROP_OUT,
 MDCNN_VIEW_PENDING) = range(11)
MDCNN_OPT_CONV_PATH, MDCNN_OPT_PROFILE, MDCNN_OPT_CONV_TILE, MDCNN_OPT_CONV_PIPE, MDCNN_OPT_CONV_XCD, MDCNN_OPT_CONV_KC, \
    MDCNN_OPT_CONV_HALO, MDCNN_OPT_CONV_HALO_SUB, MDCNN_OPT_FUSE_SKIP, MDCNN_OPT_STREAMS, MDCNN_OPT_PIPE_GROUP, MDCNN_OPT_PIPE_MODE, MDCNN_OPT_PIPE_THREADS, MDCNN_OPT_CONV_F32_MFMA = range(14)
KERNEL_CLASSES = ["shift", "step1", "lists", "conv_mfma", "conv_plain", "identity", "readout", "pool"]
FLAG_N, FLAG_U, FLAG_M = 1, 2, 4
STATE_UNSEEN, STATE_DIRTY = 1, 2

STATUS_NAMES = {0: "OK", 1: "ERR_NULL", 2: "ERR_SHAPE", 3: "ERR_DTYPE", 4: "ERR_ALIGN",
                5: "ERR_SIZE", 6: "ERR_STATE", 7: "ERR_HIP"}

EXPORTS = ["mdcnn_conv_border", "mdcnn_conv_tiles", "mdcnn_buffer_bytes", "mdcnn_create_buffer", "mdcnn_destroy_buffer",
           "mdcnn_shift_camera", "mdcnn_set_crop", "mdcnn_layer_forward", "mdcnn_layer_forward_noalloc", "mdcnn_net_create", "mdcnn_net_destroy",
           "mdcnn_frame", "mdcnn_frame_crop", "mdcnn_frame_batch", "mdcnn_frame_batch_crop", "mdcnn_frame_plan", "mdcnn_frames", "mdcnn_frames_batch", "mdcnn_frames_crop", "mdcnn_frames_masked", "mdcnn_frames_plan", "mdcnn_input_mask", "mdcnn_read_view", "mdcnn_write_view", "mdcnn_set_option", "mdcnn_profile_read", "mdcnn_profile_read_launches", "mdcnn_bench_copy", "mdcnn_bench_mfma",
           "mdcnn_pack_weights", "mdcnn_last_error", "mdcnn_version"]


class mdcnn_buffer_desc(C.Structure):
    _fields_ = [("H", C.c_int), ("W", C.c_int), ("C", C.c_int), ("dtype", C.c_int), ("kind", C.c_int),
                ("border", C.c_int * 4), ("tile", C.c_int), ("relu", C.c_int), ("theta", C.c_float),
                ("bias_dev", C.c_void_p), ("origin_y", C.c_int), ("origin_x", C.c_int), ("pool_prev", C.c_int), ("crops", C.c_int),
                ("truncation_free", C.c_int)]


class mdcnn_conv_desc(C.Structure):
    _fields_ = [("k", C.c_int), ("stride", C.c_int), ("pad", C.c_int), ("Cin", C.c_int), ("Cout", C.c_int),
                ("up", C.c_int), ("w_dev", C.c_void_p), ("w_packed_dev", C.c_void_p), ("op", C.c_int)]


class mdcnn_mask_params(C.Structure):
    _fields_ = [("theta", C.c_float), ("sens_base", C.c_float), ("sens_gain", C.c_float), ("pool", C.c_int),
                ("suppress", C.c_int), ("dilate", C.c_int)]


class MdcnnError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"mdcnn {STATUS_NAMES.get(status, status)}: {msg}")
        self.status = status


_lib = None


def lib():
    """The loaded library; raises if it was not built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        vp, ip, sz = C.c_void_p, C.POINTER(C.c_int), C.c_size_t
        L.mdcnn_conv_border.argtypes = [C.c_int] * 5 + [ip, ip]
        L.mdcnn_conv_tiles.argtypes = [C.c_int] * 5 + [ip, ip, C.POINTER(C.c_longlong)]
        L.mdcnn_buffer_bytes.argtypes = [C.POINTER(mdcnn_buffer_desc), C.POINTER(sz)]
        L.mdcnn_create_buffer.argtypes = [C.POINTER(mdcnn_buffer_desc), vp, sz, C.POINTER(vp)]
        L.mdcnn_destroy_buffer.argtypes = [vp]
        L.mdcnn_shift_camera.argtypes = [C.POINTER(vp), C.c_int, C.c_int, C.c_int, vp, ip]
        L.mdcnn_set_crop.argtypes = [C.POINTER(vp), C.c_int] + [C.c_int] * 4
        L.mdcnn_frame_crop.argtypes = [vp, vp, vp] + [C.c_int] * 6 + [vp, sz, vp, ip]
        L.mdcnn_layer_forward.argtypes = [vp, vp, vp, C.POINTER(mdcnn_conv_desc), C.POINTER(vp), C.c_int, vp]
        L.mdcnn_layer_forward_noalloc.argtypes = [vp, vp, vp, C.POINTER(mdcnn_conv_desc), C.POINTER(vp), C.c_int, vp]
        L.mdcnn_net_create.argtypes = [C.POINTER(vp), C.c_int, ip, ip, C.POINTER(mdcnn_conv_desc), C.c_int,
                                       C.POINTER(vp)]
        L.mdcnn_net_destroy.argtypes = [vp]
        L.mdcnn_frame.argtypes = [vp, vp, vp, C.c_int, C.c_int, vp, sz, vp, ip]
        L.mdcnn_frame_batch.argtypes = [C.POINTER(vp), C.c_int, C.POINTER(vp), C.POINTER(vp), ip, ip, C.POINTER(vp), sz, vp, ip]
        L.mdcnn_frame_plan.argtypes = [vp, C.c_int, ip, ip, C.c_int, ip, ip]
        L.mdcnn_frames.argtypes = [vp, C.c_int, C.POINTER(vp), C.POINTER(vp), ip, ip, C.POINTER(vp), sz, C.c_int, vp, ip]
        L.mdcnn_frame_batch_crop.argtypes = [C.POINTER(vp), C.c_int, C.POINTER(vp), C.POINTER(vp), ip, ip, ip, C.POINTER(vp), C.POINTER(sz), vp, ip]
        L.mdcnn_frames_batch.argtypes = [C.POINTER(vp), C.c_int, C.c_int, C.POINTER(vp), C.POINTER(vp), ip, ip, C.POINTER(vp), sz, C.c_int, vp, ip]
        L.mdcnn_frames_crop.argtypes = [vp, C.c_int, C.POINTER(vp), C.POINTER(vp), ip, ip, ip, C.POINTER(vp), C.POINTER(sz), C.c_int, vp, ip]
        L.mdcnn_frames_masked.argtypes = [vp, C.c_int, C.POINTER(vp), C.POINTER(vp), C.POINTER(mdcnn_mask_params), C.POINTER(vp), sz, ip, ip,
                                          C.POINTER(vp), sz, C.c_int, vp, ip]
        L.mdcnn_frames_plan.argtypes = [vp, C.c_int, ip, ip, ip, C.c_int, ip, C.c_int, ip, C.c_int, ip, ip]
        L.mdcnn_input_mask.argtypes = [vp, vp, vp, C.POINTER(mdcnn_mask_params), vp, sz, vp]
        L.mdcnn_read_view.argtypes = [vp, C.c_int, vp, sz, vp]
        L.mdcnn_write_view.argtypes = [vp, C.c_int, vp, sz, vp]
        L.mdcnn_set_option.argtypes = [C.c_int, C.c_int]
        L.mdcnn_pack_weights.argtypes = [C.POINTER(mdcnn_conv_desc), C.c_int, vp, sz, vp]
        L.mdcnn_profile_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_longlong)]
        L.mdcnn_profile_read_launches.argtypes = [C.c_int, ip, ip, ip, C.POINTER(C.c_float), ip]
        L.mdcnn_bench_copy.argtypes = [vp, vp, sz, vp]
        L.mdcnn_bench_mfma.argtypes = [C.c_int, C.c_int, vp, vp, C.POINTER(C.c_double)]
        L.mdcnn_last_error.restype = C.c_char_p
        L.mdcnn_version.restype = C.c_char_p
        for name in EXPORTS:
            if name not in ("mdcnn_last_error", "mdcnn_version"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(status):
    if status != MDCNN_OK:
        raise MdcnnError(status, lib().mdcnn_last_error().decode())


def mdcnn_last_error() -> str:
    return lib().mdcnn_last_error().decode()


def mdcnn_version() -> str:
    return lib().mdcnn_version().decode()


def mdcnn_set_option(option: int, value: int):
    _check(lib().mdcnn_set_option(option, value))


def mdcnn_profile_read():
    """{class name: (milliseconds, launches)} since the last call (blocks)."""
    n = len(KERNEL_CLASSES)
    ms, cnt = (C.c_double * n)(), (C.c_longlong * n)()
    _check(lib().mdcnn_profile_read(n, ms, cnt))
    return {k: (ms[i], cnt[i]) for i, k in enumerate(KERNEL_CLASSES)}


def mdcnn_profile_read_launches():
    """[(class name, site, edge, microseconds)] of the launches since the last read, in issue order (blocks)."""
    n = C.c_int()
    cap = 1 << 16
    cls, site, edge, us = (C.c_int * cap)(), (C.c_int * cap)(), (C.c_int * cap)(), (C.c_float * cap)()
    _check(lib().mdcnn_profile_read_launches(cap, cls, site, edge, us, C.byref(n)))
    return [(KERNEL_CLASSES[cls[i]], site[i], edge[i], us[i]) for i in range(n.value)]


def mdcnn_bench_copy(src_ptr: int, dst_ptr: int, nbytes: int, stream: int = 0):
    _check(lib().mdcnn_bench_copy(src_ptr, dst_ptr, nbytes, stream))


def mdcnn_bench_mfma(iters: int, blocks: int, sink_ptr: int, stream: int = 0) -> float:
    """Launches the matrix-core loop; returns the floating-point operations of the launch."""
    f = C.c_double()
    _check(lib().mdcnn_bench_mfma(int(iters), int(blocks), sink_ptr, stream, C.byref(f)))
    return f.value


def mdcnn_conv_border(k, stride, pad, in_extent, out_extent):
    b, a = C.c_int(), C.c_int()
    _check(lib().mdcnn_conv_border(k, stride, pad, in_extent, out_extent, C.byref(b), C.byref(a)))
    return b.value, a.value


def mdcnn_buffer_bytes(desc: mdcnn_buffer_desc) -> int:
    n = C.c_size_t()
    _check(lib().mdcnn_buffer_bytes(C.byref(desc), C.byref(n)))
    return n.value


def mdcnn_create_buffer(desc: mdcnn_buffer_desc, dev_ptr: int, nbytes: int) -> int:
    h = C.c_void_p()
    _check(lib().mdcnn_create_buffer(C.byref(desc), dev_ptr, nbytes, C.byref(h)))
    return h.value


def mdcnn_destroy_buffer(buf: int):
    _check(lib().mdcnn_destroy_buffer(buf))


def _handles(bufs):
    return (C.c_void_p * len(bufs))(*bufs)


def mdcnn_shift_camera(bufs, dty: int, dtx: int, stream: int = 0) -> bool:
    r = C.c_int()
    _check(lib().mdcnn_shift_camera(_handles(bufs), len(bufs), int(dty), int(dtx), stream, C.byref(r)))
    return bool(r.value)


def mdcnn_set_crop(bufs, ty0: int, tx0: int, th: int, tw: int):
    _check(lib().mdcnn_set_crop(_handles(bufs), len(bufs), int(ty0), int(tx0), int(th), int(tw)))


def mdcnn_layer_forward(buf: int, frame_ptr, forced_ptr, edges, outs, stream: int = 0):
    n = len(edges)
    arr = (mdcnn_conv_desc * max(n, 1))(*edges)
    _check(lib().mdcnn_layer_forward(buf, frame_ptr, forced_ptr, arr, _handles(outs) if n else None, n, stream))


def mdcnn_conv_tiles(Hp: int, Wp: int, k: int, max_pixels: int, max_staged: int):
    """(th, tw, tiles) of the rectangular tiles the halo-staged convolution would use."""
    th, tw, n = C.c_int(), C.c_int(), C.c_longlong()
    _check(lib().mdcnn_conv_tiles(int(Hp), int(Wp), int(k), int(max_pixels), int(max_staged), C.byref(th), C.byref(tw), C.byref(n)))
    return th.value, tw.value, n.value


def mdcnn_layer_forward_noalloc(buf: int, frame_ptr, forced_ptr, edges, outs, stream: int = 0):
    n = len(edges)
    arr = (mdcnn_conv_desc * max(n, 1))(*edges)
    _check(lib().mdcnn_layer_forward_noalloc(buf, frame_ptr, forced_ptr, arr, _handles(outs) if n else None, n, stream))


def mdcnn_net_create(sites, edge_src, edge_dst, edges) -> int:
    h = C.c_void_p()
    n = len(edges)
    _check(lib().mdcnn_net_create(_handles(sites), len(sites), (C.c_int * n)(*edge_src), (C.c_int * n)(*edge_dst),
                                  (mdcnn_conv_desc * n)(*edges), n, C.byref(h)))
    return h.value


def mdcnn_pack_weights(edge, dtype: int, dst_ptr: int, dst_bytes: int, stream: int = 0):
    _check(lib().mdcnn_pack_weights(C.byref(edge), int(dtype), dst_ptr, dst_bytes, stream))


def mdcnn_net_destroy(net: int):
    _check(lib().mdcnn_net_destroy(net))


def mdcnn_frame(net: int, frame_ptr: int, forced_ptr, dty: int, dtx: int, out_ptr: int, out_bytes: int,
                stream: int = 0) -> bool:
    r = C.c_int()
    _check(lib().mdcnn_frame(net, frame_ptr, forced_ptr, int(dty), int(dtx), out_ptr, out_bytes, stream, C.byref(r)))
    return bool(r.value)


def mdcnn_frame_crop(net: int, frame_ptr: int, forced_ptr, dty: int, dtx: int, crop, out_ptr: int, out_bytes: int,
                     stream: int = 0) -> bool:
    """crop = (ty0, tx0, th, tw) in tiles of the view."""
    r = C.c_int()
    ty0, tx0, th, tw = (int(v) for v in crop)
    _check(lib().mdcnn_frame_crop(net, frame_ptr, forced_ptr, int(dty), int(dtx), ty0, tx0, th, tw, out_ptr, out_bytes,
                                  stream, C.byref(r)))
    return bool(r.value)


def mdcnn_frame_batch(nets, frame_ptrs, forced_ptrs, dty, dtx, out_ptrs, out_bytes: int, stream: int = 0):
    """One frame for len(nets) streams; returns the list of reset decisions."""
    n = len(nets)
    r = (C.c_int * n)()
    forced = None if forced_ptrs is None else (C.c_void_p * n)(*forced_ptrs)
    _check(lib().mdcnn_frame_batch(_handles(nets), n, (C.c_void_p * n)(*frame_ptrs), forced,
                                   (C.c_int * n)(*[int(v) for v in dty]), (C.c_int * n)(*[int(v) for v in dtx]),
                                   (C.c_void_p * n)(*out_ptrs), out_bytes, stream, r))
    return [bool(v) for v in r]


def mdcnn_frame_batch_crop(nets, frame_ptrs, forced_ptrs, dty, dtx, crops, out_ptrs, out_bytes, stream: int = 0):
    """One cropped frame for len(nets) streams, crops[b] = (ty0, tx0, th, tw); returns the list of reset decisions."""
    n = len(nets)
    r = (C.c_int * n)()
    forced = None if forced_ptrs is None else (C.c_void_p * n)(*forced_ptrs)
    flat = [int(v) for c in crops for v in c]
    _check(lib().mdcnn_frame_batch_crop(_handles(nets), n, (C.c_void_p * n)(*frame_ptrs), forced,
                                        (C.c_int * n)(*[int(v) for v in dty]), (C.c_int * n)(*[int(v) for v in dtx]), (C.c_int * (4 * n))(*flat),
                                        (C.c_void_p * n)(*out_ptrs), (C.c_size_t * n)(*[int(v) for v in out_bytes]), stream, r))
    return [bool(v) for v in r]


def mdcnn_frame_plan(net: int, streams: int = 0):
    """(stream of every launch, [launches it waits for], streams used) of a frame of `net`."""
    n, ns = C.c_int(), C.c_int()
    _check(lib().mdcnn_frame_plan(net, int(streams), None, None, 0, C.byref(n), C.byref(ns)))
    so, wo = (C.c_int * n.value)(), (C.c_int * (2 * n.value))()
    _check(lib().mdcnn_frame_plan(net, int(streams), so, wo, n.value, None, None))
    waits = [[w for w in (wo[2 * i], wo[2 * i + 1]) if w >= 0] for i in range(n.value)]
    return list(so), waits, ns.value


def mdcnn_frames(net: int, frame_ptrs, forced_ptrs, dty, dtx, out_ptrs, out_bytes: int, depth: int = 0, stream: int = 0):
    """len(frame_ptrs) consecutive frames of one video, up to `depth` in flight; returns the reset decisions."""
    n = len(frame_ptrs)
    r = (C.c_int * n)()
    forced = None if forced_ptrs is None else (C.c_void_p * n)(*forced_ptrs)
    _check(lib().mdcnn_frames(net, n, (C.c_void_p * n)(*frame_ptrs), forced,
                              (C.c_int * n)(*[int(v) for v in dty]), (C.c_int * n)(*[int(v) for v in dtx]),
                              (C.c_void_p * n)(*out_ptrs), out_bytes, int(depth), stream, r))
    return [bool(v) for v in r]


def mdcnn_frames_batch(nets, frame_ptrs, forced_ptrs, dty, dtx, out_ptrs, out_bytes: int, depth: int = 0, stream: int = 0):
    """frame_ptrs[f][b] etc.: frame f of video b; len(nets) videos, up to `depth` frames of each in flight.  Returns
    the reset decisions [f][b]."""
    nb, nf = len(nets), len(frame_ptrs)
    n = nb * nf
    flat = lambda rows: [v for row in rows for v in row]
    r = (C.c_int * n)()
    forced = None if forced_ptrs is None else (C.c_void_p * n)(*flat(forced_ptrs))
    _check(lib().mdcnn_frames_batch(_handles(nets), nb, nf, (C.c_void_p * n)(*flat(frame_ptrs)), forced,
                                    (C.c_int * n)(*[int(v) for v in flat(dty)]), (C.c_int * n)(*[int(v) for v in flat(dtx)]),
                                    (C.c_void_p * n)(*flat(out_ptrs)), out_bytes, int(depth), stream, r))
    return [[bool(r[f * nb + b]) for b in range(nb)] for f in range(nf)]


def mdcnn_frames_crop(net: int, frame_ptrs, forced_ptrs, dty, dtx, crops, out_ptrs, out_bytes, depth: int = 0, stream: int = 0):
    """mdcnn_frames with one crop (ty0, tx0, th, tw) and one output size per frame."""
    n = len(frame_ptrs)
    r = (C.c_int * n)()
    forced = None if forced_ptrs is None else (C.c_void_p * n)(*forced_ptrs)
    flat = [int(v) for c in crops for v in c]
    _check(lib().mdcnn_frames_crop(net, n, (C.c_void_p * n)(*frame_ptrs), forced,
                                   (C.c_int * n)(*[int(v) for v in dty]), (C.c_int * n)(*[int(v) for v in dtx]), (C.c_int * (4 * n))(*flat),
                                   (C.c_void_p * n)(*out_ptrs), (C.c_size_t * n)(*[int(v) for v in out_bytes]), int(depth), stream, r))
    return [bool(v) for v in r]


def mdcnn_frames_masked(net: int, frame_ptrs, roi_ptrs, prm: mdcnn_mask_params, mask_ptrs, mask_bytes: int, dty, dtx, out_ptrs,
                        out_bytes: int, depth: int = 0, stream: int = 0):
    """mdcnn_frames with the input masks made by the library (mdcnn_input_mask) into mask_ptrs."""
    n = len(frame_ptrs)
    r = (C.c_int * n)()
    roi = None if roi_ptrs is None else (C.c_void_p * n)(*roi_ptrs)
    _check(lib().mdcnn_frames_masked(net, n, (C.c_void_p * n)(*frame_ptrs), roi, C.byref(prm), (C.c_void_p * n)(*mask_ptrs), mask_bytes,
                                     (C.c_int * n)(*[int(v) for v in dty]), (C.c_int * n)(*[int(v) for v in dtx]),
                                     (C.c_void_p * n)(*out_ptrs), out_bytes, int(depth), stream, r))
    return [bool(v) for v in r]


def mdcnn_frames_plan(net: int, n_sites: int, depth: int = 0):
    """Frame pipeline of `net` as a dict: per group `first_call`, `wait_call` (call of the frame before it waits for)
    and `init_call` (call whose delta launch carries its initialisation, -1: own launch); `group_of_site`;
    `stream_of_call` (one more entry for the readout; -1: frame f on stream f % depth); `n_calls`."""
    n, nc = C.c_int(), C.c_int()
    _check(lib().mdcnn_frames_plan(net, int(depth), None, None, None, 0, None, 0, None, 0, C.byref(n), C.byref(nc)))
    a, b, c = (C.c_int * n.value)(), (C.c_int * n.value)(), (C.c_int * n.value)()
    g, so = (C.c_int * n_sites)(*([-1] * n_sites)), (C.c_int * (nc.value + 1))()
    _check(lib().mdcnn_frames_plan(net, int(depth), a, b, c, n.value, g, n_sites, so, nc.value + 1, None, None))
    return dict(first_call=list(a), wait_call=list(b), init_call=list(c), group_of_site=list(g), stream_of_call=list(so),
                n_calls=nc.value)


def mdcnn_input_mask(buf: int, frame_ptr: int, roi_ptr, prm: mdcnn_mask_params, mask_ptr: int, mask_bytes: int, stream: int = 0):
    _check(lib().mdcnn_input_mask(buf, frame_ptr, roi_ptr, C.byref(prm), mask_ptr, mask_bytes, stream))


def mdcnn_read_view(buf: int, what: int, dst_ptr: int, nbytes: int, stream: int = 0):
    _check(lib().mdcnn_read_view(buf, what, dst_ptr, nbytes, stream))


def mdcnn_write_view(buf: int, what: int, src_ptr: int, nbytes: int, stream: int = 0):
    _check(lib().mdcnn_write_view(buf, what, src_ptr, nbytes, stream))
