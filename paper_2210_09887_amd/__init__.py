"""MotionDeltaCNN hot path for AMD MI355X: HIP kernels behind a C ABI
(include/mdcnn.h), a ctypes binding with the same names, and a small helper
that instantiates a network description on the GPU."""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
