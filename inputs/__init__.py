"""Seeded synthetic workloads shared by the CPU oracle and the HIP path.

This package holds data only: network topologies with seeded weights
(`inputs.nets`) and moving-camera frame sequences (`inputs.scenes`).  None of
the method's arithmetic (ring addressing, borders, thresholds, convolution)
lives here; the oracle and the HIP binding each derive those on their own.
"""
from .nets import NetSpec, SiteSpec, EdgeSpec, build_net, CONFIG_NAMES  # noqa: F401
from .scenes import build_sequence, Sequence  # noqa: F401
