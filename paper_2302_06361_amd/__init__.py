"""libdash for MI355X: garbling and evaluating arithmetic garbled circuits over CRT residues
(Dash, arXiv 2302.06361) with hand-written HIP kernels behind the C ABI of include/dash.h.

This package is a thin binding: argument marshalling and device-buffer bookkeeping only.  Every
step of the path runs in the kernels of libdash.so; there is no CPU fallback.
"""
from .binding import (Context, Labels, Layer, DashError, lib_path,  # noqa: F401
                      DENSE, CONV2D, SUMPOOL, RELU, SCALE, SIGN, PROJ, LAMBDA_CEIL, LAMBDA_FLOOR)
from .network import GarbledNetwork, StreamedNetwork  # noqa: F401
from .grouped import ProjectionBatch  # noqa: F401
