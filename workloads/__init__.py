"""Seeded synthetic inputs and the wire format of the transfer engine.

This package is the only code shared by the CPU oracle and the HIP path. It
holds the binary layout of a transfer descriptor, the numeric values of the
error codes and flags (an interface, fixed by the C header), the five seeded
workload recipes, and a runner that drives any object exposing the engine
calls. It contains none of the method's arithmetic: no chunking, no schedule,
no allocator, no byte movement.
"""
from .format import (DESC_DTYPE, FT_HOST, FT_POOL, FT_PAGEABLE, H2P, P2H, P2P, CLASS_NAMES,
                     FT_OK, FT_EINVAL, FT_ENOMEM, FT_ERANGE, FT_EOVERLAP,
                     FT_EBUSY, FT_EHIP, FT_VALIDATE, FT_LOG, FT_PATH_DMA,
                     FT_TIMING, FT_DETACHED, FtError, make_descs)
