"""Wire format shared by both implementations: descriptor layout, codes, flags.

A descriptor is 64 bytes, little endian, and carries no pointers to follow.
The same record is declared as ``ft_desc`` in the C header; the values below
must stay equal to that header's.
"""
import numpy as np

FT_HOST = 0   # address space of pinned host memory
FT_POOL = 1   # logical byte-offset space of the device pool
FT_PAGEABLE = 2   # ordinary host memory (host side of a transfer, open jobs only): goes through the pinned ring

# link classes (one independent weighted schedule each)
H2P, P2H, P2P = 0, 1, 2
CLASS_NAMES = ("H2P", "P2H", "P2P")

FT_OK = 0
FT_EINVAL = -1
FT_ENOMEM = -2
FT_ERANGE = -3
FT_EOVERLAP = -4
FT_EBUSY = -5
FT_EHIP = -6
FT_ECLOSED = -7
FT_E2BIG = -8

FT_VALIDATE = 1 << 0   # exact overlap check of the submit
FT_LOG = 1 << 1        # per-ticket device timestamps
FT_PATH_DMA = 1 << 2   # run the same schedule on the copy engines
FT_TIMING = 1 << 3     # device events around each class's kernel
FT_DETACHED = 1 << 4   # caller's stream does not wait for the job
FT_KEEP = 1 << 5       # keep the job record after wait
FT_OPEN = 1 << 6       # trigger the chunks in batches and accept merges meanwhile

DESC_DTYPE = np.dtype([
    ("func", "<u4"),
    ("src_space", "u1"),
    ("dst_space", "u1"),
    ("flags", "<u2"),
    ("src", "<u8"),
    ("dst", "<u8"),
    ("row_bytes", "<u8"),
    ("rows", "<u8"),
    ("src_pitch", "<u8"),
    ("dst_pitch", "<u8"),
    ("_pad", "<u8"),
])
assert DESC_DTYPE.itemsize == 64


class FtError(Exception):
    """An engine call returned a negative code."""

    def __init__(self, code, what=""):
        super().__init__(f"ft error {code} {what}")
        self.code = code


def make_descs(records):
    """Pack an iterable of dicts/tuples into a DESC_DTYPE array.

    Each record is a dict with keys func, src_space, dst_space, src, dst,
    row_bytes and optionally rows, src_pitch, dst_pitch, flags.
    """
    records = list(records)
    out = np.zeros(len(records), dtype=DESC_DTYPE)
    for i, r in enumerate(records):
        out[i]["func"] = r["func"]
        out[i]["src_space"] = r["src_space"]
        out[i]["dst_space"] = r["dst_space"]
        out[i]["flags"] = r.get("flags", 0)
        out[i]["src"] = r["src"]
        out[i]["dst"] = r["dst"]
        out[i]["row_bytes"] = r["row_bytes"]
        out[i]["rows"] = r.get("rows", 1)
        out[i]["src_pitch"] = r.get("src_pitch", r["row_bytes"])
        out[i]["dst_pitch"] = r.get("dst_pitch", r["row_bytes"])
    return out
