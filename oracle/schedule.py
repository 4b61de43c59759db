"""Chunking and proportional interleave of Sec. 6.1, step by step.

Sec. 6.1 says two things about the order of work on a shared link: each
function's data is cut into small fixed-size chunks (2 MB by default), and
chunks of different functions are triggered in proportion to the bandwidth
allotted to each function. The paper does not print the interleave rule.
Reading taken here (stride scheduling): a function f with integer weight w_f
that has had s_f chunks served holds the finish tag (s_f + 1) / w_f; the next
chunk always comes from the unfinished function with the smallest tag, ties
going to the lowest function index. Per function and per link class the
payloads of its descriptors, in submission order and row-major inside a
descriptor, form one byte stream; chunk k is stream bytes [kC, (k+1)C).
"""
from fractions import Fraction

from . import HOST, POOL, PAGEABLE, H2P, P2H, P2P, OracleError, EINVAL


def link_class(src_space, dst_space):
    """Sec. 5.1 lists host<->GPU and intra-GPU passing as different methods;
    each direction of the host link and the on-device path is its own class."""
    if src_space in (HOST, PAGEABLE) and dst_space == POOL:
        return H2P
    if src_space == POOL and dst_space in (HOST, PAGEABLE):
        return P2H
    if src_space == POOL and dst_space == POOL:
        return P2P
    raise OracleError(EINVAL, "host to host is not a transfer of this engine")


def chunk_count(stream_bytes, chunk_bytes):
    return -(-stream_bytes // chunk_bytes)


def stride_order(n, w):
    """Total order of all chunks. n[f] chunks and weight w[f] per function.

    Returns a list of (f, k); position in the list is the ticket."""
    served = [0] * len(n)
    order = []
    for _ in range(sum(n)):
        best = None
        best_tag = None
        for f in range(len(n)):
            if served[f] >= n[f]:
                continue
            tag = Fraction(served[f] + 1, w[f])
            if best is None or tag < best_tag:
                best, best_tag = f, tag
        order.append((best, served[best]))
        served[best] += 1
    return order


def chunk_segments(rows_bytes, chunk_bytes, k):
    """Pieces of chunk k of one function's stream.

    rows_bytes: list of (row_bytes, rows) per descriptor of the function, in
    submission order. Returns a list of (descriptor index, row, column,
    length): maximal runs that stay inside one row of one descriptor."""
    lo = k * chunk_bytes
    hi = lo + chunk_bytes
    out = []
    base = 0
    for d, (row_bytes, rows) in enumerate(rows_bytes):
        size = row_bytes * rows
        a = max(lo, base)
        b = min(hi, base + size)
        pos = a
        while pos < b:
            p = pos - base
            r, c = divmod(p, row_bytes)
            length = min(row_bytes - c, b - pos)
            out.append((d, r, c, length))
            pos += length
        base += size
    return out
