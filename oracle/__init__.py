"""CPU oracle of the chunked, weight-interleaved transfer engine.

TEST INFRASTRUCTURE ONLY. This package is a plain, slow, single-threaded
description of what the engine computes, written from the paper's text
(FaaSTube, arxiv 2411.01830) so that the HIP path can be checked against it
byte for byte. Only the test-suite, the smoke check and the benchmark's
``cpu_baseline`` leg may import it. It shares no code with the HIP path and
never calls it.

What it follows:
  * pool.py      the pooled GPU store of Sec. 7.1 (blocks handed out from a
                 pre-allocated, growable pool instead of native allocation).
  * schedule.py  Sec. 6.1: every function's data is cut into fixed-size
                 chunks and chunks of different functions are triggered in
                 proportion to the bandwidth given to each function.
  * engine.py    Sec. 5.1: host<->GPU and intra-GPU passing are copies; the
                 chunks are transport only, so the data result is the plain
                 definition dst[i] = src[i]. Sources in ordinary host memory
                 (Sec. 6.1's circular pinned buffer) are copies like any other.
  * rate.py      Sec. 6.1, function transfer rate control: least rate from the
                 SLO, idle bandwidth to the tightest SLO, integer weights.
  * batches.py   Sec. 6.1, batched transfer triggering: the batches of a link
                 when functions arrive while it is busy.
  * store.py     Sec. 7: histogram sizing of the pool, queue-aware choice of
                 what to move to host memory and back, and the least-recently-
                 stored rule it is measured against.
  * paths.py     Sec. 6.2 / Alg. 1: contention-aware parallel paths between two
                 GPUs and chunk striping in proportion to path bandwidth.

Parity pins (all in tests/, run without a GPU): hand-derived orders under
tests/golden/, the sort-by-finish-tag brute force, a closed-form rank,
round-robin and single-function special cases, the within-one-chunk share
invariant, periodicity, per-byte coverage counts, byte-loop data movement,
NumPy strided views and a brute-force slab bitmap; for the later modules
hand-worked rates, orders, reservations and path selections (tests/golden/),
a second formulation of the batched order, NumPy's inverted-CDF percentile,
the paper's own migration example, brute-force path enumeration and SciPy's
maximum flow as an upper bound. The timed bandwidth shares have no oracle
(they depend on the machine): parity unpinned.
"""

OK = 0
EINVAL = -1
ENOMEM = -2
ERANGE = -3
EOVERLAP = -4
EBUSY = -5

HOST = 0
POOL = 1
PAGEABLE = 2   # ordinary host memory, as the source of a host->pool or the destination of a pool->host
               # transfer (Sec. 6.1: it travels through a pinned ring, which is transport and leaves
               # the result a plain copy)

H2P, P2H, P2P = 0, 1, 2

FLAG_VALIDATE = 1


class OracleError(Exception):
    def __init__(self, code, what=""):
        super().__init__(f"oracle error {code}: {what}")
        self.code = code


from .pool import Pool            # noqa: E402
from .schedule import (link_class, chunk_count, stride_order,  # noqa: E402
                       chunk_segments)
from .engine import OracleEngine  # noqa: E402
