"""Batched transfer triggering of Sec. 6.1 with functions that arrive while a
link is busy.

Sec. 6.1: a chunk transfer cannot be interrupted once triggered, so the
chunks of a link are triggered in batches (5 chunks by default); functions
that arrive meanwhile get bandwidth by having their chunks included in the
batches that follow.

Reading taken here. A link class works through a sequence of batches of at
most `batch_chunks` chunks. A job is a set of functions (stream sizes in
chunks, weights). Job 0 is there from the start; a later job carries
`arrive`, the number of batches that had already been triggered when it
showed up, so batch `arrive` is the first that may hold its chunks (jobs are
listed in the order they arrive). Whenever
jobs join at a batch boundary, the proportional order (stride order of
schedule.py) is built afresh over everything not yet triggered: the
remaining chunks of every earlier function, renumbered from where each
stands, and all chunks of the new functions; functions are ordered by (job,
function index) for the tie rule. Between arrivals the order in force is
simply continued, five chunks at a time. When the link runs dry while jobs are
still to come, the earliest of them (smallest `arrive`, then job index) starts
a new sequence at once; the others keep waiting for their batch count.

Rate control (Sec. 6.1) changes shares while functions run: when a function arrives or
leaves, the bandwidth left over moves to whichever SLO is then the tightest. A job may
therefore carry `reweight`, a list of (batches triggered when the change was made, new
weights of its functions): from the first batch not yet triggered at that moment the
order is built afresh over everything not yet triggered, exactly as for an arrival, with
the new weights in force. A change made before the job has arrived takes effect with its
arrival; a change made once the link is dry changes nothing; of two changes to one job
made at the same count of batches the later one holds.

TEST INFRASTRUCTURE ONLY (see the package docstring).
"""
from .schedule import stride_order


def batched_order(jobs, batch_chunks=5):
    """jobs: list of dicts with keys `n` (chunks per function), `w` (weights) and,
    for every job but the first, `arrive`. Returns the list of batches; a batch is
    a list of (job, function, chunk)."""
    if batch_chunks < 1:
        raise ValueError("batch_chunks")
    arrive = [0] + [jobs[j]["arrive"] for j in range(1, len(jobs))]
    if any(a > b for a, b in zip(arrive, arrive[1:])):
        raise ValueError("jobs are listed in the order they arrive")
    waiting = list(range(1, len(jobs)))
    weights = [list(job["w"]) for job in jobs]            # the weights in force
    # in time order; of two changes to one job made at the same count the later in its list holds
    changes = sorted(((at, j, list(w)) for j, job in enumerate(jobs) for at, w in job.get("reweight", [])),
                     key=lambda change: change[0])
    funcs = [(0, f) for f in range(len(jobs[0]["n"]))]   # (job, function) in tie order
    served = {(0, f): 0 for f in range(len(jobs[0]["n"]))}
    batches = []
    order = None      # the order in force: list of (index into funcs, fresh chunk number)
    pos = 0
    base = {}         # chunk number each function stood at when the order was built
    while True:
        dry = order is None or pos >= len(order)
        newly = [j for j in waiting if jobs[j]["arrive"] <= len(batches)]
        if dry and order is not None and not newly and waiting:
            newly = [waiting[0]]
        for j in newly:
            waiting.remove(j)
            for f in range(len(jobs[j]["n"])):
                funcs.append((j, f))
                served[(j, f)] = 0
        changed = False
        while changes and changes[0][0] <= len(batches):
            _, j, w = changes.pop(0)
            if len(w) != len(jobs[j]["n"]) or min(w) < 1:
                raise ValueError("reweight")
            weights[j] = w
            changed = True
        if order is None or newly or (changed and not dry):
            live = [jf for jf in funcs if served[jf] < jobs[jf[0]]["n"][jf[1]]]
            base = {jf: served[jf] for jf in live}
            n = [jobs[j]["n"][f] - served[(j, f)] for j, f in live]
            w = [weights[j][f] for j, f in live]
            order = [(live[i], k) for i, k in stride_order(n, w)]
            pos = 0
        if pos >= len(order):
            if not waiting:
                break
            continue
        batch = []
        for jf, k in order[pos:pos + batch_chunks]:
            batch.append((jf[0], jf[1], base[jf] + k))
            served[jf] += 1
        pos += len(batch)
        batches.append(batch)
    return batches
