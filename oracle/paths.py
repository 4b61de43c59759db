"""Contention-aware selection of parallel paths between two GPUs (Sec. 6.2, Alg. 1)
and the striping of chunks over the paths chosen.

Alg. 1 and the prose of Sec. 6.2. The server's links are a directed graph with a
bandwidth per link (Topo) and a matrix of what is still free (BW). For a function that
sends from g_s to g_d: (1) go through the loop-free paths from g_s to g_d, shortest
first; a path all of whose links are idle is taken, it carries the bandwidth of its
narrowest link, b_min(path), and b_min is subtracted from the free bandwidth of every
link on it; stop when g_s has no free outgoing or g_d no free incoming bandwidth.
(2) If both still have some, go through the busy paths: if the function that occupies
the path holds more bandwidth in total than the current one and can switch to another
path, it does, and the busy path goes to the current function. Chunks are then sent
over the chosen paths in proportion to each path's bandwidth.

Readings (the listing's loop guards are garbled and step 2 is only sketched):
  * the loops run "while there is a next path"; the union/intersection signs in the
    listing's conditions are "or"/"and";
  * path order: fewer hops first, then the node sequence in lexicographic order; the search
    may be cut at `max_hops` links (the paper prunes the search but does not say how);
  * a link is idle when its free bandwidth equals its full bandwidth;
  * step 2 follows the prose, not the listing (which appends every busy path): a busy path
    is taken over only if exactly one path of one other function blocks it, that function
    holds more total bandwidth than the current one, and after giving the blocking path up it
    finds an idle path between the same two GPUs that shares no link with the path wanted;
    it then moves there (keeping the narrowest-link rule) and the current function takes the
    path, which is then idle;
  * striping: stride order over the paths with the paths' bandwidths as weights (the same
    proportional rule as for functions on one link).

TEST INFRASTRUCTURE ONLY (see the package docstring).
"""
from fractions import Fraction


def simple_paths(topo, s, d, max_hops=0):
    """Every loop-free path s -> d over links with bandwidth > 0 and at most max_hops links
    (0 = no limit), by (hops, node sequence)."""
    n = len(topo)
    out = []
    limit = max_hops if max_hops else n - 1

    def walk(path, seen):
        u = path[-1]
        if u == d:
            out.append(tuple(path))
            return
        if len(path) > limit:
            return
        for v in range(n):
            if topo[u][v] > 0 and v not in seen:
                walk(path + [v], seen | {v})

    if s != d:
        walk([s], {s})
    out.sort(key=lambda p: (len(p), p))
    return out


def edges(path):
    return list(zip(path[:-1], path[1:]))


class Links:
    def __init__(self, topo, max_hops=0):
        self.max_hops = max_hops
        self.n = len(topo)
        self.topo = [list(row) for row in topo]
        self.free = [list(row) for row in topo]
        self.paths = {}          # func -> list of [path tuple, bandwidth]

    def out_free(self, g):
        return sum(self.free[g])

    def in_free(self, g):
        return sum(self.free[u][g] for u in range(self.n))

    def idle(self, path):
        return all(self.free[u][v] == self.topo[u][v] for u, v in edges(path))

    def _take(self, func, path):
        bw = min(self.topo[u][v] for u, v in edges(path))
        for u, v in edges(path):
            self.free[u][v] -= bw
        self.paths.setdefault(func, []).append([path, bw])
        return bw

    def _give_up(self, func, idx):
        path, bw = self.paths[func].pop(idx)
        for u, v in edges(path):
            self.free[u][v] += bw
        return path, bw

    def total(self, func):
        return sum(bw for _, bw in self.paths.get(func, []))

    def release(self, func):
        while self.paths.get(func):
            self._give_up(func, 0)
        self.paths.pop(func, None)

    def select(self, func, s, d):
        if func in self.paths or s == d:
            raise ValueError("function already has paths, or source is destination")
        self.paths[func] = []
        cand = simple_paths(self.topo, s, d, self.max_hops)
        saturated = lambda: self.out_free(s) == 0 or self.in_free(d) == 0
        # step 1: idle paths, shortest first
        for path in cand:
            if saturated():
                break
            if self.idle(path):
                self._take(func, path)
        # step 2: busy paths whose one occupant is richer and can move elsewhere
        if not saturated():
            for path in cand:
                if saturated():
                    break
                if any(path == p for p, _ in self.paths[func]) or self.idle(path):
                    continue
                want = set(edges(path))
                blockers = [(g, i) for g, plist in self.paths.items() if g != func
                            for i, (p, _) in enumerate(plist) if want & set(edges(p))]
                mine = any(want & set(edges(p)) for p, _ in self.paths[func])
                if mine or len(blockers) != 1:
                    continue
                g, i = blockers[0]
                if self.total(g) <= self.total(func):
                    continue
                old, old_bw = self._give_up(g, i)
                alt = None
                for q in simple_paths(self.topo, old[0], old[-1], self.max_hops):
                    if q != old and self.idle(q) and not (want & set(edges(q))):
                        alt = q
                        break
                if alt is None or not self.idle(path):
                    # put it back exactly where it was
                    for u, v in edges(old):
                        self.free[u][v] -= old_bw
                    self.paths[g].insert(i, [old, old_bw])
                    continue
                # the occupant moves; its path list keeps the position of the path it gave up
                bw = min(self.topo[u][v] for u, v in edges(alt))
                for u, v in edges(alt):
                    self.free[u][v] -= bw
                self.paths[g].insert(i, [alt, bw])
                self._take(func, path)
        return [(p, bw) for p, bw in self.paths[func]]


def stripe_chunks(path_bw, nchunks):
    """Path of every chunk: always the path with the smallest (sent + 1) / bandwidth, ties
    to the lower path index."""
    sent = [0] * len(path_bw)
    out = []
    for _ in range(nchunks):
        best = min(range(len(path_bw)), key=lambda p: (Fraction(sent[p] + 1, path_bw[p]), p))
        out.append(best)
        sent[best] += 1
    return out


def dgx_v100_like():
    """The hybrid-cube-mesh stand-in (links of 24 and 48 GB/s); an input, kept with the other synthetic inputs."""
    from workloads.traces import hybrid_cube_mesh_24_48
    return hybrid_cube_mesh_24_48()


def xgmi_full_mesh(n=8, bw=64):
    """Every GPU linked to every other by one link; an input, kept with the other synthetic inputs."""
    from workloads.traces import full_mesh
    return full_mesh(n, bw)
