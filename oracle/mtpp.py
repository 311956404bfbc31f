"""Max-throughput partitioning of a computation graph by slicing a topological order (oracle; test infrastructure).

Sections "Dynamic sharding of neural networks" and "Enhanced MTPP slicing of topological order": operations v with
work(v), sizeparam(v), sizeout(v); blocks S; bandwidth B; fast memory M;

  io(S, T)    = (1 / B) * sum of sizeout(v) over the v in S whose output some operation of T consumes   (eq. io)
  overflow(S) = max(0, sizeparam(S) + peak(S) - M) / B + peak(S) / B                                     (eq. overflow)
  f(S)        = io(V \\ S, S) + sum of work over S + overflow(S) + io(S, V \\ S)                          (eq. f)
  minimise over the slicings of the order into at most k consecutive blocks the largest f                (eq. P*, Alg. 1)

Everything here is written straight from those definitions with Python sets and brute force over all cut
positions: usable for a dozen operations.  Readings (the paper leaves these open or prints them inconsistently):
the order is Kahn's with the smallest ready index first; the printed overflow adds bytes to seconds, here both of
its terms are times at bandwidth B and the first is clamped at zero; peak(S) is the largest working set of one
operation of S (its output plus its inputs); the "heuristic adjustment" and "heuristic-based weighting" of the
listing are the identity.
"""
import itertools


def kahn_order(n, edges):
    indeg = [0] * n
    succ = [[] for _ in range(n)]
    for u, v in edges:
        succ[u].append(v)
        indeg[v] += 1
    ready = sorted(v for v in range(n) if indeg[v] == 0)
    order = []
    while ready:
        v = ready.pop(0)
        order.append(v)
        for w in succ[v]:
            indeg[w] -= 1
            if indeg[w] == 0:
                ready.append(w)
        ready.sort()
    assert len(order) == n, "the graph has a cycle"
    return order


def io(S, T, edges, sizeout, B):
    producers = {u for (u, v) in edges if u in S and v in T}
    return sum(sizeout[u] for u in producers) / B


def peak(S, edges, sizeout):
    best = 0.0
    for v in S:
        best = max(best, sizeout[v] + sum(sizeout[u] for u in {a for (a, b) in edges if b == v}))
    return best


def block_cost(S, n, edges, work, sizeparam, sizeout, B, M):
    S = set(S)
    rest = set(range(n)) - S
    pk = peak(S, edges, sizeout)
    overflow = max(0.0, sum(sizeparam[v] for v in S) + pk - M) / B + pk / B
    return io(rest, S, edges, sizeout, B) + sum(work[v] for v in S) + overflow + io(S, rest, edges, sizeout, B)


def slice_order(n, edges, work, sizeparam, sizeout, k, B, M, order=None):
    """Best slicing of the order into at most k blocks: (bottleneck cost, list of blocks as lists of operations).
    Ties go to fewer blocks, then to the lexicographically smallest cut positions."""
    order = kahn_order(n, edges) if order is None else list(order)
    best = None
    for blocks in range(1, min(k, n) + 1):
        for cuts in itertools.combinations(range(1, n), blocks - 1):
            bounds = [0, *cuts, n]
            parts = [order[bounds[i]:bounds[i + 1]] for i in range(blocks)]
            cost = max(block_cost(p, n, edges, work, sizeparam, sizeout, B, M) for p in parts)
            if best is None or cost < best[0]:
                best = (cost, parts)
    return best
