"""libmtpp.so (host only) against the partitioning oracle: Kahn's order and every block cost exactly as defined,
the bottleneck of the best slicing equal to brute force over all cut positions, the returned blocks a valid
slicing that attains it; larger graphs against properties; error returns."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import mtpp as oracle
from paper_2407_19775_amd import mtpp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.skipif(not os.path.exists(mtpp.LIB_PATH), reason="libmtpp.so not built")


def random_dag(rng, n, p):
    perm = rng.permutation(n)                     # a hidden order, so that indices are not already sorted
    edges = [(int(perm[a]), int(perm[b])) for a in range(n) for b in range(a + 1, n) if rng.random() < p]
    if rng.random() < 0.5 and edges:
        edges.append(edges[0])                    # a duplicate edge counts once
    work = rng.uniform(0.5, 5.0, n)
    sizeparam = rng.uniform(0.0, 10.0, n)
    sizeout = rng.uniform(0.0, 6.0, n)
    return edges, work, sizeparam, sizeout


def test_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "mtpp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(mtpp_[a-z0-9_]+)\s*\(", text)))
    L = ctypes.CDLL(mtpp.LIB_PATH)
    assert names == sorted(mtpp.EXPORTS)
    for name in names:
        assert hasattr(L, name)


@pytest.mark.parametrize("seed", range(12))
def test_against_brute_force(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 10))
    edges, work, sp, so = random_dag(rng, n, float(rng.choice([0.15, 0.4, 0.8])))
    B, M = float(rng.uniform(0.5, 4.0)), float(rng.choice([0.0, 8.0, 30.0, 1e9]))
    order = mtpp.kahn_order(n, edges)
    assert order.tolist() == oracle.kahn_order(n, edges)
    for first in range(n):
        for last in range(first, n):
            want = oracle.block_cost(order[first:last + 1].tolist(), n, edges, work, sp, so, B, M)
            got = mtpp.block_cost(n, edges, work, sp, so, order, first, last, B, M)
            assert abs(got - want) <= 1e-12 * max(1.0, abs(want)), (first, last)
    for k in (1, 2, 3, n, n + 3):
        want, parts = oracle.slice_order(n, edges, work.tolist(), sp.tolist(), so.tolist(), k, B, M)
        got, ends = mtpp.slice_order(n, edges, work, sp, so, k, B, M)
        assert abs(got - want) <= 1e-12 * max(1.0, abs(want)), k
        # the blocks: a slicing of the order into at most k non-empty runs whose largest cost is the bottleneck
        assert 1 <= ends.size <= min(k, n) and ends[-1] == n and np.all(np.diff(np.concatenate([[0], ends])) > 0)
        starts = np.concatenate([[0], ends[:-1]])
        costs = [oracle.block_cost(order[a:b].tolist(), n, edges, work, sp, so, B, M) for a, b in zip(starts, ends)]
        assert abs(max(costs) - want) <= 1e-12 * max(1.0, abs(want))
        assert ends.size == len(parts)            # ties go to fewer blocks on both sides


def test_a_given_order_is_used_and_checked():
    edges = [(0, 1), (0, 2), (1, 3), (2, 3)]
    w, sp, so = [1.0, 2.0, 3.0, 4.0], [3.0, 5.0, 7.0, 2.0], [8.0, 4.0, 2.0, 1.0]
    for order in ([0, 1, 2, 3], [0, 2, 1, 3]):
        want, _ = oracle.slice_order(4, edges, w, sp, so, 2, 2.0, 10.0, order=order)
        got, ends = mtpp.slice_order(4, edges, w, sp, so, 2, 2.0, 10.0, order=order)
        assert got == want
    with pytest.raises(mtpp.MtppError):
        mtpp.slice_order(4, edges, w, sp, so, 2, 2.0, 10.0, order=[1, 0, 2, 3])      # 1 before its input 0
    with pytest.raises(mtpp.MtppError):
        mtpp.slice_order(4, edges, w, sp, so, 2, 2.0, 10.0, order=[0, 1, 1, 3])      # not a permutation
    with pytest.raises(mtpp.MtppError):
        mtpp.kahn_order(3, [(0, 1), (1, 2), (2, 0)])                                 # a cycle
    with pytest.raises(mtpp.MtppError):
        mtpp.slice_order(4, edges, w, sp, so, 0, 2.0, 10.0)                          # k < 1
    with pytest.raises(mtpp.MtppError):
        mtpp.slice_order(4, edges, w, sp, so, 2, 0.0, 10.0)                          # no bandwidth
    with pytest.raises(mtpp.MtppError):
        mtpp.slice_order(4, [(0, 7)], w, sp, so, 2, 2.0, 10.0)                       # edge to a missing operation


def test_a_layered_network_of_a_thousand_operations():
    # a transformer-like chain of blocks with skip connections: properties that hold at any size
    rng = np.random.default_rng(3)
    n = 1000
    edges = [(i, i + 1) for i in range(n - 1)] + [(i, i + 4) for i in range(0, n - 4, 4)]
    work = rng.uniform(1.0, 2.0, n)
    sp = rng.uniform(0.0, 4.0, n)
    so = rng.uniform(0.5, 1.0, n)
    B, M = 8.0, 64.0
    whole, _ = mtpp.slice_order(n, edges, work, sp, so, 1, B, M)
    order = mtpp.kahn_order(n, edges)
    assert order.tolist() == list(range(n))
    assert abs(whole - mtpp.block_cost(n, edges, work, sp, so, order, 0, n - 1, B, M)) < 1e-9
    prev = whole
    for k in (2, 4, 8, 16, 64):
        cost, ends = mtpp.slice_order(n, edges, work, sp, so, k, B, M)
        assert cost <= prev + 1e-12 and ends.size <= k and ends[-1] == n
        starts = np.concatenate([[0], ends[:-1]])
        costs = [mtpp.block_cost(n, edges, work, sp, so, order, int(a), int(b) - 1, B, M) for a, b in zip(starts, ends)]
        assert abs(max(costs) - cost) < 1e-9
        assert cost >= work.sum() / k                                # no slicing beats a perfect split of the work
        prev = cost
