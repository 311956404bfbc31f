"""Pins for the partitioning oracle: a chain with a closed form, the cost terms on a hand-worked diamond, and
properties that hold for every graph."""
import numpy as np

from oracle import mtpp


def test_kahn_order_smallest_ready_first():
    edges = [(3, 1), (3, 0), (0, 2), (1, 2), (4, 2)]
    assert mtpp.kahn_order(5, edges) == [3, 0, 1, 4, 2]
    assert mtpp.kahn_order(3, []) == [0, 1, 2]


def test_cost_terms_on_a_diamond_by_hand():
    # 0 -> 1, 0 -> 2, 1 -> 3, 2 -> 3; sizeout = [8, 4, 2, 1], B = 2, M = 10
    edges = [(0, 1), (0, 2), (1, 3), (2, 3)]
    so, sp, w = [8.0, 4.0, 2.0, 1.0], [3.0, 5.0, 7.0, 2.0], [1.0, 2.0, 3.0, 4.0]
    # block {1, 2}: input is operation 0's output, once although both consume it: 8 / 2 = 4
    assert mtpp.io({0, 3}, {1, 2}, edges, so, 2.0) == 4.0
    # its outputs go to 3: (4 + 2) / 2 = 3
    assert mtpp.io({1, 2}, {0, 3}, edges, so, 2.0) == 3.0
    # working sets: op 1: 4 + 8 = 12, op 2: 2 + 8 = 10 -> peak 12; parameters 12; overflow = (12 + 12 - 10) / 2 + 12 / 2 = 13
    assert mtpp.peak({1, 2}, edges, so) == 12.0
    assert mtpp.block_cost({1, 2}, 4, edges, w, sp, so, 2.0, 10.0) == 4.0 + 5.0 + 13.0 + 3.0
    # a block that fits in fast memory pays only peak / B as overflow: {3}: peak 1 + 4 + 2 = 7, parameters 2
    assert mtpp.block_cost({3}, 4, edges, w, sp, so, 2.0, 10.0) == 3.0 + 4.0 + 3.5 + 0.0


def test_chain_without_memory_pressure_has_a_closed_form():
    # a chain of equal operations, nothing to stream (huge M, zero-size tensors): f(S) = sum of work, and the best
    # slicing into at most k blocks is the most even one: ceil(n / k) operations in the largest block
    n = 9
    edges = [(i, i + 1) for i in range(n - 1)]
    for k in (1, 2, 3, 4, 9, 12):
        cost, parts = mtpp.slice_order(n, edges, [1.0] * n, [0.0] * n, [0.0] * n, k, 1.0, 1e9)
        assert cost == -(-n // min(k, n))
        assert [v for p in parts for v in p] == list(range(n)) and len(parts) <= k


def test_more_blocks_never_hurt_and_one_block_is_the_whole_graph():
    rng = np.random.default_rng(0)
    for trial in range(5):
        n = 8
        edges = [(u, v) for u in range(n) for v in range(u + 1, n) if rng.random() < 0.3]
        w, sp, so = rng.uniform(1, 5, n).tolist(), rng.uniform(0, 8, n).tolist(), rng.uniform(0, 4, n).tolist()
        costs = [mtpp.slice_order(n, edges, w, sp, so, k, 2.0, 12.0)[0] for k in (1, 2, 3, 4)]
        assert costs[0] == mtpp.block_cost(range(n), n, edges, w, sp, so, 2.0, 12.0)
        assert all(costs[i + 1] <= costs[i] for i in range(3))
        # every block of the best slicing is a run of the order, so no edge points backwards between blocks
        cost, parts = mtpp.slice_order(n, edges, w, sp, so, 3, 2.0, 12.0)
        where = {v: i for i, p in enumerate(parts) for v in p}
        assert all(where[u] <= where[v] for u, v in edges)
