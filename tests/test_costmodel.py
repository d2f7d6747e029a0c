"""The alpha-beta cost model: each inequality the paper derives (Sec. III-D) must agree with a
direct comparison of the two cost expressions it was derived from; single costs are checked
against values worked by hand from the table of primitives (Sec. II-A)."""

import math
import random

import pytest

from paper_2312_02493_amd import costmodel as cm


def test_hand_values():
    # N = 8 (log2 = 3), alpha = 1 ms, beta = 1 ns/byte, M = 1e6 bytes
    a, b, m, n = 1e-3, 1e-9, 1e6, 8
    assert cm.cost_ps(a, b, m, n) == pytest.approx(2e-3 + 14e-3)
    assert cm.cost_ring_allreduce(a, b, m, n) == pytest.approx(14e-3 + 1.75e-3)
    assert cm.cost_tree_allreduce(a, b, m, n) == pytest.approx(6e-3 + 6e-3)
    assert cm.cost_broadcast(a, b, m, n) == pytest.approx(3e-3 + 3e-3)
    assert cm.cost_allgather(a, b, m, n) == pytest.approx(3e-3 + 7e-3)
    # AR-Topk at c = 0.1: M*c = 1e5 bytes
    assert cm.cost_artopk_ring(a, b, m, n, 0.1) == pytest.approx(1e-3 * (14 + 3) + 1e-4 * (1.75 + 3))
    assert cm.cost_artopk_tree(a, b, m, n, 0.1) == pytest.approx(3 * 3e-3 + 3 * 3 * 1e-4)
    assert cm.cost_topk_allgather(a, b, m, n, 0.1) == pytest.approx(3e-3 + 2e-4 * 7)


def test_inequalities_match_direct_comparison():
    rng = random.Random(7)
    for _ in range(4000):
        n = rng.choice([3, 4, 5, 8, 16, 31, 64])
        alpha = 10 ** rng.uniform(-6, -1)
        beta = 10 ** rng.uniform(-11, -7)
        m = 10 ** rng.uniform(5, 10)
        c = 10 ** rng.uniform(-3, -1)
        ring, tree = cm.cost_artopk_ring(alpha, beta, m, n, c), cm.cost_artopk_tree(alpha, beta, m, n, c)
        ag = cm.cost_topk_allgather(alpha, beta, m, n, c)
        if abs(ring - tree) > 1e-9 * max(ring, tree):
            assert cm.ring_beats_tree(alpha, beta, m, n, c) == (ring < tree)
        if abs(ring - ag) > 1e-9 * max(ring, ag):
            assert cm.ring_beats_allgather(alpha, beta, m, n, c) == (ring < ag)
        if abs(tree - ag) > 1e-9 * max(tree, ag):
            assert cm.tree_beats_allgather(alpha, beta, m, n, c) == (tree < ag)
        assert cm.choose_collective(alpha, beta, m, n, c) == min(
            (ag, "AG"), (ring, "ART-Ring"), (tree, "ART-Tree"))[1]


def test_regimes():
    # high latency, small message: all-gather's single log(N) latency term wins
    assert cm.choose_collective(1e-1, 1e-9, 1e6, 8, 0.001) == "AG"
    # low latency, large message: the bandwidth-optimal ring wins
    assert cm.choose_collective(1e-6, 1e-9, 4e9, 8, 0.1) == "ART-Ring"
    assert math.isclose(cm.cost_artopk_tree(0.0, 1.0, 1.0, 2, 1.0), 3.0)
