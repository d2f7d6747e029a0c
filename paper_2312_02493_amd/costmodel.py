"""alpha-beta communication cost model and collective chooser (host-side, closed forms).

Follows the paper's Table "Bandwidth Complexity and Communication Cost of
Primitives" (Sec. II-A) and its communication-cost analysis of AR-Topk
(Sec. III-D): alpha is the latency in seconds, beta the seconds per byte
(1 / bandwidth), M the gradient size in bytes, N the number of workers, c the
compression ratio.  Logarithms are base 2.  This decides WHEN the compressor
step of this library is the right tool; it moves no data itself.
"""

from __future__ import annotations

import math


def _log2(n: int) -> float:
    return math.log2(n)


# ---- Table of primitives (Sec. II-A) --------------------------------------
def cost_ps(alpha: float, beta: float, m: float, n: int) -> float:
    return 2 * alpha + 2 * (n - 1) * m * beta


def cost_ring_allreduce(alpha: float, beta: float, m: float, n: int) -> float:
    return 2 * (n - 1) * alpha + 2 * (n - 1) / n * m * beta


def cost_tree_allreduce(alpha: float, beta: float, m: float, n: int) -> float:
    return 2 * alpha * _log2(n) + 2 * _log2(n) * m * beta


def cost_broadcast(alpha: float, beta: float, m: float, n: int) -> float:
    return alpha * _log2(n) + _log2(n) * m * beta


def cost_allgather(alpha: float, beta: float, m: float, n: int) -> float:
    return alpha * _log2(n) + (n - 1) * m * beta


# ---- compressed exchange (Sec. III-D) ---------------------------------------
def cost_topk_allgather(alpha: float, beta: float, m: float, n: int, c: float) -> float:
    """Values and indices of every worker (2*M*c bytes each) through AllGather."""
    return cost_allgather(alpha, beta, 2 * m * c, n)


def cost_artopk_ring(alpha: float, beta: float, m: float, n: int, c: float) -> float:
    """Broadcast of the leader's indices (M*c bytes) + ring all-reduce of the values."""
    return cost_broadcast(alpha, beta, m * c, n) + cost_ring_allreduce(alpha, beta, m * c, n)


def cost_artopk_tree(alpha: float, beta: float, m: float, n: int, c: float) -> float:
    """Broadcast of the leader's indices (M*c bytes) + tree all-reduce of the values."""
    return cost_broadcast(alpha, beta, m * c, n) + cost_tree_allreduce(alpha, beta, m * c, n)


# ---- the paper's three inequalities on alpha / beta --------------------------
def ring_beats_tree(alpha: float, beta: float, m: float, n: int, c: float) -> bool:
    """AR-Topk with ring reduction is cheaper than with tree reduction (needs N >= 3)."""
    lg = _log2(n)
    return alpha / beta < (lg - (n - 1) / n) / (n - 1 - lg) * m * c


def ring_beats_allgather(alpha: float, beta: float, m: float, n: int, c: float) -> bool:
    lg = _log2(n)
    return alpha / beta < (1 - 1 / n - lg / (2 * (n - 1))) * m * c


def tree_beats_allgather(alpha: float, beta: float, m: float, n: int, c: float) -> bool:
    lg = _log2(n)
    return alpha / beta < ((n - 1) / lg - 1.5) * m * c


def choose_collective(alpha: float, beta: float, m: float, n: int, c: float) -> str:
    """'AG', 'ART-Ring' or 'ART-Tree': the cheapest way to exchange the compressed update."""
    costs = {
        "AG": cost_topk_allgather(alpha, beta, m, n, c),
        "ART-Ring": cost_artopk_ring(alpha, beta, m, n, c),
        "ART-Tree": cost_artopk_tree(alpha, beta, m, n, c),
    }
    return min(costs, key=costs.get)
