"""CPU oracle for one AR-Topk compressor step with error feedback.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition of what
the GPU library must compute.  Nothing in the product path may import it; only
the tests, the smoke check and the benchmark's CPU-baseline leg do.  It shares
no code with the HIP kernels and imports nothing from them.

Everything here is single-threaded NumPy written straight from the method's
definition:

* error feedback                 -- Sec. II-C, error-feedback equations
* Top-k by magnitude, k entries  -- Sec. II-C (top k% with values + indices),
                                    Sec. III-A, Alg. 1 (Topk call)
* leader choice STAR / VAR       -- Sec. III-B, Alg. 1 (worker selection branch)
* gather at the shared indices   -- Alg. 1 (indexing G with the broadcast ix)
* residual rewrite               -- Alg. 1 (residual = G - g~), EF equations
* reduction of the k values      -- Alg. 1 (AllReduce), here a sum over the
                                    workers in rank order 0..W-1
* dense update                   -- Alg. 1 (model update consumes g~ on the
                                    full parameter vector)
* 16-bit gradient storage        -- not in the paper: a gradient stored as
                                    bfloat16 / float16 is widened exactly to
                                    float32 and the step above applies

Readings taken where the paper leaves a choice open (each also listed in the
design notes of the repository):

* "variance" of a worker is the population variance (divide by n) of its
  dense error-fed vector, accumulated in float64 in two passes (MODE_VAR_G
  takes it of the raw gradient instead; MODE_VAR_TOPK is Alg. 1's printed
  squared norm of the worker's own Top-k values);
* Top-k ranks by |value| using the raw 31 magnitude bits, ties go to the
  lowest index, and the k indices are reported in ascending order;
* the VAR leader is the first (lowest-rank) worker attaining the maximum;
* the reduced value is a plain sum (no 1/W), float32, added in rank order;
* a selected position of a residual becomes +0.0, every other position keeps
  the bits of the error-fed gradient.

All functions are pinned by tests that do not re-use these formulas: brute
force ranking and subset enumeration on tiny inputs, a hand-worked example,
closed forms for the variance, a cancellation triple for the summation order,
library routines on special cases.  Nothing here is "parity unpinned".
"""

from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

MODE_STAR = 0
MODE_VAR = 1
MODE_FIXED = 2
MODE_VAR_TOPK = 3
MODE_VAR_G = 4

_MAG_MASK = np.uint32(0x7FFFFFFF)


# --------------------------------------------------------------------------
# Gradients stored in 16 bits: exact widening to float32 before anything else
# --------------------------------------------------------------------------
def widen_gradient(bits16: np.ndarray, kind: str) -> np.ndarray:
    """float32 values of 16-bit gradient storage given as uint16 bit patterns.

    'bf16': the 16 bits are the upper half of the float32 (sign, 8 exponent
    bits, 7 mantissa bits), the lower half is zero.  'f16': IEEE binary16,
    every value of which (subnormals included) is a float32 value; NumPy's
    conversion is used as the step.
    """
    b = np.ascontiguousarray(bits16, dtype=np.uint16)
    if kind == "bf16":
        return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)
    if kind == "f16":
        return b.view(np.float16).astype(np.float32)
    raise ValueError("kind must be 'bf16' or 'f16'")


# --------------------------------------------------------------------------
# k from the compression ratio  (Sec. II-C: ceil(k*G/100) values and indices)
# --------------------------------------------------------------------------
def k_from_ratio(rho: float, n: int) -> int:
    """Number of kept entries for keep-fraction ``rho`` of ``n`` elements.

    One IEEE double multiply followed by a ceiling, clamped to [1, n].
    """
    k = int(math.ceil(float(rho) * float(n)))
    return max(1, min(int(n), k))


# --------------------------------------------------------------------------
# error feedback  (Sec. II-C, first EF equation; Alg. 1, first loop line)
# --------------------------------------------------------------------------
def ef_add(g: np.ndarray, residual: np.ndarray) -> np.ndarray:
    """acc = g + residual, one float32 addition per element."""
    g = np.asarray(g, dtype=np.float32)
    residual = np.asarray(residual, dtype=np.float32)
    return np.add(g, residual, dtype=np.float32)


# --------------------------------------------------------------------------
# leader choice  (Sec. III-B; Alg. 1 worker-selection branch)
# --------------------------------------------------------------------------
def variance(x: np.ndarray) -> float:
    """Population variance of a float32 vector, float64, two passes."""
    xd = np.asarray(x, dtype=np.float32).astype(np.float64)
    n = xd.size
    mean = float(xd.sum() / n)          # pass 1
    dev = xd - mean
    return float((dev * dev).sum() / n)  # pass 2


def topk_sqnorm(acc: np.ndarray, idx: np.ndarray) -> float:
    """Squared 2-norm (float64) of the values a worker's own Top-k keeps -- the
    scalar Alg. 1 writes into var[r] for the VAR-Topk leader choice."""
    v = np.asarray(acc, np.float32)[np.asarray(idx, np.int64)].astype(np.float64)
    return float((v * v).sum())


def leader_star(step: int, w: int) -> int:
    """Round-robin leader: the step counter modulo the number of workers."""
    return int(step) % int(w)


def leader_var(variances: Sequence[float]) -> int:
    """First worker (lowest rank) whose variance equals the maximum."""
    best = 0
    for r in range(1, len(variances)):
        if variances[r] > variances[best]:
            best = r
    return best


# --------------------------------------------------------------------------
# Top-k by magnitude  (Sec. II-C, Sec. III-A, Alg. 1 Topk call)
# --------------------------------------------------------------------------
def magnitude_keys(x: np.ndarray) -> np.ndarray:
    """The 31 magnitude bits of every float32 as an unsigned integer.

    For finite values the integer order of these keys equals the order of the
    absolute values; +x and -x share a key, and so do +0.0 and -0.0.
    """
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return bits & _MAG_MASK


def topk_indices(acc: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest |acc|, lowest index first among equal keys.

    Full stable sort on "how far below the largest possible key" so that equal
    keys stay in index order; the first k of that order are the winners and
    are returned sorted ascending (int32).
    """
    n = acc.size
    if not (1 <= k <= n):
        raise ValueError("k out of range")
    keys = magnitude_keys(acc)
    descending = (_MAG_MASK - keys)
    order = np.argsort(descending, kind="stable")
    winners = np.sort(order[:k])
    return winners.astype(np.int32)


def topk_indices_segmented(acc: np.ndarray, seg_off: Sequence[int],
                           seg_k: Sequence[int]) -> np.ndarray:
    """Layer-wise selection: an independent Top-k inside every segment.

    ``seg_off`` has one more entry than there are segments; segment s covers
    [seg_off[s], seg_off[s+1]) and contributes seg_k[s] global indices.  The
    concatenation in segment order is ascending.
    """
    out: List[np.ndarray] = []
    for s in range(len(seg_k)):
        lo, hi = int(seg_off[s]), int(seg_off[s + 1])
        local = topk_indices(acc[lo:hi], int(seg_k[s]))
        out.append((local.astype(np.int64) + lo).astype(np.int32))
    return np.concatenate(out) if out else np.zeros(0, np.int32)


# --------------------------------------------------------------------------
# gather, ordered sum, scatter, residual  (Alg. 1, lines after the Broadcast)
# --------------------------------------------------------------------------
def gather(accs: Sequence[np.ndarray], idx: np.ndarray) -> np.ndarray:
    """vals[w][m] = acc_w[idx[m]] for every worker."""
    return np.stack([np.asarray(a, np.float32)[idx] for a in accs], axis=0)


def ordered_sum(vals: np.ndarray) -> np.ndarray:
    """Float32 sum over workers taken strictly in rank order 0, 1, ..., W-1."""
    total = vals[0].astype(np.float32, copy=True)
    for w in range(1, vals.shape[0]):
        total = np.add(total, vals[w], dtype=np.float32)
    return total


def scatter_update(n: int, idx: np.ndarray, summed: np.ndarray) -> np.ndarray:
    """Dense update: zero everywhere except update[idx[m]] = summed[m]."""
    update = np.zeros(n, dtype=np.float32)
    update[idx] = summed
    return update


def residual_rewrite(acc: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """New residual: acc with the communicated positions set to +0.0."""
    res = np.array(acc, dtype=np.float32, copy=True)
    res[idx] = np.float32(0.0)
    return res


# --------------------------------------------------------------------------
# one whole step  (Alg. 1 loop body, W workers side by side)
# --------------------------------------------------------------------------
class StepResult:
    __slots__ = ("leader", "variances", "idx", "vals", "sum", "update",
                 "residual", "acc")

    def __init__(self):
        self.leader = -1
        self.variances: Optional[List[float]] = None
        self.idx = None
        self.vals = None
        self.sum = None
        self.update = None
        self.residual = None
        self.acc = None


def step(g: Sequence[np.ndarray], residual: Sequence[np.ndarray], k: int,
         mode: int, step_no: int = 0, fixed_leader: int = 0,
         seg_off: Optional[Sequence[int]] = None,
         seg_k: Optional[Sequence[int]] = None,
         keep_acc: bool = False) -> StepResult:
    """One AR-Topk step for W simulated workers.

    ``g`` and ``residual`` are W float32 vectors of equal length.  With
    ``seg_off``/``seg_k`` the selection is per segment (one leader for the
    whole concatenation); otherwise ``k`` entries of the whole vector are kept.
    """
    w = len(g)
    n = int(np.asarray(g[0]).size)
    out = StepResult()

    accs = [ef_add(g[r], residual[r]) for r in range(w)]

    if mode == MODE_STAR:
        out.leader = leader_star(step_no, w)
    elif mode == MODE_VAR:
        out.variances = [variance(a) for a in accs]
        out.leader = leader_var(out.variances)
    elif mode == MODE_VAR_G:
        # the other reading of "largest gradient variance" (Sec. III-B): the variance of the
        # raw gradient, before the residual is added
        out.variances = [variance(np.asarray(x, dtype=np.float32)) for x in g]
        out.leader = leader_var(out.variances)
    elif mode == MODE_VAR_TOPK:
        # Alg. 1 as printed: Topk on every worker first, the squared norm of each
        # worker's own k values decides the leader (first maximum)
        own = [topk_indices(a, k) for a in accs]
        out.variances = [topk_sqnorm(a, i) for a, i in zip(accs, own)]
        out.leader = leader_var(out.variances)
    elif mode == MODE_FIXED:
        out.leader = int(fixed_leader)
    else:
        raise ValueError("unknown mode")

    lead_acc = accs[out.leader]
    if seg_off is not None:
        out.idx = topk_indices_segmented(lead_acc, seg_off, seg_k)
    else:
        out.idx = topk_indices(lead_acc, k)

    out.vals = gather(accs, out.idx)
    out.sum = ordered_sum(out.vals)
    out.update = scatter_update(n, out.idx, out.sum)
    out.residual = [residual_rewrite(a, out.idx) for a in accs]
    if keep_acc:
        out.acc = accs
    return out


# --------------------------------------------------------------------------
# neighbours of the step: compression gain and the sparse model update
# --------------------------------------------------------------------------
def compression_gain(acc: np.ndarray, idx: np.ndarray) -> float:
    """||g_c||^2 / ||g_e||^2 for one worker (Sec. II-C, statistical efficiency
    of compression): g_e is the error-fed gradient ``acc``, g_c keeps only the
    communicated positions.  float64 sums of squares."""
    a = np.asarray(acc, dtype=np.float32).astype(np.float64)
    kept = a[np.asarray(idx, dtype=np.int64)]
    total = float((a * a).sum())
    return float((kept * kept).sum()) / total if total > 0.0 else 0.0


def apply_update(weights: np.ndarray, idx: np.ndarray, summed: np.ndarray, eta: float) -> np.ndarray:
    """Alg. 1 model update restricted to the communicated positions:
    w[idx] = w[idx] - eta * g~ in float32 (product rounded, then difference)."""
    w = np.array(weights, dtype=np.float32, copy=True)
    i = np.asarray(idx, dtype=np.int64)
    step = np.multiply(np.float32(eta), np.asarray(summed, np.float32), dtype=np.float32)
    w[i] = np.subtract(w[i], step, dtype=np.float32)
    return w


# --------------------------------------------------------------------------
# O(n) uniqueness certificate for a claimed Top-k index set
# --------------------------------------------------------------------------
def topk_certificate(acc: np.ndarray, idx: np.ndarray, k: int) -> Tuple[bool, str]:
    """Decide in O(n) whether ``idx`` is THE Top-k set of ``acc``.

    Exactly one size-k set S satisfies: with T the smallest key inside S, every
    key above T lies in S, and among keys equal to T the members of S are the
    ones with the lowest indices.  Checking those conditions (plus size, order
    and range) is therefore the same as comparing with the full-sort answer,
    without sorting n elements.
    """
    n = acc.size
    idx = np.asarray(idx)
    if idx.size != k:
        return False, "wrong count"
    if k == 0:
        return True, ""
    idx64 = idx.astype(np.int64)
    if idx64[0] < 0 or idx64[-1] >= n:
        return False, "index out of range"
    if k > 1 and not bool(np.all(idx64[1:] > idx64[:-1])):
        return False, "not strictly ascending"
    keys = magnitude_keys(acc)
    sel_keys = keys[idx64]
    t = sel_keys.min()
    n_above = int(np.count_nonzero(keys > t))
    n_above_in = int(np.count_nonzero(sel_keys > t))
    if n_above != n_above_in:
        return False, "a key above the threshold is missing"
    eq_in = idx64[sel_keys == t]
    if n_above + eq_in.size != k:
        return False, "count mismatch"
    # members at the threshold must be exactly the first eq_in.size equals
    eq_all = np.flatnonzero(keys == t)
    if not np.array_equal(eq_all[:eq_in.size], eq_in):
        return False, "ties not taken lowest-index first"
    return True, ""
