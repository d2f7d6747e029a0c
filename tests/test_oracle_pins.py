"""Pins for the CPU oracle: every check here is independent of the oracle's own
formulas (brute force, hand-worked values, closed forms, library routines on
special cases, invariants).  A dropped term, a wrong sign, a wrong tie rule or
a transposed operand in the oracle fails at least one of them."""

import itertools
import math
import os

import numpy as np
import pytest

from oracle import artopk_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _bits(x):
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)


def _abs_key(v):
    """Magnitude ordering key computed without bit tricks (finite values)."""
    return abs(float(v))


# ---------------------------------------------------------------- golden trace
def _load_trace():
    d = {}
    with open(os.path.join(GOLDEN, "worked_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = line.split(":")
            d[key.strip()] = [float(t) for t in val.split()]
    return d


def test_hand_worked_trace_star():
    t = _load_trace()
    w, n, k = int(t["W"][0]), int(t["N"][0]), int(t["k"][0])
    res = [np.zeros(n, np.float32) for _ in range(w)]
    for s in (1, 2):
        g = [np.asarray(t[f"step{s}.g{r}"], np.float32) for r in range(w)]
        out = orc.step(g, res, k, orc.MODE_STAR, step_no=s, keep_acc=True)
        assert out.leader == int(t[f"step{s}.leader"][0])
        assert out.idx.tolist() == [int(v) for v in t[f"step{s}.idx"]]
        for r in range(w):
            assert out.vals[r].tolist() == t[f"step{s}.vals{r}"]
            assert out.residual[r].tolist() == t[f"step{s}.res{r}"]
            # residual zeros are +0.0, never -0.0
            assert not np.any(_bits(out.residual[r])[out.idx] != 0)
            if f"step{s}.acc{r}" in t:
                assert out.acc[r].tolist() == t[f"step{s}.acc{r}"]
        assert out.sum.tolist() == t[f"step{s}.sum"]
        assert out.update.tolist() == t[f"step{s}.update"]
        res = out.residual


def test_hand_worked_trace_var():
    t = _load_trace()
    n, k = int(t["N"][0]), int(t["k"][0])
    g = [np.asarray(t[f"step2.g{r}"], np.float32) for r in range(2)]
    res = [np.asarray(t[f"step1.res{r}"], np.float32) for r in range(2)]
    out = orc.step(g, res, k, orc.MODE_VAR, step_no=2)
    assert out.variances[0] == pytest.approx(t["step2.var0"][0], rel=1e-14)
    assert out.variances[1] == pytest.approx(t["step2.var1"][0], rel=1e-14)
    assert out.leader == 0
    assert out.idx.tolist() == [int(v) for v in t["step2.idx"]]
    assert out.sum.tolist() == t["step2.sum"]


def test_k_table():
    with open(os.path.join(GOLDEN, "k_table.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            n, rho, k = line.split()
            assert orc.k_from_ratio(float(rho), int(n)) == int(k)
    assert orc.k_from_ratio(0.5, 3) == 2
    assert orc.k_from_ratio(1e-9, 10) == 1
    assert orc.k_from_ratio(1.0, 10) == 10


# ---------------------------------------------------------------- Top-k pins
def _brute_rank_select(x, k):
    """Rank every element by counting who beats it; O(n^2), no sort."""
    n = len(x)
    sel = []
    for j in range(n):
        beat = 0
        for u in range(n):
            if _abs_key(x[u]) > _abs_key(x[j]) or (_abs_key(x[u]) == _abs_key(x[j]) and u < j):
                beat += 1
        if beat < k:
            sel.append(j)
    return sel


def _rand_small(rng, n):
    kind = rng.integers(0, 4)
    if kind == 0:
        x = rng.standard_normal(n)
    elif kind == 1:   # heavy ties, both signs, zeros of both signs
        x = rng.choice([-2.0, -1.0, -0.0, 0.0, 1.0, 2.0, 0.5, -0.5], n)
    elif kind == 2:   # all equal magnitude
        x = rng.choice([-3.25, 3.25], n)
    else:             # mostly distinct with a few planted duplicates
        x = rng.standard_normal(n)
        x[rng.integers(0, n)] = -x[rng.integers(0, n)]
    return x.astype(np.float32)


def test_topk_brute_force_rank():
    rng = np.random.default_rng(1)
    for _ in range(400):
        n = int(rng.integers(1, 21))
        x = _rand_small(rng, n)
        for k in {1, n, int(rng.integers(1, n + 1))}:
            assert orc.topk_indices(x, k).tolist() == _brute_rank_select(x, k)


def test_topk_subset_enumeration():
    """The unique size-k subset whose every member beats every non-member."""
    rng = np.random.default_rng(2)
    for _ in range(60):
        n = int(rng.integers(2, 11))
        x = _rand_small(rng, n)
        k = int(rng.integers(1, n + 1))

        def beats(a, b):
            return _abs_key(x[a]) > _abs_key(x[b]) or (_abs_key(x[a]) == _abs_key(x[b]) and a < b)

        good = [list(s) for s in itertools.combinations(range(n), k)
                if all(beats(a, b) for a in s for b in range(n) if b not in s)]
        assert len(good) == 1
        assert orc.topk_indices(x, k).tolist() == good[0]


def test_topk_distinct_equals_argpartition():
    rng = np.random.default_rng(3)
    x = rng.standard_normal(50_000).astype(np.float32)
    x = x[np.unique(np.abs(x), return_index=True)[1]]     # distinct magnitudes
    rng.shuffle(x)
    k = 777
    lib = np.sort(np.argpartition(-np.abs(x.astype(np.float64)), k - 1)[:k])
    assert np.array_equal(orc.topk_indices(x, k), lib)


def test_topk_invariants_and_certificate():
    rng = np.random.default_rng(4)
    x = (rng.standard_normal(200_000) * 1e-3).astype(np.float32)
    q = rng.random(x.size) < 0.3
    x[q] = (np.rint(x[q] * 1024) / 1024).astype(np.float32)   # many ties
    for k in (1, 17, 2000, 150_000, x.size):
        idx = orc.topk_indices(x, k)
        assert idx.size == k and idx.dtype == np.int32
        assert np.all(np.diff(idx.astype(np.int64)) > 0)
        mask = np.zeros(x.size, bool)
        mask[idx] = True
        if k < x.size:
            assert np.abs(x[mask]).min() >= np.abs(x[~mask]).max()
        ok, why = orc.topk_certificate(x, idx, k)
        assert ok, why


def test_certificate_rejects_wrong_sets():
    """The certificate is itself pinned: on tiny inputs it accepts exactly the
    brute-force answer and rejects every other size-k subset."""
    rng = np.random.default_rng(5)
    for _ in range(40):
        n = int(rng.integers(2, 9))
        x = _rand_small(rng, n)
        k = int(rng.integers(1, n + 1))
        truth = _brute_rank_select(x, k)
        for s in itertools.combinations(range(n), k):
            ok, _ = orc.topk_certificate(x, np.asarray(s, np.int32), k)
            assert ok == (list(s) == truth)


def test_magnitude_key_special_values():
    x = np.array([0.0, -0.0, 1e-45, -1e-45, 1.0, -1.0, np.inf, -np.inf], np.float32)
    k = orc.magnitude_keys(x)
    assert k[0] == k[1] == 0
    assert k[2] == k[3] == 1          # smallest denormal keeps its order
    assert k[4] == k[5] and k[6] == k[7] and k[6] > k[4] > k[2]
    # sign must not matter: -x ties with +x and the lower index wins
    y = np.array([-4.0, 4.0, 4.0, -4.0], np.float32)
    assert orc.topk_indices(y, 2).tolist() == [0, 1]


def test_segmented_topk_is_per_segment():
    rng = np.random.default_rng(6)
    x = rng.standard_normal(300).astype(np.float32)
    off = [0, 7, 8, 120, 300]
    ks = [3, 1, 10, 25]
    idx = orc.topk_indices_segmented(x, off, ks)
    pos = 0
    for s in range(4):
        want = [off[s] + j for j in _brute_rank_select(x[off[s]:off[s + 1]], ks[s])]
        assert idx[pos:pos + ks[s]].tolist() == want
        pos += ks[s]
    assert pos == idx.size


# ---------------------------------------------------------------- variance pins
def test_variance_library_and_closed_forms():
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(100_003) * 0.01 + 0.003).astype(np.float32)
    assert orc.variance(x) == pytest.approx(np.var(x.astype(np.float64)), rel=1e-13)
    assert orc.variance(np.full(1000, 3.5, np.float32)) == 0.0
    n = 4097
    ramp = np.arange(n, dtype=np.float32)
    assert orc.variance(ramp) == pytest.approx((n * n - 1) / 12.0, rel=1e-13)
    # shift invariance with an exactly representable shift
    y = np.arange(1024, dtype=np.float32)
    assert orc.variance(y + np.float32(4096.0)) == pytest.approx(orc.variance(y), rel=1e-13)
    # population, not sample: two points +-1 have variance 1, not 2
    assert orc.variance(np.array([1.0, -1.0], np.float32)) == 1.0


def test_leader_rules():
    assert [orc.leader_star(i, 4) for i in (1, 2, 3, 4, 5)] == [1, 2, 3, 0, 1]
    # every rank leads exactly once in W consecutive steps
    assert sorted(orc.leader_star(i, 8) for i in range(11, 19)) == list(range(8))
    assert orc.leader_var([1.0, 3.0, 3.0, 2.0]) == 1      # first maximum
    assert orc.leader_var([5.0]) == 0
    assert orc.leader_var([0.0, 0.0, 1e-30]) == 2


# ---------------------------------------------------------------- sum / EF pins
def test_ordered_sum_is_left_to_right():
    big = np.float32(2.0 ** 24)
    vals = np.array([[big], [1.0], [-big]], np.float32)
    assert orc.ordered_sum(vals)[0] == 0.0            # (2^24 + 1) - 2^24 = 0 in fp32
    assert orc.ordered_sum(vals[[0, 2, 1]])[0] == 1.0  # a different order differs
    assert np.array_equal(orc.ordered_sum(vals[:1]), vals[0])   # W = 1
    rng = np.random.default_rng(8)
    ints = rng.integers(-1000, 1000, (8, 500)).astype(np.float32)
    assert np.array_equal(orc.ordered_sum(ints), ints.astype(np.int64).sum(0).astype(np.float32))


def test_ef_add_is_single_fp32_add():
    g = np.array([1.0, 1e-8, 3.0, -0.0], np.float32)
    r = np.array([1e-8, 1.0, -3.0, 0.0], np.float32)
    acc = orc.ef_add(g, r)
    assert acc.dtype == np.float32
    assert acc.tolist() == [1.0, 1.0, 0.0, 0.0]
    assert _bits(acc)[3] == 0                          # -0 + +0 = +0
    z = np.zeros(5, np.float32)
    h = np.array([1.5, -2.0, 1e-40, 0.0, 7.0], np.float32)   # includes a denormal
    assert np.array_equal(_bits(orc.ef_add(h, z)), _bits(h))


def test_step_invariants_multi_step():
    rng = np.random.default_rng(9)
    w, n, k = 4, 5000, 50
    res = [np.zeros(n, np.float32) for _ in range(w)]
    led = []
    for s in range(1, 2 * w + 1):
        g = [(rng.standard_normal(n) * 0.01).astype(np.float32) for _ in range(w)]
        out = orc.step(g, res, k, orc.MODE_STAR, step_no=s, keep_acc=True)
        led.append(out.leader)
        for r in range(w):
            acc = np.add(g[r], res[r], dtype=np.float32)       # EF uses last step's residual
            assert np.array_equal(_bits(acc), _bits(out.acc[r]))
            sent = np.zeros(n, np.float32)
            sent[out.idx] = out.vals[r]
            # at every position exactly one of {sent, residual} carries acc's bits
            assert np.array_equal(_bits(np.add(sent, out.residual[r], dtype=np.float32)), _bits(acc))
            on = np.zeros(n, bool)
            on[out.idx] = True
            assert not _bits(out.residual[r])[on].any()
            assert np.array_equal(_bits(out.residual[r])[~on], _bits(acc)[~on])
            assert np.array_equal(out.vals[r], acc[out.idx])
        # the leader's own row holds magnitudes >= everything it left behind
        la = np.abs(out.acc[out.leader])
        off = np.ones(n, bool)
        off[out.idx] = False
        assert la[out.idx].min() >= la[off].max()
        assert not out.update[off].any()
        assert np.array_equal(out.update[out.idx], out.sum)
        res = out.residual
    assert led[:w] == [1, 2, 3, 0] and sorted(led[:w]) == list(range(w))


def test_step_k_equals_n_is_dense_ordered_allreduce():
    rng = np.random.default_rng(10)
    w, n = 3, 257
    g = [rng.standard_normal(n).astype(np.float32) for _ in range(w)]
    res = [np.zeros(n, np.float32) for _ in range(w)]
    out = orc.step(g, res, n, orc.MODE_FIXED, fixed_leader=2)
    dense = np.add(np.add(g[0], g[1], dtype=np.float32), g[2], dtype=np.float32)
    assert np.array_equal(out.update, dense)
    assert all(not r.any() for r in out.residual)


def test_var_mode_picks_largest_spread():
    rng = np.random.default_rng(11)
    n = 20000
    g = [(rng.standard_normal(n) * s).astype(np.float32) for s in (0.5, 2.0, 1.0)]
    res = [np.zeros(n, np.float32) for _ in range(3)]
    out = orc.step(g, res, 10, orc.MODE_VAR)
    assert out.leader == 1
    assert out.variances[1] == pytest.approx(np.var(g[1].astype(np.float64)), rel=1e-12)
    # selection was made on the leader: its row dominates its own leftovers
    assert np.array_equal(out.idx, orc.topk_indices(g[1], 10))


# ---------------------------------------------------------------- gain / sparse update pins
def test_gain_and_sparse_update_hand_values():
    t = _load_trace()
    acc0 = np.asarray(t["step1.g0"], np.float32)          # residual is zero at step 1
    idx = np.asarray(t["step1.idx"], np.int32)
    assert orc.compression_gain(acc0, idx) == pytest.approx(t["step1.gain0"][0], rel=1e-14)
    w_after = orc.apply_update(np.asarray(t["step1.w_before"], np.float32), idx,
                               np.asarray(t["step1.sum"], np.float32), t["step1.eta"][0])
    assert w_after.tolist() == t["step1.w_after"]


def test_gain_closed_forms():
    n = 1000
    x = np.where(np.arange(n) % 2 == 0, 2.0, -2.0).astype(np.float32)     # equal magnitudes
    for k in (1, 10, n):
        idx = orc.topk_indices(x, k)
        assert orc.compression_gain(x, idx) == pytest.approx(k / n, rel=1e-14)
    rng = np.random.default_rng(30)
    y = rng.standard_normal(5000).astype(np.float32)
    idx = orc.topk_indices(y, 50)
    g = orc.compression_gain(y, idx)
    kept = np.zeros_like(y)
    kept[idx] = y[idx]
    assert g == pytest.approx(np.linalg.norm(kept.astype(np.float64)) ** 2 / np.linalg.norm(y.astype(np.float64)) ** 2,
                              rel=1e-12)
    res = orc.residual_rewrite(y, idx)                     # gain from the step's outputs: V / (V + R)
    v = float((y[idx].astype(np.float64) ** 2).sum())
    r = float((res.astype(np.float64) ** 2).sum())
    assert g == pytest.approx(v / (v + r), rel=1e-12)
    assert 0.0 < g < 1.0 and orc.compression_gain(y, orc.topk_indices(y, 500)) > g   # grows with k


def test_sparse_update_equals_dense_update():
    rng = np.random.default_rng(31)
    n, k, eta = 4000, 77, 0.037
    w = rng.standard_normal(n).astype(np.float32)
    idx = np.sort(rng.choice(n, k, replace=False)).astype(np.int32)
    s = rng.standard_normal(k).astype(np.float32)
    dense = np.subtract(w, np.multiply(np.float32(eta), orc.scatter_update(n, idx, s), dtype=np.float32),
                        dtype=np.float32)
    assert np.array_equal(_bits(orc.apply_update(w, idx, s, eta)), _bits(dense))


def test_literal_alg1_leader_rule_hand_values():
    t = _load_trace()
    k = int(t["k"][0])
    g = [np.asarray(t[f"step2.g{r}"], np.float32) for r in range(2)]
    res = [np.asarray(t[f"step1.res{r}"], np.float32) for r in range(2)]
    out = orc.step(g, res, k, orc.MODE_VAR_TOPK, step_no=2)
    assert out.variances == [t["step2.topk_sqnorm0"][0], t["step2.topk_sqnorm1"][0]]
    assert out.leader == int(t["step2.topk_leader"][0])
    assert out.idx.tolist() == [int(v) for v in t["step2.topk_idx"]]
    assert out.sum.tolist() == t["step2.topk_sum"]
    # the squared norm of a worker's own Top-k is the largest any k-subset can have
    rng = np.random.default_rng(50)
    x = rng.standard_normal(12).astype(np.float32)
    best = max(float((x[list(s)].astype(np.float64) ** 2).sum()) for s in itertools.combinations(range(12), 4))
    assert orc.topk_sqnorm(x, orc.topk_indices(x, 4)) == pytest.approx(best, rel=1e-15)


# --------------------------------------------------------------------------
# 16-bit gradient storage: the widening is pinned by decoding the fields by hand
# --------------------------------------------------------------------------
def test_widen_f16_all_bit_patterns_against_field_decoding():
    bits = np.arange(1 << 16, dtype=np.uint32)
    sign = np.where(bits >> 15, -1.0, 1.0)
    e = (bits >> 10) & 0x1F
    m = (bits & 0x3FF).astype(np.float64)
    normal = sign * np.ldexp(1.0 + m / 1024.0, e.astype(np.int64) - 15)
    sub = sign * np.ldexp(m / 1024.0, -14)
    want = np.where(e == 0, sub, normal)
    got = orc.widen_gradient(bits.astype(np.uint16), "f16")
    finite = e != 31
    assert got.dtype == np.float32
    assert np.array_equal(got[finite].astype(np.float64), want[finite])       # exact, subnormals included
    assert np.array_equal(np.signbit(got[finite]), bits[finite] >> 15 == 1)   # -0.0 keeps its sign
    inf = (e == 31) & (bits & 0x3FF == 0)
    assert np.all(np.isinf(got[inf])) and np.array_equal(got[inf] < 0, bits[inf] >> 15 == 1)
    assert np.all(np.isnan(got[(e == 31) & (bits & 0x3FF != 0)]))


def test_widen_bf16_known_values_and_round_trip():
    known = {0x3F80: 1.0, 0xC000: -2.0, 0x0000: 0.0, 0x3DCC: 0.099609375, 0x7F80: np.inf, 0xFF80: -np.inf,
             0x0001: 2.0 ** -133, 0x0080: 2.0 ** -126, 0x7F7F: (2.0 - 2.0 ** -7) * 2.0 ** 127}
    b = np.array(list(known), dtype=np.uint16)
    got = orc.widen_gradient(b, "bf16")
    assert got.dtype == np.float32
    assert np.array_equal(got.astype(np.float64), np.array(list(known.values())))
    every = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    wide = orc.widen_gradient(every, "bf16")
    assert np.array_equal(wide.view(np.uint32) >> 16, every.astype(np.uint32))  # the bits are the upper half
    assert np.all(wide.view(np.uint32) & 0xFFFF == 0)                             # nothing is invented below


def test_raw_gradient_variance_rule_differs_from_the_error_fed_one():
    # worker 0: small gradient, large stale residual; worker 1: larger gradient, no residual.
    # The error-fed vector of worker 0 varies more, the raw gradient of worker 1 does.
    g = [np.array([0.1, -0.1, 0.1, -0.1], np.float32), np.array([1.0, -1.0, 1.0, -1.0], np.float32)]
    res = [np.array([5.0, -5.0, 0.0, 0.0], np.float32), np.zeros(4, np.float32)]
    a = orc.step(g, res, 1, orc.MODE_VAR)
    b = orc.step(g, res, 1, orc.MODE_VAR_G)
    assert a.leader == 0 and b.leader == 1
    # population variances by hand: g0 -> 0.01, g1 -> 1 (float32 0.1 is not exact, hence the tolerance)
    assert abs(b.variances[0] - 0.01) < 1e-8 and b.variances[1] == 1.0
    # everything after the leader choice is the same machinery: index of the largest |acc| of the leader
    assert list(a.idx) == [0] and list(b.idx) == [0]
    assert a.sum[0] == np.float32(np.float32(0.1) + np.float32(5.0)) + np.float32(1.0)
