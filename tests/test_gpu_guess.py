"""GPU parity of the selection route that samples a threshold guess before the
fused pass (Sec. III-B leaves the Top-k method open; every route must give the
oracle's result bit for bit).

On long vectors the library samples each worker's g + residual, guesses a
lower bound on the key of the k-th largest magnitude, lets the fused pass mark
the elements that reach it, and builds the survivor list from the marks.  The
guess can be wrong in both directions; then the library must notice and take
the full route.  The route is switched on here for short vectors through the
library's option ARTOPK_OPT_GUESS_MIN_N (artopk_set_option).
"""

import math

import numpy as np
import pytest

import artopk_inputs as inp
from oracle import artopk_oracle as orc
from tests import gpu_util
from tests.gpu_util import GpuRunner, assert_step_matches, top_two_gap

pytestmark = pytest.mark.gpu


@pytest.fixture(params=["pieces", "mask_only"])
def guess_on(monkeypatch, request):
    """The guess route on short vectors, in both of its forms for a leader known up front: the
    fused pass hands the marked elements on tile by tile (the default), or leaves only the mask."""
    monkeypatch.setitem(gpu_util.OPTIONS, "guess_min_n", 4096)
    monkeypatch.setitem(gpu_util.OPTIONS, "stage_tiles", 2 if request.param == "pieces" else 0)


def _sample_positions(n):
    """The elements the library samples: `runs` runs of 16 consecutive elements."""
    runs = min(16384, n // 64)
    stride = n // runs
    starts = (np.arange(runs, dtype=np.int64) * stride) & ~np.int64(15)
    return (starts[:, None] + np.arange(16, dtype=np.int64)[None, :]).ravel()


def _m_hi(n, k):
    runs = min(16384, n // 64)
    expect = k * (runs * 16) / n
    return int(math.ceil(expect + 6.0 * math.sqrt(expect) + 8.0))


def _run_steps(runner, gen, w, n, k, mode, steps, expect_mask, fixed_leader=0):
    res = [np.zeros(n, dtype=np.float32) for _ in range(w)]
    for step_no in range(1, steps + 1):
        g = [gen(step_no, r) for r in range(w)]
        want = orc.step(g, res, k, mode, step_no=step_no, fixed_leader=fixed_leader)
        if mode == orc.MODE_VAR:
            assert top_two_gap(want.variances) > 1e-4
        runner.load_g(g)
        got = runner.step(k, mode, step_no, fixed_leader=fixed_leader)
        info = runner.ctx.select_info()
        assert gpu_util.FORCED or (info["guessed"] == 1), info
        if expect_mask is not None:
            want_mask = expect_mask[step_no - 1] if isinstance(expect_mask, (list, tuple)) else expect_mask
            assert gpu_util.FORCED or (info["from_mask"] == want_mask), (step_no, info)
        assert_step_matches(got, want, mode)
        res = want.residual


@pytest.mark.parametrize("rho", [0.01, 0.001])
def test_guess_star_three_steps_with_ragged_tail(guess_on, rho):
    n, w = (1 << 20) + 3, 4
    wl = inp.workload(1, n=n, w=w)
    k = wl.k(rho)
    runner = GpuRunner(w, n, k)
    _run_steps(runner, lambda s, r: wl.gen(s, r), w, n, k, orc.MODE_STAR, 3, expect_mask=1)


def test_guess_var_workers_of_different_scale(guess_on):
    n, w = 1_500_001, 8
    wl = inp.workload(2, n=n, w=w)
    k = wl.k(0.01)
    runner = GpuRunner(w, n, k)
    _run_steps(runner, lambda s, r: wl.gen(s, r), w, n, k, orc.MODE_VAR, 3, expect_mask=1)


def test_guess_var_leader_changes_every_step(guess_on):
    n, w = 600_000, 4
    wl = inp.workload(1, n=n, w=w)
    k = wl.k(0.01)
    runner = GpuRunner(w, n, k)

    def gen(step_no, r):
        scale = np.float32(3.0 if r == (step_no * 3) % w else 1.0)
        return wl.gen(step_no, r) * scale

    _run_steps(runner, gen, w, n, k, orc.MODE_VAR, 4, expect_mask=1)


def test_guess_sample_too_small_for_a_bound(guess_on):
    # k so close to n / 32 that the wanted sample rank still fits, on a vector barely long enough
    # to be sampled: exercises the route where a slot may end up without a bound
    n, w = 16_384, 2
    wl = inp.workload(1, n=n, w=w)
    k = n // 32
    runner = GpuRunner(w, n, k)
    _run_steps(runner, lambda s, r: wl.gen(s, r), w, n, k, orc.MODE_STAR, 2, expect_mask=None)


def test_guess_heavy_tails_fixed_leader(guess_on):
    n, w = 3_000_000, 3
    wl = inp.workload(4, n=n, w=w)
    k = wl.k(0.001)
    runner = GpuRunner(w, n, k)
    _run_steps(runner, lambda s, r: wl.gen(s, r), w, n, k, orc.MODE_FIXED, 2, expect_mask=1, fixed_leader=2)


def test_guess_ties_on_the_threshold(guess_on):
    # a tenth of the values lie on a coarse grid; k is put inside a plateau so the tie rule decides
    n, w = 2_000_000, 2
    wl = inp.workload(5, n=n, w=w)
    g0 = wl.gen(1, 1)  # the leader of step 1
    key = g0.view(np.uint32) & np.uint32(0x7FFFFFFF)
    q = np.float32(3.0 / 1024.0).view(np.uint32)
    above, equal = int((key > q).sum()), int((key == q).sum())
    assert equal >= 4
    k = above + equal // 2
    assert k * 32 <= n
    runner = GpuRunner(w, n, k)
    _run_steps(runner, lambda s, r: wl.gen(s, r), w, n, k, orc.MODE_STAR, 1, expect_mask=None)


def test_guess_too_high_takes_the_full_route(guess_on):
    # large values sit only on sampled elements, enough of them to lift the guess above the
    # true threshold, but fewer than k in the whole vector
    n, w, k = 1 << 20, 2, 10_000
    rng = np.random.default_rng(11)
    pos = _sample_positions(n)
    m_hi = _m_hi(n, k)
    assert m_hi + 64 < k

    def gen(step_no, r):
        x = (1e-6 * rng.standard_normal(n)).astype(np.float32)
        x[pos[: m_hi + 64]] = np.float32(1.0) + np.arange(m_hi + 64, dtype=np.float32) * np.float32(1e-3)
        return x

    runner = GpuRunner(w, n, k)
    _run_steps(runner, gen, w, n, k, orc.MODE_STAR, 2, expect_mask=0)


def test_guess_too_low_list_over_capacity(guess_on):
    # two magnitudes only: the guessed bound admits 60 % of the vector, far beyond the list
    n, w, k = 1 << 20, 2, 5_000
    rng = np.random.default_rng(12)

    def gen(step_no, r):
        x = np.where(rng.random(n) < 0.6, 1.0, 0.5).astype(np.float32)
        x *= np.where(rng.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
        return x

    runner = GpuRunner(w, n, k)
    _run_steps(runner, gen, w, n, k, orc.MODE_STAR, 1, expect_mask=0)


def test_guess_all_equal_vector(guess_on):
    n, w, k = 300_000, 2, 1_000
    runner = GpuRunner(w, n, k)
    _run_steps(runner, lambda s, r: np.full(n, 0.25, dtype=np.float32), w, n, k, orc.MODE_STAR, 1, expect_mask=0)


def test_guess_marks_in_the_elements_behind_the_last_group(guess_on):
    n, w, k = (1 << 19) + 3, 2, 600
    rng = np.random.default_rng(13)

    def gen(step_no, r):
        x = (1e-2 * rng.standard_normal(n)).astype(np.float32)
        x[-3:] = np.array([5.0, -7.0, 6.0], dtype=np.float32)
        return x

    runner = GpuRunner(w, n, k)
    _run_steps(runner, gen, w, n, k, orc.MODE_STAR, 2, expect_mask=1)


def test_guess_infinities_and_nans_are_the_largest(guess_on):
    n, w, k = 1 << 18, 2, 300
    rng = np.random.default_rng(14)

    def gen(step_no, r):
        x = rng.standard_normal(n).astype(np.float32)
        x[1000:1300:3] = np.float32(np.inf)
        x[5000:5100:2] = np.float32(-np.inf)
        return x

    runner = GpuRunner(w, n, k)
    _run_steps(runner, gen, w, n, k, orc.MODE_STAR, 1, expect_mask=None)


def test_guess_is_off_for_short_vectors_by_default():
    n, w = 1 << 20, 2
    wl = inp.workload(1, n=n, w=w)
    k = wl.k(0.01)
    runner = GpuRunner(w, n, k)
    g = [wl.gen(1, r) for r in range(w)]
    runner.load_g(g)
    runner.step(k, orc.MODE_STAR, 1)
    assert gpu_util.FORCED or (runner.ctx.select_info()["guessed"] == 0)


def test_guess_literal_leader_rule_every_worker_selects_from_its_mask(guess_on):
    """Alg. 1 as printed (every worker runs Top-k, the largest squared norm of the own k values
    leads) on the guess route: every worker's list comes from its own mask."""
    n, w = 400_003, 5
    wl = inp.workload(2, n=n, w=w)
    k = wl.k(0.01)
    runner = GpuRunner(w, n, k)
    _run_steps(runner, lambda s, r: wl.gen(s, r), w, n, k, orc.MODE_VAR_TOPK, 3, expect_mask=1)


@pytest.mark.parametrize("mode", ["star", "var"])
def test_guess_kept_elements_clustered_in_two_tiles(guess_on, mode):
    """All large magnitudes sit in one stretch across a tile border of the fused pass: most tiles
    mark nothing, two mark thousands, and the sample sees the stretch in a few of its runs only."""
    n, w, k = 40 * 32768 + 3, 4, 5_000
    rng = np.random.default_rng(22)

    def gen(step_no, r):
        x = (1e-3 * (1.0 + 0.3 * r) * rng.standard_normal(n)).astype(np.float32)
        lo = 18 * 32768 - 2500
        x[lo:lo + 5200] = (1.0 + rng.random(5200)).astype(np.float32)
        return x

    runner = GpuRunner(w, n, k)
    _run_steps(runner, gen, w, n, k, orc.MODE_STAR if mode == "star" else orc.MODE_VAR, 2, expect_mask=None)


@pytest.mark.parametrize("n", [16_384, 32_768, 32_769, 3 * 32_768 + 2, 9 * 32_768 - 1, 17 * 32_768 + 131])
def test_guess_pieces_ragged_lengths(guess_on, n):
    """Vector lengths around the tile and slab borders of the staged pieces (a slab is eight tiles)."""
    w = 2
    wl = inp.workload(1, n=n, w=w)
    k = max(1, n // 200)
    runner = GpuRunner(w, n, k)
    _run_steps(runner, lambda s, r: wl.gen(s, r), w, n, k, orc.MODE_STAR, 2, expect_mask=None)


@pytest.mark.parametrize("rho", [0.1, 0.05])
def test_guess_pieces_dense_keep(guess_on, rho):
    """One element in ten kept: with the pieces the guess route also serves selections this dense
    (without them it stands back for the histogram route)."""
    n, w = 1_200_003, 3
    wl = inp.workload(4, n=n, w=w)
    k = wl.k(rho)
    runner = GpuRunner(w, n, k)
    res = [np.zeros(n, dtype=np.float32) for _ in range(w)]
    for step_no in (1, 2, 3):
        g = [wl.gen(step_no, r) for r in range(w)]
        want = orc.step(g, res, k, orc.MODE_STAR, step_no=step_no)
        runner.load_g(g)
        got = runner.step(k, orc.MODE_STAR, step_no)
        info = runner.ctx.select_info()
        staged = gpu_util.OPTIONS["stage_tiles"] != 0
        assert gpu_util.FORCED or (info["guessed"] == (1 if staged else 0)), info
        if staged:
            assert gpu_util.FORCED or (info["from_mask"] == 1), info
        assert_step_matches(got, want, orc.MODE_STAR)
        res = want.residual


@pytest.mark.parametrize("where", ["one_tile_overflows", "every_eighth_tile_overflows", "all_in_last_tile"])
def test_guess_pieces_tiles_with_more_marks_than_a_piece_holds(guess_on, where):
    """Tiles whose marks exceed the piece size report an overflow and their slab is built from the
    mask, next to slabs built from pieces."""
    n, w, k = 37 * 32768 + 77, 2, 6_000
    rng = np.random.default_rng(31)

    def gen(step_no, r):
        x = (1e-3 * rng.standard_normal(n)).astype(np.float32)
        big = lambda m: ((1.0 + rng.random(m)) * np.where(rng.random(m) < 0.5, -1.0, 1.0)).astype(np.float32)
        if where == "one_tile_overflows":
            lo = 9 * 32768 + 100
            x[lo:lo + 4000] = big(4000)
            x[::997] = big(len(x[::997]))
        elif where == "every_eighth_tile_overflows":
            for t in range(3, 37, 8):
                x[t * 32768 + 5: t * 32768 + 1505] = big(1500)
        else:
            x[36 * 32768 + 10: 36 * 32768 + 5010] = big(5000)
            x[n - 2] = np.float32(9.0)
        return x

    runner = GpuRunner(w, n, k)
    _run_steps(runner, gen, w, n, k, orc.MODE_STAR, 2, expect_mask=None)
