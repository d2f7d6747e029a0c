"""GPU parity: the HIP path, called through the C ABI binding, against the CPU
oracle on the same seeded inputs -- bit-exact for indices, gathered values,
ordered sums, updates and residuals; variance within 1e-5 relative."""

import numpy as np
import pytest

import artopk_inputs as inp
from oracle import artopk_oracle as orc
from tests import gpu_util
from tests.gpu_util import GpuRunner, assert_step_matches, bits, top_two_gap

pytestmark = pytest.mark.gpu

VAR_GAP = 1e-4   # leader must agree wherever the top two variances differ by more


def _run_workload(wl, rho, steps, n_print=True):
    k = wl.k(rho)
    seg_off = None if wl.seg_off is None else [int(v) for v in wl.seg_off]
    seg_k = None if wl.seg_off is None else [int(v) for v in wl.seg_k(rho)]
    run = GpuRunner(wl.w, wl.n, k, max_segments=1 if seg_k is None else len(seg_k))
    res = [np.zeros(wl.n, np.float32) for _ in range(wl.w)]
    mode = orc.MODE_STAR if wl.mode == inp.MODE_STAR else orc.MODE_VAR
    for s in range(1, steps + 1):
        g = [wl.gen(s, r) for r in range(wl.w)]
        want = orc.step(g, res, k, mode, step_no=s, seg_off=seg_off, seg_k=seg_k)
        if mode == orc.MODE_VAR:
            assert top_two_gap(want.variances) > VAR_GAP, "generator must keep the variance gap"
        run.load_g(g)
        got = run.step(k, mode, s, seg_off=seg_off, seg_k=seg_k)
        print(f"[{wl.name}] n={wl.n} rho={rho} step={s} leader={want.leader} k={k}", flush=True)
        assert_step_matches(got, want, mode)
        res = want.residual


def test_c1_full_star_three_steps():
    _run_workload(inp.workload(1), 0.01, 3)


@pytest.mark.parametrize("rho", [0.01, 0.001])
def test_c2_shrunk_var(rho):
    _run_workload(inp.workload(2, n=1_000_003), rho, 4)


def test_c3_shrunk_segmented_var():
    wl = inp.workload(3, n=600_000)
    _run_workload(wl, 0.01, 3)


@pytest.mark.parametrize("rho", [0.1, 0.01, 0.001])
def test_c4_shrunk_star(rho):
    _run_workload(inp.workload(4, n=2_000_006), rho, 5)


def test_c5_shrunk_var_with_ties():
    _run_workload(inp.workload(5, n=3_000_001), 0.001, 3)


def test_c5_tie_plateau_threshold():
    """k chosen so that the threshold falls inside a plateau of equal keys."""
    wl = inp.workload(5, n=2_500_000, w=3)
    g = [wl.gen(1, r) for r in range(3)]
    q = np.float32(3.0 / 1024.0)
    keys = orc.magnitude_keys(g[1])
    qk = orc.magnitude_keys(np.array([q], np.float32))[0]
    n_eq = int((keys == qk).sum())
    assert n_eq > 10
    k = int((keys > qk).sum()) + n_eq // 2
    run = GpuRunner(3, wl.n, k)
    run.load_g(g)
    res = [np.zeros(wl.n, np.float32) for _ in range(3)]
    want = orc.step(g, res, k, orc.MODE_FIXED, fixed_leader=1)
    got = run.step(k, orc.MODE_FIXED, 0, fixed_leader=1)
    assert_step_matches(got, want, orc.MODE_FIXED)


# ------------------------------------------------------------------ edge cases
def _one_step(g, res, k, mode=orc.MODE_FIXED, leader=0, step_no=0):
    w, n = len(g), g[0].size
    run = GpuRunner(w, n, k)
    run.load_g(g)
    run.load_res(res)
    want = orc.step(g, res, k, mode, step_no=step_no, fixed_leader=leader)
    got = run.step(k, mode, step_no, fixed_leader=leader)
    assert_step_matches(got, want, mode)
    got["info"] = run.ctx.select_info()
    return got, want


@pytest.mark.parametrize("n", [1, 2, 3, 5, 63, 64, 255, 1025, 16384, 16385, 40001])
def test_tiny_and_ragged_sizes(n):
    rng = np.random.default_rng(n)
    g = [rng.standard_normal(n).astype(np.float32) for _ in range(2)]
    res = [rng.standard_normal(n).astype(np.float32) * 0.1 for _ in range(2)]
    for k in sorted({1, n, max(1, n // 3)}):
        _one_step(g, res, k, leader=1)


def test_all_equal_vector_takes_lowest_indices():
    n = 1_200_000          # more equal keys than the survivor list can hold
    g = [np.full(n, 0.25, np.float32), np.full(n, -0.25, np.float32)]
    g[0][::7] = -0.25
    res = [np.zeros(n, np.float32), np.zeros(n, np.float32)]
    for k in (1, 5000, n - 1):
        got, _ = _one_step(g, res, k, leader=0)
        assert np.array_equal(got["idx"], np.arange(k, dtype=np.int32))


def test_two_valued_and_sign_pairs():
    rng = np.random.default_rng(12)
    n = 300_007
    x = rng.choice(np.array([1.5, -1.5, 0.75, -0.75], np.float32), n)
    y = rng.standard_normal(n).astype(np.float32)
    res = [np.zeros(n, np.float32), np.zeros(n, np.float32)]
    n_big = int((np.abs(x) == 1.5).sum())
    for k in (1, n_big - 3, n_big, n_big + 3, n):
        _one_step([x, y], res, k, leader=0)


def test_denormals_zeros_and_huge_values():
    rng = np.random.default_rng(13)
    n = 100_003
    x = rng.standard_normal(n).astype(np.float32)
    x[::5] = 0.0
    x[1::5] = -0.0
    x[2::50] = np.float32(1e-40)          # denormal
    x[3::50] = np.float32(-3e-41)
    x[7] = np.float32(3e38)
    x[9] = np.float32(-np.inf)
    y = (rng.standard_normal(n) * 1e-39).astype(np.float32)    # all denormal
    res = [np.zeros(n, np.float32), (rng.standard_normal(n) * 1e-39).astype(np.float32)]
    for k, leader in ((10, 0), (n // 2, 0), (n - 5, 0), (100, 1), (n, 1)):
        _one_step([x, y], res, k, leader=leader)


def test_sum_order_is_rank_order():
    n = 4096
    big = np.float32(2.0 ** 24)
    g = [np.full(n, big, np.float32), np.ones(n, np.float32), np.full(n, -big, np.float32)]
    res = [np.zeros(n, np.float32) for _ in range(3)]
    got, _ = _one_step(g, res, 17, leader=1)
    assert not got["sum"].any()           # (2^24 + 1) - 2^24 == 0 only in rank order


def test_var_leader_and_values():
    rng = np.random.default_rng(14)
    n = 777_777
    g = [(rng.standard_normal(n) * s + m).astype(np.float32) for s, m in
         ((0.5, 0.0), (1.0, 5.0), (2.0, -3.0), (1.5, 100.0))]
    res = [np.zeros(n, np.float32) for _ in range(4)]
    got, want = _one_step(g, res, 1234, mode=orc.MODE_VAR)
    assert got["leader"] == 2


def test_k_equals_n_dense_allreduce():
    rng = np.random.default_rng(15)
    n = 70_001
    g = [rng.standard_normal(n).astype(np.float32) for _ in range(5)]
    res = [np.zeros(n, np.float32) for _ in range(5)]
    got, _ = _one_step(g, res, n, leader=3)
    assert all(not r.any() for r in got["residual"])


# ------------------------------------------------------------------ single entry points
def test_entry_points_one_by_one():
    import torch
    import paper_2312_02493_amd as lib

    rng = np.random.default_rng(16)
    w, n, k = 3, 500_003, 4321
    dev = torch.device("cuda:0")
    acc_h = [(rng.standard_normal(n) * (1 + r)).astype(np.float32) for r in range(w)]
    acc = [torch.from_numpy(a).to(dev) for a in acc_h]
    ctx = lib.Context(w, n, k, max_segments=8)

    var = torch.zeros(w, dtype=torch.float64, device=dev)
    am = torch.zeros(1, dtype=torch.int32, device=dev)
    ctx.artopk_variance(acc, var, am)
    ctx.status()
    ref = np.array([orc.variance(a) for a in acc_h])
    np.testing.assert_allclose(var.cpu().numpy(), ref, rtol=1e-5)
    assert int(am.item()) == orc.leader_var(list(ref))

    idx = torch.full((k,), -1, dtype=torch.int32, device=dev)
    ctx.artopk_select_topk(acc[1], k, idx)
    ctx.status()
    want_idx = orc.topk_indices(acc_h[1], k)
    assert np.array_equal(idx.cpu().numpy(), want_idx)

    seg_off = [0, 17, 100_000, 100_001, 350_000, n]
    seg_k = [5, 1000, 1, 2000, 1315]
    assert sum(seg_k) == k
    idx2 = torch.full((k,), -1, dtype=torch.int32, device=dev)
    ctx.artopk_select_topk(acc[2], k, idx2, seg_off=seg_off, seg_k=seg_k)
    ctx.status()
    assert np.array_equal(idx2.cpu().numpy(), orc.topk_indices_segmented(acc_h[2], seg_off, seg_k))

    vals = torch.empty(w * k, dtype=torch.float32, device=dev)
    summed = torch.empty(k, dtype=torch.float32, device=dev)
    ctx.artopk_gather_sum(acc, idx, k, vals, summed)
    ctx.status()
    want_vals = orc.gather(acc_h, want_idx)
    want_sum = orc.ordered_sum(want_vals)
    assert np.array_equal(bits(vals.cpu().numpy().reshape(w, k)), bits(want_vals))
    assert np.array_equal(bits(summed.cpu().numpy()), bits(want_sum))
    for a, h in zip(acc, acc_h):                      # gather must not modify its input
        assert np.array_equal(bits(a.cpu().numpy()), bits(h))

    upd = torch.full((n,), float("nan"), dtype=torch.float32, device=dev)
    ctx.artopk_scatter_residual(acc, idx, k, summed, upd)
    ctx.status()
    assert np.array_equal(bits(upd.cpu().numpy()), bits(orc.scatter_update(n, want_idx, want_sum)))
    for a, h in zip(acc, acc_h):
        assert np.array_equal(bits(a.cpu().numpy()), bits(orc.residual_rewrite(h, want_idx)))


def test_invalid_arguments_are_rejected():
    import torch
    import paper_2312_02493_amd as lib

    dev = torch.device("cuda:0")
    n = 1024
    ctx = lib.Context(2, n, 100)
    x = [torch.zeros(n, device=dev), torch.zeros(n, device=dev)]
    idx = torch.zeros(100, dtype=torch.int32, device=dev)
    s = torch.zeros(100, device=dev)
    u = torch.zeros(n, device=dev)
    with pytest.raises(lib.ArTopkError) as e:
        ctx.artopk_step(x, x, 0, lib.ARTOPK_STAR, 1, idx, s, u)            # k < 1
    assert e.value.code == -1
    with pytest.raises(lib.ArTopkError):
        ctx.artopk_step(x, x, 101, lib.ARTOPK_STAR, 1, idx, s, u)          # k > max_k
    with pytest.raises(lib.ArTopkError):
        ctx.artopk_step(x, x, 10, 9, 1, idx, s, u)                         # unknown mode
    with pytest.raises(lib.ArTopkError):
        ctx.artopk_step(x + x, x + x, 10, lib.ARTOPK_STAR, 1, idx, s, u)   # W > max_w
    with pytest.raises(lib.ArTopkError):
        ctx.artopk_select_topk(x[0][1:], 10, idx)                          # misaligned
    with pytest.raises(lib.ArTopkError):
        ctx.artopk_select_topk(x[0], 10, idx, seg_off=[0, 500, n], seg_k=[5, 6])   # sum(seg_k) != k
    ctx.status()


# ------------------------------------------------------------------ segmented selection, edge cases
def _segmented_select(x, seg_off, seg_k, max_segments=None):
    import torch
    import paper_2312_02493_amd as lib

    dev = torch.device("cuda:0")
    k = int(sum(seg_k))
    ctx = lib.Context(1, x.size, k, max_segments=max_segments or len(seg_k))
    xd = torch.from_numpy(x).to(dev)
    idx = torch.full((k,), -1, dtype=torch.int32, device=dev)
    ctx.artopk_select_topk(xd, k, idx, seg_off=[int(v) for v in seg_off], seg_k=[int(v) for v in seg_k])
    ctx.status()
    want = orc.topk_indices_segmented(x, seg_off, seg_k)
    got = idx.cpu().numpy()
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, f"segmented idx differs first at {bad[:5]}: got {got[bad[:5]]} want {want[bad[:5]]}"
    return ctx, xd, idx


def test_segments_tiny_ragged_and_many():
    rng = np.random.default_rng(21)
    sizes = [1, 2, 3, 5, 1, 64, 63, 4097, 8191, 8193, 1, 30000, 7, 16385]
    sizes += [int(v) for v in rng.integers(1, 300, 400)]            # several hundred small layers
    off = np.concatenate([[0], np.cumsum(sizes)])
    n = int(off[-1])
    x = rng.standard_normal(n).astype(np.float32)
    x[rng.integers(0, n, n // 10)] = 0.5                             # planted ties
    ks = [max(1, int(np.ceil(0.05 * s))) for s in sizes]
    ks[7] = sizes[7]                                                 # one segment kept entirely
    ks[9] = 1
    _segmented_select(x, off, ks)


def test_segments_with_degenerate_members():
    """One all-equal segment larger than its survivor list (forces the deeper array passes for
    that segment only), one all-zero segment, next to ordinary ones."""
    rng = np.random.default_rng(22)
    sizes = [50_000, 700_000, 123_457, 300_000, 9]
    off = np.concatenate([[0], np.cumsum(sizes)])
    n = int(off[-1])
    x = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    x[off[1]:off[2]] = np.float32(-0.125)                            # all equal (sign ignored)
    x[off[1] + 5:off[2]:3] = np.float32(0.125)
    x[off[3]:off[4]] = 0.0                                           # all zero
    ks = [500, 40_000, 1235, 17, 9]
    ctx, xd, idx = _segmented_select(x, off, ks)
    got = idx.cpu().numpy()
    assert np.array_equal(got[500:40_500], np.arange(off[1], off[1] + 40_000, dtype=np.int32))
    # the same context must serve a different layout afterwards (descriptor table is re-uploaded)
    off2 = [0, 100_000, n]
    ks2 = [10, 41_751]
    idx.fill_(-1)
    ctx.artopk_select_topk(xd, sum(ks2), idx, seg_off=off2, seg_k=ks2)
    ctx.status()
    assert np.array_equal(idx.cpu().numpy(), orc.topk_indices_segmented(x, off2, ks2))


def test_segmented_step_star_fixed_leader():
    rng = np.random.default_rng(23)
    sizes = [3000, 1, 50_000, 20_001, 64]
    off = [int(v) for v in np.concatenate([[0], np.cumsum(sizes)])]
    n = off[-1]
    ks = [30, 1, 777, 200, 64]
    k = sum(ks)
    w = 3
    g = [rng.standard_normal(n).astype(np.float32) for _ in range(w)]
    res = [(rng.standard_normal(n) * 0.3).astype(np.float32) for _ in range(w)]
    run = GpuRunner(w, n, k, max_segments=len(ks))
    for step_no in (1, 2):
        run.load_g(g)
        run.load_res(res)
        want = orc.step(g, res, k, orc.MODE_STAR, step_no=step_no, seg_off=off, seg_k=ks)
        got = run.step(k, orc.MODE_STAR, step_no, seg_off=off, seg_k=ks)
        assert_step_matches(got, want, orc.MODE_STAR)
        res = want.residual


# ------------------------------------------------------------------ neighbours of the step
def test_compression_gain_and_sparse_update():
    import torch

    rng = np.random.default_rng(40)
    w, n, k = 4, 600_013, 5001            # k odd: the rows of vals are not 16-byte aligned
    g = [(rng.standard_normal(n) * (1 + r)).astype(np.float32) for r in range(w)]
    res = [(rng.standard_normal(n) * 0.5).astype(np.float32) for _ in range(w)]
    run = GpuRunner(w, n, k)
    run.load_g(g)
    run.load_res(res)
    want = orc.step(g, res, k, orc.MODE_VAR, keep_acc=True)
    got = run.step(k, orc.MODE_VAR, 0)
    assert_step_matches(got, want, orc.MODE_VAR)
    gain = torch.zeros(w, dtype=torch.float64, device=run.dev)
    run.ctx.artopk_compression_gain(run.res, run.vals, k, gain)
    run.ctx.status()
    ref = np.array([orc.compression_gain(want.acc[r], want.idx) for r in range(w)])
    # float64 sums of squares on both sides, summed in a different order
    np.testing.assert_allclose(gain.cpu().numpy(), ref, rtol=1e-10)

    weights_h = rng.standard_normal(n).astype(np.float32)
    weights = torch.from_numpy(weights_h).to(run.dev)
    eta = 0.0123
    run.ctx.artopk_apply_update(weights, run.idx, run.sum, k, eta)
    run.ctx.status()
    assert np.array_equal(bits(weights.cpu().numpy()), bits(orc.apply_update(weights_h, want.idx, want.sum, eta)))


@pytest.mark.parametrize("mode,rho", [("star", 0.001), ("star", 0.05), ("var", 0.01), ("var_topk", 0.01)])
def test_step_without_the_dense_update_feeds_the_sparse_model_update(mode, rho):
    """update_out = NULL: the step leaves out the dense update (Alg. 1 update line taken in its
    sparse form), everything else is the step of the oracle, and artopk_apply_update on
    (idx, sum) changes the weights exactly as the dense update would.  A buffer passed in an
    earlier call must stay untouched."""
    import torch
    import paper_2312_02493_amd as lib

    mode_lib = {"star": lib.ARTOPK_STAR, "var": lib.ARTOPK_VAR, "var_topk": lib.ARTOPK_VAR_TOPK}[mode]
    mode_orc = {"star": orc.MODE_STAR, "var": orc.MODE_VAR, "var_topk": orc.MODE_VAR_TOPK}[mode]
    n, w = 250_007, 3
    wl = inp.workload(2, n=n, w=w)
    k = wl.k(rho)
    run = GpuRunner(w, n, k)
    res = [np.zeros(n, dtype=np.float32) for _ in range(w)]
    weights_h = np.random.default_rng(77).standard_normal(n).astype(np.float32)
    weights = torch.from_numpy(weights_h).to(run.dev)
    eta = 0.05
    for step_no in (1, 2):
        g = [wl.gen(step_no, r) for r in range(w)]
        want = orc.step(g, res, k, mode_orc, step_no=step_no)
        run.load_g(g)
        run.idx.fill_(-1)
        run.sum.fill_(float("nan"))
        run.update.fill_(float("nan"))
        run.ctx.artopk_step(run.g, run.res, k, mode_lib, step_no, run.idx, run.sum, None, vals_out=run.vals,
                            leader_out=run.leader, var_out=run.var)
        run.ctx.artopk_apply_update(weights, run.idx, run.sum, k, eta)
        run.ctx.status()
        assert int(run.leader.item()) == want.leader
        assert np.array_equal(run.idx[:k].cpu().numpy(), want.idx)
        assert np.array_equal(bits(run.sum[:k].cpu().numpy()), bits(want.sum))
        assert np.array_equal(bits(run.vals[: w * k].cpu().numpy().reshape(w, k)), bits(want.vals))
        for r in range(w):
            assert np.array_equal(bits(run.res[r].cpu().numpy()), bits(want.residual[r])), f"residual {r}"
        assert bool(torch.isnan(run.update).all()), "the dense update was written"
        # the dense form w - eta * update (update is +0.0 off the kept indices) gives the same weights
        dense = np.subtract(weights_h, np.multiply(np.float32(eta), want.update, dtype=np.float32), dtype=np.float32)
        weights_h = orc.apply_update(weights_h, want.idx, want.sum, eta)
        assert np.array_equal(bits(dense), bits(weights_h))
        assert np.array_equal(bits(weights.cpu().numpy()), bits(weights_h))
        res = want.residual


def test_topk_workers_and_literal_leader_rule():
    import torch
    import paper_2312_02493_amd as lib

    rng = np.random.default_rng(41)
    w, n, k = 5, 300_011, 2999
    g = [(rng.standard_normal(n) * (1.0 + 0.1 * ((r * 3) % w))).astype(np.float32) for r in range(w)]
    res = [(rng.standard_normal(n) * 0.2).astype(np.float32) for _ in range(w)]
    acc = [orc.ef_add(a, b) for a, b in zip(g, res)]
    dev = torch.device("cuda:0")
    ctx = lib.Context(w, n, k)
    acc_d = [torch.from_numpy(a).to(dev) for a in acc]
    idx = torch.full((w * k,), -1, dtype=torch.int32, device=dev)
    vals = torch.empty(w * k, dtype=torch.float32, device=dev)
    sq = torch.zeros(w, dtype=torch.float64, device=dev)
    am = torch.full((1,), -1, dtype=torch.int32, device=dev)
    ctx.artopk_topk_workers(acc_d, k, idx, vals, sq, am)
    ctx.status()
    want_idx = [orc.topk_indices(a, k) for a in acc]
    want_sq = [orc.topk_sqnorm(a, i) for a, i in zip(acc, want_idx)]
    got_idx = idx.cpu().numpy().reshape(w, k)
    got_vals = vals.cpu().numpy().reshape(w, k)
    for r in range(w):
        assert np.array_equal(got_idx[r], want_idx[r]), f"worker {r} indices"
        assert np.array_equal(bits(got_vals[r]), bits(acc[r][want_idx[r].astype(np.int64)])), f"worker {r} values"
    np.testing.assert_allclose(sq.cpu().numpy(), want_sq, rtol=1e-12)
    assert int(am.item()) == orc.leader_var(want_sq)

    # the whole step with the literal leader rule
    run = GpuRunner(w, n, k)
    run.load_g(g)
    run.load_res(res)
    want = orc.step(g, res, k, orc.MODE_VAR_TOPK)
    got = run.step(k, orc.MODE_VAR_TOPK, 0)
    assert got["leader"] == want.leader
    np.testing.assert_allclose(got["var"], want.variances, rtol=1e-12)
    assert_step_matches(got, want, orc.MODE_FIXED)


def test_generic_path_with_host_known_leader(monkeypatch):
    """STAR / FIXED normally take the leader-first pipeline; the library's switch back to the
    generic pipeline (histogram for the leader only inside the all-worker pass, scattered gather)
    must give the same bits."""
    monkeypatch.setitem(gpu_util.OPTIONS, "leader_first", 0)
    rng = np.random.default_rng(42)
    w, n, k = 4, 450_003, 4500
    g = [rng.standard_normal(n).astype(np.float32) for _ in range(w)]
    res = [(rng.standard_normal(n) * 0.4).astype(np.float32) for _ in range(w)]
    run = GpuRunner(w, n, k)
    assert run.ctx.get_option(2) == 0   # ARTOPK_OPT_LEADER_FIRST
    for step_no in (5, 6):
        run.load_g(g)
        run.load_res(res)
        want = orc.step(g, res, k, orc.MODE_STAR, step_no=step_no)
        got = run.step(k, orc.MODE_STAR, step_no)
        assert_step_matches(got, want, orc.MODE_STAR)
        res = want.residual


def test_two_runs_give_identical_bits():
    rng = np.random.default_rng(43)
    w, n, k = 3, 700_001, 7000
    g = [(rng.standard_normal(n) * 1e-3).astype(np.float32) for _ in range(w)]
    g[1][::3] = np.float32(2.0 ** -10)              # many ties at one magnitude
    res = [np.zeros(n, np.float32) for _ in range(w)]
    outs = []
    for _ in range(2):
        run = GpuRunner(w, n, k)
        run.load_g(g)
        run.load_res(res)
        outs.append(run.step(k, orc.MODE_VAR, 1))
    a, b = outs
    assert a["leader"] == b["leader"] and np.array_equal(a["idx"], b["idx"])
    assert np.array_equal(bits(a["sum"]), bits(b["sum"])) and np.array_equal(bits(a["update"]), bits(b["update"]))
    assert np.array_equal(a["var"].view(np.uint64), b["var"].view(np.uint64))


@pytest.mark.parametrize("rule", ["star", "var", "star_all_workers_first"])
def test_bucketed_layout_16mi_elements(rule, monkeypatch):
    """Fixed-size buckets (64 MB = 16 Mi float32 each, the granularity the paper's
    communication measurements use) are just a segment table.  40 M elements: the fused pass
    strides over the tiles; with the round-robin leader its pass and the segments' selection
    run first and the other worker follows in one pass (or, with that switched off, all
    workers' pass first).  Two steps, residual carried."""
    if rule == "star_all_workers_first":
        monkeypatch.setitem(gpu_util.OPTIONS, "leader_first", 0)
    mode = orc.MODE_VAR if rule == "var" else orc.MODE_STAR
    wl = inp.workload(4, n=40_000_007, w=2)
    bucket = 16 * 1024 * 1024
    off = list(range(0, wl.n, bucket)) + [wl.n]
    ks = [int(np.ceil(0.001 * (off[i + 1] - off[i]))) for i in range(len(off) - 1)]
    k = sum(ks)
    res = [np.zeros(wl.n, np.float32) for _ in range(2)]
    run = GpuRunner(2, wl.n, k, max_segments=len(ks))
    for step_no in (1, 2):
        g = [wl.gen(step_no, r, threads=8) * np.float32(1.0 + 0.05 * r) for r in range(2)]
        run.load_g(g)
        want = orc.step(g, res, k, mode, step_no=step_no, seg_off=off, seg_k=ks)
        if mode == orc.MODE_VAR:
            assert top_two_gap(want.variances) > 1e-4
        got = run.step(k, mode, step_no, seg_off=off, seg_k=ks)
        assert_step_matches(got, want, mode)
        res = want.residual


@pytest.mark.parametrize("rule,route", [("var", "histogram"), ("var", "guess"), ("star", "histogram"), ("star", "guess"),
                                        ("star", "pieces"), ("counter", "histogram"), ("counter", "guess")])
def test_step_captured_in_a_hip_graph_replays_like_eager_steps(rule, route, monkeypatch):
    """One step recorded into a HIP graph (through torch's capture) and replayed three times,
    with host work and synchronisation between the replays: every replay must be the next step
    of the oracle, residual carried.  The step allocates nothing, clears its scratch with a fill
    kernel (no memset nodes) and takes every data-dependent decision on the device.  Under the
    round-robin rule the recorded leader (step 1 -> worker 1) is the one every replay uses, unless
    the iteration counter lives on the device (rule "counter"): then replay r is step 1 + r with the
    next worker of the round leading.  The dense update is written in its tile-by-tile form on the
    guess route."""
    import torch
    import paper_2312_02493_amd as lib

    if route in ("guess", "pieces"):
        monkeypatch.setitem(gpu_util.OPTIONS, "guess_min_n", 4096)
        monkeypatch.setitem(gpu_util.OPTIONS, "update_tiles_min_n", 1)
        # the leader's fused pass hands the marked elements on tile by tile, or leaves only the mask
        monkeypatch.setitem(gpu_util.OPTIONS, "stage_tiles", 2 if route == "pieces" else 0)
    mode_lib = {"var": lib.ARTOPK_VAR, "star": lib.ARTOPK_STAR, "counter": lib.ARTOPK_STAR_COUNTER}[rule]
    mode_orc = orc.MODE_VAR if rule == "var" else orc.MODE_STAR
    n, w = 200_003, 4
    wl = inp.workload(2, n=n, w=w)
    k = wl.k(0.01)
    dev = torch.device("cuda:0")
    side = torch.cuda.Stream()
    g_np = [wl.gen(1, r) for r in range(w)]
    with torch.cuda.stream(side):
        ctx = gpu_util.make_context(w, n, k, 1, stream=side.cuda_stream)
        g = [torch.from_numpy(a).to(dev) for a in g_np]
        res = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(w)]
        idx = torch.empty(k, dtype=torch.int32, device=dev)
        summed = torch.empty(k, dtype=torch.float32, device=dev)
        update = torch.empty(n, dtype=torch.float32, device=dev)
        vals = torch.empty(w * k, dtype=torch.float32, device=dev)
        leader = torch.zeros(1, dtype=torch.int32, device=dev)
        var = torch.zeros(w, dtype=torch.float64, device=dev)

        def step():
            ctx.artopk_step(g, res, k, mode_lib, 1, idx, summed, update, vals_out=vals, leader_out=leader,
                            var_out=var)

        step()  # warm-up outside the capture
        side.synchronize()
        ctx.status()
        for r in res:
            r.zero_()
        ctx.set_step_counter(1)  # the warm-up step has advanced it
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        for r in res:
            r.zero_()
        side.synchronize()

        want_res = [np.zeros(n, dtype=np.float32) for _ in range(w)]
        for replay in range(3):
            want = orc.step(g_np, want_res, k, mode_orc, step_no=1 + replay if rule == "counter" else 1)
            if rule == "counter":
                assert want.leader == (1 + replay) % w
            if rule == "var":
                assert top_two_gap(want.variances) > 1e-4
            graph.replay()
            side.synchronize()
            ctx.status()
            got = {
                "leader": int(leader.item()), "var": var.cpu().numpy().copy(), "idx": idx.cpu().numpy(),
                "sum": summed.cpu().numpy(), "update": update.cpu().numpy(),
                "residual": [r.cpu().numpy() for r in res], "vals": vals.cpu().numpy().reshape(w, k),
            }
            assert_step_matches(got, want, mode_orc)
            assert gpu_util.FORCED or (ctx.select_info()["guessed"] == (0 if route == "histogram" else 1))
            want_res = want.residual
            _ = torch.ones(1000, device=dev).sum().item()  # unrelated eager work between the replays


@pytest.mark.parametrize("route", ["histogram", "guess", "segments"])
def test_round_robin_leader_from_the_counter_on_the_device(route, monkeypatch):
    """ARTOPK_STAR_COUNTER: the iteration counter of the round-robin rule (Alg. 1, STAR branch) is
    kept by the context on the device, the `step` argument is ignored, and every call moves the
    counter on.  Four steps from counter 5 with three workers (leaders 2, 0, 1, 2), fresh gradients
    and the residual carried, against the oracle's STAR steps 5..8; then the counter is set back."""
    import paper_2312_02493_amd as lib

    if route == "guess":
        monkeypatch.setitem(gpu_util.OPTIONS, "guess_min_n", 4096)
    n, w = 150_011, 3
    wl = inp.workload(2, n=n, w=w)
    seg_off = seg_k = None
    if route == "segments":
        seg_off = [0, 40_000, 40_003, 99_999, n]
        seg_k = [400, 1, 600, 500]
        k = sum(seg_k)
    else:
        k = wl.k(0.01)
    run = GpuRunner(w, n, k, max_segments=4)
    run.ctx.set_step_counter(5)
    res = [np.zeros(n, dtype=np.float32) for _ in range(w)]
    for step_no in (5, 6, 7, 8, 1):
        if step_no == 1:
            run.ctx.set_step_counter(1)
        g = [wl.gen(step_no, r) for r in range(w)]
        want = orc.step(g, res, k, orc.MODE_STAR, step_no=step_no, seg_off=seg_off, seg_k=seg_k)
        assert want.leader == step_no % w
        run.load_g(g)
        got = run.step(k, lib.ARTOPK_STAR_COUNTER, 123_456, seg_off=seg_off, seg_k=seg_k)  # step argument unused
        assert_step_matches(got, want, orc.MODE_STAR)
        if route != "segments":
            assert gpu_util.FORCED or (run.ctx.select_info()["guessed"] == (1 if route == "guess" else 0))
        res = want.residual


@pytest.mark.parametrize("case", ["all_equal", "two_valued", "normal"])
def test_many_kept_entries_zeroed_inside_the_selection(case):
    """With 32 k >= N and the leader known up front the leader's residual is zeroed inside the
    selection kernels.  all_equal: the level-1 survivors overflow the list, so the deeper array
    passes run and the final pass does all the zeroing; two_valued: a large tie class sits in the
    threshold digit; normal: the usual split between the two kernels."""
    n, w, k = 200_003, 3, 50_000
    rng = np.random.default_rng(5)

    def gen():
        if case == "all_equal":
            return np.full(n, -0.5, dtype=np.float32)
        if case == "two_valued":
            x = np.where(rng.random(n) < 0.2, 2.0, 1.0).astype(np.float32)   # 40 k large, 10 k of the ties kept
            return x * np.where(rng.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
        return rng.standard_normal(n).astype(np.float32)

    run = GpuRunner(w, n, k)
    res = [np.zeros(n, dtype=np.float32) for _ in range(w)]
    for step_no in (1, 2, 3):
        g = [gen() for _ in range(w)]
        want = orc.step(g, res, k, orc.MODE_STAR, step_no=step_no)
        run.load_g(g)
        got = run.step(k, orc.MODE_STAR, step_no)
        assert_step_matches(got, want, orc.MODE_STAR)
        res = want.residual


@pytest.mark.parametrize("layout", ["flat", "segmented", "flat_guess"])
def test_leader_by_variance_of_the_raw_gradient(layout, monkeypatch):
    """Mode VAR_G: the leader is the worker whose raw gradient varies most (the other reading of
    Sec. III-B's "largest gradient variance").  Gradient scales rotate over the steps while the
    residuals go stale, so the raw-gradient rule and the error-fed rule disagree on the way."""
    if layout == "flat_guess":
        monkeypatch.setitem(gpu_util.OPTIONS, "guess_min_n", 4096)
    n, w = 120_001, 4
    wl = inp.workload(1, n=n, w=w)
    seg_off = seg_k = None
    k = wl.k(0.01)
    if layout == "segmented":
        seg_off = np.array([0, 30_000, 30_007, 90_000, n], dtype=np.int64)
        seg_k = np.array([300, 3, 600, 301], dtype=np.int64)
        k = int(seg_k.sum())
    run = GpuRunner(w, n, k, 1 if seg_k is None else len(seg_k))
    res = [np.zeros(n, dtype=np.float32) for _ in range(w)]
    res[2] = wl.gen(99, 2) * np.float32(6.0)  # worker 2 starts with a large stale residual
    run.load_res(res)
    disagreements = 0
    for step_no in range(1, 6):
        g = [wl.gen(step_no, r) * np.float32(1.0 + 0.5 * ((r + step_no) % w)) for r in range(w)]
        want = orc.step(g, res, k, orc.MODE_VAR_G, step_no=step_no, seg_off=seg_off, seg_k=seg_k)
        other = orc.step(g, res, k, orc.MODE_VAR, step_no=step_no, seg_off=seg_off, seg_k=seg_k)
        disagreements += int(want.leader != other.leader)
        assert top_two_gap(want.variances) > 1e-4
        run.load_g(g)
        got = run.step(k, orc.MODE_VAR_G, step_no,
                       seg_off=None if seg_off is None else [int(v) for v in seg_off],
                       seg_k=None if seg_k is None else [int(v) for v in seg_k])
        assert_step_matches(got, want, orc.MODE_VAR_G)
        res = want.residual
    assert disagreements >= 1


@pytest.mark.parametrize("case", ["all_equal", "two_valued_many_ties", "one_top_digit", "one_top_digit_guess",
                                  "one_top_digit_pieces"])
def test_deeper_array_passes_on_a_long_degenerate_vector(case, monkeypatch):
    """Vectors short enough to fit the survivor list whole never take the deeper array passes, so
    they are exercised here on a vector of 5 M elements whose level-1 survivors overflow the list.
    all_equal / two_valued: not even the level-2 survivors fit, the level-3 array pass writes the
    outputs itself; one_top_digit: every magnitude shares the top 12 key bits and differs below,
    so the level-2 array pass writes the list and the final pass reads it (also behind a guess
    that cannot work, since the whole vector reaches any bound in that digit; with pieces the
    bound is refined by a second digit, the guess holds and no array pass is needed)."""
    n, w, k = 5_000_003, 2, 60_000
    rng = np.random.default_rng(77)
    if case in ("one_top_digit_guess", "one_top_digit_pieces"):
        monkeypatch.setitem(gpu_util.OPTIONS, "guess_min_n", 4096)
        monkeypatch.setitem(gpu_util.OPTIONS, "stage_tiles", 0 if case == "one_top_digit_guess" else 1)

    def gen():
        if case == "all_equal":
            return np.full(n, 0.75, dtype=np.float32)
        if case.startswith("one_top_digit"):   # [1, 1.0625): exponent and the first four mantissa bits equal
            x = (1.0 + 0.0625 * rng.random(n)).astype(np.float32)
            x = np.minimum(x, np.float32(1.0624999))
            return x * np.where(rng.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
        x = np.where(rng.random(n) < 0.004, 3.0, 1.0).astype(np.float32)  # ~20 k large, 40 k of 4.98 M ties kept
        return x * np.where(rng.random(n) < 0.5, -1.0, 1.0).astype(np.float32)

    run = GpuRunner(w, n, k)
    res = [np.zeros(n, dtype=np.float32) for _ in range(w)]
    for step_no in (1, 2):
        g = [gen() for _ in range(w)]
        want = orc.step(g, res, k, orc.MODE_STAR, step_no=step_no)
        run.load_g(g)
        got = run.step(k, orc.MODE_STAR, step_no)
        info = run.ctx.select_info()
        if case == "one_top_digit_pieces":
            assert gpu_util.FORCED or (info["guessed"] == 1 and info["from_mask"] == 1), info
        elif step_no == 1:  # (at step 2 the residual has split the tie class and the list fits again)
            assert gpu_util.FORCED or (info["list_level"] == 0)   # the deeper array passes wrote the list
        assert_step_matches(got, want, orc.MODE_STAR)
        res = want.residual


@pytest.mark.parametrize("where", ["front", "middle", "back", "two_islands", "one_dense_tile"])
def test_kept_indices_clustered_in_few_tiles(where):
    """The other workers' streaming pass takes the kept indices tile by tile (32768 elements).
    Here all of them sit in one or two places, so most tiles have none, some have more indices
    than the block has threads, and the runs of empty tiles before, between and behind are long;
    the vector ends in a ragged group whose elements are kept in the `back` case."""
    n, w = 40 * 32768 + 3, 4
    rng = np.random.default_rng(21)
    k = {"front": 900, "middle": 5_000, "back": 700, "two_islands": 2_600, "one_dense_tile": 30_000}[where]

    def gen():
        x = (1e-3 * rng.standard_normal(n)).astype(np.float32)
        big = lambda m: (1.0 + rng.random(m)).astype(np.float32) * np.where(rng.random(m) < 0.5, -1.0, 1.0).astype(np.float32)
        if where == "front":
            x[:1000] = big(1000)
        elif where == "middle":                      # straddles the border of tiles 17 and 18
            lo = 18 * 32768 - 2500
            x[lo:lo + 5200] = big(5200)
        elif where == "back":
            x[-800:] = big(800)
        elif where == "two_islands":
            x[5 * 32768 + 100:5 * 32768 + 1500] = big(1400)
            x[33 * 32768 - 700:33 * 32768 + 700] = big(1400)
        else:                                        # nearly every element of tile 9 is kept
            x[9 * 32768 + 50:9 * 32768 + 50 + 31_000] = big(31_000)
        return x

    run = GpuRunner(w, n, k)
    res = [np.zeros(n, dtype=np.float32) for _ in range(w)]
    for step_no in (1, 2):
        g = [gen() for _ in range(w)]
        want = orc.step(g, res, k, orc.MODE_STAR, step_no=step_no)
        run.load_g(g)
        got = run.step(k, orc.MODE_STAR, step_no)
        assert_step_matches(got, want, orc.MODE_STAR)
        res = want.residual


@pytest.mark.parametrize("n", [3, 32768, 32769, 5 * 32768 + 2, 300_001])
def test_dense_update_streamed_tile_by_tile(n, monkeypatch):
    """The dense update of long, sparsely kept vectors is written as zeros tile by tile with the
    values stored behind them; switched on here for short vectors.  Covers a vector shorter than
    a group of four, exact and ragged tile ends, kept entries on tile borders and at both ends,
    under a rule that gathers entry by entry (VAR) and one that streams the other workers (STAR);
    also the stand-alone scatter entry point."""
    import torch
    monkeypatch.setitem(gpu_util.OPTIONS, "update_tiles_min_n", 1)
    w = 3
    rng = np.random.default_rng(31)
    kk = min(n, max(n // 200, 12)) if n > 12 else 2   # few enough kept entries for the streamed form when n is not tiny

    def gen(scale):
        x = (scale * rng.standard_normal(n)).astype(np.float32)
        x[0] = 9.0
        x[n - 1] = -8.0
        for border in range(32768, n, 32768):
            x[border - 1] = 7.0
            if border < n:
                x[border] = -7.5
        return x

    for mode in (orc.MODE_VAR, orc.MODE_STAR):
        run = GpuRunner(w, n, kk)
        res = [np.zeros(n, dtype=np.float32) for _ in range(w)]
        for step_no in (1, 2):
            g = [gen(1.0 + 0.5 * r) for r in range(w)]
            want = orc.step(g, res, kk, mode, step_no=step_no)
            if mode == orc.MODE_VAR:
                assert top_two_gap(want.variances) > 1e-4
            run.load_g(g)
            got = run.step(kk, mode, step_no)
            assert_step_matches(got, want, mode)
            res = want.residual
        # stand-alone: residual rewrite + dense update from the step's own idx and sum
        upd = torch.full((n,), float("nan"), dtype=torch.float32, device=run.dev)
        run.ctx.artopk_scatter_residual(run.res, run.idx[:kk], kk, run.sum[:kk], upd)
        run.ctx.status()
        assert np.array_equal(bits(upd.cpu().numpy()), bits(want.update))


@pytest.mark.parametrize("guess", [False, True])
def test_ordinary_loads_and_stores_give_the_same_bits(guess, monkeypatch):
    """The streaming passes use non-temporal loads and stores by default; the library's switch to
    ordinary ones must not change a bit, on either selection route and under either kind of leader."""
    monkeypatch.setitem(gpu_util.OPTIONS, "nontemporal", 0)
    if guess:
        monkeypatch.setitem(gpu_util.OPTIONS, "guess_min_n", 4096)
    w, n = 3, 6 * 32768 + 77
    wl = inp.workload(2, n=n, w=w)
    k = wl.k(0.01)
    for mode in (orc.MODE_VAR, orc.MODE_STAR):
        run = GpuRunner(w, n, k)
        res = [np.zeros(n, dtype=np.float32) for _ in range(w)]
        for step_no in (1, 2):
            g = [wl.gen(step_no, r) for r in range(w)]
            want = orc.step(g, res, k, mode, step_no=step_no)
            if mode == orc.MODE_VAR:
                assert top_two_gap(want.variances) > 1e-4
            run.load_g(g)
            got = run.step(k, mode, step_no)
            assert gpu_util.FORCED or (run.ctx.select_info()["guessed"] == (1 if guess else 0))
            assert_step_matches(got, want, mode)
            res = want.residual


# ------------------------------------------------------------------ variance against awkward data
@pytest.mark.parametrize("case", ["outlier_first", "outlier_first_four", "common_offset", "outlier_last"])
@pytest.mark.parametrize("route", ["stand_alone", "step_histogram", "step_guess"])
def test_variance_is_not_spoilt_by_one_element_or_an_offset(case, route, monkeypatch):
    """The per-worker variance (Sec. III-B leader rule) must stay within 1e-5 of the two-pass
    float64 definition whatever sits at the start of a vector: an element a million standard
    deviations out at index 0 (or the first four, or the last one), or a common offset a
    thousand standard deviations large.  Checked through artopk_variance and through a variance-
    rule step on both selection routes (the step's fused passes accumulate their own sums)."""
    import torch

    rng = np.random.default_rng(77)
    w, n, k = 3, 1_200_003, 1200
    sigma = [1.0e-3, 1.2e-3, 1.5e-3]
    g = [(rng.standard_normal(n) * s).astype(np.float32) for s in sigma]
    if case == "outlier_first":
        for r in range(w):
            g[r][0] = np.float32(1.0e6 * sigma[r])
    elif case == "outlier_first_four":
        for r in range(w):
            g[r][:4] = np.float32(-1.0e6 * sigma[r])
    elif case == "outlier_last":
        for r in range(w):
            g[r][-1] = np.float32(1.0e6 * sigma[r])
    else:
        g = [(x.astype(np.float64) + 1.0).astype(np.float32) for x in g]
    ref = np.array([orc.variance(x) for x in g])
    assert top_two_gap(ref) > VAR_GAP
    if route == "stand_alone":
        dev = torch.device("cuda:0")
        ctx = gpu_util.make_context(w, n, k)
        x = [torch.from_numpy(a).to(dev) for a in g]
        var = torch.zeros(w, dtype=torch.float64, device=dev)
        am = torch.full((1,), -1, dtype=torch.int32, device=dev)
        ctx.artopk_variance(x, var, am)
        ctx.status()
        np.testing.assert_allclose(var.cpu().numpy(), ref, rtol=1e-5, atol=0.0)
        assert int(am.item()) == orc.leader_var(list(ref))
        return
    if route == "step_guess":
        monkeypatch.setitem(gpu_util.OPTIONS, "guess_min_n", 4096)
    res = [np.zeros(n, np.float32) for _ in range(w)]
    got, want = _one_step(g, res, k, mode=orc.MODE_VAR)
    assert gpu_util.FORCED or (got["info"]["guessed"] == (1 if route == "step_guess" else 0))
    np.testing.assert_allclose(got["var"], ref, rtol=1e-5, atol=0.0)


# ------------------------------------------------------------------ boundary rules
def test_overlapping_buffers_are_rejected():
    """A buffer a call writes must not overlap any other buffer of the call: the in-place EF add
    and the scatter would otherwise corrupt silently.  Read-only buffers may be shared."""
    import torch
    import paper_2312_02493_amd as lib

    dev = torch.device("cuda:0")
    n, k, w = 4096, 64, 2
    ctx = lib.Context(w, n, k)
    g = [torch.randn(n, device=dev) for _ in range(w)]
    res = [torch.zeros(n, device=dev) for _ in range(w)]
    big = torch.zeros(2 * n, device=dev)
    idx = torch.zeros(k, dtype=torch.int32, device=dev)
    s = torch.zeros(k, device=dev)
    u = torch.zeros(n, device=dev)
    vals = torch.zeros(w * k, device=dev)

    def rejected(fn):
        with pytest.raises(lib.ArTopkError) as e:
            fn()
        assert e.value.code == -1 and "overlap" in str(e.value), str(e.value)

    rejected(lambda: ctx.artopk_step(g, g, k, lib.ARTOPK_STAR, 1, idx, s, u))                     # g[w] is residual[w]
    rejected(lambda: ctx.artopk_step(g, [res[0], res[0]], k, lib.ARTOPK_STAR, 1, idx, s, u))      # one residual twice
    rejected(lambda: ctx.artopk_step(g, [big[:n], big[n - 4:2 * n - 4]], k, lib.ARTOPK_STAR, 1, idx, s, u))  # partial overlap
    rejected(lambda: ctx.artopk_step(g, res, k, lib.ARTOPK_STAR, 1, idx, s, res[1]))              # update inside a residual
    rejected(lambda: ctx.artopk_step(g, res, k, lib.ARTOPK_STAR, 1, idx, s, u, vals_out=s))       # vals_out over sum_out
    rejected(lambda: ctx.artopk_step(g, res, k, lib.ARTOPK_STAR, 1, idx, idx.view(torch.float32), u))  # sum_out is idx_out
    rejected(lambda: ctx.artopk_gather_sum(res, idx, k, vals, vals[:k]))
    rejected(lambda: ctx.artopk_scatter_residual(res, idx, k, s, res[0]))
    rejected(lambda: ctx.artopk_select_topk(res[0], k, res[0][:k].view(torch.int32)))
    # two workers reading one gradient buffer is allowed, and nothing above was enqueued or spoilt the context
    ctx.artopk_step([g[0], g[0]], res, k, lib.ARTOPK_STAR, 1, idx, s, u, vals_out=vals)
    ctx.status()
    want = orc.step([g[0].cpu().numpy()] * 2, [np.zeros(n, np.float32)] * 2, k, orc.MODE_STAR, step_no=1)
    assert np.array_equal(idx.cpu().numpy(), want.idx)
    assert np.array_equal(bits(u.cpu().numpy()), bits(want.update))


def test_options_are_validated_and_reported():
    import paper_2312_02493_amd as lib

    ctx = lib.Context(2, 4096, 16)
    assert ctx.get_option(lib.ARTOPK_OPT_GUESS_MIN_N) == 1 << 25
    assert ctx.get_option(lib.ARTOPK_OPT_UPDATE_TILES_MIN_N) == 1 << 22
    assert ctx.get_option(lib.ARTOPK_OPT_LEADER_FIRST) == 1
    assert ctx.get_option(lib.ARTOPK_OPT_NONTEMPORAL) == 1
    assert ctx.get_option(lib.ARTOPK_OPT_STAGE_TILES) == 1
    for key, bad in ((lib.ARTOPK_OPT_GUESS_MIN_N, 0), (lib.ARTOPK_OPT_GUESS_MIN_N, (1 << 31) + 1),
                     (lib.ARTOPK_OPT_UPDATE_TILES_MIN_N, -5), (lib.ARTOPK_OPT_LEADER_FIRST, 2),
                     (lib.ARTOPK_OPT_NONTEMPORAL, -1), (lib.ARTOPK_OPT_STAGE_TILES, 3), (99, 1)):
        with pytest.raises(lib.ArTopkError) as e:
            ctx.set_option(key, bad)
        assert e.value.code == -1
    ctx.set_option(lib.ARTOPK_OPT_GUESS_MIN_N, 4096)
    assert ctx.get_option(lib.ARTOPK_OPT_GUESS_MIN_N) == 4096
