"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI
binding and compare it with the CPU oracle bit for bit."""

import numpy as np

from oracle import artopk_oracle as orc


# Route switches applied to every context these helpers create (name -> value; a test changes
# them with monkeypatch.setitem, so that they revert when it ends).  The routes give identical
# results, so every parity test may run on any of them.
OPTIONS = {}
# Switches forced for the whole session (pytest --artopk-option): a test's checks of WHICH route ran
# are then off, its comparisons of the results are not.
FORCED = set()
_OPTION_KEYS = {"guess_min_n": 0, "update_tiles_min_n": 1, "leader_first": 2, "nontemporal": 3, "stage_tiles": 4}


def make_context(*args, **kwargs):
    """lib.Context(...) with the current OPTIONS applied through artopk_set_option."""
    import paper_2312_02493_amd as lib

    ctx = lib.Context(*args, **kwargs)
    for name, value in OPTIONS.items():
        ctx.set_option(_OPTION_KEYS[name], value)
    return ctx


def bits(x):
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)


class GpuRunner:
    """Keeps W gradient / residual tensors on the GPU and steps them."""

    def __init__(self, w, n, max_k, max_segments=1):
        import torch
        import paper_2312_02493_amd as lib

        self.torch, self.lib = torch, lib
        self.w, self.n = w, n
        dev = torch.device("cuda:0")
        self.dev = dev
        self.ctx = make_context(w, n, max_k, max_segments)
        self.g = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(w)]
        self.res = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(w)]
        self.update = torch.empty(n, dtype=torch.float32, device=dev)
        self.leader = torch.full((1,), -7, dtype=torch.int32, device=dev)
        self.var = torch.zeros(w, dtype=torch.float64, device=dev)
        self.max_k = max_k
        self.idx = torch.empty(max_k, dtype=torch.int32, device=dev)
        self.vals = torch.empty(w * max_k, dtype=torch.float32, device=dev)
        self.sum = torch.empty(max_k, dtype=torch.float32, device=dev)

    def load_g(self, arrays):
        for t, a in zip(self.g, arrays):
            t.copy_(self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)))

    def load_res(self, arrays):
        for t, a in zip(self.res, arrays):
            t.copy_(self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)))

    def step(self, k, mode, step_no, fixed_leader=0, seg_off=None, seg_k=None, want_vals=True):
        t = self.torch
        self.idx.fill_(-1)
        self.sum.fill_(float("nan"))
        self.update.fill_(float("nan"))
        self.ctx.artopk_step(self.g, self.res, k, mode, step_no, self.idx, self.sum, self.update,
                             vals_out=self.vals if want_vals else None, leader_out=self.leader,
                             var_out=self.var, fixed_leader=fixed_leader, seg_off=seg_off, seg_k=seg_k)
        self.ctx.status()
        t.cuda.synchronize()
        out = {
            "leader": int(self.leader.item()),
            "var": self.var.cpu().numpy().copy(),
            "idx": self.idx[:k].cpu().numpy(),
            "sum": self.sum[:k].cpu().numpy(),
            "update": self.update.cpu().numpy(),
            "residual": [r.cpu().numpy() for r in self.res],
        }
        if want_vals:
            out["vals"] = self.vals[: self.w * k].cpu().numpy().reshape(self.w, k)
        return out


def assert_step_matches(got, want: "orc.StepResult", mode, var_rtol=1e-5):
    """Bit-exact comparison of one GPU step with the oracle's."""
    assert got["leader"] == want.leader, (got["leader"], want.leader, got["var"], want.variances)
    if mode in (orc.MODE_VAR, orc.MODE_VAR_G):
        ref = np.asarray(want.variances)
        # variance within 1e-5 relative (both sides fp64; the GPU sums in one shifted pass)
        np.testing.assert_allclose(got["var"], ref, rtol=var_rtol, atol=0.0)
    assert got["idx"].dtype == np.int32
    bad = np.flatnonzero(got["idx"] != want.idx)
    assert bad.size == 0, f"idx differs at {bad[:5]}: got {got['idx'][bad[:5]]} want {want.idx[bad[:5]]} (k={want.idx.size})"
    if "vals" in got:
        assert np.array_equal(bits(got["vals"]), bits(want.vals)), "vals differ"
    assert np.array_equal(bits(got["sum"]), bits(want.sum)), "sum differs"
    assert np.array_equal(bits(got["update"]), bits(want.update)), "update differs"
    for r in range(len(want.residual)):
        assert np.array_equal(bits(got["residual"][r]), bits(want.residual[r])), f"residual {r} differs"


def top_two_gap(variances):
    v = np.sort(np.asarray(variances, dtype=np.float64))[::-1]
    return float((v[0] - v[1]) / v[0]) if len(v) > 1 and v[0] > 0 else 1.0
