"""GPU parity of the step on gradients stored in 16 bits (bfloat16 / float16).

The library widens every gradient value exactly to float32 and then runs the
step of Alg. 1 as for float32 gradients; the oracle is handed the widened
values (oracle.widen_gradient, pinned on the CPU against a hand decoding of the
fields) and everything is compared bit for bit.
"""

import numpy as np
import pytest

import artopk_inputs as inp
from oracle import artopk_oracle as orc
from tests import gpu_util
from tests.gpu_util import GpuRunner, assert_step_matches, top_two_gap

pytestmark = pytest.mark.gpu


def _to_bits16(x32, kind):
    """16-bit storage of float32 test data (rounding to nearest; how is irrelevant to the check)."""
    if kind == "f16":
        with np.errstate(over="ignore"):
            return x32.astype(np.float16).view(np.uint16)
    u = x32.view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16          # round to nearest even on the dropped half
    return r.astype(np.uint16)


class Runner16(GpuRunner):
    def __init__(self, kind, *a, **kw):
        super().__init__(*a, **kw)
        t = self.torch
        self.kind = kind
        self.tdtype = t.bfloat16 if kind == "bf16" else t.float16
        self.g_type = self.lib.ARTOPK_G_BF16 if kind == "bf16" else self.lib.ARTOPK_G_F16
        self.g16 = [t.empty(self.n, dtype=self.tdtype, device=self.dev) for _ in range(self.w)]

    def load_bits(self, arrays):
        t = self.torch
        for dst, b in zip(self.g16, arrays):
            dst.copy_(t.from_numpy(np.ascontiguousarray(b).view(np.int16)).view(self.tdtype))

    def step16(self, k, mode, step_no, fixed_leader=0, seg_off=None, seg_k=None):
        t = self.torch
        self.idx.fill_(-1)
        self.sum.fill_(float("nan"))
        self.update.fill_(float("nan"))
        self.ctx.artopk_step_g16(self.g16, self.g_type, self.res, k, mode, step_no, self.idx, self.sum, self.update,
                                 vals_out=self.vals, leader_out=self.leader, var_out=self.var,
                                 fixed_leader=fixed_leader, seg_off=seg_off, seg_k=seg_k)
        self.ctx.status()
        t.cuda.synchronize()
        return {
            "leader": int(self.leader.item()),
            "var": self.var.cpu().numpy().copy(),
            "idx": self.idx[:k].cpu().numpy(),
            "sum": self.sum[:k].cpu().numpy(),
            "update": self.update.cpu().numpy(),
            "residual": [r.cpu().numpy() for r in self.res],
            "vals": self.vals[: self.w * k].cpu().numpy().reshape(self.w, k),
        }


def _run(kind, wl, n, w, k, mode, steps, seg_off=None, seg_k=None, scale=1.0, spice=None):
    runner = Runner16(kind, w, n, k, 1 if seg_k is None else len(seg_k))
    res = [np.zeros(n, dtype=np.float32) for _ in range(w)]
    for step_no in range(1, steps + 1):
        bits = []
        for r in range(w):
            x = wl.gen(step_no, r) * np.float32(scale)
            if spice is not None:
                spice(x, r)
            bits.append(_to_bits16(x, kind))
        g = [orc.widen_gradient(b, kind) for b in bits]
        want = orc.step(g, res, k, mode, step_no=step_no, seg_off=seg_off, seg_k=seg_k)
        if mode == orc.MODE_VAR:
            assert top_two_gap(want.variances) > 1e-4
        runner.load_bits(bits)
        got = runner.step16(k, mode, step_no, seg_off=None if seg_off is None else [int(v) for v in seg_off],
                            seg_k=None if seg_k is None else [int(v) for v in seg_k])
        assert_step_matches(got, want, mode)
        res = want.residual
    return runner


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_g16_star_three_steps_ragged(kind):
    n, w = 300_003, 4
    wl = inp.workload(1, n=n, w=w)
    _run(kind, wl, n, w, wl.k(0.01), orc.MODE_STAR, 3)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_g16_var_three_steps(kind):
    n, w = 500_001, 8
    wl = inp.workload(2, n=n, w=w)
    _run(kind, wl, n, w, wl.k(0.01), orc.MODE_VAR, 3)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_g16_segmented_var(kind):
    n, w = 400_000, 4
    wl = inp.workload(3, n=n, w=w)
    # float16 cannot hold the smallest Laplace scales as normals: scaled up, the values still
    # span normals and subnormals
    _run(kind, wl, n, w, wl.k(0.01), orc.MODE_VAR, 2, seg_off=wl.seg_off, seg_k=wl.seg_k(0.01),
         scale=64.0 if kind == "f16" else 1.0)


def test_g16_f16_subnormals_infinities_and_signed_zero():
    n, w = 70_001, 2
    wl = inp.workload(1, n=n, w=w)

    def spice(x, r):
        x[10:2000:7] = np.float32(3e-6)        # float16 subnormal range
        x[11:2000:7] = np.float32(-6e-8)       # the smallest subnormal, negative
        x[5000:5040] = np.float32(1e6)         # overflows to +inf in float16
        x[6000:6010] = np.float32(-0.0)

    _run("f16", wl, n, w, 700, orc.MODE_STAR, 2, spice=spice)


@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_g16_guess_route(kind, monkeypatch):
    monkeypatch.setitem(gpu_util.OPTIONS, "guess_min_n", 4096)
    n, w = (1 << 20) + 2, 3
    wl = inp.workload(1, n=n, w=w)
    runner = _run(kind, wl, n, w, wl.k(0.001), orc.MODE_STAR, 2)
    info = runner.ctx.select_info()
    assert gpu_util.FORCED or (info["guessed"] == 1 and info["from_mask"] == 1), info


def test_g16_rejects_float32_type_and_misaligned_rows():
    import torch
    import paper_2312_02493_amd as lib

    n, w, k = 4096, 2, 16
    dev = torch.device("cuda:0")
    ctx = lib.Context(w, n, k)
    g = [torch.zeros(n + 8, dtype=torch.bfloat16, device=dev) for _ in range(w)]
    res = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(w)]
    idx = torch.empty(k, dtype=torch.int32, device=dev)
    s = torch.empty(k, dtype=torch.float32, device=dev)
    upd = torch.empty(n, dtype=torch.float32, device=dev)
    with pytest.raises(lib.ArTopkError):
        ctx.artopk_step_g16([t[:n] for t in g], lib.ARTOPK_G_F32, res, k, lib.ARTOPK_STAR, 1, idx, s, upd)
    with pytest.raises(lib.ArTopkError):  # rows starting 2 bytes off an 8-byte boundary
        ctx.artopk_step_g16([t[1:n + 1] for t in g], lib.ARTOPK_G_BF16, res, k, lib.ARTOPK_STAR, 1, idx, s, upd)
    ctx.status()
