"""Seeded synthetic gradients for the AR-Topk compressor workloads.

This package only draws random numbers and lays them out; it contains none of
the compressor's arithmetic and is imported by neither the oracle nor the HIP
binding.  Tests, the smoke check and the benchmark use it to hand the *same
bits* to both sides.

Recipe.  Every array is cut into chunks of CHUNK elements.  Chunk c of worker
r at step i of workload cfg is drawn from

    numpy.random.Generator(PCG64(SeedSequence([BASE_SEED, cfg, i, r, c])))

in float64 and cast once to float32 (r = 255 names a stream shared by all
workers, r = 254 the stream that lays out segments).  Chunks are independent,
so any sub-range can be produced, on any number of threads, with identical
bits.  Steps are counted from 1 as in Alg. 1 of the paper.

Workloads 3 and 5 draw every worker from the same distribution; to keep the
VAR-Topk leader well defined their worker r is scaled by (1 + 0.01 r) and
(1 + 0.004 r) respectively, so the per-worker variances differ by far more than
the sampling noise of the variance estimate (about 5e-4 and 5e-5 relative).

The five workloads stand in for the real gradients of the models the paper
trains and for its 1e8 / 1e9 element tensors: same element counts, fp32,
bell-shaped / heavy-tailed value distributions concentrated in a few binades,
distinct per-worker variances where the leader rule needs them, and exact
magnitude ties where the tie rule needs them.
"""

from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

BASE_SEED = 23120249
CHUNK = 1 << 22
SHARED_STREAM = 255
LAYOUT_STREAM = 254

MODE_STAR = 0
MODE_VAR = 1


def _rng(cfg: int, step: int, worker: int, chunk: int) -> np.random.Generator:
    ss = np.random.SeedSequence([BASE_SEED, int(cfg), int(step), int(worker), int(chunk)])
    return np.random.Generator(np.random.PCG64(ss))


@dataclass
class Workload:
    cfg: int
    name: str
    n: int
    w: int
    mode: int
    rhos: Sequence[float]
    steps: int
    seg_off: Optional[np.ndarray] = None      # int64, nseg+1
    seg_scale: Optional[np.ndarray] = None    # float64, nseg (cfg 3)
    seed_bump: int = 0                         # added to cfg in the seed on reseed
    note: str = ""
    _elem_scale_cache: dict = field(default_factory=dict, repr=False)

    # -- segment helpers ---------------------------------------------------
    def seg_k(self, rho: float) -> Optional[np.ndarray]:
        if self.seg_off is None:
            return None
        sizes = np.diff(self.seg_off)
        ks = [max(1, min(int(s), int(math.ceil(float(rho) * float(s))))) for s in sizes]
        return np.asarray(ks, dtype=np.int64)

    def k(self, rho: float) -> int:
        if self.seg_off is not None:
            return int(self.seg_k(rho).sum())
        return max(1, min(self.n, int(math.ceil(float(rho) * float(self.n)))))

    # -- drawing -------------------------------------------------------------
    def _chunk(self, step: int, worker: int, c: int) -> np.ndarray:
        lo = c * CHUNK
        m = min(CHUNK, self.n - lo)
        cfg = self.cfg + 1000 * self.seed_bump
        if self.cfg == 1:
            x = 0.01 * _rng(cfg, step, worker, c).standard_normal(m)
        elif self.cfg == 2:
            zs = _rng(cfg, step, SHARED_STREAM, c).standard_normal(m)
            zw = _rng(cfg, step, worker, c).standard_normal(m)
            s_w = 0.5 * 2.0 ** (worker / 3.5)
            x = 0.01 * zs + (0.01 * s_w) * zw
        elif self.cfg == 3:
            lap = _rng(cfg, step, worker, c).laplace(0.0, 1.0, m)
            x = lap * ((1.0 + 0.01 * worker) * self._elem_scale(lo, lo + m))
        elif self.cfg == 4:
            x = 1e-3 * _rng(cfg, step, worker, c).standard_t(3.0, m)
        elif self.cfg == 5:
            r = _rng(cfg, step, worker, c)
            x = (1e-3 * (1.0 + 0.004 * worker)) * r.standard_normal(m)
            u = r.random(m)
            q = np.rint(x * 1024.0) / 1024.0
            x = np.where(u < 0.1, q, x)
        else:
            raise ValueError("unknown workload")
        return x.astype(np.float32)

    def _elem_scale(self, lo: int, hi: int) -> np.ndarray:
        s0 = int(np.searchsorted(self.seg_off, lo, side="right") - 1)
        s1 = int(np.searchsorted(self.seg_off, hi, side="left"))
        bounds = np.clip(self.seg_off[s0:s1 + 1], lo, hi)
        return np.repeat(self.seg_scale[s0:s1], np.diff(bounds))

    def gen(self, step: int, worker: int, lo: int = 0, hi: Optional[int] = None,
            threads: int = 1) -> np.ndarray:
        """float32 gradient of ``worker`` at ``step`` restricted to [lo, hi)."""
        hi = self.n if hi is None else hi
        out = np.empty(hi - lo, dtype=np.float32)
        self.gen_into(out, step, worker, lo, hi, threads)
        return out

    def gen_into(self, out: np.ndarray, step: int, worker: int, lo: int = 0,
                 hi: Optional[int] = None, threads: int = 1) -> None:
        hi = self.n if hi is None else hi
        c0, c1 = lo // CHUNK, (hi + CHUNK - 1) // CHUNK

        def one(c: int) -> None:
            a = max(lo, c * CHUNK)
            b = min(hi, (c + 1) * CHUNK)
            x = self._chunk(step, worker, c)
            out[a - lo:b - lo] = x[a - c * CHUNK:b - c * CHUNK]

        if threads <= 1 or c1 - c0 <= 1:
            for c in range(c0, c1):
                one(c)
        else:
            with ThreadPoolExecutor(max_workers=threads) as ex:
                list(ex.map(one, range(c0, c1)))


def _segments(cfg: int, n_total: int, nseg: int, lo_size: float, hi_size: float):
    """Segment sizes log-uniform in [lo_size, hi_size], rescaled to n_total."""
    r = _rng(cfg, 0, LAYOUT_STREAM, 0)
    u = r.uniform(math.log(lo_size), math.log(hi_size), nseg)
    raw = np.exp(u)
    f = n_total / raw.sum()
    sizes = np.maximum(1, np.floor(raw * f).astype(np.int64))
    sizes[int(np.argmax(sizes))] += n_total - int(sizes.sum())
    scale = np.exp(r.uniform(math.log(1e-4), math.log(1e-1), nseg))
    off = np.zeros(nseg + 1, dtype=np.int64)
    off[1:] = np.cumsum(sizes)
    assert off[-1] == n_total and sizes.min() >= 1
    return off, scale


_FULL_N = {1: 1_048_576, 2: 11_689_512, 3: 25_557_032, 4: 138_357_544, 5: 1_000_000_000}
_FULL_W = {1: 4, 2: 8, 3: 8, 4: 4, 5: 8}


def workload(cfg: int, n: Optional[int] = None, w: Optional[int] = None,
             seed_bump: int = 0) -> Workload:
    """Workload ``cfg`` (1..5), optionally shrunk to ``n`` elements / ``w`` workers.

    A shrunk workload keeps the value distribution and structure and differs
    only in size; it is what the oracle can finish in seconds.
    """
    n = _FULL_N[cfg] if n is None else int(n)
    w = _FULL_W[cfg] if w is None else int(w)
    if cfg == 1:
        return Workload(1, "c1-flat-1M-star", n, w, MODE_STAR, (0.01,), 3, seed_bump=seed_bump,
                        note="N(0,0.01^2) iid")
    if cfg == 2:
        return Workload(2, "c2-resnet18-var", n, w, MODE_VAR, (0.01, 0.001), 10, seed_bump=seed_bump,
                        note="shared + per-worker normal, s_w=0.5*2^(w/3.5)")
    if cfg == 3:
        nseg = 54 if n >= 54 * 64 else max(1, n // 64)
        hi_size = 2.4e6 * (n / _FULL_N[3])
        off, scale = _segments(3 + 1000 * seed_bump, n, nseg, 64.0 if n == _FULL_N[3] else 8.0,
                               max(hi_size, 64.0))
        return Workload(3, "c3-resnet50-layerwise-var", n, w, MODE_VAR, (0.01,), 5, seg_off=off,
                        seg_scale=scale, seed_bump=seed_bump, note="54 Laplace tensors")
    if cfg == 4:
        return Workload(4, "c4-vgg16-star", n, w, MODE_STAR, (0.1, 0.01, 0.001), 5,
                        seed_bump=seed_bump, note="1e-3 * Student-t(3)")
    if cfg == 5:
        return Workload(5, "c5-1B-var", n, w, MODE_VAR, (0.001,), 3, seed_bump=seed_bump,
                        note="N(0,1e-3^2), 10% on the 2^-10 grid")
    raise ValueError("cfg must be 1..5")


def bits_checksum(x: np.ndarray) -> int:
    """XOR of the uint32 views, for logging that two sides saw the same bits."""
    v = np.ascontiguousarray(x).view(np.uint32)
    return int(np.bitwise_xor.reduce(v)) if v.size else 0
