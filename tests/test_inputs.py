"""Host-side checks of the seeded input generators (no compressor arithmetic)."""

import numpy as np

import artopk_inputs as inp


def test_subrange_and_threads_give_identical_bits():
    wl = inp.workload(5, n=3 * inp.CHUNK + 12345, w=2)
    full = wl.gen(1, 1)
    part = wl.gen(1, 1, lo=inp.CHUNK - 7, hi=2 * inp.CHUNK + 99, threads=4)
    assert np.array_equal(full[inp.CHUNK - 7:2 * inp.CHUNK + 99].view(np.uint32), part.view(np.uint32))
    again = wl.gen(1, 1, threads=3)
    assert inp.bits_checksum(full) == inp.bits_checksum(again)
    assert not np.array_equal(full, wl.gen(2, 1))
    assert not np.array_equal(full, wl.gen(1, 0))


def test_full_sizes_and_k():
    assert inp.workload(1).k(0.01) == 10486
    assert inp.workload(2).k(0.001) == 11690
    assert inp.workload(4).k(0.1) == 13835755
    assert inp.workload(5).k(0.001) == 1000000
    w3 = inp.workload(3)
    assert w3.seg_off[-1] == 25_557_032 and len(w3.seg_off) == 55
    assert np.diff(w3.seg_off).min() >= 1
    ks = w3.seg_k(0.01)
    assert np.all(ks >= 1) and np.all(ks <= np.diff(w3.seg_off))
    assert 255_571 <= ks.sum() <= 255_571 + 54


def test_value_structure():
    w2 = inp.workload(2, n=200_000)
    v = [float(np.var(w2.gen(1, r).astype(np.float64))) for r in range(8)]
    assert all(b > a for a, b in zip(v, v[1:]))          # distinct, increasing spreads
    w5 = inp.workload(5, n=400_000)
    x = w5.gen(1, 0).astype(np.float64) * 1024.0
    on_grid = np.mean(x == np.rint(x))
    assert 0.08 < on_grid < 0.12                          # ~10 % forced onto the 2^-10 grid
    w3 = inp.workload(3, n=100_000)
    x3 = w3.gen(1, 0)
    assert x3.size == 100_000 and np.isfinite(x3).all()
