"""ctypes binding of libartopk.so.  Same names as the C ABI; marshalling only.

PyTorch is used for device memory (tensor.data_ptr()) and for the stream handle;
no step of the compressor runs in PyTorch.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))

ARTOPK_STAR, ARTOPK_VAR, ARTOPK_FIXED, ARTOPK_VAR_TOPK, ARTOPK_VAR_G = 0, 1, 2, 3, 4
ARTOPK_STAR_COUNTER = 5
ARTOPK_G_F32, ARTOPK_G_BF16, ARTOPK_G_F16 = 0, 1, 2
ARTOPK_OPT_GUESS_MIN_N, ARTOPK_OPT_UPDATE_TILES_MIN_N, ARTOPK_OPT_LEADER_FIRST, ARTOPK_OPT_NONTEMPORAL = 0, 1, 2, 3
ARTOPK_OPT_STAGE_TILES = 4
PROF_NAMES = ("pass_a", "select", "gather", "update", "total")

_SYMBOLS = (
    "artopk_create", "artopk_destroy", "artopk_last_error", "artopk_status", "artopk_variance",
    "artopk_select_topk", "artopk_gather_sum", "artopk_scatter_residual", "artopk_step",
    "artopk_set_profile", "artopk_get_profile", "artopk_version", "artopk_compression_gain",
    "artopk_apply_update", "artopk_topk_workers", "artopk_select_info", "artopk_step_g16",
    "artopk_set_option", "artopk_get_option", "artopk_variance_static", "artopk_set_step_counter",
    "artopk_scratch_bytes",
)


class ArTopkError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"artopk error {code}: {text}")
        self.code = code


def lib_path() -> str:
    return os.path.join(HERE, "libartopk.so")


def exported_symbols():
    return _SYMBOLS


_lib = None


def load_library():
    """Load libartopk.so; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2312_02493_amd.build`")
    lib = C.CDLL(path)
    vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
    lib.artopk_create.argtypes = [C.POINTER(vp), i32, i64, i64, i32, vp]
    lib.artopk_destroy.argtypes = [vp]
    lib.artopk_last_error.argtypes = [vp]
    lib.artopk_last_error.restype = C.c_char_p
    lib.artopk_status.argtypes = [vp]
    lib.artopk_variance.argtypes = [vp, vp, i32, i64, vp, vp]
    lib.artopk_select_topk.argtypes = [vp, vp, i64, i32, vp, vp, i64, vp]
    lib.artopk_gather_sum.argtypes = [vp, vp, i32, i64, vp, i64, vp, vp]
    lib.artopk_scatter_residual.argtypes = [vp, vp, i32, i64, vp, i64, vp, vp]
    lib.artopk_step.argtypes = [vp, vp, vp, i32, i64, i32, vp, vp, i64, i32, u64, i32, vp, vp, vp, vp, vp, vp]
    lib.artopk_step_g16.argtypes = [vp, vp, i32, vp, i32, i64, i32, vp, vp, i64, i32, u64, i32, vp, vp, vp, vp, vp,
                                    vp]
    lib.artopk_topk_workers.argtypes = [vp, vp, i32, i64, i64, vp, vp, vp, vp]
    lib.artopk_compression_gain.argtypes = [vp, vp, i32, i64, vp, i64, vp]
    lib.artopk_apply_update.argtypes = [vp, vp, i64, vp, vp, i64, C.c_float]
    lib.artopk_set_profile.argtypes = [vp, i32]
    lib.artopk_get_profile.argtypes = [vp, C.POINTER(C.c_float), i32]
    lib.artopk_select_info.argtypes = [vp, C.POINTER(i32), i32]
    lib.artopk_set_option.argtypes = [vp, i32, i64]
    lib.artopk_get_option.argtypes = [vp, i32, C.POINTER(i64)]
    lib.artopk_variance_static.argtypes = [vp, i32, i64, vp, vp, vp]
    lib.artopk_set_step_counter.argtypes = [vp, C.c_uint64]
    lib.artopk_scratch_bytes.argtypes = [i32, i64, i64, i32]
    lib.artopk_version.restype = i32
    lib.artopk_scratch_bytes.restype = i64
    for name in _SYMBOLS:
        if name not in ("artopk_last_error", "artopk_version", "artopk_scratch_bytes"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _ptr_table(tensors: Sequence):
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = int(t.data_ptr())
    return arr


def _i64_array(values):
    if values is None:
        return None
    arr = (C.c_int64 * len(values))()
    for i, v in enumerate(values):
        arr[i] = int(v)
    return arr


def artopk_scratch_bytes(max_w: int, max_n: int, max_k: int, max_segments: int = 1) -> int:
    """Device bytes a Context of these limits allocates (-1: limits refused); needs no GPU."""
    return int(load_library().artopk_scratch_bytes(int(max_w), int(max_n), int(max_k), int(max_segments)))


def artopk_variance_static(x: Sequence, var_out, argmax_out=None, stream: Optional[int] = None):
    """The context-free variance call that allocates nothing (enqueued on `stream`, default: torch's current)."""
    import torch

    lib = load_library()
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    rc = lib.artopk_variance_static(_ptr_table(x), len(x), x[0].numel(), _ptr(var_out), _ptr(argmax_out),
                                    C.c_void_p(stream))
    if rc != 0:
        raise ArTopkError(rc, lib.artopk_last_error(None).decode())


class Context:
    """Owns one artopk_ctx bound to the current torch stream of the current device."""

    def __init__(self, max_w: int, max_n: int, max_k: int, max_segments: int = 1, stream: Optional[int] = None):
        import torch

        if not torch.cuda.is_available():
            raise RuntimeError("the AR-Topk library needs a GPU; there is no CPU path")
        self._lib = load_library()
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        self._h = C.c_void_p()
        rc = self._lib.artopk_create(C.byref(self._h), max_w, max_n, max_k, max_segments, C.c_void_p(stream))
        if rc != 0:
            raise ArTopkError(rc, "artopk_create failed")

    # -- plumbing ------------------------------------------------------------
    def _check(self, rc: int):
        if rc != 0:
            raise ArTopkError(rc, self._lib.artopk_last_error(self._h).decode())

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.artopk_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def status(self):
        self._check(self._lib.artopk_status(self._h))

    def set_profile(self, level: int):
        """0 off, 1 events around pass A only, 2 events at every stage boundary."""
        self._check(self._lib.artopk_set_profile(self._h, int(level)))

    def set_option(self, key: int, value: int):
        self._check(self._lib.artopk_set_option(self._h, int(key), int(value)))

    def set_step_counter(self, value: int):
        self._check(self._lib.artopk_set_step_counter(self._h, int(value)))

    def get_option(self, key: int) -> int:
        out = C.c_int64()
        self._check(self._lib.artopk_get_option(self._h, int(key), C.byref(out)))
        return int(out.value)

    def select_info(self) -> dict:
        buf = (C.c_int32 * 5)()
        self._check(self._lib.artopk_select_info(self._h, buf, 5))
        return {"guessed": int(buf[0]), "from_mask": int(buf[1]), "list_count": int(buf[2]),
                "list_level": int(buf[3]), "dominant_workers": int(buf[4])}

    def get_profile(self) -> dict:
        buf = (C.c_float * len(PROF_NAMES))()
        self._check(self._lib.artopk_get_profile(self._h, buf, len(PROF_NAMES)))
        return {name: float(buf[i]) for i, name in enumerate(PROF_NAMES)}

    # -- the five entry points ---------------------------------------------
    def artopk_variance(self, x: Sequence, var_out, argmax_out=None):
        n = x[0].numel()
        self._check(self._lib.artopk_variance(self._h, _ptr_table(x), len(x), n, _ptr(var_out), _ptr(argmax_out)))

    def artopk_select_topk(self, acc, k: int, idx_out, seg_off=None, seg_k=None):
        nseg = 1 if seg_off is None else len(seg_k)
        self._check(self._lib.artopk_select_topk(self._h, _ptr(acc), acc.numel(), nseg, _i64_array(seg_off),
                                                 _i64_array(seg_k), k, _ptr(idx_out)))

    def artopk_gather_sum(self, acc: Sequence, idx, k: int, vals_out, sum_out):
        n = acc[0].numel()
        self._check(self._lib.artopk_gather_sum(self._h, _ptr_table(acc), len(acc), n, _ptr(idx), k,
                                                _ptr(vals_out), _ptr(sum_out)))

    def artopk_scatter_residual(self, residual: Sequence, idx, k: int, summed, update):
        n = residual[0].numel()
        self._check(self._lib.artopk_scatter_residual(self._h, _ptr_table(residual), len(residual), n, _ptr(idx), k,
                                                      _ptr(summed), _ptr(update)))

    def artopk_topk_workers(self, acc: Sequence, k: int, idx_out, vals_out=None, sqnorm_out=None, argmax_out=None):
        n = acc[0].numel()
        self._check(self._lib.artopk_topk_workers(self._h, _ptr_table(acc), len(acc), n, k, _ptr(idx_out),
                                                  _ptr(vals_out), _ptr(sqnorm_out), _ptr(argmax_out)))

    def artopk_compression_gain(self, residual: Sequence, vals, k: int, gain_out):
        n = residual[0].numel()
        self._check(self._lib.artopk_compression_gain(self._h, _ptr_table(residual), len(residual), n, _ptr(vals),
                                                      k, _ptr(gain_out)))

    def artopk_apply_update(self, weights, idx, summed, k: int, eta: float):
        self._check(self._lib.artopk_apply_update(self._h, _ptr(weights), weights.numel(), _ptr(idx), _ptr(summed),
                                                  k, C.c_float(eta)))

    def artopk_step(self, g: Sequence, residual: Sequence, k: int, mode: int, step: int, idx_out, sum_out,
                    update_out, vals_out=None, leader_out=None, var_out=None, fixed_leader: int = 0,
                    seg_off=None, seg_k=None):
        n = g[0].numel()
        nseg = 1 if seg_off is None else len(seg_k)
        self._check(self._lib.artopk_step(self._h, _ptr_table(g), _ptr_table(residual), len(g), n, nseg,
                                          _i64_array(seg_off), _i64_array(seg_k), k, mode, step, fixed_leader,
                                          _ptr(leader_out), _ptr(var_out), _ptr(idx_out), _ptr(vals_out),
                                          _ptr(sum_out), _ptr(update_out)))

    def artopk_step_g16(self, g: Sequence, g_type: int, residual: Sequence, k: int, mode: int, step: int, idx_out,
                        sum_out, update_out, vals_out=None, leader_out=None, var_out=None, fixed_leader: int = 0,
                        seg_off=None, seg_k=None):
        n = g[0].numel()
        nseg = 1 if seg_off is None else len(seg_k)
        self._check(self._lib.artopk_step_g16(self._h, _ptr_table(g), g_type, _ptr_table(residual), len(g), n, nseg,
                                              _i64_array(seg_off), _i64_array(seg_k), k, mode, step, fixed_leader,
                                              _ptr(leader_out), _ptr(var_out), _ptr(idx_out), _ptr(vals_out),
                                              _ptr(sum_out), _ptr(update_out)))
