"""ctypes binding of the DPPF C-ABI library (include/dppf.h, include/dppf_util.h).

Argument marshalling only: every step of the round runs in the library's HIP kernels.
PyTorch supplies device memory (``tensor.data_ptr()``) and the stream; nothing here computes.
There is no fallback: if the native library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "libdppf.so")
_lib = None

KERNEL_NAMES = {0: "reduce", 1: "step_reduce", 2: "finalize", 3: "update", 4: "local_step", 5: "mean",
                6: "step_update", 7: "update_exact", 8: "seq_reduce", 9: "seq_update", 10: "adamw_step",
                11: "adamw_reduce"}


class DppfError(RuntimeError):
    pass


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load libdppf.so (built in-tree by ``python -m paper_2507_20424_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise DppfError(f"{_LIB_PATH} is missing: build it with `python -m paper_2507_20424_amd.build`; "
                        "there is no CPU fallback")
    lib = ctypes.CDLL(_LIB_PATH)
    c_fpp = ctypes.POINTER(ctypes.c_void_p)
    vp, f, i64 = ctypes.c_void_p, ctypes.c_float, ctypes.c_int64
    sigs = {
        "dppf_strerror": (ctypes.c_char_p, [ctypes.c_int]),
        "dppf_last_hip_error": (ctypes.c_int, []),
        "dppf_plan_create": (ctypes.c_int, [ctypes.POINTER(vp), ctypes.c_int, ctypes.c_int, ctypes.POINTER(i64)]),
        "dppf_plan_destroy": (ctypes.c_int, [vp]),
        "dppf_plan_dim": (i64, [vp]),
        "dppf_sweep_tile_elems": (ctypes.c_int, [ctypes.c_int]),
        "dppf_layout_tiles": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, ctypes.POINTER(i64), ctypes.POINTER(i64),
                                             ctypes.POINTER(i64), ctypes.POINTER(i64), i64,
                                             ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(i64),
                                             ctypes.POINTER(ctypes.c_int32)]),
        "dppf_replica_mean": (ctypes.c_int, [vp, c_fpp, c_fpp, vp]),
        "dppf_dist_norms": (ctypes.c_int, [vp, c_fpp, c_fpp, vp, vp]),
        "dppf_pull_push_round": (ctypes.c_int, [vp, c_fpp, f, f, vp, vp, c_fpp, vp]),
        "dppf_local_sgd_step": (ctypes.c_int, [vp, c_fpp, c_fpp, c_fpp, f, f, f, vp]),
        "dppf_round": (ctypes.c_int, [vp, c_fpp, c_fpp, c_fpp, f, f, f, f, f, vp, vp, c_fpp, vp]),
        "dppf_pull_push_round_flat": (ctypes.c_int, [vp, vp, i64, f, f, vp, vp, vp, vp]),
        "dppf_local_sgd_step_flat": (ctypes.c_int, [vp, vp, vp, vp, i64, f, f, f, vp]),
        "dppf_round_flat": (ctypes.c_int, [vp, vp, vp, vp, i64, f, f, f, f, f, vp, vp, vp, vp]),
        "dppf_pull_push_round_flat_static": (ctypes.c_int, [vp, ctypes.c_int, i64, i64, f, f, vp, vp, vp]),
        "dppf_pull_push_round_exact": (ctypes.c_int, [vp, c_fpp, f, f, vp, vp, vp]),
        "dppf_pull_then_push": (ctypes.c_int, [vp, c_fpp, c_fpp, f, f, ctypes.c_int, vp, vp]),
        "dppf_local_adamw_step": (ctypes.c_int, [vp, c_fpp, c_fpp, c_fpp, c_fpp, f, f, f, f, f, i64, vp]),
        "dppf_round_adamw": (ctypes.c_int, [vp, c_fpp, c_fpp, c_fpp, c_fpp, f, f, f, f, f, i64, f, f, vp, vp, vp]),
        "dppf_plan_average_norm": (ctypes.c_int, [vp, vp, vp]),
        "dppf_round_statistics": (ctypes.c_int, [vp, ctypes.c_int, f, f, vp, vp, vp]),
        "dppf_push_schedule": (f, [ctypes.c_int, f, i64, i64]),
        "dppf_util_copy": (ctypes.c_int, [vp, vp, i64, vp]),
        "dppf_util_stream_probe": (ctypes.c_int, [vp, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                  ctypes.c_int, ctypes.c_int, vp]),
        "dppf_util_stream_probe_grouped": (ctypes.c_int, [vp, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                          ctypes.c_int, ctypes.c_int, ctypes.c_int, vp]),
        "dppf_plan_timing_enable": (ctypes.c_int, [vp, ctypes.c_int]),
        "dppf_plan_timing_read": (ctypes.c_int, [vp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(f), ctypes.c_int]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc < 0:
        lib = load()
        msg = lib.dppf_strerror(rc).decode()
        raise DppfError(f"{what}: {msg} (code {rc}, hip error {lib.dppf_last_hip_error()})")


class PointerTable:
    """A host array of device pointers, built once and reused across calls.

    ``tensors`` is either a list of M lists of T tensors (per-worker table, worker-major) or a
    flat list of T tensors (per-model table).  The tensors are kept alive by the table."""

    def __init__(self, tensors: Sequence):
        if len(tensors) > 0 and isinstance(tensors[0], (list, tuple)):
            flat = [t for row in tensors for t in row]
        else:
            flat = list(tensors)
        self.keep = flat
        self.n = len(flat)
        self.array = (ctypes.c_void_p * max(self.n, 1))()
        for i, t in enumerate(flat):
            self.array[i] = t.data_ptr() if hasattr(t, "data_ptr") else int(t)

    @property
    def ptr(self):
        return ctypes.cast(self.array, ctypes.POINTER(ctypes.c_void_p))


def _table(obj) -> Optional[PointerTable]:
    if obj is None or isinstance(obj, PointerTable):
        return obj
    return PointerTable(obj)


def _tptr(tab: Optional[PointerTable]):
    return tab.ptr if tab is not None else None


def _dev(t) -> Optional[int]:
    if t is None:
        return None
    return t.data_ptr() if hasattr(t, "data_ptr") else int(t)


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if hasattr(stream, "cuda_stream"):
        return stream.cuda_stream or None
    return int(stream) or None


class Plan:
    """Shape-dependent state of the library for M workers and a list of tensor sizes."""

    def __init__(self, M: int, numel: Sequence[int]):
        lib = load()
        self.M, self.T = int(M), len(numel)
        self.numel = [int(n) for n in numel]
        arr = (ctypes.c_int64 * max(self.T, 1))(*self.numel)
        handle = ctypes.c_void_p()
        _check(lib.dppf_plan_create(ctypes.byref(handle), self.M, self.T, arr), "dppf_plan_create")
        self._h = handle
        self._lib = lib

    def close(self) -> None:
        if getattr(self, "_h", None):
            self._lib.dppf_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def d(self) -> int:
        return int(self._lib.dppf_plan_dim(self._h))

    def _expect(self, tab: PointerTable, n: int, name: str) -> None:
        if tab.n != n:
            raise DppfError(f"{name}: table has {tab.n} pointers, the plan needs {n}")

    # ---- steps of the round
    def replica_mean(self, x, xbar, stream=None) -> None:
        x, xbar = _table(x), _table(xbar)
        self._expect(x, self.M * self.T, "x"); self._expect(xbar, self.T, "xbar")
        _check(self._lib.dppf_replica_mean(self._h, x.ptr, xbar.ptr, _stream(stream)), "dppf_replica_mean")

    def dist_norms(self, x, r_out, xbar=None, stream=None) -> None:
        x, xbar = _table(x), _table(xbar)
        self._expect(x, self.M * self.T, "x")
        if xbar is not None:
            self._expect(xbar, self.T, "xbar")
        _check(self._lib.dppf_dist_norms(self._h, x.ptr, _tptr(xbar), _dev(r_out), _stream(stream)),
               "dppf_dist_norms")

    def pull_push_round(self, x, pull, push, r_out=None, c_out=None, xbar_out=None, stream=None) -> None:
        x, xbar_out = _table(x), _table(xbar_out)
        self._expect(x, self.M * self.T, "x")
        if xbar_out is not None:
            self._expect(xbar_out, self.T, "xbar_out")
        _check(self._lib.dppf_pull_push_round(self._h, x.ptr, pull, push, _dev(r_out), _dev(c_out),
                                              _tptr(xbar_out), _stream(stream)), "dppf_pull_push_round")

    def local_sgd_step(self, x, v, g, lr, momentum, weight_decay=0.0, stream=None) -> None:
        x, v, g = _table(x), _table(v), _table(g)
        for tab, name in ((x, "x"), (v, "v"), (g, "g")):
            self._expect(tab, self.M * self.T, name)
        _check(self._lib.dppf_local_sgd_step(self._h, x.ptr, v.ptr, g.ptr, lr, momentum, weight_decay,
                                             _stream(stream)), "dppf_local_sgd_step")

    def round(self, x, v, g, lr, momentum, weight_decay, pull, push, r_out=None, c_out=None,
              xbar_out=None, stream=None) -> None:
        x, v, g, xbar_out = _table(x), _table(v), _table(g), _table(xbar_out)
        for tab, name in ((x, "x"), (v, "v"), (g, "g")):
            self._expect(tab, self.M * self.T, name)
        if xbar_out is not None:
            self._expect(xbar_out, self.T, "xbar_out")
        _check(self._lib.dppf_round(self._h, x.ptr, v.ptr, g.ptr, lr, momentum, weight_decay, pull, push,
                                    _dev(r_out), _dev(c_out), _tptr(xbar_out), _stream(stream)), "dppf_round")

    # ---- variants of the round and of the local step
    def pull_push_round_exact(self, x, pull, push_r, r_out=None, c_out=None, stream=None) -> None:
        x = _table(x)
        self._expect(x, self.M * self.T, "x")
        _check(self._lib.dppf_pull_push_round_exact(self._h, x.ptr, pull, push_r, _dev(r_out), _dev(c_out),
                                                    _stream(stream)), "dppf_pull_push_round_exact")

    def pull_then_push(self, x, x_c, pull, push, push_from="average", r_post_out=None, stream=None) -> None:
        x, x_c = _table(x), _table(x_c)
        self._expect(x, self.M * self.T, "x"); self._expect(x_c, self.T, "x_c")
        code = {"average": 0, "consensus": 1}[push_from]
        _check(self._lib.dppf_pull_then_push(self._h, x.ptr, x_c.ptr, pull, push, code, _dev(r_post_out),
                                             _stream(stream)), "dppf_pull_then_push")

    def local_adamw_step(self, x, m1, m2, g, lr, beta1, beta2, eps, weight_decay, step, stream=None) -> None:
        x, m1, m2, g = _table(x), _table(m1), _table(m2), _table(g)
        for tab, name in ((x, "x"), (m1, "m1"), (m2, "m2"), (g, "g")):
            self._expect(tab, self.M * self.T, name)
        _check(self._lib.dppf_local_adamw_step(self._h, x.ptr, m1.ptr, m2.ptr, g.ptr, lr, beta1, beta2, eps,
                                               weight_decay, step, _stream(stream)), "dppf_local_adamw_step")

    def round_adamw(self, x, m1, m2, g, lr, beta1, beta2, eps, weight_decay, step, pull, push, r_out=None,
                    c_out=None, stream=None) -> None:
        x, m1, m2, g = _table(x), _table(m1), _table(m2), _table(g)
        for tab, name in ((x, "x"), (m1, "m1"), (m2, "m2"), (g, "g")):
            self._expect(tab, self.M * self.T, name)
        _check(self._lib.dppf_round_adamw(self._h, x.ptr, m1.ptr, m2.ptr, g.ptr, lr, beta1, beta2, eps,
                                          weight_decay, step, pull, push, _dev(r_out), _dev(c_out),
                                          _stream(stream)), "dppf_round_adamw")

    # ---- flat forms (T == 1); x, v, g are [M, ld] tensors or raw device addresses
    def pull_push_round_flat(self, x, ld, pull, push, r_out=None, c_out=None, xbar_out=None, stream=None):
        _check(self._lib.dppf_pull_push_round_flat(self._h, _dev(x), ld, pull, push, _dev(r_out), _dev(c_out),
                                                   _dev(xbar_out), _stream(stream)), "dppf_pull_push_round_flat")

    def local_sgd_step_flat(self, x, v, g, ld, lr, momentum, weight_decay=0.0, stream=None):
        _check(self._lib.dppf_local_sgd_step_flat(self._h, _dev(x), _dev(v), _dev(g), ld, lr, momentum,
                                                  weight_decay, _stream(stream)), "dppf_local_sgd_step_flat")

    def round_flat(self, x, v, g, ld, lr, momentum, weight_decay, pull, push, r_out=None, c_out=None,
                   xbar_out=None, stream=None):
        _check(self._lib.dppf_round_flat(self._h, _dev(x), _dev(v), _dev(g), ld, lr, momentum, weight_decay,
                                         pull, push, _dev(r_out), _dev(c_out), _dev(xbar_out),
                                         _stream(stream)), "dppf_round_flat")

    def average_norm(self, out, stream=None) -> None:
        """out[0] (device) = ||x_A|| of the most recent round enqueued on this plan."""
        _check(self._lib.dppf_plan_average_norm(self._h, _dev(out), _stream(stream)), "dppf_plan_average_norm")

    # ---- per-kernel timing
    def timing_enable(self, enable: bool = True) -> None:
        _check(self._lib.dppf_plan_timing_enable(self._h, 1 if enable else 0), "dppf_plan_timing_enable")

    def timing_read(self, cap: int = 4096) -> List[tuple]:
        ids = (ctypes.c_int * cap)()
        ms = (ctypes.c_float * cap)()
        n = self._lib.dppf_plan_timing_read(self._h, ids, ms, cap)
        _check(n, "dppf_plan_timing_read")
        return [(KERNEL_NAMES.get(ids[i], str(ids[i])), float(ms[i])) for i in range(n)]


def pull_push_round_flat_static(x, M: int, d: int, ld: int, pull: float, push: float, r_out=None, c_out=None,
                                stream=None) -> None:
    """The plain round on one [M, ld] buffer without a plan and without any allocation."""
    _check(load().dppf_pull_push_round_flat_static(_dev(x), M, d, ld, pull, push, _dev(r_out), _dev(c_out),
                                                   _stream(stream)), "dppf_pull_push_round_flat_static")


def util_copy(dst, src, n: int, stream=None) -> None:
    """Plain device copy of n floats through the library's load/store path (measurement aid)."""
    _check(load().dppf_util_copy(_dev(dst), _dev(src), n, _stream(stream)), "dppf_util_copy")


def round_statistics(r, M: int, pull: float, push: float, out, avg_norm=None, stream=None) -> None:
    """out[0] = mean distance, out[1..M] = pull strengths, out[M+1..2M] = push strength; with avg_norm
    (device, 1 float) also out[2M+1] = ||x_A|| and out[2M+2] = mean distance / ||x_A||.  out: device, 2M+3."""
    _check(load().dppf_round_statistics(_dev(r), M, pull, push, _dev(avg_norm), _dev(out), _stream(stream)),
           "dppf_round_statistics")


SCHEDULES = {"fixed": 0, "decreasing": 1, "increasing": 2}


def push_schedule(kind: str, push: float, t: int, t_total: int) -> float:
    return float(load().dppf_push_schedule(SCHEDULES[kind], push, t, t_total))


def util_stream_probe(base, stride: int, n: int, reads: int, writes: int, inplace: bool, blocks_per_cu: int,
                      on_demand: bool = False, stream=None) -> None:
    """Launch the library's streaming probe (measurement aid, see include/dppf_util.h)."""
    _check(load().dppf_util_stream_probe(_dev(base), stride, n, reads, writes, 1 if inplace else 0, blocks_per_cu,
                                         1 if on_demand else 0, _stream(stream)), "dppf_util_stream_probe")


def util_stream_probe_grouped(base, stride: int, n: int, groups: int, reads_per_group: int, vectors: int,
                              ahead: int, blocks_per_cu: int, on_demand: bool = False, stream=None) -> None:
    """Launch the streaming probe that takes its arrays group by group (see include/dppf_util.h)."""
    _check(load().dppf_util_stream_probe_grouped(_dev(base), stride, n, groups, reads_per_group, vectors, ahead,
                                                 blocks_per_cu, 1 if on_demand else 0, _stream(stream)),
           "dppf_util_stream_probe_grouped")


def sweep_tile_elems(M: int) -> int:
    """Elements per tile of the round's sweeps for M workers.  Host only."""
    n = load().dppf_sweep_tile_elems(M)
    _check(n, "dppf_sweep_tile_elems")
    return n


STEP_TILE_ELEMS = 4096


def layout_tiles(numel: Sequence[int], tile_elems: int = STEP_TILE_ELEMS):
    """(d, nfull, tiles) for a tensor list cut into tiles of tile_elems elements; tiles = list of
    (tensor, offset, count).  Host only."""
    lib = load()
    T = len(numel)
    arr = (ctypes.c_int64 * max(T, 1))(*[int(n) for n in numel])
    d, nfull, ntiles = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(lib.dppf_layout_tiles(tile_elems, T, arr, ctypes.byref(d), ctypes.byref(nfull), ctypes.byref(ntiles), 0,
                                 None, None, None), "dppf_layout_tiles")
    n = ntiles.value
    tt, to, tc = (ctypes.c_int32 * max(n, 1))(), (ctypes.c_int64 * max(n, 1))(), (ctypes.c_int32 * max(n, 1))()
    _check(lib.dppf_layout_tiles(tile_elems, T, arr, ctypes.byref(d), ctypes.byref(nfull), ctypes.byref(ntiles), n, tt,
                                 to, tc), "dppf_layout_tiles")
    return d.value, nfull.value, [(tt[i], to[i], tc[i]) for i in range(n)]
