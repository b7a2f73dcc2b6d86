"""TEST INFRASTRUCTURE: ctypes access to the plain CPU oracle (oracle/tacos_oracle.c).

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It imports nothing from the product package and the product imports nothing
from here.  `build()` compiles the C file with gcc; `synthesize()` runs it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tacos_oracle.c")
_LIB = os.path.join(_HERE, "libtacos_oracle.so")

ALL_GATHER, REDUCE_SCATTER, ALL_REDUCE, BROADCAST, REDUCE = 0, 1, 2, 3, 4
OK, E_INVAL, E_UNREACHABLE, E_OVERFLOW, E_NOMEM = 0, -1, -2, -3, -4

XFER_DTYPE = np.dtype([("t_ps", "<u8"), ("src", "<u4"), ("dst", "<u4"),
                       ("chunk", "<u4"), ("link", "<u4")])


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle returned error code {code}")
        self.code = code


class _CResult(ctypes.Structure):
    _fields_ = [
        ("collective_time_ps", ctypes.c_uint64),
        ("n_xfers", ctypes.c_uint64),
        ("n_events", ctypes.c_uint64),
        ("n_attempts", ctypes.c_uint64),
        ("digest", ctypes.c_uint64),
        ("pass_time_ps", ctypes.c_uint64 * 2),
        ("pass_events", ctypes.c_uint64 * 2),
        ("n_stored", ctypes.c_uint64),
        ("xfers", ctypes.c_void_p),
        ("n_event_times", ctypes.c_uint64),
        ("event_times", ctypes.c_void_p),
        ("event_matches", ctypes.c_void_p),
    ]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, popcount instruction, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-mpopcnt", "-fopenmp", "-Wall", "-Wextra",
                               "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.orc_synthesize.restype = ctypes.c_int
        L.orc_synthesize.argtypes = [
            ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64,
            ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_uint32, ctypes.POINTER(ctypes.POINTER(_CResult))]
        L.orc_result_free.restype = None
        L.orc_result_free.argtypes = [ctypes.POINTER(_CResult)]
        L.orc_philox4x32_10.restype = None
        L.orc_philox4x32_10.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.orc_mix.restype = ctypes.c_uint64
        L.orc_mix.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32]
        L.orc_link_cost.restype = ctypes.c_int
        L.orc_link_cost.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                                    ctypes.POINTER(ctypes.c_uint64)]
        L.orc_max_threads.restype = ctypes.c_int
        L.orc_set_progress.restype = None
        L.orc_set_progress.argtypes = [ctypes.c_uint64]
        L.orc_set_keep_windows.restype = None
        L.orc_set_keep_windows.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        _lib = L
    return _lib


@dataclass
class OracleResult:
    collective_time_ps: int
    n_xfers: int
    n_events: int
    n_attempts: int
    digest: int
    pass_time_ps: tuple
    pass_events: tuple
    xfers: np.ndarray          # XFER_DTYPE, canonical order (time, link id)
    event_times: np.ndarray    # uint64, matching sweeps of the last pass
    event_matches: np.ndarray  # uint32


def philox4x32_10(ctr, key) -> tuple:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return tuple(int(x) for x in out)


def mix(t_ps: int, link: int, chunk: int) -> int:
    return int(lib().orc_mix(t_ps, link, chunk))


def link_cost(alpha_ps: int, beta_fs_per_B: int, chunk_bytes: int):
    out = ctypes.c_uint64(0)
    ok = lib().orc_link_cost(alpha_ps, beta_fs_per_B, chunk_bytes, ctypes.byref(out))
    return int(out.value) if ok else None


def set_progress(every: int) -> None:
    """Print a line on stderr every `every` matching sweeps (0 = silent)."""
    lib().orc_set_progress(int(every))


def set_keep_windows(stride: int, block: int) -> None:
    """Forward pass: store the blocks of `block` records starting at keep_first + k * stride
    instead of one window (stride 0 = one window again)."""
    lib().orc_set_keep_windows(int(stride), int(block))


def max_threads() -> int:
    return int(lib().orc_max_threads())


def synthesize(n_npus, row_ptr, col_idx, alpha_ps, beta_fs_per_B, chunks_per_npu, chunk_bytes,
               collective, seed, max_events: int = 0, keep_first: int = 0,
               keep_xfers: int = (1 << 64) - 1, n_threads: int = 1,
               link_order: int = 0, matching: int = 0, root: int = 0) -> OracleResult:
    rp = np.ascontiguousarray(row_ptr, dtype=np.uint32)
    ci = np.ascontiguousarray(col_idx, dtype=np.uint32)
    al = np.ascontiguousarray(alpha_ps, dtype=np.uint64)
    be = np.ascontiguousarray(beta_fs_per_B, dtype=np.uint64)
    res = ctypes.POINTER(_CResult)()
    rc = lib().orc_synthesize(int(n_npus), rp.ctypes.data, ci.ctypes.data, al.ctypes.data,
                              be.ctypes.data, int(chunks_per_npu), int(chunk_bytes),
                              int(collective), int(seed), int(max_events), int(keep_first),
                              int(keep_xfers), int(n_threads), int(link_order), int(matching),
                              int(root), ctypes.byref(res))
    if rc != OK:
        raise OracleError(rc)
    try:
        r = res.contents
        n = int(r.n_stored)
        if n:
            buf = (ctypes.c_char * (n * XFER_DTYPE.itemsize)).from_address(r.xfers)
            xf = np.frombuffer(buf, dtype=XFER_DTYPE).copy()
        else:
            xf = np.zeros(0, dtype=XFER_DTYPE)
        ne = int(r.n_event_times)
        if ne:
            et = np.frombuffer((ctypes.c_char * (ne * 8)).from_address(r.event_times),
                               dtype=np.uint64).copy()
            em = np.frombuffer((ctypes.c_char * (ne * 4)).from_address(r.event_matches),
                               dtype=np.uint32).copy()
        else:
            et = np.zeros(0, dtype=np.uint64)
            em = np.zeros(0, dtype=np.uint32)
        return OracleResult(int(r.collective_time_ps), int(r.n_xfers), int(r.n_events),
                            int(r.n_attempts), int(r.digest),
                            (int(r.pass_time_ps[0]), int(r.pass_time_ps[1])),
                            (int(r.pass_events[0]), int(r.pass_events[1])), xf, et, em)
    finally:
        lib().orc_result_free(res)


def synthesize_workload(w, **kw) -> OracleResult:
    """Run the oracle on an object with .topo/.chunks_per_npu/.chunk_bytes/.collective/.seed."""
    t = w.topo
    return synthesize(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B,
                      w.chunks_per_npu, w.chunk_bytes, w.collective, w.seed, **kw)
