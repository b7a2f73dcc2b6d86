"""Thin ctypes binding of the C ABI in include/tacos.h (argument marshalling only).

Every step of the synthesis runs in the HIP kernels of libtacos_hip.so; this module
converts numpy arrays to the C structs and back.  There is no CPU fallback: if the
shared library has not been built, loading raises; without a HIP device every call
raises TacosError(TACOS_E_DEVICE).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtacos_hip.so")

TACOS_ALL_GATHER, TACOS_REDUCE_SCATTER, TACOS_ALL_REDUCE, TACOS_BROADCAST, TACOS_REDUCE = 0, 1, 2, 3, 4
TACOS_OK = 0
TACOS_E_INVAL, TACOS_E_UNREACHABLE, TACOS_E_OVERFLOW, TACOS_E_NOMEM, TACOS_E_DEVICE = -1, -2, -3, -4, -5
TACOS_LINK_ORDER_ID, TACOS_LINK_ORDER_COST = 0, 1
TACOS_MATCH_LINK_CENTRIC, TACOS_MATCH_POSTCONDITION = 0, 1
TACOS_MAX_CHUNKS = 262144
TACOS_MAX_CHUNKS_IN_REGISTERS = 65536
TACOS_NO_CHUNK = 0xFFFFFFFF

XFER_DTYPE = np.dtype([("t_ps", "<u8"), ("src", "<u4"), ("dst", "<u4"),
                       ("chunk", "<u4"), ("link", "<u4")])

# every symbol include/tacos.h declares
EXPORTS = [
    "tacos_synthesize", "tacos_seed_search", "tacos_result_collective_time_ps", "tacos_result_num_xfers",
    "tacos_result_num_events", "tacos_result_num_passes", "tacos_result_pass_time_ps",
    "tacos_result_pass_events", "tacos_result_read", "tacos_result_event_trace",
    "tacos_result_link_counts", "tacos_result_digest", "tacos_result_kernel_ms", "tacos_result_kernel_launches",
    "tacos_result_wall_ms", "tacos_result_device_bytes", "tacos_result_free",
    "tacos_strerror", "tacos_last_error", "tacos_link_costs", "tacos_link_costs_static", "tacos_version",
    "tacos_result_link_busy", "tacos_unwind_switch", "tacos_ideal_bound",
]


class _Topology(ctypes.Structure):
    _fields_ = [("n_npus", ctypes.c_uint32), ("n_links", ctypes.c_uint32),
                ("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p),
                ("alpha_ps", ctypes.c_void_p), ("beta_fs_per_B", ctypes.c_void_p)]


class _Options(ctypes.Structure):
    _fields_ = [("stream", ctypes.c_void_p), ("max_events", ctypes.c_uint64),
                ("time_kernels", ctypes.c_uint32), ("launch_mode", ctypes.c_uint32),
                ("link_order", ctypes.c_uint32), ("matching", ctypes.c_uint32),
                ("root", ctypes.c_uint32)]


class _Ideal(ctypes.Structure):
    _fields_ = [("collective_bytes", ctypes.c_uint64), ("bandwidth_term_ps", ctypes.c_uint64),
                ("diameter_ps", ctypes.c_uint64), ("ideal_ps", ctypes.c_uint64),
                ("pass_bandwidth_term_ps", ctypes.c_uint64 * 2), ("pass_bottleneck_npu", ctypes.c_uint32 * 2)]


class TacosError(RuntimeError):
    def __init__(self, code: int, text: str, detail: str = ""):
        super().__init__(f"tacos error {code}: {text}" + (f" [{detail}]" if detail else ""))
        self.code = code


_lib = None


def load() -> ctypes.CDLL:
    """Load libtacos_hip.so (built in-tree by __graft_entry__.build()); no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build the HIP library first "
                          "(python -c 'import __graft_entry__ as g; g.build()')")
    L = ctypes.CDLL(LIB_PATH)
    u64, u32, vp, i32 = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_int
    L.tacos_synthesize.restype = i32
    L.tacos_synthesize.argtypes = [ctypes.POINTER(_Topology), u32, u64, i32, u64,
                                   ctypes.POINTER(_Options), ctypes.POINTER(vp)]
    L.tacos_seed_search.restype = i32
    L.tacos_seed_search.argtypes = [ctypes.POINTER(_Topology), u32, u64, i32, vp, u32,
                                    ctypes.POINTER(_Options), vp, vp, ctypes.POINTER(u32)]
    for name in ("collective_time_ps", "num_xfers", "num_events", "digest", "kernel_launches",
                 "device_bytes"):
        f = getattr(L, "tacos_result_" + name)
        f.restype, f.argtypes = u64, [vp]
    L.tacos_result_num_passes.restype, L.tacos_result_num_passes.argtypes = u32, [vp]
    for name in ("pass_time_ps", "pass_events"):
        f = getattr(L, "tacos_result_" + name)
        f.restype, f.argtypes = u64, [vp, u32]
    for name in ("kernel_ms", "wall_ms"):
        f = getattr(L, "tacos_result_" + name)
        f.restype, f.argtypes = ctypes.c_double, [vp]
    L.tacos_result_read.restype, L.tacos_result_read.argtypes = i32, [vp, u64, u64, vp]
    L.tacos_result_event_trace.restype, L.tacos_result_event_trace.argtypes = i32, [vp, u32, vp, vp]
    L.tacos_result_link_counts.restype, L.tacos_result_link_counts.argtypes = i32, [vp, u32, vp]
    L.tacos_result_free.restype, L.tacos_result_free.argtypes = None, [vp]
    L.tacos_strerror.restype, L.tacos_strerror.argtypes = ctypes.c_char_p, [i32]
    L.tacos_last_error.restype, L.tacos_last_error.argtypes = ctypes.c_char_p, []
    L.tacos_link_costs.restype, L.tacos_link_costs.argtypes = i32, [ctypes.POINTER(_Topology), u64, vp]
    L.tacos_result_link_busy.restype = i32
    L.tacos_result_link_busy.argtypes = [vp, u32, vp, ctypes.POINTER(u64), ctypes.POINTER(u64), ctypes.POINTER(u64)]
    L.tacos_unwind_switch.restype = i32
    L.tacos_unwind_switch.argtypes = [u32, u32, u64, u64, vp, vp, vp, vp]
    L.tacos_ideal_bound.restype = i32
    L.tacos_ideal_bound.argtypes = [ctypes.POINTER(_Topology), u32, u64, i32, u32, ctypes.POINTER(_Ideal)]
    L.tacos_link_costs_static.restype = i32
    L.tacos_link_costs_static.argtypes = [ctypes.POINTER(_Topology), u64, vp]
    L.tacos_version.restype, L.tacos_version.argtypes = ctypes.c_char_p, []
    _lib = L
    return L


def _raise(code: int):
    L = load()
    raise TacosError(code, L.tacos_strerror(code).decode(), L.tacos_last_error().decode())


def _topology_struct(n_npus, row_ptr, col_idx, alpha_ps, beta_fs_per_B):
    rp = np.ascontiguousarray(row_ptr, dtype=np.uint32)
    ci = np.ascontiguousarray(col_idx, dtype=np.uint32)
    al = np.ascontiguousarray(alpha_ps, dtype=np.uint64)
    be = np.ascontiguousarray(beta_fs_per_B, dtype=np.uint64)
    t = _Topology(int(n_npus), int(ci.shape[0]), rp.ctypes.data, ci.ctypes.data,
                  al.ctypes.data, be.ctypes.data)
    return t, (rp, ci, al, be)  # keep the arrays alive with the struct


class TacosResult:
    """Owner of a tacos_result_t handle."""

    def __init__(self, handle: int):
        self._h = ctypes.c_void_p(handle)

    def _req(self):
        if not self._h:
            raise ValueError("result already freed")
        return self._h

    @property
    def collective_time_ps(self) -> int:
        return int(load().tacos_result_collective_time_ps(self._req()))

    @property
    def num_xfers(self) -> int:
        return int(load().tacos_result_num_xfers(self._req()))

    @property
    def num_events(self) -> int:
        return int(load().tacos_result_num_events(self._req()))

    @property
    def num_passes(self) -> int:
        return int(load().tacos_result_num_passes(self._req()))

    def pass_time_ps(self, i: int) -> int:
        return int(load().tacos_result_pass_time_ps(self._req(), i))

    def pass_events(self, i: int) -> int:
        return int(load().tacos_result_pass_events(self._req(), i))

    @property
    def digest(self) -> int:
        return int(load().tacos_result_digest(self._req()))

    @property
    def kernel_ms(self) -> float:
        return float(load().tacos_result_kernel_ms(self._req()))

    @property
    def kernel_launches(self) -> int:
        return int(load().tacos_result_kernel_launches(self._req()))

    @property
    def wall_ms(self) -> float:
        return float(load().tacos_result_wall_ms(self._req()))

    @property
    def device_bytes(self) -> int:
        return int(load().tacos_result_device_bytes(self._req()))

    def read(self, first: int = 0, count: Optional[int] = None) -> np.ndarray:
        """tacos_result_read: transfers [first, first+count) in canonical order."""
        if count is None:
            count = self.num_xfers - first
        out = np.zeros(int(count), dtype=XFER_DTYPE)
        rc = load().tacos_result_read(self._req(), int(first), int(count), out.ctypes.data)
        if rc != TACOS_OK:
            _raise(rc)
        return out

    def event_trace(self, pass_index: int = 0):
        n = self.pass_events(pass_index)
        t = np.zeros(n, dtype=np.uint64)
        m = np.zeros(n, dtype=np.uint32)
        rc = load().tacos_result_event_trace(self._req(), pass_index, t.ctypes.data, m.ctypes.data)
        if rc != TACOS_OK:
            _raise(rc)
        return t, m

    def link_counts(self, pass_index: int, n_links: int) -> np.ndarray:
        """tacos_result_link_counts: transfers carried by every link in one pass."""
        out = np.zeros(int(n_links), dtype=np.uint64)
        rc = load().tacos_result_link_counts(self._req(), pass_index, out.ctypes.data)
        if rc != TACOS_OK:
            _raise(rc)
        return out

    def link_busy(self, pass_index: int, n_links: int):
        """tacos_result_link_busy: (busy_ps[n_links], sum, min, max) of one pass, python ints."""
        out = np.zeros(int(n_links), dtype=np.uint64)
        s, mn, mx = ctypes.c_uint64(0), ctypes.c_uint64(0), ctypes.c_uint64(0)
        rc = load().tacos_result_link_busy(self._req(), pass_index, out.ctypes.data, ctypes.byref(s),
                                           ctypes.byref(mn), ctypes.byref(mx))
        if rc != TACOS_OK:
            _raise(rc)
        return out, int(s.value), int(mn.value), int(mx.value)

    def free(self):
        if self._h:
            load().tacos_result_free(self._h)
            self._h = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.free()


def tacos_synthesize(n_npus, row_ptr, col_idx, alpha_ps, beta_fs_per_B, chunks_per_npu,
                     chunk_bytes, collective, seed, stream: int = 0, max_events: int = 0,
                     time_kernels: bool = False, launch_mode: int = 0,
                     link_order: int = 0, matching: int = 0, root: int = 0) -> TacosResult:
    """tacos_synthesize of include/tacos.h.  `stream` is a raw hipStream_t value (for a
    torch stream: torch.cuda.current_stream().cuda_stream); 0 = the null stream."""
    L = load()
    topo, keep = _topology_struct(n_npus, row_ptr, col_idx, alpha_ps, beta_fs_per_B)
    opts = _Options(ctypes.c_void_p(int(stream) or None), int(max_events), 1 if time_kernels else 0,
                    int(launch_mode), int(link_order), int(matching), int(root))
    out = ctypes.c_void_p(None)
    rc = L.tacos_synthesize(ctypes.byref(topo), int(chunks_per_npu), int(chunk_bytes),
                            int(collective), int(seed), ctypes.byref(opts), ctypes.byref(out))
    del keep
    if rc != TACOS_OK:
        _raise(rc)
    return TacosResult(out.value)


def tacos_seed_search(n_npus, row_ptr, col_idx, alpha_ps, beta_fs_per_B, chunks_per_npu,
                      chunk_bytes, collective, seeds, stream: int = 0, launch_mode: int = 0,
                      link_order: int = 0, matching: int = 0, root: int = 0):
    """tacos_seed_search of include/tacos.h: (time_ps[n_seeds], num_events[n_seeds], best index)."""
    L = load()
    topo, keep = _topology_struct(n_npus, row_ptr, col_idx, alpha_ps, beta_fs_per_B)
    opts = _Options(ctypes.c_void_p(int(stream) or None), 0, 0, int(launch_mode), int(link_order),
                    int(matching), int(root))
    seeds = np.ascontiguousarray(np.asarray(seeds, dtype=np.uint64))
    times = np.zeros(len(seeds), dtype=np.uint64)
    events = np.zeros(len(seeds), dtype=np.uint64)
    best = ctypes.c_uint32(0)
    rc = L.tacos_seed_search(ctypes.byref(topo), int(chunks_per_npu), int(chunk_bytes), int(collective),
                             seeds.ctypes.data if len(seeds) else None, len(seeds), ctypes.byref(opts),
                             times.ctypes.data, events.ctypes.data, ctypes.byref(best))
    del keep
    if rc != TACOS_OK:
        _raise(rc)
    return times, events, int(best.value)


def tacos_link_costs(n_npus, row_ptr, col_idx, alpha_ps, beta_fs_per_B, chunk_bytes) -> np.ndarray:
    L = load()
    topo, keep = _topology_struct(n_npus, row_ptr, col_idx, alpha_ps, beta_fs_per_B)
    out = np.zeros(topo.n_links, dtype=np.uint64)
    rc = L.tacos_link_costs(ctypes.byref(topo), int(chunk_bytes), out.ctypes.data)
    del keep
    if rc != TACOS_OK:
        _raise(rc)
    return out


def tacos_link_costs_static(n_npus, row_ptr, col_idx, alpha_ps, beta_fs_per_B, chunk_bytes) -> np.ndarray:
    """tacos_link_costs_static of include/tacos.h (allocates no device memory)."""
    L = load()
    topo, keep = _topology_struct(n_npus, row_ptr, col_idx, alpha_ps, beta_fs_per_B)
    out = np.zeros(topo.n_links, dtype=np.uint64)
    rc = L.tacos_link_costs_static(ctypes.byref(topo), int(chunk_bytes), out.ctypes.data)
    del keep
    if rc != TACOS_OK:
        _raise(rc)
    return out


def tacos_unwind_switch(n_npus: int, degree: int, alpha_ps: int, beta_fs_per_B: int):
    """tacos_unwind_switch of include/tacos.h: (row_ptr, col_idx, alpha_ps, beta_fs_per_B) arrays."""
    n, d = int(n_npus), int(degree)
    n_links = max(0, n * d) if n >= 2 and 1 <= d <= n - 1 else 1
    row_ptr = np.zeros(max(n, 0) + 1, dtype=np.uint32)
    col = np.zeros(n_links, dtype=np.uint32)
    al = np.zeros(n_links, dtype=np.uint64)
    be = np.zeros(n_links, dtype=np.uint64)
    rc = load().tacos_unwind_switch(n, d, int(alpha_ps), int(beta_fs_per_B), row_ptr.ctypes.data, col.ctypes.data,
                                    al.ctypes.data, be.ctypes.data)
    if rc != TACOS_OK:
        _raise(rc)
    return row_ptr, col, al, be


def tacos_ideal_bound(n_npus, row_ptr, col_idx, alpha_ps, beta_fs_per_B, chunks_per_npu, chunk_bytes, collective,
                      with_diameter: bool = True) -> dict:
    """tacos_ideal_bound of include/tacos.h as a dict of python ints."""
    topo, keep = _topology_struct(n_npus, row_ptr, col_idx, alpha_ps, beta_fs_per_B)
    out = _Ideal()
    rc = load().tacos_ideal_bound(ctypes.byref(topo), int(chunks_per_npu), int(chunk_bytes), int(collective),
                                  1 if with_diameter else 0, ctypes.byref(out))
    del keep
    if rc != TACOS_OK:
        _raise(rc)
    n_pass = 2 if collective == TACOS_ALL_REDUCE else 1
    return {"collective_bytes": int(out.collective_bytes), "bandwidth_term_ps": int(out.bandwidth_term_ps),
            "diameter_ps": int(out.diameter_ps), "ideal_ps": int(out.ideal_ps),
            "pass_bandwidth_term_ps": [int(out.pass_bandwidth_term_ps[i]) for i in range(n_pass)],
            "pass_bottleneck_npu": [int(out.pass_bottleneck_npu[i]) for i in range(n_pass)]}


def tacos_version() -> str:
    return load().tacos_version().decode()


def seed_search_workload(w, seeds, **kw):
    """Convenience: tacos_seed_search on a workload object (its own seed is not used)."""
    t = w.topo
    return tacos_seed_search(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B,
                             w.chunks_per_npu, w.chunk_bytes, w.collective, seeds, **kw)


def synthesize_best_of(w, seeds, **kw):
    """Best of several seeds with its schedule: tacos_seed_search over `seeds`, then
    tacos_synthesize with the winning seed.  Returns (result, best seed, times)."""
    skw = {k: v for k, v in kw.items() if k in ("stream", "link_order", "matching")}
    times, _, best = seed_search_workload(w, seeds, **skw)
    t = w.topo
    seed = int(np.asarray(seeds, dtype=np.uint64)[best])
    r = tacos_synthesize(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B,
                         w.chunks_per_npu, w.chunk_bytes, w.collective, seed, **kw)
    return r, seed, times


def synthesize_workload(w, **kw) -> TacosResult:
    """Convenience: run on an object with .topo/.chunks_per_npu/.chunk_bytes/.collective/.seed."""
    t = w.topo
    return tacos_synthesize(t.n_npus, t.row_ptr, t.col_idx, t.alpha_ps, t.beta_fs_per_B,
                            w.chunks_per_npu, w.chunk_bytes, w.collective, w.seed, **kw)
