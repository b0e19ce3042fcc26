"""Loader for the CPU oracle (``ap_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by
the ``cpu_baseline`` leg of ``bench.py``.  The product package never imports this
module, and this module never imports the product's binding or kernels.

``build()`` compiles the C file with gcc into ``oracle/libap_oracle.so``;
``Oracle`` wraps one problem (trace + replica table + SLOs) for ctypes calls.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ap_oracle.c")
_LIB = os.path.join(_HERE, "libap_oracle.so")


class OrcReplica(C.Structure):
    _fields_ = [("prefill_base_us", C.c_uint32), ("prefill_per_tok_us", C.c_uint32),
                ("decode_base_us", C.c_uint32), ("decode_per_kctx_us", C.c_uint32),
                ("t_on_us", C.c_uint64), ("t_off_us", C.c_uint64)]


class OrcMetrics(C.Structure):
    _fields_ = [("sum_e2e_us", C.c_uint64), ("sum_ttft_us", C.c_uint64), ("sum_tpot_us", C.c_uint64),
                ("makespan_us", C.c_uint64), ("p99_ttft_us", C.c_uint64), ("p99_tpot_us", C.c_uint64),
                ("p99_e2e_us", C.c_uint64), ("slo_ok", C.c_uint32), ("n_rejected", C.c_uint32)]


class OrcProblem(C.Structure):
    _fields_ = [("R", C.c_uint32), ("arrival_us", C.c_void_p), ("prompt_len", C.c_void_p),
                ("out_len", C.c_void_p), ("M", C.c_uint32), ("replicas", C.c_void_p), ("B", C.c_uint32),
                ("slo_ttft_us", C.c_uint64), ("slo_tpot_us", C.c_uint64), ("penalty_us", C.c_uint64),
                ("n_types", C.c_uint32), ("rep_type", C.c_void_p), ("prefill_tab", C.c_void_p),
                ("tpot_tab", C.c_void_p)]


class OrcDetail(C.Structure):
    _fields_ = [("start_us", C.c_void_p), ("finish_us", C.c_void_p), ("ttft_us", C.c_void_p),
                ("tpot_us", C.c_void_p), ("e2e_us", C.c_void_p), ("rejected", C.c_void_p)]


METRICS_DTYPE = np.dtype([("sum_e2e_us", "<u8"), ("sum_ttft_us", "<u8"), ("sum_tpot_us", "<u8"),
                          ("makespan_us", "<u8"), ("p99_ttft_us", "<u8"), ("p99_tpot_us", "<u8"),
                          ("p99_e2e_us", "<u8"), ("slo_ok", "<u4"), ("n_rejected", "<u4")])
assert METRICS_DTYPE.itemsize == 64 and C.sizeof(OrcMetrics) == 64


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2; it is a checker, never tuned).  AP_ORACLE_LIB in the environment
    names a library built elsewhere to be loaded instead (the sanitizer build of tests/test_oracle_sanitizers.py)."""
    if os.environ.get("AP_ORACLE_LIB"):
        return os.environ["AP_ORACLE_LIB"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", "-pthread",
                        _SRC, "-o", _LIB], check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_hist_bin.argtypes = [C.c_uint64]
        L.orc_hist_bin.restype = C.c_uint32
        L.orc_hist_lower.argtypes = [C.c_uint32]
        L.orc_hist_lower.restype = C.c_uint64
        L.orc_eval_row.argtypes = [C.POINTER(OrcProblem), C.c_void_p, C.POINTER(OrcMetrics), C.c_void_p]
        L.orc_eval_row.restype = C.c_int
        L.orc_eval_batch.argtypes = [C.POINTER(OrcProblem), C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p]
        L.orc_eval_batch.restype = C.c_int
        L.orc_child_row.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        L.orc_child_row.restype = None
        _lib = L
    return _lib


def hist_bin(v: int) -> int:
    return int(lib().orc_hist_bin(int(v)))


def hist_lower(b: int) -> int:
    return int(lib().orc_hist_lower(int(b)))


class Oracle:
    """One problem instance: trace arrays, replica table, B, SLOs, penalty."""

    def __init__(self, arrival_us, prompt_len, out_len, coef, t_on_us, t_off_us, B,
                 slo_ttft_us, slo_tpot_us, penalty_us):
        self.arrival = np.ascontiguousarray(arrival_us, dtype=np.uint64)
        self.prompt = np.ascontiguousarray(prompt_len, dtype=np.int32)
        self.out = np.ascontiguousarray(out_len, dtype=np.int32)
        coef = np.asarray(coef, dtype=np.uint32).reshape(-1, 4)
        self.M = int(coef.shape[0])
        self.R = int(self.arrival.shape[0])
        self.replicas = (OrcReplica * self.M)()
        for m in range(self.M):
            a, b, c, d = (int(x) for x in coef[m])
            self.replicas[m] = OrcReplica(a, b, c, d, int(t_on_us[m]), int(t_off_us[m]))
        self.problem = OrcProblem(self.R, self.arrival.ctypes.data, self.prompt.ctypes.data,
                                  self.out.ctypes.data, self.M,
                                  C.cast(self.replicas, C.c_void_p).value, int(B),
                                  int(slo_ttft_us), int(slo_tpot_us), int(penalty_us), 0, None, None, None)

    def set_cost_tables(self, rep_type, prefill_us, tpot_us) -> "Oracle":
        """Switch to the tabulated cost model: ``rep_type`` uint32[M], tables uint32[T][R] (microseconds of
        prefill, microseconds per output token).  The windows of the replica table stay in force."""
        self.rep_type = np.ascontiguousarray(rep_type, dtype=np.uint32)
        self.prefill_tab = np.ascontiguousarray(prefill_us, dtype=np.uint32)
        self.tpot_tab = np.ascontiguousarray(tpot_us, dtype=np.uint32)
        assert self.rep_type.shape == (self.M,) and self.prefill_tab.ndim == 2
        assert self.prefill_tab.shape == self.tpot_tab.shape and self.prefill_tab.shape[1] == self.R
        assert int(self.rep_type.max()) < self.prefill_tab.shape[0]
        self.problem.n_types = self.prefill_tab.shape[0]
        self.problem.rep_type = self.rep_type.ctypes.data
        self.problem.prefill_tab = self.prefill_tab.ctypes.data
        self.problem.tpot_tab = self.tpot_tab.ctypes.data
        return self

    @classmethod
    def from_trace(cls, tr, **override):
        kw = dict(arrival_us=tr.arrival_us, prompt_len=tr.prompt_len, out_len=tr.out_len, coef=tr.coef,
                  t_on_us=tr.t_on_us, t_off_us=tr.t_off_us, B=tr.B, slo_ttft_us=tr.slo_ttft_us,
                  slo_tpot_us=tr.slo_tpot_us, penalty_us=tr.penalty_us)
        kw.update(override)
        return cls(**kw)

    def eval_row(self, row, detail: bool = False):
        row = np.ascontiguousarray(row, dtype=np.uint16)
        assert row.shape == (self.R,)
        m = OrcMetrics()
        if not detail:
            rc = lib().orc_eval_row(C.byref(self.problem), row.ctypes.data, C.byref(m), None)
            if rc:
                raise RuntimeError(f"orc_eval_row failed: {rc}")
            return _metrics_to_record(m)
        arrs = {k: np.zeros(self.R, dtype=np.uint64) for k in ("start_us", "finish_us", "ttft_us", "tpot_us", "e2e_us")}
        rej = np.zeros(self.R, dtype=np.uint8)
        det = OrcDetail(*(arrs[k].ctypes.data for k in ("start_us", "finish_us", "ttft_us", "tpot_us", "e2e_us")),
                        rej.ctypes.data)
        rc = lib().orc_eval_row(C.byref(self.problem), row.ctypes.data, C.byref(m), C.byref(det))
        if rc:
            raise RuntimeError(f"orc_eval_row failed: {rc}")
        arrs["rejected"] = rej.astype(bool)
        return _metrics_to_record(m), arrs

    def eval_batch(self, assign, nthreads: int = 1) -> np.ndarray:
        assign = np.ascontiguousarray(assign, dtype=np.uint16)
        assert assign.ndim == 2 and assign.shape[1] == self.R
        out = np.zeros(assign.shape[0], dtype=METRICS_DTYPE)
        rc = lib().orc_eval_batch(C.byref(self.problem), assign.ctypes.data, assign.shape[0], int(nthreads),
                                  out.ctypes.data)
        if rc:
            raise RuntimeError(f"orc_eval_batch failed: {rc}")
        return out

    def eval_children(self, parent, edit_first, edit_request, edit_replica, nthreads: int = 1) -> np.ndarray:
        """Children of ``parent`` given as edit lists: their rows by the child-row rule, then ``eval_batch``."""
        return self.eval_batch(child_rows(parent, edit_first, edit_request, edit_replica), nthreads)


def child_rows(parent, edit_first, edit_request, edit_replica) -> np.ndarray:
    """Rows of the children of ``parent``: child c applies edits ``edit_first[c] .. edit_first[c+1]``
    (none when that range is empty or reversed) front to back."""
    parent = np.ascontiguousarray(parent, dtype=np.uint16)
    first = np.ascontiguousarray(edit_first, dtype=np.uint32)
    request = np.ascontiguousarray(edit_request, dtype=np.uint32)
    replica = np.ascontiguousarray(edit_replica, dtype=np.uint16)
    assert first.ndim == 1 and first.shape[0] >= 1 and request.shape == replica.shape
    n_children, R = first.shape[0] - 1, parent.shape[0]
    rows = np.empty((n_children, R), dtype=np.uint16)
    for c in range(n_children):
        lo, hi = int(first[c]), int(first[c + 1])
        n = max(0, hi - lo)
        assert n == 0 or hi <= request.shape[0]
        lib().orc_child_row(parent.ctypes.data, R, request.ctypes.data + 4 * lo, replica.ctypes.data + 2 * lo,
                            n, rows[c].ctypes.data)
    return rows


def _metrics_to_record(m: OrcMetrics) -> np.ndarray:
    rec = np.zeros((), dtype=METRICS_DTYPE)
    for name in METRICS_DTYPE.names:
        rec[name] = getattr(m, name)
    return rec
