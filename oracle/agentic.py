"""Loader for the agentic-workflow oracle (``agentic_oracle.c``).  TEST INFRASTRUCTURE ONLY."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "agentic_oracle.c")
_LIB = os.path.join(_HERE, "libagentic_oracle.so")


class AgoProblem(C.Structure):
    _fields_ = [("W", C.c_uint32), ("K", C.c_uint32), ("arrival_us", C.c_void_p), ("slo_us", C.c_void_p),
                ("wf", C.c_void_p), ("in_len", C.c_void_p), ("out_len", C.c_void_p), ("pred_first", C.c_void_p),
                ("pred", C.c_void_p), ("P", C.c_uint32), ("Q", C.c_uint32), ("pa", C.c_void_p), ("pb", C.c_void_p),
                ("qc", C.c_void_p), ("qd", C.c_void_p), ("cap", C.c_void_p), ("penalty_permille", C.c_uint64)]


class AgoDetail(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("release_us", "pre_start_us", "pre_end_us", "dec_start_us", "done_us", "failed")]


METRICS_DTYPE = np.dtype([("sum_ratio_permille", "<u8"), ("p95_permille", "<u8"), ("p99_permille", "<u8"),
                          ("makespan_us", "<u8"), ("n_late", "<u4"), ("n_failed", "<u4")])
assert METRICS_DTYPE.itemsize == 40


def build(force: bool = False) -> str:
    """AP_AGENTIC_ORACLE_LIB in the environment names a library built elsewhere to be loaded instead."""
    if os.environ.get("AP_AGENTIC_ORACLE_LIB"):
        return os.environ["AP_AGENTIC_ORACLE_LIB"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", _SRC, "-o", _LIB], check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.ago_eval.argtypes = [C.POINTER(AgoProblem), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ago_eval.restype = C.c_int
        L.ago_eval_batch.argtypes = [C.POINTER(AgoProblem), C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p]
        L.ago_eval_batch.restype = C.c_int
        _lib = L
    return _lib


class AgenticOracle:
    """One problem: workflows, calls with their predecessor lists, instances, penalty ratio."""

    def __init__(self, arrival_us, slo_us, wf, in_len, out_len, pred_first, pred, pa, pb, qc, qd, cap, penalty_permille):
        u64 = lambda a: np.ascontiguousarray(a, dtype=np.uint64)
        u32 = lambda a: np.ascontiguousarray(a, dtype=np.uint32)
        self.a = dict(arrival_us=u64(arrival_us), slo_us=u64(slo_us), wf=u32(wf), in_len=u32(in_len), out_len=u32(out_len),
                      pred_first=u32(pred_first), pred=u32(np.append(np.asarray(pred, dtype=np.uint32), np.uint32(0))),
                      pa=u32(pa), pb=u32(pb), qc=u32(qc), qd=u32(qd), cap=u32(cap))
        self.W, self.K = self.a["arrival_us"].shape[0], self.a["wf"].shape[0]
        ptr = {k: v.ctypes.data for k, v in self.a.items()}
        self.problem = AgoProblem(self.W, self.K, ptr["arrival_us"], ptr["slo_us"], ptr["wf"], ptr["in_len"], ptr["out_len"],
                                  ptr["pred_first"], ptr["pred"], self.a["pa"].shape[0], self.a["qc"].shape[0], ptr["pa"],
                                  ptr["pb"], ptr["qc"], ptr["qd"], ptr["cap"], int(penalty_permille))

    @classmethod
    def from_workload(cls, wl, **override):
        kw = {k: wl[k] for k in ("arrival_us", "slo_us", "wf", "in_len", "out_len", "pred_first", "pred", "pa", "pb", "qc",
                                 "qd", "cap", "penalty_permille")}
        kw.update(override)
        return cls(**kw)

    def eval(self, pre_inst, dec_inst, key, detail: bool = False):
        pre = np.ascontiguousarray(pre_inst, dtype=np.uint16)
        dec = np.ascontiguousarray(dec_inst, dtype=np.uint16)
        key = np.ascontiguousarray(key, dtype=np.uint32)
        assert pre.shape == dec.shape == key.shape == (self.K,)
        out = np.zeros(1, dtype=METRICS_DTYPE)
        if not detail:
            rc = lib().ago_eval(C.byref(self.problem), pre.ctypes.data, dec.ctypes.data, key.ctypes.data, out.ctypes.data, None)
            assert rc == 0
            return out[0]
        arrs = {n: np.zeros(self.K, dtype=np.uint64) for n in ("release_us", "pre_start_us", "pre_end_us", "dec_start_us", "done_us")}
        failed = np.zeros(self.K, dtype=np.uint8)
        det = AgoDetail(*(arrs[n].ctypes.data for n in ("release_us", "pre_start_us", "pre_end_us", "dec_start_us", "done_us")),
                        failed.ctypes.data)
        rc = lib().ago_eval(C.byref(self.problem), pre.ctypes.data, dec.ctypes.data, key.ctypes.data, out.ctypes.data, C.byref(det))
        assert rc == 0
        arrs["failed"] = failed.astype(bool)
        return out[0], arrs

    def eval_batch(self, pre_inst, dec_inst, key) -> np.ndarray:
        pre = np.ascontiguousarray(pre_inst, dtype=np.uint16)
        dec = np.ascontiguousarray(dec_inst, dtype=np.uint16)
        key = np.ascontiguousarray(key, dtype=np.uint32)
        assert pre.ndim == 2 and pre.shape == dec.shape == key.shape and pre.shape[1] == self.K
        out = np.zeros(pre.shape[0], dtype=METRICS_DTYPE)
        rc = lib().ago_eval_batch(C.byref(self.problem), pre.ctypes.data, dec.ctypes.data, key.ctypes.data, pre.shape[0],
                                  out.ctypes.data)
        assert rc == 0
        return out
