"""ctypes binding of ``libautopoiesis_eval.so``: the same names as the C ABI
(``include/autopoiesis_eval.h``), argument marshalling only.  Every step of the
evaluation runs in the library's HIP kernels; PyTorch is used by callers for device
memory and streams.  There is no fallback: a missing library raises at load time.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libautopoiesis_eval.so")

AP_OK, AP_ERR_INVALID, AP_ERR_RANGE, AP_ERR_ALLOC, AP_ERR_DEVICE, AP_ERR_STATE = range(6)
AP_MAX_SLOTS = 64
AP_MAX_REPLICAS = 1024

# numpy views of the ABI structs
REPLICA_DTYPE = np.dtype([("prefill_base_us", "<u4"), ("prefill_per_tok_us", "<u4"), ("decode_base_us", "<u4"),
                          ("decode_per_kctx_us", "<u4"), ("t_on_us", "<u8"), ("t_off_us", "<u8")])
METRICS_DTYPE = np.dtype([("sum_e2e_us", "<u8"), ("sum_ttft_us", "<u8"), ("sum_tpot_us", "<u8"),
                          ("makespan_us", "<u8"), ("p99_ttft_us", "<u8"), ("p99_tpot_us", "<u8"),
                          ("p99_e2e_us", "<u8"), ("slo_ok", "<u4"), ("n_rejected", "<u4")])
TYPED_REPLICA_DTYPE = np.dtype({"names": ["type", "t_on_us", "t_off_us"], "formats": ["<u4", "<u8", "<u8"],
                                "offsets": [0, 8, 16], "itemsize": 24})
MODEL_DTYPE = np.dtype([(n, "<u4") for n in ("layers", "hidden", "intermediate", "vocab", "heads", "kv_heads", "weight_bits")])
GPU_DTYPE = np.dtype({"names": ["mem_bytes", "flops", "hbm_bytes_per_s", "pcie_bytes_per_s", "link_intra_bytes_per_s",
                                "link_inter_bytes_per_s", "gpus_per_node"],
                      "formats": ["<f8"] * 6 + ["<u4"], "offsets": [0, 8, 16, 24, 32, 40, 48], "itemsize": 56})
GROUP_DTYPE = np.dtype([(n, "<u4") for n in ("model", "gpu", "tp", "batch")])
PLACEMENT_DTYPE = np.dtype([("tp", "<u4"), ("count", "<u4")])
AGENTIC_METRICS_DTYPE = np.dtype([("sum_ratio_permille", "<u8"), ("p95_permille", "<u8"), ("p99_permille", "<u8"),
                                  ("makespan_us", "<u8"), ("n_late", "<u4"), ("n_failed", "<u4")])
BREAKDOWN_DTYPE = np.dtype([("total_ns", "<u8"), ("sum_stale_ns", "<u8"), ("sum_reconfig_ns", "<u8"), ("sum_serve_ns", "<u8"),
                            ("sched_ns", "<u8"), ("n_intervals", "<u4"), ("reserved", "<u4")])
assert REPLICA_DTYPE.itemsize == 32 and METRICS_DTYPE.itemsize == 64 and MODEL_DTYPE.itemsize == 28


class ApSlo(C.Structure):
    _fields_ = [("ttft_us", C.c_uint64), ("tpot_us", C.c_uint64), ("penalty_us", C.c_uint64)]


class ApError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {ap_status_str(status)} (status {status})")


_lib = None


def lib() -> C.CDLL:
    """Load the HIP library built in-tree; raise if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2604_07144_amd.build` "
                                    "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        L.ap_workload_create.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.POINTER(C.c_void_p)]
        L.ap_workload_create.restype = C.c_int
        L.ap_costmodel_set.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.POINTER(ApSlo)]
        L.ap_costmodel_set.restype = C.c_int
        L.ap_costtable_set.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.POINTER(ApSlo), C.c_void_p,
                                       C.c_void_p, C.c_uint32]
        L.ap_costtable_set.restype = C.c_int
        L.ap_eval_candidates.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p]
        L.ap_eval_candidates.restype = C.c_int
        L.ap_eval_counts_get.argtypes = [C.c_void_p, C.c_void_p]
        L.ap_eval_counts_get.restype = C.c_int
        L.ap_parent_set.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32]
        L.ap_parent_set.restype = C.c_int
        L.ap_eval_children.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p,
                                       C.c_void_p]
        L.ap_eval_children.restype = C.c_int
        L.ap_roofline_tables.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_uint32,
                                         C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.ap_roofline_tables.restype = C.c_int
        L.ap_roofline_costs.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32,
                                        C.c_void_p, C.c_void_p]
        L.ap_roofline_costs.restype = C.c_int
        L.ap_costtable_set_roofline.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p,
                                                C.c_uint32, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32]
        L.ap_costtable_set_roofline.restype = C.c_int
        L.ap_trace_time.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p,
                                    C.c_void_p]
        L.ap_trace_time.restype = C.c_int
        L.ap_trace_time_static.argtypes = L.ap_trace_time.argtypes
        L.ap_trace_time_static.restype = C.c_int
        L.ap_agentic_create.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint32, C.c_uint64,
                                        C.POINTER(C.c_void_p)]
        L.ap_agentic_create.restype = C.c_int
        L.ap_agentic_eval.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p]
        L.ap_agentic_eval.restype = C.c_int
        L.ap_agentic_destroy.argtypes = [C.c_void_p]
        L.ap_agentic_destroy.restype = C.c_int
        L.ap_workload_destroy.argtypes = [C.c_void_p]
        L.ap_workload_destroy.restype = C.c_int
        L.ap_status_str.argtypes = [C.c_int]
        L.ap_status_str.restype = C.c_char_p
        L.ap_hist_bin.argtypes = [C.c_uint64]
        L.ap_hist_bin.restype = C.c_uint32
        L.ap_hist_lower.argtypes = [C.c_uint32]
        L.ap_hist_lower.restype = C.c_uint64
        _lib = L
    return _lib


def ap_status_str(status: int) -> str:
    return lib().ap_status_str(int(status)).decode()


def ap_hist_bin(value_us: int) -> int:
    return int(lib().ap_hist_bin(int(value_us)))


def ap_hist_lower(bin_index: int) -> int:
    return int(lib().ap_hist_lower(int(bin_index)))


def _check(status: int, where: str) -> None:
    if status != AP_OK:
        raise ApError(status, where)


def ap_workload_create(arrival_us, prompt_len, out_len) -> int:
    """Host arrays in, opaque workload handle out."""
    arrival = np.ascontiguousarray(arrival_us, dtype=np.uint64)
    prompt = np.ascontiguousarray(prompt_len, dtype=np.int32)
    out = np.ascontiguousarray(out_len, dtype=np.int32)
    if not (arrival.ndim == prompt.ndim == out.ndim == 1 and arrival.shape == prompt.shape == out.shape):
        raise ValueError("arrival_us, prompt_len and out_len must be 1-D arrays of one length")
    handle = C.c_void_p()
    _check(lib().ap_workload_create(arrival.ctypes.data, prompt.ctypes.data, out.ctypes.data,
                                    arrival.shape[0], C.byref(handle)), "ap_workload_create")
    return handle.value


def make_replicas(coef, t_on_us, t_off_us) -> np.ndarray:
    """Pack (a, b, c, d) rows and windows into an array of ap_replica."""
    coef = np.asarray(coef, dtype=np.uint32).reshape(-1, 4)
    rep = np.zeros(coef.shape[0], dtype=REPLICA_DTYPE)
    rep["prefill_base_us"], rep["prefill_per_tok_us"] = coef[:, 0], coef[:, 1]
    rep["decode_base_us"], rep["decode_per_kctx_us"] = coef[:, 2], coef[:, 3]
    rep["t_on_us"] = np.asarray(t_on_us, dtype=np.uint64)
    rep["t_off_us"] = np.asarray(t_off_us, dtype=np.uint64)
    return rep


def ap_costmodel_set(workload: int, replicas: np.ndarray, B: int, slo_ttft_us: int, slo_tpot_us: int,
                     penalty_us: int) -> None:
    replicas = np.ascontiguousarray(replicas, dtype=REPLICA_DTYPE)
    slo = ApSlo(int(slo_ttft_us), int(slo_tpot_us), int(penalty_us))
    _check(lib().ap_costmodel_set(workload, replicas.ctypes.data, replicas.shape[0], int(B), C.byref(slo)),
           "ap_costmodel_set")


def ap_costtable_set(workload: int, rep_type, t_on_us, t_off_us, B: int, slo_ttft_us: int, slo_tpot_us: int,
                     penalty_us: int, prefill_us, tpot_us) -> None:
    """Host arrays in: replica types and windows (length M), cost tables uint32[T][R]."""
    rep = np.zeros(len(rep_type), dtype=TYPED_REPLICA_DTYPE)
    rep["type"] = np.asarray(rep_type, dtype=np.uint32)
    rep["t_on_us"] = np.asarray(t_on_us, dtype=np.uint64)
    rep["t_off_us"] = np.asarray(t_off_us, dtype=np.uint64)
    prefill = np.ascontiguousarray(prefill_us, dtype=np.uint32)
    tpot = np.ascontiguousarray(tpot_us, dtype=np.uint32)
    if prefill.ndim != 2 or prefill.shape != tpot.shape:
        raise ValueError("prefill_us and tpot_us must be 2-D arrays [n_types][R] of one shape")
    slo = ApSlo(int(slo_ttft_us), int(slo_tpot_us), int(penalty_us))
    _check(lib().ap_costtable_set(workload, rep.ctypes.data, rep.shape[0], int(B), C.byref(slo), prefill.ctypes.data,
                                  tpot.ctypes.data, prefill.shape[0]), "ap_costtable_set")


def ap_eval_candidates(workload: int, d_assign_ptr: int, n_candidates: int, d_out_ptr: int, stream: int = 0) -> None:
    """Device pointers (ints) in; asynchronous on ``stream`` (a hipStream_t as int, 0 = default)."""
    _check(lib().ap_eval_candidates(workload, C.c_void_p(d_assign_ptr), int(n_candidates), C.c_void_p(d_out_ptr),
                                    C.c_void_p(stream)), "ap_eval_candidates")


def ap_eval_counts_get(workload: int):
    """Returns (candidates scored since the cost model was set, those that went through the exact replay kernels)."""
    out = (C.c_uint64 * 2)()
    _check(lib().ap_eval_counts_get(workload, out), "ap_eval_counts_get")
    return int(out[0]), int(out[1])


def ap_parent_set(workload: int, parent, max_children: int) -> None:
    """Host uint16[R] parent row in; sizes the device rows for up to ``max_children`` children."""
    parent = np.ascontiguousarray(parent, dtype=np.uint16)
    if parent.ndim != 1:
        raise ValueError("parent must be a 1-D array of replica ids")
    _check(lib().ap_parent_set(workload, parent.ctypes.data, int(max_children)), "ap_parent_set")


def ap_eval_children(workload: int, d_edit_first_ptr: int, d_edit_request_ptr: int, d_edit_replica_ptr: int,
                     n_children: int, d_out_ptr: int, stream: int = 0) -> None:
    """Device pointers (ints) in; asynchronous on ``stream`` (a hipStream_t as int, 0 = default)."""
    _check(lib().ap_eval_children(workload, C.c_void_p(d_edit_first_ptr), C.c_void_p(d_edit_request_ptr),
                                  C.c_void_p(d_edit_replica_ptr), int(n_children), C.c_void_p(d_out_ptr),
                                  C.c_void_p(stream)), "ap_eval_children")


def _roofline_args(models, gpus, groups):
    models = np.ascontiguousarray(models, dtype=MODEL_DTYPE)
    gpus = np.ascontiguousarray(gpus, dtype=GPU_DTYPE)
    groups = np.ascontiguousarray(groups, dtype=GROUP_DTYPE)
    return models, gpus, groups


def ap_roofline_tables(models, gpus, groups, max_seq: int):
    """Structured arrays in (MODEL_DTYPE, GPU_DTYPE, GROUP_DTYPE); returns prefill_ns[G][max_seq+1],
    decode_prefix_ns[G][max_seq+2], weight_bytes[G], feasible[G]."""
    models, gpus, groups = _roofline_args(models, gpus, groups)
    G = groups.shape[0]
    prefill_ns = np.zeros((G, max_seq + 1), dtype=np.uint64)
    prefix_ns = np.zeros((G, max_seq + 2), dtype=np.uint64)
    weight = np.zeros(G, dtype=np.float64)
    feasible = np.zeros(G, dtype=np.uint8)
    _check(lib().ap_roofline_tables(models.ctypes.data, models.shape[0], gpus.ctypes.data, gpus.shape[0],
                                    groups.ctypes.data, G, int(max_seq), prefill_ns.ctypes.data, prefix_ns.ctypes.data,
                                    weight.ctypes.data, feasible.ctypes.data), "ap_roofline_tables")
    return prefill_ns, prefix_ns, weight, feasible


def ap_roofline_costs(workload: int, n_requests: int, models, gpus, groups):
    """Returns prefill_us[G][R], tpot_us[G][R] (uint32) for the workload's requests."""
    models, gpus, groups = _roofline_args(models, gpus, groups)
    G = groups.shape[0]
    prefill_us = np.zeros((G, n_requests), dtype=np.uint32)
    tpot_us = np.zeros((G, n_requests), dtype=np.uint32)
    _check(lib().ap_roofline_costs(workload, models.ctypes.data, models.shape[0], gpus.ctypes.data, gpus.shape[0],
                                   groups.ctypes.data, G, prefill_us.ctypes.data, tpot_us.ctypes.data), "ap_roofline_costs")
    return prefill_us, tpot_us


def ap_costtable_set_roofline(workload: int, rep_type, t_on_us, t_off_us, B: int, slo_ttft_us: int, slo_tpot_us: int,
                              penalty_us: int, models, gpus, groups) -> None:
    """Roofline cost tables computed into the workload's own device buffers and attached as its cost model;
    group g is replica type g."""
    models, gpus, groups = _roofline_args(models, gpus, groups)
    rep = np.zeros(len(rep_type), dtype=TYPED_REPLICA_DTYPE)
    rep["type"] = np.asarray(rep_type, dtype=np.uint32)
    rep["t_on_us"] = np.asarray(t_on_us, dtype=np.uint64)
    rep["t_off_us"] = np.asarray(t_off_us, dtype=np.uint64)
    slo = ApSlo(int(slo_ttft_us), int(slo_tpot_us), int(penalty_us))
    _check(lib().ap_costtable_set_roofline(workload, rep.ctypes.data, rep.shape[0], int(B), C.byref(slo), models.ctypes.data,
                                           models.shape[0], gpus.ctypes.data, gpus.shape[0], groups.ctypes.data,
                                           groups.shape[0]), "ap_costtable_set_roofline")


AP_LOAD_DEPLOYED, AP_LOAD_CHANGED = 0, 1


def ap_trace_time(models, pcie_coef, gpus, d_plans_ptr: int, d_n_intervals_ptr: int, d_sched_ns_ptr: int,
                  d_stale_ns_ptr: int, d_serve_ns_ptr: int, n_candidates: int, n_max: int, d_out_ptr: int,
                  load_scope: int = AP_LOAD_DEPLOYED, stream: int = 0) -> None:
    """Host descriptors (structured arrays, float64 coefficients), device pointers (ints) for the rest."""
    models = np.ascontiguousarray(models, dtype=MODEL_DTYPE)
    gpus = np.ascontiguousarray(gpus, dtype=GPU_DTYPE)
    coef = np.ascontiguousarray(pcie_coef, dtype=np.float64)
    if coef.shape != (models.shape[0],):
        raise ValueError("one PCIe coefficient per model")
    _check(lib().ap_trace_time(models.ctypes.data, coef.ctypes.data, models.shape[0], gpus.ctypes.data, gpus.shape[0],
                               C.c_void_p(d_plans_ptr), C.c_void_p(d_n_intervals_ptr), C.c_void_p(d_sched_ns_ptr),
                               C.c_void_p(d_stale_ns_ptr), C.c_void_p(d_serve_ns_ptr), int(n_candidates), int(n_max),
                               int(load_scope), C.c_void_p(d_out_ptr), C.c_void_p(stream)), "ap_trace_time")


def ap_trace_time_static(models, pcie_coef, gpus, d_plans_ptr: int, d_n_intervals_ptr: int, d_sched_ns_ptr: int,
                         d_stale_ns_ptr: int, d_serve_ns_ptr: int, n_candidates: int, n_max: int, d_out_ptr: int,
                         load_scope: int = AP_LOAD_DEPLOYED, stream: int = 0) -> None:
    """ap_trace_time without allocation or waiting: asynchronous on ``stream``."""
    models = np.ascontiguousarray(models, dtype=MODEL_DTYPE)
    gpus = np.ascontiguousarray(gpus, dtype=GPU_DTYPE)
    coef = np.ascontiguousarray(pcie_coef, dtype=np.float64)
    if coef.shape != (models.shape[0],):
        raise ValueError("one PCIe coefficient per model")
    _check(lib().ap_trace_time_static(models.ctypes.data, coef.ctypes.data, models.shape[0], gpus.ctypes.data, gpus.shape[0],
                                      C.c_void_p(d_plans_ptr), C.c_void_p(d_n_intervals_ptr), C.c_void_p(d_sched_ns_ptr),
                                      C.c_void_p(d_stale_ns_ptr), C.c_void_p(d_serve_ns_ptr), int(n_candidates), int(n_max),
                                      int(load_scope), C.c_void_p(d_out_ptr), C.c_void_p(stream)), "ap_trace_time_static")


def ap_agentic_create(arrival_us, slo_us, wf, in_len, out_len, pred_first, pred, pa, pb, qc, qd, cap,
                      penalty_permille: int) -> int:
    """Host arrays in (instances as parallel coefficient arrays), opaque handle out."""
    arrival = np.ascontiguousarray(arrival_us, dtype=np.uint64)
    slo = np.ascontiguousarray(slo_us, dtype=np.uint64)
    wf, in_len, out_len = (np.ascontiguousarray(x, dtype=np.uint32) for x in (wf, in_len, out_len))
    pred_first = np.ascontiguousarray(pred_first, dtype=np.uint32)
    pred = np.append(np.asarray(pred, dtype=np.uint32), np.uint32(0))          # a valid pointer even when empty
    prefill = np.ascontiguousarray(np.stack([np.asarray(pa, np.uint32), np.asarray(pb, np.uint32)], axis=1))
    decode = np.ascontiguousarray(np.stack([np.asarray(qc, np.uint32), np.asarray(qd, np.uint32), np.asarray(cap, np.uint32)], axis=1))
    if arrival.shape != slo.shape or not (wf.shape == in_len.shape == out_len.shape) or pred_first.shape != (wf.shape[0] + 1,):
        raise ValueError("array lengths do not fit together")
    handle = C.c_void_p()
    _check(lib().ap_agentic_create(arrival.ctypes.data, slo.ctypes.data, arrival.shape[0], wf.ctypes.data, in_len.ctypes.data,
                                   out_len.ctypes.data, pred_first.ctypes.data, pred.ctypes.data, wf.shape[0],
                                   prefill.ctypes.data, prefill.shape[0], decode.ctypes.data, decode.shape[0],
                                   int(penalty_permille), C.byref(handle)), "ap_agentic_create")
    return handle.value


def ap_agentic_eval(handle: int, d_prefill_ptr: int, d_decode_ptr: int, d_key_ptr: int, n_candidates: int, d_out_ptr: int,
                    stream: int = 0) -> None:
    _check(lib().ap_agentic_eval(handle, C.c_void_p(d_prefill_ptr), C.c_void_p(d_decode_ptr), C.c_void_p(d_key_ptr),
                                 int(n_candidates), C.c_void_p(d_out_ptr), C.c_void_p(stream)), "ap_agentic_eval")


def ap_agentic_destroy(handle: int) -> None:
    _check(lib().ap_agentic_destroy(handle), "ap_agentic_destroy")


def ap_workload_destroy(workload: int) -> None:
    _check(lib().ap_workload_destroy(workload), "ap_workload_destroy")
