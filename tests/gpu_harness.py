"""Shared plumbing for the GPU parity tests: run rows through the C ABI and through the
oracle, compare byte for byte.  (Not a test module.)"""
from __future__ import annotations

import numpy as np
import torch

from oracle import Oracle
from paper_2604_07144_amd import binding


class GpuWorkload:
    """A workload handle of the HIP library with its cost model set from a Trace."""

    def __init__(self, tr, tables=None, **override):
        """``tables=(rep_type, prefill_us[T][R], tpot_us[T][R])`` selects the tabulated cost model (the trace's
        coefficients are then unused); otherwise the linear one with the trace's coefficients."""
        kw = dict(B=tr.B, slo_ttft_us=tr.slo_ttft_us, slo_tpot_us=tr.slo_tpot_us, penalty_us=tr.penalty_us,
                  coef=tr.coef, t_on_us=tr.t_on_us, t_off_us=tr.t_off_us)
        kw.update(override)
        self.R = tr.R
        self.handle = binding.ap_workload_create(tr.arrival_us, tr.prompt_len, tr.out_len)
        try:
            if tables is None:
                binding.ap_costmodel_set(self.handle, binding.make_replicas(kw["coef"], kw["t_on_us"], kw["t_off_us"]),
                                         kw["B"], kw["slo_ttft_us"], kw["slo_tpot_us"], kw["penalty_us"])
            else:
                binding.ap_costtable_set(self.handle, tables[0], kw["t_on_us"], kw["t_off_us"], kw["B"],
                                         kw["slo_ttft_us"], kw["slo_tpot_us"], kw["penalty_us"], tables[1], tables[2])
        except Exception:
            self.close()
            raise

    def eval_device(self, d_assign: torch.Tensor, d_out: torch.Tensor | None = None) -> torch.Tensor:
        """d_assign: CUDA tensor [C, R] of 2-byte elements.  Returns the CUDA result tensor [C, 8] int64."""
        assert d_assign.is_cuda and d_assign.element_size() == 2 and d_assign.is_contiguous()
        assert d_assign.shape[1] == self.R
        C = d_assign.shape[0]
        if d_out is None:
            d_out = torch.full((C, 8), -1, dtype=torch.int64, device=d_assign.device)
        binding.ap_eval_candidates(self.handle, d_assign.data_ptr(), C, d_out.data_ptr(),
                                   torch.cuda.current_stream().cuda_stream)
        return d_out

    def eval(self, rows: np.ndarray) -> np.ndarray:
        rows = np.ascontiguousarray(rows, dtype=np.uint16)
        d_assign = torch.from_numpy(rows.view(np.int16)).cuda()
        d_out = self.eval_device(d_assign)
        torch.cuda.synchronize()
        return to_records(d_out)

    def counts(self):
        """(candidates scored, candidates that went through the exact replay kernels) since the cost model was set."""
        return binding.ap_eval_counts_get(self.handle)

    def set_parent(self, parent: np.ndarray, max_children: int) -> None:
        binding.ap_parent_set(self.handle, parent, max_children)

    def eval_children_device(self, d_first: torch.Tensor, d_request: torch.Tensor, d_replica: torch.Tensor,
                             d_out: torch.Tensor | None = None) -> torch.Tensor:
        """Edit lists as CUDA tensors (int32 [C+1], int32 [E], int16 [E]); returns the CUDA result tensor."""
        assert d_first.is_cuda and d_first.element_size() == 4 and d_request.element_size() == 4
        assert d_replica.element_size() == 2 and d_request.shape == d_replica.shape
        C = d_first.shape[0] - 1
        if d_out is None:
            d_out = torch.full((C, 8), -1, dtype=torch.int64, device=d_first.device)
        binding.ap_eval_children(self.handle, d_first.data_ptr(), d_request.data_ptr(), d_replica.data_ptr(), C,
                                 d_out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        return d_out

    def eval_children(self, first: np.ndarray, request: np.ndarray, replica: np.ndarray) -> np.ndarray:
        d_out = self.eval_children_device(*edit_lists_to_device(first, request, replica))
        torch.cuda.synchronize()
        return to_records(d_out)

    def close(self):
        if self.handle is not None:
            binding.ap_workload_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def edit_lists_to_device(first, request, replica):
    """Upload edit lists; the two edit arrays get one spare element so that their pointers are valid when empty."""
    first = np.ascontiguousarray(first, dtype=np.uint32)
    request = np.concatenate([np.ascontiguousarray(request, dtype=np.uint32), np.zeros(1, np.uint32)])
    replica = np.concatenate([np.ascontiguousarray(replica, dtype=np.uint16), np.zeros(1, np.uint16)])
    return (torch.from_numpy(first.view(np.int32)).cuda(), torch.from_numpy(request.view(np.int32)).cuda(),
            torch.from_numpy(replica.view(np.int16)).cuda())


def to_records(d_out: torch.Tensor) -> np.ndarray:
    return d_out.cpu().numpy().view(binding.METRICS_DTYPE).reshape(-1)


def oracle_for(tr, **override) -> Oracle:
    return Oracle.from_trace(tr, **override)


def assert_same(got: np.ndarray, want: np.ndarray, what: str = "") -> None:
    """Bit-exact comparison of metric records; on failure name the first differing row and fields."""
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if got.tobytes() == want.tobytes():
        return
    for c in range(got.shape[0]):
        if got[c] != want[c]:
            diff = {n: (int(got[c][n]), int(want[c][n])) for n in got.dtype.names if got[c][n] != want[c][n]}
            raise AssertionError(f"{what}: row {c} differs (gpu, oracle): {diff}")
    raise AssertionError(f"{what}: records differ in padding only")
