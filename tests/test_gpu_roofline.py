"""GPU parity for the roofline cost tables (``ap_roofline_tables`` / ``ap_roofline_costs``), through the C ABI,
against ``oracle/roofline.py``.  The kernels do the same IEEE double operations in the same order as the oracle
(no fused multiply-add) and round to whole nanoseconds before anything is summed, so the bar is bit equality
of every table entry; sums of decode steps are integers."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import roofline as rf                          # noqa: E402
from paper_2604_07144_amd import binding, traces          # noqa: E402
from tests.gpu_harness import GpuWorkload, assert_same, oracle_for   # noqa: E402

MODELS = [rf.Model(32, 4096, 11008, 32000, 32, 32, 16),          # 7B-class, multi-head attention
          rf.Model(32, 4096, 14336, 128256, 32, 8, 16),          # 8B-class, grouped-query attention
          rf.Model(80, 8192, 28672, 128256, 64, 8, 8),           # 70B-class, 8-bit weights
          rf.Model(2, 64, 100, 7, 4, 1, 4)]                      # tiny, odd sizes, 4-bit
GPUS = [rf.Gpu(288e9, 2.5e15, 8e12, 128e9, 1.075e12, 50e9, 8),
        rf.Gpu(80e9, 989e12, 3.35e12, 64e9, 450e9, 25e9, 8),
        rf.Gpu(24e9, 82.6e12, 1.008e12, 32e9, 32e9, 12.5e9, 2)]


def _pack(models, gpus, groups):
    m = np.array([(x.layers, x.hidden, x.intermediate, x.vocab, x.heads, x.kv_heads, x.weight_bits) for x in models],
                 dtype=binding.MODEL_DTYPE)
    g = np.zeros(len(gpus), dtype=binding.GPU_DTYPE)
    for i, x in enumerate(gpus):
        g[i] = (x.mem_bytes, x.flops, x.hbm_bytes_per_s, x.pcie_bytes_per_s, x.link_intra_bytes_per_s,
                x.link_inter_bytes_per_s, x.gpus_per_node)
    q = np.array([(x.model, x.gpu, x.tp, x.batch) for x in groups], dtype=binding.GROUP_DTYPE)
    return m, g, q


def _all_groups():
    return [rf.Group(z, g, t, b) for z in range(len(MODELS)) for g in range(len(GPUS)) for t in (1, 2, 4, 16)
            for b in (1, 8, 64)]


@pytest.mark.parametrize("max_seq", [1, 255, 256, 257, 5000])
def test_tables_bit_exact(max_seq):
    torch.cuda.init()
    groups = _all_groups()
    want_pre, want_prefix = rf.tables(MODELS, GPUS, groups, max_seq)
    got_pre, got_prefix, weight, feasible = binding.ap_roofline_tables(*_pack(MODELS, GPUS, groups), max_seq)
    assert got_pre.shape == want_pre.shape and got_prefix.shape == want_prefix.shape
    bad = np.argwhere(got_pre != want_pre)
    assert bad.size == 0, (groups[bad[0][0]], int(bad[0][1]), int(got_pre[tuple(bad[0])]), int(want_pre[tuple(bad[0])]))
    bad = np.argwhere(got_prefix != want_prefix)
    assert bad.size == 0, (groups[bad[0][0]], int(bad[0][1]), int(got_prefix[tuple(bad[0])]), int(want_prefix[tuple(bad[0])]))
    assert weight.tolist() == [rf.weight_bytes(MODELS[x.model]) for x in groups]
    assert feasible.tolist() == [int(rf.feasible(MODELS[x.model], GPUS[x.gpu], x.tp)) for x in groups]
    assert 0 < int(feasible.sum()) < len(groups)                   # both verdicts occur


def test_long_tables_bit_exact():
    """A million sequence lengths for one compute-heavy and one memory-heavy group: the prefix sums run through
    thousands of tiles and reach 2^47 ns."""
    torch.cuda.init()
    groups = [rf.Group(2, 1, 8, 64), rf.Group(3, 2, 1, 1)]
    max_seq = 1 << 20
    want_pre, want_prefix = rf.tables(MODELS, GPUS, groups, max_seq)
    got_pre, got_prefix, _, _ = binding.ap_roofline_tables(*_pack(MODELS, GPUS, groups), max_seq)
    assert (got_pre == want_pre).all() and (got_prefix == want_prefix).all()
    assert int(want_prefix[0, -1]) > 1 << 47


def test_request_costs_and_the_replay_on_top_of_them():
    """Tables for three replica types of a trace, computed on the device, handed to ap_costtable_set, and the
    replay's records compared with the oracle's tabulated branch fed with the oracle's own tables."""
    tr = traces.make_trace(3, C=32, R=2000, M=12)        # short enough for 32-bit microseconds at these speeds
    groups = [rf.Group(1, 0, 1, 8), rf.Group(1, 1, 2, 8), rf.Group(0, 0, 4, 16)]
    want_pre, want_tpot = rf.request_costs(MODELS, GPUS, groups, tr.prompt_len, tr.out_len)
    rep_type = (np.arange(tr.M) % 3).astype(np.uint32)
    rows = tr.assignment_rows(0, 32)
    with GpuWorkload(tr) as g:
        got_pre, got_tpot = binding.ap_roofline_costs(g.handle, tr.R, *_pack(MODELS, GPUS, groups))
        assert (got_pre == want_pre).all() and (got_tpot == want_tpot).all()
        assert int(want_pre.min()) > 0 and int(want_tpot.min()) > 0 and len(np.unique(want_pre[0])) > 100
        binding.ap_costtable_set(g.handle, rep_type, tr.t_on_us, tr.t_off_us, tr.B, tr.slo_ttft_us, tr.slo_tpot_us,
                                 tr.penalty_us, got_pre, got_tpot)
        got = g.eval(rows)
    want = oracle_for(tr).set_cost_tables(rep_type, want_pre, want_tpot).eval_batch(rows, nthreads=8)
    assert_same(got, want, "replay on roofline tables")


def test_tables_that_stay_on_the_device_and_the_chain_on_one_stream():
    """Roofline tables -> replay -> trace time without a table or a record crossing to the host in between:
    ap_costtable_set_roofline fills the workload's own table buffers, ap_eval_candidates leaves its records on the
    device, one torch operation on the same stream turns makespans into serving times, and ap_trace_time_static
    (which neither allocates nor waits) adds them up.  The oracle chain: roofline.request_costs ->
    Oracle.set_cost_tables / eval_batch -> reconfig.trace_time."""
    from oracle import reconfig as rc
    tr = traces.make_trace(3, C=48, R=2000, M=12)
    groups = [rf.Group(1, 0, 1, 8), rf.Group(1, 1, 2, 8), rf.Group(0, 0, 4, 16)]
    rep_type = (np.arange(tr.M) % 3).astype(np.uint32)
    rows = tr.assignment_rows(0, 48)
    n_cand, N = 16, 3                                        # candidate c serves interval i under row 3 c + i
    models, gpus = MODELS[:2], GPUS[:2]
    coef = [5.3, 7.0]
    rng = np.random.default_rng(11)
    options = np.array([(0, 0), (1, 1), (2, 1), (4, 2)], dtype=np.uint32)
    plans = options[rng.integers(0, len(options), size=(n_cand, N, len(models), len(gpus)))]
    n_intervals = np.full(n_cand, N, dtype=np.uint32)
    sched = rng.integers(0, 10**9, size=n_cand).astype(np.uint64)
    stale = rng.integers(0, 10**9, size=(n_cand, N)).astype(np.uint64)
    m, g, q = _pack(MODELS, GPUS, groups)
    m2, g2, _ = _pack(models, gpus, [rf.Group(0, 0, 1, 1)])

    handle = binding.ap_workload_create(tr.arrival_us, tr.prompt_len, tr.out_len)
    try:
        for _ in range(2):                                   # the second call reuses every buffer of the first
            binding.ap_costtable_set_roofline(handle, rep_type, tr.t_on_us, tr.t_off_us, tr.B, tr.slo_ttft_us,
                                              tr.slo_tpot_us, tr.penalty_us, m, g, q)
        stream = torch.cuda.current_stream().cuda_stream
        d_assign = torch.from_numpy(np.ascontiguousarray(rows, dtype=np.uint16).view(np.int16)).cuda()
        d_plans = torch.from_numpy(np.ascontiguousarray(plans).view(np.int32)).cuda()
        d_n = torch.from_numpy(n_intervals.view(np.int32)).cuda()
        d_sched = torch.from_numpy(sched.view(np.int64)).cuda()
        d_stale = torch.from_numpy(stale.view(np.int64)).cuda()
        d_metrics = torch.full((48, 8), -1, dtype=torch.int64, device="cuda")
        d_total = torch.full((n_cand, 6), -1, dtype=torch.int64, device="cuda")
        torch.cuda.synchronize()                             # inputs are in place; nothing below waits for the device
        binding.ap_eval_candidates(handle, d_assign.data_ptr(), 48, d_metrics.data_ptr(), stream)
        d_serve = (d_metrics[:, 3] * 1000).reshape(n_cand, N).contiguous()       # makespan_us -> t_serve in ns
        binding.ap_trace_time_static(m2, coef, g2, d_plans.data_ptr(), d_n.data_ptr(), d_sched.data_ptr(),
                                     d_stale.data_ptr(), d_serve.data_ptr(), n_cand, N, d_total.data_ptr(),
                                     binding.AP_LOAD_DEPLOYED, stream)
        torch.cuda.synchronize()
        got_metrics = d_metrics.cpu().numpy().view(binding.METRICS_DTYPE).reshape(-1)
        got = d_total.cpu().numpy().view(binding.BREAKDOWN_DTYPE).reshape(-1)
    finally:
        binding.ap_workload_destroy(handle)

    want_pre, want_tpot = rf.request_costs(MODELS, GPUS, groups, tr.prompt_len, tr.out_len)
    want_metrics = oracle_for(tr).set_cost_tables(rep_type, want_pre, want_tpot).eval_batch(rows, nthreads=8)
    assert_same(got_metrics, want_metrics, "replay on tables that never left the device")
    serve = (want_metrics["makespan_us"].astype(np.uint64) * np.uint64(1000)).reshape(n_cand, N)
    tau = rc.transfer_ns(models, coef, gpus)
    for c in range(n_cand):
        n, s_stale, s_reconfig, s_serve, total = rc.trace_time(tau, plans[c], n_intervals[c], sched[c], stale[c], serve[c],
                                                               "deployed")
        assert tuple(int(x) for x in got[c]) == (total, s_stale, s_reconfig, s_serve, int(sched[c]), n, 0), c
    assert len(set(int(x) for x in got["sum_reconfig_ns"])) > 4 and int(got["sum_serve_ns"].min()) > 0


def test_chained_tables_error_paths():
    tr = traces.make_trace(3, C=4, R=300, M=6)
    m, g, q = _pack(MODELS, GPUS, [rf.Group(1, 0, 1, 8), rf.Group(0, 0, 4, 16)])
    handle = binding.ap_workload_create(tr.arrival_us, tr.prompt_len, tr.out_len)
    try:
        def status(rep_type, groups=q, B=tr.B):
            with pytest.raises(binding.ApError) as e:
                binding.ap_costtable_set_roofline(handle, rep_type, tr.t_on_us, tr.t_off_us, B, tr.slo_ttft_us,
                                                  tr.slo_tpot_us, tr.penalty_us, m, g, groups)
            return e.value.status
        assert status(np.array([0, 1, 2, 0, 1, 0], np.uint32)) == binding.AP_ERR_INVALID       # type 2 of 2 groups
        bad = q.copy()
        bad["model"] = 9
        assert status(np.zeros(6, np.uint32), bad) == binding.AP_ERR_INVALID
        assert status(np.zeros(6, np.uint32), B=0) == binding.AP_ERR_INVALID
        # a 70B-class model on one slow GPU: a service time of hours does not fit 32-bit microseconds
        slow = _pack(MODELS, GPUS, [rf.Group(2, 2, 1, 64)])[2]
        assert status(np.zeros(6, np.uint32), slow) == binding.AP_ERR_RANGE
        d_assign = torch.zeros((1, tr.R), dtype=torch.int16, device="cuda")
        d_out = torch.zeros((1, 8), dtype=torch.int64, device="cuda")
        with pytest.raises(binding.ApError) as e:           # the failed call left no cost model behind
            binding.ap_eval_candidates(handle, d_assign.data_ptr(), 1, d_out.data_ptr(), 0)
        assert e.value.status == binding.AP_ERR_STATE
    finally:
        binding.ap_workload_destroy(handle)


def test_error_paths():
    torch.cuda.init()
    m, g, q = _pack(MODELS[:1], GPUS[:1], [rf.Group(0, 0, 1, 1)])

    def status(models, gpus, groups, max_seq=10):
        with pytest.raises(binding.ApError) as e:
            binding.ap_roofline_tables(models, gpus, groups, max_seq)
        return e.value.status

    for field, value in (("model", 1), ("gpu", 1), ("tp", 0), ("batch", 0)):
        bad = q.copy()
        bad[field] = value
        assert status(m, g, bad) == binding.AP_ERR_INVALID
    for field in ("layers", "heads", "weight_bits"):
        bad = m.copy()
        bad[field] = 0
        assert status(bad, g, q) == binding.AP_ERR_INVALID
    bad = m.copy()
    bad["kv_heads"] = 64                                            # more key-value heads than heads
    assert status(bad, g, q) == binding.AP_ERR_INVALID
    bad = g.copy()
    bad["hbm_bytes_per_s"] = 0.0
    assert status(m, bad, q) == binding.AP_ERR_INVALID
    assert status(m, g, q, max_seq=0) == binding.AP_ERR_INVALID
    assert status(m, g, q, max_seq=(1 << 24) + 1) == binding.AP_ERR_RANGE
    binding.ap_roofline_tables(m, g, q, 10)                         # and the valid call still works
