"""GPU parity for the reconfiguration cost and end-to-end trace time (``ap_trace_time``), through the C ABI,
against ``oracle/reconfig.py``: integer nanoseconds, so every field must be equal."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import reconfig as rc                          # noqa: E402
from oracle import roofline as rf                          # noqa: E402
from paper_2604_07144_amd import binding                  # noqa: E402
from tests.test_gpu_roofline import GPUS, MODELS, _pack    # noqa: E402


SCOPES = {"deployed": binding.AP_LOAD_DEPLOYED, "changed": binding.AP_LOAD_CHANGED}


def run(models, coef, gpus, plans, n_intervals, sched, stale, serve, scope="deployed"):
    """plans: uint32 [C][N][Z][G][2]; returns the records as a structured array."""
    C, N = plans.shape[0], plans.shape[1]
    m, g, _ = _pack(models, gpus, [rf.Group(0, 0, 1, 1)])
    d_plans = torch.from_numpy(np.ascontiguousarray(plans, dtype=np.uint32).view(np.int32)).cuda()
    d_n = torch.from_numpy(np.asarray(n_intervals, dtype=np.uint32).view(np.int32)).cuda()
    d_sched = torch.from_numpy(np.asarray(sched, dtype=np.uint64).view(np.int64)).cuda()
    d_stale = torch.from_numpy(np.ascontiguousarray(stale, dtype=np.uint64).view(np.int64)).cuda()
    d_serve = torch.from_numpy(np.ascontiguousarray(serve, dtype=np.uint64).view(np.int64)).cuda()
    d_out = torch.full((C, 6), -1, dtype=torch.int64, device="cuda")
    binding.ap_trace_time(m, coef, g, d_plans.data_ptr(), d_n.data_ptr(), d_sched.data_ptr(), d_stale.data_ptr(),
                          d_serve.data_ptr(), C, N, d_out.data_ptr(), SCOPES[scope], torch.cuda.current_stream().cuda_stream)
    return d_out.cpu().numpy().view(binding.BREAKDOWN_DTYPE).reshape(-1)


def check(models, coef, gpus, plans, n_intervals, sched, stale, serve, scope="deployed"):
    got = run(models, coef, gpus, plans, n_intervals, sched, stale, serve, scope)
    tau = rc.transfer_ns(models, coef, gpus)
    for c in range(plans.shape[0]):
        n, s_stale, s_reconfig, s_serve, total = rc.trace_time(tau, plans[c], n_intervals[c], sched[c], stale[c], serve[c],
                                                               scope)
        want = (total, s_stale, s_reconfig, s_serve, int(sched[c]), n, 0)
        assert tuple(int(x) for x in got[c]) == want, (scope, c, got[c], want)
    return got


def test_random_plan_sequences():
    rng = np.random.default_rng(5)
    C, N, Z, G = 700, 6, len(MODELS), len(GPUS)
    options = np.array([(0, 0), (0, 0), (1, 1), (2, 1), (2, 2), (8, 1), (16, 4), (3, 0)], dtype=np.uint32)
    plans = options[rng.integers(0, len(options), size=(C, N, Z, G))]
    keep = rng.random((C, N)) < 0.35                                   # often a plan repeats its predecessor
    for i in range(1, N):
        plans[:, i][keep[:, i]] = plans[:, i - 1][keep[:, i]]
    n_intervals = rng.integers(0, N + 3, size=C).astype(np.uint32)      # 0 and values beyond N are clamped
    sched = rng.integers(0, 10**10, size=C).astype(np.uint64)
    stale = rng.integers(0, 10**10, size=(C, N)).astype(np.uint64)
    serve = rng.integers(0, 10**11, size=(C, N)).astype(np.uint64)
    got = check(MODELS, [5.3, 7.0, 11.5, 1.0], GPUS, plans, n_intervals, sched, stale, serve)
    assert (got["sum_reconfig_ns"] == 0).any() and (got["sum_reconfig_ns"] > 0).any()
    other = check(MODELS, [5.3, 7.0, 11.5, 1.0], GPUS, plans, n_intervals, sched, stale, serve, "changed")
    assert (other["sum_reconfig_ns"] < got["sum_reconfig_ns"]).any()    # an unchanged model loads slowest somewhere
    assert (other["sum_reconfig_ns"] <= got["sum_reconfig_ns"]).all()


def test_two_models_where_the_scopes_differ_on_gpu():
    """Model 0 changes its TP degree, model 1 (the larger one) stays: the loading cost as printed is the larger model's
    transfer time, the changed-only scope gives the smaller model's."""
    models, gpus = MODELS[:2], GPUS[:1]
    plans = np.array([[[[(2, 1)], [(4, 1)]], [[(4, 1)], [(4, 1)]]]], dtype=np.uint32)       # [1][2][2][1][2]
    args = (models, [1.0, 1.0], gpus, plans, np.array([2], np.uint32), np.array([7], np.uint64),
            np.array([[0, 11]], np.uint64), np.array([[13, 17]], np.uint64))
    tau = rc.transfer_ns(models, [1.0, 1.0], gpus)
    both = {scope: int(check(*args, scope)["sum_reconfig_ns"][0]) for scope in SCOPES}
    assert both["deployed"] == int(tau[0, 0]) + int(max(tau[0, 0], tau[1, 0]))
    assert both["changed"] == 2 * int(tau[0, 0])
    assert both["deployed"] != both["changed"]


def test_printed_worked_numbers_on_gpu():
    """System prompt Example C (13 GB over 32 and 64 GB/s: 0.41 s + 0.20 s) and the rows of Table 1."""
    small = rf.Model(40, 5120, 13824, 32000, 40, 40, 8)
    gpus = [rf.Gpu(80e9, 1e15, 3e12, 32e9, 4e11, 5e10, 8), rf.Gpu(80e9, 1e15, 3e12, 64e9, 4e11, 5e10, 8)]
    coef = [13e9 / rf.weight_bytes(small)]
    plans = np.array([[[[(1, 1), (0, 0)]], [[(0, 0), (1, 1)]]]], dtype=np.uint32)          # [1][2][1][2][2]
    got = check([small], coef, gpus, plans, np.array([2], np.uint32), np.array([0], np.uint64),
                np.zeros((1, 2), np.uint64), np.zeros((1, 2), np.uint64))
    assert round(int(got["sum_reconfig_ns"][0]) / 1e9, 2) == 0.61
    rows = ((2, 7.6, 12.0, 25.2, 44.8), (5, 5.5, 4.0, 24.0, 33.5), (1, 10.0, 17.0, 23.0, 50.0))
    N = 6
    plans = np.zeros((3, N, 1, 2, 2), dtype=np.uint32)
    n_intervals, stale, serve = np.zeros(3, np.uint32), np.zeros((3, N), np.uint64), np.zeros((3, N), np.uint64)
    gpus_t, coefs = [], None
    for c, (n_resched, s_stale, s_reconfig, s_serve, _) in enumerate(rows):
        n = n_resched + 1
        n_intervals[c] = n
        for i in range(N):
            plans[c, i, 0, 0] = (1 + (i % 2), 1)                       # the TP degree flips every interval
        stale[c, 1:n] = int(round(s_stale / n_resched * 1e9))
        serve[c, :n] = int(round(s_serve / n * 1e9))
    # one GPU type per row would need different transfer times; instead give each row its own call
    for c, (n_resched, s_stale, s_reconfig, s_serve, total) in enumerate(rows):
        want_tau = s_reconfig / n_resched / 2                          # termination + loading = twice tau
        gpus_c = [rf.Gpu(80e9, 1e15, 3e12, rf.weight_bytes(small) / want_tau, 4e11, 5e10, 8)] * 2
        got = check([small], [1.0], gpus_c, plans[c:c + 1], n_intervals[c:c + 1], np.array([0], np.uint64),
                    stale[c:c + 1], serve[c:c + 1])
        assert [round(int(got[k][0]) / 1e9, 1) for k in ("sum_stale_ns", "sum_reconfig_ns", "sum_serve_ns", "total_ns")] == \
            [s_stale, s_reconfig, s_serve, total]


def test_error_paths():
    torch.cuda.init()
    m, g, _ = _pack(MODELS[:1], GPUS[:1], [rf.Group(0, 0, 1, 1)])
    buf = torch.zeros(64, dtype=torch.int64, device="cuda")
    ptr = buf.data_ptr()

    def status(models, coef, gpus, C=1, N=1, hole=None, scope=0):
        args = [models, coef, gpus, ptr, ptr, ptr, ptr, ptr, C, N, ptr, scope]
        if hole is not None:
            args[hole] = 0
        with pytest.raises(binding.ApError) as e:
            binding.ap_trace_time(*args)
        return e.value.status

    assert status(m, [0.0], g) == binding.AP_ERR_INVALID             # coefficient must be positive
    bad = g.copy()
    bad["pcie_bytes_per_s"] = 0.0
    assert status(m, [1.0], bad) == binding.AP_ERR_INVALID
    assert status(m, [1.0], g, N=0) == binding.AP_ERR_INVALID
    assert status(m, [1.0], g, scope=2) == binding.AP_ERR_INVALID
    for hole in (3, 4, 5, 6, 7, 10):
        assert status(m, [1.0], g, hole=hole) == binding.AP_ERR_INVALID
    binding.ap_trace_time(m, [1.0], g, ptr, ptr, ptr, ptr, ptr, 0, 1, ptr)      # C == 0: nothing to do
