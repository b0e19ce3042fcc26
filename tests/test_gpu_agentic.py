"""GPU parity for candidate plans of agentic workflows (``ap_agentic_*``), through the C ABI, against the
serial CPU oracle: integer work, so every field of every record must be equal."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle.agentic import AgenticOracle                   # noqa: E402
from paper_2604_07144_amd import binding, traces          # noqa: E402

FIELDS = ("arrival_us", "slo_us", "wf", "in_len", "out_len", "pred_first", "pred", "pa", "pb", "qc", "qd", "cap",
          "penalty_permille")


def gpu_eval(wl, pre, dec, key):
    handle = binding.ap_agentic_create(*(wl[f] for f in FIELDS))
    try:
        C = pre.shape[0]
        d_pre = torch.from_numpy(np.ascontiguousarray(pre, dtype=np.uint16).view(np.int16)).cuda()
        d_dec = torch.from_numpy(np.ascontiguousarray(dec, dtype=np.uint16).view(np.int16)).cuda()
        d_key = torch.from_numpy(np.ascontiguousarray(key, dtype=np.uint32).view(np.int32)).cuda()
        d_out = torch.full((C, 5), -1, dtype=torch.int64, device="cuda")
        binding.ap_agentic_eval(handle, d_pre.data_ptr(), d_dec.data_ptr(), d_key.data_ptr(), C, d_out.data_ptr(),
                                torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        return d_out.cpu().numpy().view(binding.AGENTIC_METRICS_DTYPE).reshape(-1)
    finally:
        binding.ap_agentic_destroy(handle)


def both(wl, pre, dec, key, what):
    got = gpu_eval(wl, pre, dec, key)
    want = AgenticOracle.from_workload(wl).eval_batch(pre, dec, key)
    for c in range(pre.shape[0]):
        assert got[c].tolist() == want[c].tolist(), (what, c, got[c], want[c])
    return got


def tiny(P=1, cap=300):
    return dict(arrival_us=[0], slo_us=[10000], wf=[0, 0, 0], in_len=[100, 200, 50], out_len=[10, 5, 20],
                pred_first=[0, 0, 1, 2], pred=[0, 0], pa=[100] * P, pb=[1] * P, qc=[10], qd=[0], cap=[cap],
                penalty_permille=77_000)


def test_hand_worked_schedules_on_gpu():
    rows = lambda *r: tuple(np.array([x], dtype=t) for x, t in zip(r, (np.uint16, np.uint16, np.uint32)))
    got = both(tiny(), *rows([0, 0, 0], [0, 0, 0], [0, 1, 0]), "one prefill instance")
    assert (int(got["sum_ratio_permille"][0]), int(got["makespan_us"][0])) == (80, 800)
    got = both(tiny(P=2, cap=250), *rows([0, 0, 1], [0, 0, 0], [0, 0, 0]), "budget blocks admission")
    assert int(got["makespan_us"][0]) == 700
    got = both(tiny(P=2, cap=150), *rows([0, 0, 1], [0, 0, 0], [0, 0, 0]), "a call that never fits")
    assert (int(got["sum_ratio_permille"][0]), int(got["n_failed"][0])) == (77_000, 1)
    both(tiny(P=2), *rows([9, 0, 1], [0, 0, 9], [0, 0, 0]), "unknown instances")


def test_token_budget_near_the_32_bit_limit():
    """Two calls of 3e9 tokens each on a decode instance whose budget is 2^32 - 1: together they exceed it (and the
    32-bit sum of their sizes wraps round), so the second waits for the first to leave."""
    wl = dict(arrival_us=[0, 0], slo_us=[10**6, 10**6], wf=[0, 1], in_len=[3_000_000_000, 3_000_000_000], out_len=[5, 7],
              pred_first=[0, 0, 0], pred=[], pa=[10], pb=[0], qc=[1000], qd=[0], cap=[2**32 - 1], penalty_permille=50_000)
    rows = tuple(np.array([x], dtype=t) for x, t in zip(([0, 0], [0, 0], [0, 1]), (np.uint16, np.uint16, np.uint32)))
    got = both(wl, *rows, "budget near 2^32")
    # prefill 10 us each, one at a time: decode of call 0 runs 10..5010, call 1 (ready at 20) is admitted at 5010
    assert int(got["makespan_us"][0]) == 5010 + 7000 and int(got["n_failed"][0]) == 0


@pytest.mark.parametrize("seed,W,P,Q,capacity,rate,mean_calls", [
    (0, 64, 4, 4, 16384, 20.0, 5.0),        # the paper-shaped slice, light
    (1, 64, 2, 2, 3000, 200.0, 5.0),        # contended on both stages, some ids outside the cluster
    (2, 64, 1, 3, 9000, 80.0, 5.0),
    (3, 64, 3, 1, 12000, 500.0, 5.0),
    (4, 1, 1, 1, 20000, 10.0, 1.0),         # one workflow
    (5, 33, 5, 7, 6000, 300.0, 9.0),        # odd sizes
    (6, 200, 64, 64, 4000, 2000.0, 5.0),    # as many instances as lanes, about a thousand calls
    (7, 64, 4, 4, 1200, 50.0, 3.0),         # tiny budgets: many calls can never fit
])
def test_random_workloads(seed, W, P, Q, capacity, rate, mean_calls):
    wl = traces.make_agentic(seed, W, P=P, Q=Q, capacity=capacity, rate=rate, mean_calls=mean_calls)
    K = len(wl["wf"])
    assert K <= 1024
    pre, dec, key = traces.draw_agentic_candidates(seed, 48, K, P, Q, key_range=[1 << 20, 40][seed % 2], bad_ids=seed == 1)
    got = both(wl, pre, dec, key, f"seed {seed} K={K}")
    assert len({tuple(r) for r in got.tolist()}) > 1 or W == 1


def test_largest_supported_sizes():
    """1024 workflows of one call each on 64 + 64 instances: every documented limit at once."""
    rng = np.random.default_rng(11)
    W = K = 1024
    wl = dict(arrival_us=np.sort(rng.integers(0, 2_000_000, W)).astype(np.uint64), slo_us=rng.integers(1, 10**6, W).astype(np.uint64),
              wf=np.arange(K, dtype=np.uint32), in_len=rng.integers(1, 4000, K).astype(np.uint32),
              out_len=rng.integers(1, 300, K).astype(np.uint32), pred_first=np.zeros(K + 1, np.uint32), pred=np.zeros(0, np.uint32),
              pa=rng.integers(1, 3000, 64).astype(np.uint32), pb=rng.integers(0, 4, 64).astype(np.uint32),
              qc=rng.integers(1, 50, 64).astype(np.uint32), qd=rng.integers(0, 9, 64).astype(np.uint32),
              cap=rng.integers(2000, 9000, 64).astype(np.uint32), penalty_permille=5000)
    pre, dec, key = traces.draw_agentic_candidates(3, 12, K, 64, 64, key_range=7, bad_ids=True)
    both(wl, pre, dec, key, "1024 workflows, 1024 calls, 64 + 64 instances")
    # a dependency chain through all 1024 calls of one workflow
    chain = dict(wl, arrival_us=[5], slo_us=[10**9], wf=np.zeros(K, np.uint32), pred_first=np.concatenate([[0], np.arange(K)]).astype(np.uint32),
                 pred=np.arange(K - 1, dtype=np.uint32))
    both(chain, pre, dec, key, "one chain of 1024 calls")


def test_error_paths():
    torch.cuda.init()
    wl = traces.make_agentic(0, 8)

    def status(**change):
        args = dict(wl)
        args.update(change)
        with pytest.raises(binding.ApError) as e:
            binding.ap_agentic_create(*(args[f] for f in FIELDS))
        return e.value.status

    bad = wl["wf"].copy(); bad[0] = 99
    assert status(wf=bad) == binding.AP_ERR_INVALID
    bad = wl["in_len"].copy(); bad[1] = 0
    assert status(in_len=bad) == binding.AP_ERR_INVALID
    bad = wl["slo_us"].copy(); bad[2] = 0
    assert status(slo_us=bad) == binding.AP_ERR_INVALID
    if len(wl["pred"]):
        bad = wl["pred"].copy(); bad[0] = len(wl["wf"]) - 1          # a predecessor that is not earlier
        assert status(pred=bad) == binding.AP_ERR_INVALID
    assert status(pa=[0] * 4, pb=[0] * 4) == binding.AP_ERR_INVALID          # a stage that takes no time
    assert status(pa=[0xFFFFFFFF] * 4) == binding.AP_ERR_RANGE               # times beyond 32 bits
    assert status(pa=[1] * 65, pb=[1] * 65) == binding.AP_ERR_RANGE          # more instances than supported
    h = binding.ap_agentic_create(*(wl[f] for f in FIELDS))
    with pytest.raises(binding.ApError) as e:
        binding.ap_agentic_eval(h, 0, 0, 0, 1, 0)
    assert e.value.status == binding.AP_ERR_INVALID
    binding.ap_agentic_eval(h, 0, 0, 0, 0, 0)                                 # C == 0
    binding.ap_agentic_destroy(h)
