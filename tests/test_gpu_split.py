"""GPU parity for replicas that differ or have availability windows, where the library cuts every replica's trace
into a listed part (replayed one queue per lane) and a streamed part (scored on arrival): every branch of that path
against the CPU oracle, byte for byte, through the C ABI; ``ap_eval_counts_get`` tells which candidates the path
settled itself and which it handed to the general replay."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from paper_2604_07144_amd import binding, traces          # noqa: E402
from tests.gpu_harness import GpuWorkload, assert_same, oracle_for   # noqa: E402

U64MAX = 0xFFFFFFFFFFFFFFFF
STD, FAST, SLOW = traces.COEF_STANDARD, traces.COEF_FAST, traces.COEF_SLOW


def elastic(n, M, B, rate, seed, *, closing=True, **kw):
    """Poisson arrivals at `rate` per second, lognormal lengths, three kinds of replica in turn, windows drawn
    inside the trace (closing=False: replicas come up but never leave)."""
    rng = np.random.default_rng(seed)
    arrival = (np.floor(np.cumsum(rng.exponential(1.0 / rate, n)) * 1e6) + 123_456_789).astype(np.uint64)
    prompt = np.clip(np.floor(rng.lognormal(6.0, 1.0, n)), 16, 4096)
    out = np.clip(np.floor(rng.lognormal(5.0, 1.0, n)), 1, 1024)
    xy = rng.integers(int(arrival[0]), int(arrival[-1]) + 1, size=(M, 2)).astype(np.uint64)
    t_on = xy.min(1)
    t_off = xy.max(1) if closing else np.full(M, U64MAX, dtype=np.uint64)
    return traces.custom_trace(arrival, prompt, out, [[STD, FAST, SLOW][m % 3] for m in range(M)], t_on, t_off, B=B, **kw)


def rows(C, n, hi, seed):
    return np.random.default_rng(seed).integers(0, hi, size=(C, n)).astype(np.uint16)


def both(tr, r, what, **override):
    with GpuWorkload(tr, **override) as g:
        got = g.eval(r)
        counts = g.counts()
    assert_same(got, oracle_for(tr, **override).eval_batch(r, nthreads=8), what)
    assert counts[0] == r.shape[0]
    return got, counts


def test_elastic_cluster_settled_without_the_general_replay():
    """A calm trace (far fewer requests in service than slots): backlogs behind t_on are replayed from their lists,
    the rest is scored on arrival, a third of the requests is rejected, so the p99 values are the penalty."""
    tr = elastic(20000, 48, 64, 1200.0, seed=1)
    got, (scored, replayed) = both(tr, rows(70, tr.R, 48, seed=2), "elastic, calm")
    assert replayed == 0 and int(got["n_rejected"].min()) > tr.R // 100
    got, (_, replayed) = both(tr, rows(5, tr.R, 50, seed=3), "elastic, calm, some unknown replica ids", B=16)
    assert replayed == 0


def test_replicas_that_never_leave_need_the_histograms():
    """No window closes: nothing is rejected, so the percentiles come from the histograms - streamed requests counted
    in LDS, listed ones added in device memory."""
    tr = elastic(15000, 24, 32, 900.0, seed=4, closing=False)
    got, (_, replayed) = both(tr, rows(40, tr.R, 24, seed=5), "elastic, nobody leaves")
    assert replayed <= 4 and int(got["n_rejected"].max()) == 0          # the split is a guess: a few may be handed back
    assert int(got["p99_ttft_us"].min()) > 100_000                      # waiting behind t_on dominates the tail


def test_candidates_that_avoid_closed_replicas_among_candidates_that_do_not():
    """Most rows spread requests over all replicas (many rejections: no histograms needed); two rows use only replicas
    that are up throughout, so they reject nothing and are streamed a second time with histograms."""
    tr = elastic(12000, 20, 64, 800.0, seed=6)
    t_on, t_off = tr.t_on_us.copy(), tr.t_off_us.copy()
    t_on[[3, 7]], t_off[[3, 7]] = 0, U64MAX
    r = rows(30, tr.R, 20, seed=7)
    r[4] = np.where(np.arange(tr.R) % 2 == 0, 3, 7)
    r[11] = 7
    got, (_, replayed) = both(tr, r, "mixed need for histograms", t_on_us=t_on, t_off_us=t_off)
    assert int(got["n_rejected"][4]) == 0 and int(got["n_rejected"][11]) == 0 and int(got["n_rejected"][0]) > 120
    assert replayed <= 3


def test_a_backlog_far_beyond_the_guess_goes_to_the_general_replay():
    """Every request on one replica that comes up late: its backlog is twenty times what an even spread would give,
    it has not drained where the streamed part begins, and the candidate is handed to the general replay."""
    tr = elastic(16000, 20, 64, 600.0, seed=8, closing=False)
    middle = int(np.argsort(tr.t_on_us)[8])                             # comes up some way into the trace
    r = rows(12, tr.R, 20, seed=9)
    r[5] = middle
    got, (_, replayed) = both(tr, r, "one overloaded replica")
    assert 1 <= replayed <= 3


def test_dense_trace_lists_every_request():
    """More requests in service than a replica has slots at almost any moment: nothing can be scored on arrival, every
    request that is not rejected goes through its replica's list."""
    tr = elastic(9000, 6, 8, 20000.0, seed=10)
    got, (_, replayed) = both(tr, rows(10, tr.R, 6, seed=11), "dense, windows")
    assert replayed == 0
    tr = elastic(9000, 6, 5, 20000.0, seed=12, closing=False, slo_ttft_us=4000, slo_tpot_us=40)
    both(tr, rows(10, tr.R, 7, seed=13), "dense, no rejections, tight objectives")


def test_small_penalty_keeps_the_histograms():
    """A penalty latency below the served latencies: rejected requests do not sit on top of the histogram, so the
    percentiles are never read off the penalty."""
    tr = elastic(10000, 16, 64, 700.0, seed=14, penalty_us=900)
    both(tr, rows(16, tr.R, 16, seed=15), "penalty below the latencies")


def test_more_candidates_than_one_batch_of_scratch():
    """The scratch area holds a fixed number of candidates' lists (about 4 GiB / 0.9 MiB here); a call with more
    candidates is worked off in batches."""
    tr = elastic(60000, 64, 64, 2500.0, seed=16)
    C = 5400
    r = rows(C, tr.R, 64, seed=17)
    with GpuWorkload(tr) as g:
        got = g.eval(r)
    pick = np.unique(np.concatenate([np.arange(0, C, 37), np.arange(C - 450, C)]))
    assert_same(got[pick], oracle_for(tr).eval_batch(r[pick], nthreads=8), "several batches")


@pytest.mark.parametrize("n,M,B", [(1, 3, 2), (63, 5, 64), (1024, 64, 64), (1025, 65, 8), (4097, 100, 33), (2047, 2, 1)])
def test_tile_and_table_edges(n, M, B):
    tr = elastic(n, M, B, 2000.0, seed=n + M)
    both(tr, rows(9, n, M + 1, seed=n), f"edges n={n} M={M} B={B}")
    still = elastic(n, M, B, 2000.0, seed=n + M + 1, closing=False)
    both(still, rows(9, n, M, seed=n + 1), f"edges, nobody leaves n={n} M={M} B={B}")


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_windows_and_objectives(seed):
    """Shapes, loads, windows and objectives drawn at random: calm to heavily overloaded, one to three kinds of
    replica, windows inside, around and outside the trace, penalties above and below the served latencies, rows with
    unknown replica ids and rows that name a single replica."""
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.choice([1, 2, 65, 700, 1024, 3000, 5000]))
    M = int(rng.choice([1, 2, 7, 33, 64, 65, 140]))
    B = int(rng.choice([1, 2, 7, 8, 16, 31, 64]))
    per_slot = float(rng.choice([0.02, 0.2, 1.0, 5.0]))                 # requests in service per slot, roughly
    rate = max(50.0, per_slot * M * B / 0.012)                          # a request is in service for about 12 ms
    closing = bool(rng.integers(0, 2))
    kw = {}
    if rng.integers(0, 3) == 0:
        kw["penalty_us"] = int(rng.choice([1, 900, 50_000]))
    if rng.integers(0, 3) == 0:
        kw["slo_ttft_us"], kw["slo_tpot_us"] = int(rng.choice([0, 4000, 10**9])), int(rng.choice([0, 40, 10**6]))
    tr = elastic(n, M, B, rate, seed=2000 + seed, closing=closing, **kw)
    t_on, t_off = tr.t_on_us.copy(), tr.t_off_us.copy()
    for m in range(M):                                                  # some windows that do not cut the trace
        pick = rng.integers(0, 8)
        if pick == 0:
            t_on[m], t_off[m] = 0, U64MAX
        elif pick == 1:
            t_on[m], t_off[m] = 0, int(tr.arrival_us[0])                # closed before the first arrival
        elif pick == 2:
            t_on[m] = t_off[m]                                          # empty
        elif pick == 3:
            t_on[m], t_off[m] = int(tr.arrival_us[-1]) + 1, U64MAX      # up after the last arrival
    if rng.integers(0, 4) == 0:                                         # one kind only
        override = dict(coef=[STD] * M, t_on_us=t_on, t_off_us=t_off)
    else:
        override = dict(t_on_us=t_on, t_off_us=t_off)
    r = rows(9, n, M + int(rng.integers(0, 3)), seed=3000 + seed)
    r[3] = int(rng.integers(0, M))
    both(tr, r, f"random seed={seed} n={n} M={M} B={B} rate={rate:.0f} closing={closing} {kw}", **override)


@pytest.mark.parametrize("n,M,B,rate", [(6000, 8, 4, 1500.0), (20000, 128, 64, 400000.0), (1500, 3, 64, 12000.0)])
def test_identical_replicas_under_load_go_through_the_lists(n, M, B, rate):
    """Identical replicas that are up throughout, with a quarter of the slots or more in service on average: the
    screen that proves nobody waits would pass hardly any candidate, so every queue is replayed from its list and
    the histograms are filled from the bins the replay leaves."""
    rng = np.random.default_rng(n)
    arrival = (np.floor(np.cumsum(rng.exponential(1.0 / rate, n)) * 1e6) + 5).astype(np.uint64)
    prompt = np.clip(np.floor(rng.lognormal(6.0, 1.0, n)), 16, 4096)
    out = np.clip(np.floor(rng.lognormal(5.0, 1.0, n)), 1, 1024)
    tr = traces.custom_trace(arrival, prompt, out, [STD] * M, np.zeros(M, np.uint64), np.full(M, U64MAX, np.uint64), B=B)
    r = rows(70, n, M, seed=n + 1)
    r[9] = 0                                                            # everything on one replica
    got, (_, replayed) = both(tr, r, f"identical replicas under load n={n} M={M} B={B}")
    assert replayed == 0 and int(got["n_rejected"].max()) == 0
    assert int(got["p99_ttft_us"][9]) > int(np.median(got["p99_ttft_us"]))


def _tables(tr, n_types, seed, scale=1.0):
    """Arbitrary cost tables: per type and request a prefill time and a time per token, unrelated to the lengths."""
    rng = np.random.default_rng(seed)
    prefill = (rng.integers(200, 30_000, size=(n_types, tr.R)) * scale).astype(np.uint32)
    tpot = (rng.integers(5, 120, size=(n_types, tr.R)) * scale).astype(np.uint32)
    return prefill, tpot


@pytest.mark.parametrize("n,M,B,rate,closing,n_types", [
    (20000, 48, 64, 1200.0, True, 3),        # calm, windows: backlogs listed, the rest scored on arrival
    (15000, 24, 32, 900.0, False, 2),        # nobody leaves: histograms from both parts
    (9000, 6, 8, 20000.0, True, 4),          # dense: every request listed
    (70000, 40, 16, 3000.0, True, 1),        # one type, R >= 65536
    (2047, 130, 33, 2000.0, True, 5),        # more than 64 replicas, ragged tile
])
def test_tabulated_cost_model_through_the_lists(n, M, B, rate, closing, n_types):
    """The listed / streamed evaluation with service times read from tables (two loads per streamed request; the
    list replay stages its replica type's entries next to the request records)."""
    tr = elastic(n, M, B, rate, seed=n + M, closing=closing)
    rep_type = (np.arange(M) * 7 % n_types).astype(np.uint32)
    prefill, tpot = _tables(tr, n_types, seed=n)
    r = rows(11, n, M + 1, seed=n + 2)
    r[4] = M - 1
    with GpuWorkload(tr, tables=(rep_type, prefill, tpot)) as g:
        got = g.eval(r)
        scored, replayed = g.counts()
    want = oracle_for(tr).set_cost_tables(rep_type, prefill, tpot).eval_batch(r, nthreads=8)
    assert_same(got, want, f"tables through the lists n={n} M={M} B={B}")
    assert scored == 11 and replayed <= 3                               # handed back at most the odd overloaded row


def test_tabulated_identical_replicas_under_load():
    """One type, always up, crowded: the tabulated form of the saturated case."""
    n, M, B = 12000, 16, 8
    rng = np.random.default_rng(5)
    arrival = (np.floor(np.cumsum(rng.exponential(1.0 / 30000.0, n)) * 1e6) + 5).astype(np.uint64)
    prompt = np.clip(np.floor(rng.lognormal(6.0, 1.0, n)), 16, 4096)
    out = np.clip(np.floor(rng.lognormal(5.0, 1.0, n)), 1, 1024)
    tr = traces.custom_trace(arrival, prompt, out, [STD] * M, np.zeros(M, np.uint64), np.full(M, U64MAX, np.uint64), B=B)
    prefill, tpot = _tables(tr, 1, seed=6)
    rep_type = np.zeros(M, np.uint32)
    r = rows(20, n, M, seed=7)
    with GpuWorkload(tr, tables=(rep_type, prefill, tpot)) as g:
        got = g.eval(r)
        _, replayed = g.counts()
    assert_same(got, oracle_for(tr).set_cost_tables(rep_type, prefill, tpot).eval_batch(r, nthreads=8), "tables, crowded")
    assert replayed == 0


@pytest.mark.parametrize("closing", [True, False])
def test_records_do_not_depend_on_what_else_is_in_the_call(closing):
    """The scratch area keeps the last call's lists, bins and histograms: a row's record must be the same whatever
    rows surround it, in whatever order, and on a repeated call (closing=False: every candidate needs the bins)."""
    tr = elastic(9000, 20, 32, 1500.0, seed=40, closing=closing)
    r = rows(200, tr.R, 21, seed=41)
    r[17] = 3
    with GpuWorkload(tr) as g:
        whole = g.eval(r)
        perm = np.random.default_rng(1).permutation(200)
        assert_same(g.eval(r[perm]), whole[perm], "permuted")
        assert_same(g.eval(r[150:]), whole[150:], "a tail of the rows, after a larger call")
        assert_same(g.eval(r[17:18]), whole[17:18], "one row")
        assert_same(g.eval(r[:129]), whole[:129], "129 rows: two wavefronts of queues and a ragged third")
        assert_same(g.eval(r), whole, "the same call again")
    assert_same(whole, oracle_for(tr).eval_batch(r, nthreads=8), "against the oracle")


@pytest.mark.parametrize("closing", [True, False])
def test_captured_in_a_graph_and_replayed(closing):
    """The listed / streamed evaluation is kernel launches only (no clears, no copies), so the call can be captured;
    replays with new assignments in between, eager work and synchronisations around them, each against the oracle."""
    from tests.gpu_harness import to_records
    tr = elastic(7000, 18, 32, 1500.0, seed=50, closing=closing)
    C = 70
    orc = oracle_for(tr)
    with GpuWorkload(tr) as g:
        d_assign = torch.zeros((C, tr.R), dtype=torch.int16, device="cuda")
        d_out = torch.full((C, 8), -1, dtype=torch.int64, device="cuda")
        g.eval_device(d_assign, d_out)                                   # eager warm-up call
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            g.eval_device(d_assign, d_out)
        for it in range(4):
            r = rows(C, tr.R, 18 + (it % 2), seed=60 + it)
            r[0] = it % 18                                               # one overloaded replica: handed back
            d_assign.copy_(torch.from_numpy(r.view(np.int16)).cuda())
            d_out.fill_(-1)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert_same(to_records(d_out), orc.eval_batch(r, nthreads=8), f"replay {it}")
            assert_same(g.eval(r), to_records(d_out), f"eager call after replay {it}")


def test_switching_cost_models_on_one_workload():
    """One workload, its cost model replaced again and again: windows and three kinds (listed / streamed), the same as
    tables, identical replicas that are always up (screening), a slot count that makes the trace crowded (everything
    listed), and back.  Every set call re-plans kernels and scratch; no evaluation may see the previous plan."""
    tr = elastic(8000, 24, 32, 4000.0, seed=70)
    r = rows(40, tr.R, 25, seed=71)
    M = tr.M
    always = dict(t_on_us=np.zeros(M, np.uint64), t_off_us=np.full(M, U64MAX, np.uint64), coef=[STD] * M)
    rep_type = (np.arange(M) % 3).astype(np.uint32)
    prefill, tpot = _tables(tr, 3, seed=72)
    handle = binding.ap_workload_create(tr.arrival_us, tr.prompt_len, tr.out_len)
    d_assign = torch.from_numpy(np.ascontiguousarray(r).view(np.int16)).cuda()
    d_out = torch.zeros((40, 8), dtype=torch.int64, device="cuda")

    def run():
        from tests.gpu_harness import to_records
        d_out.fill_(-1)
        binding.ap_eval_candidates(handle, d_assign.data_ptr(), 40, d_out.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        return to_records(d_out)

    def linear(B, **kw):
        binding.ap_costmodel_set(handle, binding.make_replicas(kw.get("coef", tr.coef), kw.get("t_on_us", tr.t_on_us),
                                                               kw.get("t_off_us", tr.t_off_us)),
                                 B, tr.slo_ttft_us, tr.slo_tpot_us, tr.penalty_us)
        return oracle_for(tr, B=B, **kw).eval_batch(r, nthreads=8)

    def tables(B):
        binding.ap_costtable_set(handle, rep_type, tr.t_on_us, tr.t_off_us, B, tr.slo_ttft_us, tr.slo_tpot_us,
                                 tr.penalty_us, prefill, tpot)
        return oracle_for(tr, B=B).set_cost_tables(rep_type, prefill, tpot).eval_batch(r, nthreads=8)

    try:
        for round_ in range(2):
            want = linear(32)
            assert_same(run(), want, f"windows, three kinds (round {round_})")
            want = tables(32)
            assert_same(run(), want, f"the same windows, tables (round {round_})")
            want = linear(64, **always)
            assert_same(run(), want, f"identical replicas, always up (round {round_})")
            want = linear(1, **always)
            assert_same(run(), want, f"one slot per replica: crowded (round {round_})")
            want = tables(2)
            assert_same(run(), want, f"tables, two slots (round {round_})")
    finally:
        binding.ap_workload_destroy(handle)
