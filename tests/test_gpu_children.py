"""GPU parity for sparse candidates: children of a parent row given as edit lists
(``ap_parent_set`` / ``ap_eval_children``), through the C ABI, against the CPU oracle's
child-row rule followed by its replay, bit for bit.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from paper_2604_07144_amd import binding, traces          # noqa: E402
from tests.gpu_harness import (GpuWorkload, assert_same, edit_lists_to_device, oracle_for,   # noqa: E402
                               to_records)

U64MAX = 0xFFFFFFFFFFFFFFFF
STD, FAST, SLOW = traces.COEF_STANDARD, traces.COEF_FAST, traces.COEF_SLOW


def _mk(n, M, B, gap, seed, coef=None, t_on=None, t_off=None, **kw):
    rng = np.random.default_rng(seed)
    arrival = (np.cumsum(rng.integers(0, gap + 1, n)) + 1_000_000_007).astype(np.uint64)
    coef = coef or [[STD, FAST, SLOW][m % 3] for m in range(M)]
    return traces.custom_trace(arrival, rng.integers(1, 6000, n), rng.integers(1, 500, n), coef, t_on, t_off, B=B, **kw)


def both(tr, parent, lists, what, max_children=None, **override):
    first, request, replica = lists
    n_children = len(first) - 1
    with GpuWorkload(tr, **override) as g:
        g.set_parent(parent, max_children or max(1, n_children))
        got = g.eval_children(first, request, replica)
    want = oracle_for(tr, **override).eval_children(parent, first, request, replica, nthreads=8)
    assert_same(got, want, what)
    return got


# ------------------------------------------------------------------ hand-made lists
@pytest.mark.parametrize("coef", [[STD] * 4, [STD, FAST, SLOW, STD]], ids=["identical_replicas", "three_replica_types"])
def test_hand_made_lists(coef):
    """Empty list, repeated request (last edit wins), request outside the trace, unknown replica id, and a
    reversed range, with and without the shortcut for identical replicas."""
    tr = traces.custom_trace([0, 100, 200, 300, 400, 500], [100, 1024, 1025, 16, 700, 90], [10, 100, 1, 20, 5, 60],
                             coef, B=2)
    parent = np.array([0, 1, 2, 3, 0, 1], dtype=np.uint16)
    request = np.array([2, 5, 4, 4, 4, 6, 0xFFFFFFFF, 1, 0, 1, 2, 3, 4, 5], dtype=np.uint32)
    replica = np.array([3, 0, 1, 2, 3, 9, 9, 0xFFFF, 0, 0, 0, 0, 0, 0], dtype=np.uint16)
    first = np.array([0, 0, 2, 5, 8, 14, 8], dtype=np.uint32)        # the last child's range is reversed
    got = both(tr, parent, (first, request, replica), "hand-made lists")
    assert got[0] == got[5]                                          # no edits twice: the parent's record
    assert int(got[3]["n_rejected"]) == 1                            # the unknown id
    assert int(got[4]["sum_ttft_us"]) > int(got[0]["sum_ttft_us"])   # everything on one replica with two slots queues


# ------------------------------------------------------------------ both sides of the shortcut
def test_children_that_pass_and_children_that_need_their_row():
    n, M, B = 6000, 16, 8
    tr = _mk(n, M, B, 4000, seed=5, coef=[STD] * M)                  # light load, identical replicas
    parent = (np.arange(n) % M).astype(np.uint16)
    rng = np.random.default_rng(9)
    lists_req, lists_rep = [], []
    # 0: nothing; 1: three scattered edits; 2: 40 consecutive requests to replica 3 (more than the room: needs
    # its row, and queues); 3: 200 edits spread evenly (too many for the bound, yet no request waits);
    # 4: an unknown id; 5: an edit outside the trace only; 6: a long unsorted list with repeats
    lists_req.append(np.zeros(0, np.uint32)); lists_rep.append(np.zeros(0, np.uint16))
    lists_req.append(np.array([10, 3000, 5999], np.uint32)); lists_rep.append(np.array([1, 2, 3], np.uint16))
    lists_req.append(np.arange(1000, 1040, dtype=np.uint32)); lists_rep.append(np.full(40, 3, np.uint16))
    lists_req.append(np.arange(0, 6000, 30, dtype=np.uint32)); lists_rep.append((np.arange(200) % M).astype(np.uint16))
    lists_req.append(np.array([77], np.uint32)); lists_rep.append(np.array([M], np.uint16))
    lists_req.append(np.array([n], np.uint32)); lists_rep.append(np.array([0], np.uint16))
    lists_req.append(rng.integers(0, 300, 1000).astype(np.uint32)); lists_rep.append(rng.integers(0, M, 1000).astype(np.uint16))
    first = np.concatenate([[0], np.cumsum([len(x) for x in lists_req])]).astype(np.uint32)
    got = both(tr, parent, (first, np.concatenate(lists_req), np.concatenate(lists_rep)), "pass / row / replay")
    assert got[0] == got[1] == got[3] == got[5]                      # contention-free: one and the same record
    assert int(got[2]["sum_ttft_us"]) > int(got[0]["sum_ttft_us"])
    assert int(got[4]["n_rejected"]) == 1


@pytest.mark.parametrize("M,B,gap", [(16, 8, 4000), (128, 64, 100)], ids=["one_wavefront_screen", "eight_wavefront_screen"])
def test_calls_that_leave_work_for_the_replay_alternate_with_calls_that_leave_none(M, B, gap):
    """The kernels of a call tell each other through a word in device memory whether any candidate is still to
    be replayed, and consecutive calls on one workload take two such words in turn: every order of calls that
    do and do not leave such candidates, dense and as children, must give the oracle's records."""
    n = 5000
    tr = _mk(n, M, B, gap, seed=11, coef=[STD] * M)
    parent = (np.arange(n) % M).astype(np.uint16)
    crowded = parent.copy()
    crowded[1000:1000 + 6 * B] = 3                                    # more requests at once than replica 3 has slots
    rows_free = np.stack([parent, np.roll(parent, 1)])
    rows_wait = np.stack([parent, crowded, np.roll(parent, 2)])
    # children: none needs its row / the second one does
    free_lists = (np.array([0, 0, 2], np.uint32), np.array([5, 4000], np.uint32), np.array([1, 2], np.uint16))
    wait_lists = (np.array([0, 1, 1 + 6 * B, 1 + 6 * B], np.uint32),
                  np.concatenate([[9], np.arange(1000, 1000 + 6 * B)]).astype(np.uint32),
                  np.concatenate([[0], np.full(6 * B, 3)]).astype(np.uint16))
    orc = oracle_for(tr)
    want = {"free": orc.eval_batch(rows_free, nthreads=4), "wait": orc.eval_batch(rows_wait, nthreads=4),
            "free_children": orc.eval_children(parent, *free_lists, nthreads=4),
            "wait_children": orc.eval_children(parent, *wait_lists, nthreads=4)}
    assert int(want["wait"][1]["sum_ttft_us"]) > int(want["wait"][0]["sum_ttft_us"])          # somebody does wait
    assert int(want["wait_children"][1]["sum_ttft_us"]) > int(want["wait_children"][0]["sum_ttft_us"])
    order = ["wait", "free", "free", "wait", "wait", "free_children", "wait_children", "free_children", "free",
             "wait_children", "wait_children", "free", "wait", "free_children", "free_children", "wait", "free"]
    with GpuWorkload(tr) as g:
        g.set_parent(parent, 3)
        for step, kind in enumerate(order):
            if kind == "free":
                got = g.eval(rows_free)
            elif kind == "wait":
                got = g.eval(rows_wait)
            else:
                got = g.eval_children(*(free_lists if kind == "free_children" else wait_lists))
            assert_same(got, want[kind], f"call {step} ({kind})")


@pytest.mark.parametrize("burst_at", [2040, 4090, 5983], ids=["first_tile_boundary", "second_tile_boundary", "end"])
@pytest.mark.parametrize("B", [16, 17], ids=["burst_overflows", "burst_just_fits"])
def test_parent_depth_across_the_tiles_of_a_long_replica_list(B, burst_at):
    """One replica holds 6000 requests, which the parent analysis counts in tiles of 2048; 17 of them arrive in
    the same microsecond, straddling a tile boundary (or at the very end).  With 17 slots the parent is still
    contention-free and its children are settled from their lists; with 16 it is not, and every child must go
    through the dense path: a depth that lost the requests of the earlier tile would certify wrongly."""
    n, M = 6000, 2
    arrival = (np.arange(n, dtype=np.uint64) * 3000 + 1_000_000_007)
    arrival[burst_at:burst_at + 17] = arrival[burst_at]
    arrival[burst_at + 17:] += 200_000                              # the burst has drained before the next arrival
    tr = traces.custom_trace(arrival, np.full(n, 16), np.full(n, 1), [STD] * M, B=B)
    parent = np.zeros(n, np.uint16)
    first = np.array([0, 0, 1, 3, 4], np.uint32)
    request = np.array([10, burst_at + 3, burst_at + 20, 100], np.uint32)
    replica = np.array([1, 1, 1, 0], np.uint16)
    got = both(tr, parent, (first, request, replica), f"long list B={B} burst at {burst_at}")
    want_wait = B == 16
    assert (int(got[0]["sum_ttft_us"]) > n * 2048) == want_wait      # 2048 us of prefill each when nobody waits


def test_parent_that_queues_or_names_unknown_replicas():
    """No shortcut when the parent itself is not contention-free, or names a replica outside the table."""
    n, M, B = 3000, 4, 2
    tr = _mk(n, M, B, 300, seed=6, coef=[SLOW] * M)                  # heavy load: the parent queues
    parent = (np.arange(n) % M).astype(np.uint16)
    lists = traces.draw_edit_lists(11, 20, n, M, 12.0)
    both(tr, parent, lists, "queueing parent")
    light = _mk(n, M, 8, 20000, seed=6, coef=[FAST] * M)
    parent2 = parent.copy()
    parent2[1234] = M + 3
    got = both(light, parent2, lists, "parent with an unknown id")
    assert (got["n_rejected"] >= 0).all() and int(got["n_rejected"].max()) == 1
    # an edit can repair the parent's unknown id
    got = both(light, parent2, (np.array([0, 1], np.uint32), np.array([1234], np.uint32), np.array([0], np.uint16)),
               "repaired")
    assert int(got["n_rejected"][0]) == 0


@pytest.mark.parametrize("n,M,B,edits", [(4096, 8, 4, 3 * 4096), (1000, 3, 64, 2500), (777, 5, 1, 64 * 7)])
def test_lists_longer_than_the_trace(n, M, B, edits):
    """Many batches per child, most requests edited several times: the last edit must win across batches."""
    tr = _mk(n, M, B, 2000, seed=n, coef=[STD] * M)
    parent = np.zeros(n, np.uint16)
    lists = traces.draw_edit_lists(n, 6, n, M, float(edits), request_range=n + 5, replica_range=M + 1)
    both(tr, parent, lists, f"long lists n={n}")


# ------------------------------------------------------------------ random shapes
@pytest.mark.parametrize("seed", range(120))
def test_random_shapes_against_the_oracle(seed):
    rng = np.random.default_rng(5000 + seed)
    n = int(rng.choice([1, 7, 8, 63, 64, 65, 500, 512, 513, 1023, 1025, 3000, 4096, 9000]))
    M = int(rng.choice([1, 2, 3, 5, 8, 13, 33, 64, 128, 257, 600, 1024]))
    B = int(rng.choice([1, 2, 3, 8, 16, 31, 32, 48, 64]))
    gap = int(10 ** rng.uniform(1.0, 5.0))
    homogeneous = bool(rng.integers(0, 4))                           # mostly: that is where the shortcut applies
    windows = (not homogeneous) and bool(rng.integers(0, 2))
    t_on = t_off = None
    if windows:
        span = max(1, n * gap // 2)
        xy = rng.integers(0, span + 1, size=(M, 2)) + 1_000_000_007
        t_on, t_off = xy.min(1).astype(np.uint64), xy.max(1).astype(np.uint64)
    tr = _mk(n, M, B, gap, seed=seed, coef=[FAST] * M if homogeneous else None, t_on=t_on, t_off=t_off,
             penalty_us=int(rng.choice([1, 5_000_000, 3_600_000_000])))
    kind = int(rng.integers(0, 3))
    parent = [(np.arange(n) % M), rng.integers(0, M, n), np.zeros(n)][kind].astype(np.uint16)
    n_children = int(rng.integers(1, 40))
    mean = float(rng.choice([0.0, 1.0, 5.0, 70.0, n / 8 + 1]))
    lists = traces.draw_edit_lists(seed, n_children, n, M, mean, request_range=n + int(rng.integers(0, 2)) * 3,
                                   replica_range=M + int(rng.integers(0, 2)), sorted_lists=bool(rng.integers(0, 2)))
    both(tr, parent, lists, f"random n={n} M={M} B={B} gap={gap} homogeneous={homogeneous} windows={windows} "
                            f"parent={kind} children={n_children} mean={mean}",
         max_children=n_children + int(rng.integers(0, 3)))


# ------------------------------------------------------------------ the three-kernel replay behind it
def test_children_with_large_replica_tables():
    n, M, B = 5000, 1024, 64
    tr = _mk(n, M, B, 300, seed=8)                                   # three replica types: every child replayed
    parent = (np.arange(n) % M).astype(np.uint16)
    both(tr, parent, traces.draw_edit_lists(3, 9, n, M, 50.0), "M=1024 B=64 mixed")
    same = _mk(n, M, B, 300, seed=8, coef=[STD] * M)
    lists = traces.draw_edit_lists(4, 9, n, M, 50.0)
    lists[2][: int(lists[0][1])] = 5                                 # child 0 sends all its edits to replica 5
    both(same, parent, lists, "M=1024 B=64 identical")


# ------------------------------------------------------------------ state and errors
def test_state_and_error_paths():
    tr = _mk(500, 4, 4, 3000, seed=2, coef=[STD] * 4)
    parent = (np.arange(500) % 4).astype(np.uint16)
    lists = traces.draw_edit_lists(1, 5, 500, 4, 6.0)
    d_first, d_request, d_replica = edit_lists_to_device(*lists)
    d_out = torch.zeros((5, 8), dtype=torch.int64, device="cuda")

    def status_of(fn, *a):
        with pytest.raises(binding.ApError) as e:
            fn(*a)
        return e.value.status

    handle = binding.ap_workload_create(tr.arrival_us, tr.prompt_len, tr.out_len)
    try:
        assert status_of(binding.ap_parent_set, handle, parent, 5) == binding.AP_ERR_STATE      # no cost model yet
        rep = binding.make_replicas(tr.coef, tr.t_on_us, tr.t_off_us)
        binding.ap_costmodel_set(handle, rep, tr.B, tr.slo_ttft_us, tr.slo_tpot_us, tr.penalty_us)
        args = (handle, d_first.data_ptr(), d_request.data_ptr(), d_replica.data_ptr(), 5, d_out.data_ptr())
        assert status_of(binding.ap_eval_children, *args) == binding.AP_ERR_STATE               # no parent yet
        assert status_of(binding.ap_parent_set, handle, parent, 0) == binding.AP_ERR_INVALID
        binding.ap_parent_set(handle, parent, 4)
        assert status_of(binding.ap_eval_children, *args) == binding.AP_ERR_RANGE               # 5 children > 4
        binding.ap_parent_set(handle, parent, 5)
        for hole in (1, 2, 3, 5):
            bad = list(args)
            bad[hole] = 0
            assert status_of(binding.ap_eval_children, *bad) == binding.AP_ERR_INVALID
        binding.ap_eval_children(handle, d_first.data_ptr(), d_request.data_ptr(), d_replica.data_ptr(), 0, 0)   # C == 0
        binding.ap_eval_children(*args)
        torch.cuda.synchronize()
        want = oracle_for(tr).eval_children(parent, *lists)
        assert_same(to_records(d_out), want, "after the error probes")
        # a new cost model discards the parent; setting it again brings the path back with the new model
        binding.ap_costmodel_set(handle, rep, 1, tr.slo_ttft_us, tr.slo_tpot_us, tr.penalty_us)
        assert status_of(binding.ap_eval_children, *args) == binding.AP_ERR_STATE
        binding.ap_parent_set(handle, parent, 5)
        binding.ap_eval_children(*args)
        torch.cuda.synchronize()
        assert_same(to_records(d_out), oracle_for(tr, B=1).eval_children(parent, *lists), "B=1 after replacing the model")
        # a second parent on the same workload, fewer children than the rows were sized for
        parent2 = np.zeros(500, np.uint16)
        binding.ap_parent_set(handle, parent2, 3)
        d_out.fill_(-1)
        binding.ap_eval_children(handle, d_first.data_ptr(), d_request.data_ptr(), d_replica.data_ptr(), 3, d_out.data_ptr())
        torch.cuda.synchronize()
        want = oracle_for(tr, B=1).eval_children(parent2, lists[0][:4], lists[1], lists[2])
        assert_same(to_records(d_out)[:3], want, "second parent")
        assert (d_out[3:] == -1).all()                               # only the first three records were written
        # the dense call still works beside it
        rows = np.stack([parent, parent2])
        d_rows = torch.from_numpy(rows.view(np.int16)).cuda()
        binding.ap_eval_candidates(handle, d_rows.data_ptr(), 2, d_out.data_ptr())
        torch.cuda.synchronize()
        assert_same(to_records(d_out)[:2], oracle_for(tr, B=1).eval_batch(rows), "dense beside children")
    finally:
        binding.ap_workload_destroy(handle)


def test_children_captured_in_a_graph_and_replayed():
    """The call launches kernels only: capture once, replay with new edit lists in the same buffers."""
    n, M, B = 4000, 8, 4
    tr = _mk(n, M, B, 2500, seed=12, coef=[STD] * M)
    parent = (np.arange(n) % M).astype(np.uint16)
    orc = oracle_for(tr)
    n_children, cap = 24, 4000
    d_first = torch.zeros(n_children + 1, dtype=torch.int32, device="cuda")
    d_request = torch.zeros(cap, dtype=torch.int32, device="cuda")
    d_replica = torch.zeros(cap, dtype=torch.int16, device="cuda")
    d_out = torch.zeros((n_children, 8), dtype=torch.int64, device="cuda")

    def load(seed):
        first, request, replica = traces.draw_edit_lists(seed, n_children, n, M, 60.0 if seed % 2 else 3.0)
        assert len(request) <= cap
        d_first.copy_(torch.from_numpy(first.view(np.int32)))
        d_request[: len(request)].copy_(torch.from_numpy(request.view(np.int32)))
        d_replica[: len(replica)].copy_(torch.from_numpy(replica.view(np.int16)))
        return orc.eval_children(parent, first, request, replica)

    with GpuWorkload(tr) as g:
        g.set_parent(parent, n_children)
        load(0)
        g.eval_children_device(d_first, d_request, d_replica, d_out)    # eager warm-up call
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):                                    # capture on torch's capture stream
            g.eval_children_device(d_first, d_request, d_replica, d_out)
        for seed in range(4):
            want = load(seed)
            d_out.fill_(-1)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert_same(to_records(d_out), want, f"graph replay {seed}")
            eager = g.eval_children_device(d_first, d_request, d_replica)
            torch.cuda.synchronize()
            assert_same(to_records(eager), want, f"eager after replay {seed}")


# ------------------------------------------------------------------ the paper-shaped workloads
def test_jsq_half_of_configs1_as_children():
    tr = traces.make_trace(1)
    lo, hi = tr.C // 2, tr.C
    parent = tr.jsq_base()
    dense = oracle_for(tr).eval_batch(tr.assignment_rows(lo, hi), nthreads=8)
    for tidy in (False, True):
        lists = tr.mutation_lists(lo, hi, tidy=tidy)
        with GpuWorkload(tr) as g:
            g.set_parent(parent, hi - lo)
            got = g.eval_children(*lists)
        assert_same(got, dense, f"configs[1] rows {lo}..{hi} tidy={tidy}")


def test_configs3_children_reduced():
    """Three replica types and windows: no shortcut, every child is written out and replayed."""
    tr = traces.make_trace(3, C=64)
    parent = tr.assignment_row(0)
    lists = traces.draw_edit_lists(33, 64, tr.R, tr.M, 0.01 * tr.R)
    both(tr, parent, lists, "configs[3], 64 children at 1 % edits")


def test_configs4_mutation_sweep_every_child():
    """configs[4] as what it is, a mutation sweep: all 16384 children of the join-shortest-queue parent from
    their edit lists (the raw draws: unsorted, with repeats), in one call, every record against the oracle's
    replay of the dense row."""
    tr = traces.make_trace(4)
    C = tr.C
    orc = oracle_for(tr)
    parent = tr.jsq_base()
    want = np.empty(C, dtype=binding.METRICS_DTYPE)
    firsts, reqs, reps = [np.zeros(1, np.uint32)], [], []
    slab = 512
    for lo in range(0, C, slab):
        hi = min(C, lo + slab)
        first, request, replica = tr.mutation_lists(lo, hi)
        want[lo:hi] = orc.eval_children(parent, first, request, replica, nthreads=16)
        firsts.append(first[1:] + firsts[-1][-1])
        reqs.append(request)
        reps.append(replica)
    lists = (np.concatenate(firsts), np.concatenate(reqs), np.concatenate(reps))
    with GpuWorkload(tr) as g:
        g.set_parent(parent, C)
        got = g.eval_children(*lists)
    assert_same(got, want, "configs[4] as children")
    assert (got["n_rejected"] == 0).all()
