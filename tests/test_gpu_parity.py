"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, bit for bit.

Integer path, so the bar is byte equality of the 64-byte records.  Small cases compare
every candidate; the full-size configurations run every candidate on the GPU, in the
launch configuration the benchmark times, and compare a sample of rows that the oracle
computes one by one.
"""
import itertools

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from paper_2604_07144_amd import binding, traces          # noqa: E402
from tests.gpu_harness import GpuWorkload, assert_same, oracle_for, to_records   # noqa: E402

U64MAX = 0xFFFFFFFFFFFFFFFF
STD, FAST, SLOW = traces.COEF_STANDARD, traces.COEF_FAST, traces.COEF_SLOW


def both(tr, rows, what, **override):
    with GpuWorkload(tr, **override) as g:
        got = g.eval(rows)
    want = oracle_for(tr, **override).eval_batch(rows, nthreads=8)
    assert_same(got, want, what)
    return got


# ------------------------------------------------------------------ hand-worked trace
def test_hand_worked_trace_on_gpu():
    tr = traces.custom_trace([0, 1000, 1500, 2000], [100, 1024, 1025, 16], [10, 100, 1, 20], [STD], B=2)
    got = both(tr, np.zeros((1, 4), np.uint16), "hand base")
    assert (int(got["sum_e2e_us"][0]), int(got["sum_ttft_us"][0]), int(got["makespan_us"][0])) == (25240, 21305, 10358)
    assert (int(got["p99_ttft_us"][0]), int(got["p99_tpot_us"][0]), int(got["p99_e2e_us"][0])) == (7744, 35, 8320)
    both(tr, np.zeros((1, 4), np.uint16), "hand B=1", B=1)
    both(tr, np.zeros((1, 4), np.uint16), "hand t_on", t_on_us=[3000])
    both(tr, np.zeros((1, 4), np.uint16), "hand t_off", t_off_us=[5000], penalty_us=1_000_000)
    both(tr, np.zeros((1, 4), np.uint16), "hand tight slo", slo_ttft_us=6000, slo_tpot_us=30)


# ------------------------------------------------------------------ brute force, tiny
@pytest.mark.parametrize("R,M,B", [(8, 3, 1), (8, 3, 2), (7, 2, 3), (6, 3, 8)])
def test_all_assignments_of_tiny_instances(R, M, B):
    rng = np.random.default_rng(100 + R + M + B)
    arrival = np.cumsum(rng.integers(0, 3000, R)).astype(np.uint64)
    tr = traces.custom_trace(arrival, rng.integers(1, 3000, R), rng.integers(1, 200, R), [STD, FAST, SLOW][:M],
                             [0, 4000, 0][:M], [U64MAX, U64MAX, 9000][:M], B=B, penalty_us=5_000_000)
    rows = np.array(list(itertools.product(range(M), repeat=R)), dtype=np.uint16)
    both(tr, rows, f"brute R={R} M={M} B={B}")


# ------------------------------------------------------------------ crafted edge traces
def _mk(n, M, B, gap, seed, coef=None, t_on=None, t_off=None, ties=False, **kw):
    rng = np.random.default_rng(seed)
    gaps = rng.integers(0, gap + 1, n)
    if ties:
        gaps[rng.random(n) < 0.5] = 0                       # many equal arrival times
    arrival = (np.cumsum(gaps) + 1_000_000_007).astype(np.uint64)   # first arrival is not 0
    coef = coef or [[STD, FAST, SLOW][m % 3] for m in range(M)]
    return traces.custom_trace(arrival, rng.integers(1, 6000, n), rng.integers(1, 500, n), coef, t_on, t_off, B=B, **kw)


def _rows(C, R, hi, seed):
    return np.random.default_rng(seed).integers(0, hi, size=(C, R)).astype(np.uint16)


@pytest.mark.parametrize("name,n,M,B,gap,C", [
    ("saturated_b1", 3000, 3, 1, 500, 12),            # single slot, long queues
    ("saturated_b8", 5000, 4, 8, 300, 12),            # spans two time chunks, ragged tail
    ("saturated_b64", 9000, 2, 64, 40, 8),            # every slot busy, state carried over three chunks
    ("saturated_b33", 4500, 5, 33, 100, 8),           # B neither a power of two nor a row multiple
    ("light_b64", 6000, 64, 64, 4000, 8),             # nobody waits
    ("ties", 2500, 6, 4, 800, 10),
    ("one_request", 1, 1, 1, 10, 3),
    ("b_exceeds_r", 40, 3, 64, 100, 6),
    ("m512_b8", 4200, 512, 8, 50, 4),                 # many replicas: most queues empty
    ("exact_chunk", 4096, 7, 16, 600, 6),             # R equal to one full chunk
    ("chunk_plus_one", 4097, 7, 16, 600, 6),
    ("m600_b32_lds_limit", 9000, 600, 32, 248, 4),    # the replay kernel's LDS plan lands exactly on the device limit
])
def test_crafted_traces(name, n, M, B, gap, C):
    tr = _mk(n, M, B, gap, seed=len(name) * 7 + n, ties=(name == "ties"))
    both(tr, _rows(C, n, M, seed=n + M), name)


@pytest.mark.parametrize("name,n,M,B,gap,C", [
    ("light_vector_rows", 8192, 16, 16, 9000, 16),     # R % 8 == 0: 16-byte loads; nobody waits
    ("light_scalar_rows", 8191, 16, 16, 9000, 16),     # R % 8 != 0: rows are not 16-byte aligned
    ("borderline", 8192, 16, 8, 1500, 32),             # some candidates pass the screen, some do not
    ("saturated", 6000, 8, 8, 100, 8),                 # every candidate fails the screen
    ("tiny_segments", 3000, 2, 2, 30000, 8),
    ("m1000", 40000, 1000, 4, 40, 4),
    ("b1_light", 5000, 40, 1, 40000, 8),               # a single screening slot per replica
    ("m1024_b2", 6000, 1024, 2, 300, 6),               # large table, two slots per replica
    ("m256_b64", 30000, 256, 64, 60, 6),               # large table, 32 slots per replica
    ("m100_b64", 20000, 100, 64, 30, 6),               # large table, 64 slots per replica, ragged tail
])
def test_homogeneous_always_on_traces_take_the_screening_path(name, n, M, B, gap, C):
    tr = _mk(n, M, B, gap, seed=n + 13, coef=[STD] * M)
    rows = _rows(C, n, M, seed=n)
    rows[0] = np.arange(n) % M                           # round robin: the most even candidate
    both(tr, rows, name)


def test_screening_with_invalid_ids_and_unaligned_batch_pointer():
    n, M = 4096, 8
    tr = _mk(n, M, 16, 9000, seed=5, coef=[FAST] * M, penalty_us=4_000_000)
    rows = _rows(9, n, M, seed=3)
    rows[2, 100] = M                                     # one unknown replica id: that request is rejected
    rows[4, -1] = 65535
    want = oracle_for(tr).eval_batch(rows)
    assert int(want["n_rejected"][2]) == 1 and int(want["n_rejected"][0]) == 0
    with GpuWorkload(tr) as g:
        assert_same(g.eval(rows), want, "invalid ids under screening")
        # a batch that starts 2 bytes into an allocation: rows are not 16-byte aligned
        flat = torch.zeros(9 * n + 1, dtype=torch.int16, device="cuda")
        flat[1:] = torch.from_numpy(rows.view(np.int16).reshape(-1)).cuda()
        d_out = g.eval_device(flat[1:].view(9, n))
        torch.cuda.synchronize()
        assert_same(to_records(d_out), want, "unaligned batch")


@pytest.mark.parametrize("n,M,B", [(4096 + 700, 8, 16), (8192 + 300, 128, 64), (5000, 1024, 2), (6000, 64, 64),
                                   (5000, 200, 64)])
def test_unknown_ids_in_otherwise_contention_free_candidates(n, M, B):
    """Light load, identical replicas: nobody waits, so the shortcut for contention-free candidates decides
    every row; a single unknown replica id anywhere in a row (first block, middle, ragged tail; the id just
    past the table, a few further on, the largest) must still be seen.  Both forms of that kernel
    (small and large replica tables)."""
    tr = _mk(n, M, B, 60_000, seed=n, coef=[STD] * M, penalty_us=7_000_000)
    rows = _rows(12, n, M, seed=B)
    for c, (pos, bad_id) in enumerate([(0, M), (1, M + 1), (700, M + 2), (2047, 65535), (4095, M + 1), (n - 1, M),
                                       (n - 1, M + 1), (n - 300, 65535), (n // 2, M + 7)]):
        rows[c, pos] = bad_id
    want = oracle_for(tr).eval_batch(rows, nthreads=8)
    assert want["n_rejected"].tolist() == [1] * 9 + [0] * 3
    assert len(set(want["sum_ttft_us"][9:].tolist())) == 1                # the valid rows are contention-free
    with GpuWorkload(tr) as g:
        assert_same(g.eval(rows), want, "unknown ids, light load")


@pytest.mark.parametrize("name,n,M,B,gap,C,homogeneous,windows", [
    ("max_table_light", 30000, 1024, 64, 60, 6, False, False),      # the largest replica table and slot count
    ("max_table_homogeneous_saturated", 40000, 1024, 64, 1, 5, True, False),   # screening off (crowded), three kernels
    ("m700_saturated", 50000, 700, 64, 1, 4, False, False),
    ("m1000_b48_windows", 45000, 1000, 48, 2, 4, False, True),
    ("m600_b40_long_trace", 70000, 600, 40, 3, 3, False, True),      # R >= 65536: 32-bit histogram counters
])
def test_large_replica_tables_take_the_queue_per_lane_path(name, n, M, B, gap, C, homogeneous, windows):
    """M * B slot times of one candidate no longer fit in LDS, so the fused replay kernel is out.  Up to 600 - 700
    replicas the listed / streamed evaluation scores these tables (one lane per queue, slot times in registers), and the
    three-kernel replay (grouping, one lane per queue with a heap in LDS, reduction) whatever it hands back - row 0 puts
    everything on eight replicas, which breaks its bound where the rest of the trace is calm; with 1000 or 1024 replicas
    the streaming kernel's per-replica counters do not fit in LDS either and the three kernels score every row."""
    rng = np.random.default_rng(n + M)
    t_on = t_off = None
    if windows:
        span = n * gap // 2
        xy = rng.integers(0, span + 1, size=(M, 2)) + 1_000_000_007
        t_on, t_off = xy.min(1).astype(np.uint64), xy.max(1).astype(np.uint64)
    tr = _mk(n, M, B, gap, seed=n + 1, coef=[STD] * M if homogeneous else None, t_on=t_on, t_off=t_off,
             penalty_us=2_000_000_000)
    rows = _rows(C, n, M + (0 if homogeneous else 2), seed=M)           # a few unknown replica ids
    rows[0] = rng.integers(0, 8, n)                                     # everything on eight replicas: deep queues
    both(tr, rows, name)


@pytest.mark.parametrize("one_very_long_request", [False, True])
def test_large_table_screening_with_both_table_forms(one_very_long_request):
    """128 identical replicas, light load: the eight-wavefront form of the contention-free shortcut.  Its table
    is read one word per two requests when the tick that needs is in proportion; a single request that runs for
    seconds in a trace of milliseconds-long ones makes that tick far too coarse, and the library falls back to
    one word per request.  Both must agree with the oracle, unknown ids and ragged tail included."""
    n, M, B = 20000 + 333, 128, 64
    rng = np.random.default_rng(5)
    arrival = (np.cumsum(rng.integers(0, 600, n)) + 77).astype(np.uint64)
    prompt = rng.integers(1, 6000, n)
    out = rng.integers(1, 500, n)
    if one_very_long_request:
        out[n // 3] = 200_000
    tr = traces.custom_trace(arrival, prompt, out, [STD] * M, B=B, penalty_us=9_000_000)
    rows = _rows(10, n, M, seed=2)
    rows[0] = np.arange(n) % M
    rows[1, 5] = M + 3                                   # unknown ids: first block, ragged tail
    rows[2, n - 1] = 65535
    rows[3, : n // 2] = 7                                # half the trace on one replica: queueing, replayed
    want = oracle_for(tr).eval_batch(rows, nthreads=8)
    assert len(set(want["sum_ttft_us"][4:].tolist())) == 1 and want["sum_ttft_us"][3] > want["sum_ttft_us"][4]
    with GpuWorkload(tr) as g:
        assert_same(g.eval(rows), want, f"large table, one_very_long_request={one_very_long_request}")


def test_lengths_beyond_16_bits_and_coarse_ticks():
    """Prompt / output lengths >= 65536 (32-bit staging in the replay kernel) and a trace long enough that the
    screening kernel's 16-bit ticks are coarser than a microsecond."""
    rng = np.random.default_rng(77)
    n, M = 6000, 6
    arrival = (np.cumsum(rng.integers(0, 40_000, n)) + 5).astype(np.uint64)           # two minutes of trace: 2 ms ticks
    prompt = rng.integers(1, 3000, n)
    out = rng.integers(1, 300, n)
    prompt[::97] = rng.integers(65536, 200_000, len(prompt[::97]))                    # a few very long prompts
    out[::89] = rng.integers(65536, 90_000, len(out[::89]))
    coef = [(50, 1, 2, 1)] * M                                                         # small coefficients keep times in range
    tr = traces.custom_trace(arrival, prompt, out, coef, B=3, slo_ttft_us=200_000, slo_tpot_us=40)
    rows = _rows(12, n, M, seed=5)
    rows[0] = 0                                                                        # one replica takes everything: queueing
    got = both(tr, rows, "long lengths, homogeneous (screened)")
    assert len(set(got["sum_ttft_us"].tolist())) > 1                                   # screened and replayed rows both occur
    mixed = traces.custom_trace(arrival, prompt, out, [(50, 1, 2, 1), (80, 2, 3, 1)] * 3, B=3)
    both(mixed, rows, "long lengths, two replica types (replayed)")


@pytest.mark.parametrize("M,B,windows", [(1024, 64, False), (700, 48, True)])
def test_three_kernel_replay_scores_every_row_when_lengths_are_long(M, B, windows):
    """A length of 65536 tokens or more rules out the 8-byte request records of the listed / streamed evaluation, and
    M * B slot times do not fit in LDS: grouping, replay (one lane per queue, heap in LDS) and reduction score every row."""
    rng = np.random.default_rng(M)
    n = 20000
    arrival = (np.cumsum(rng.integers(0, 60, n)) + 1_000_000_007).astype(np.uint64)
    prompt = rng.integers(1, 3000, n)
    out = rng.integers(1, 300, n)
    prompt[::211] = rng.integers(65536, 120_000, len(prompt[::211]))
    t_on = t_off = None
    if windows:
        xy = rng.integers(0, n * 30 + 1, size=(M, 2)) + 1_000_000_007
        t_on, t_off = xy.min(1).astype(np.uint64), xy.max(1).astype(np.uint64)
    tr = traces.custom_trace(arrival, prompt, out, [[(50, 1, 2, 1), (80, 2, 3, 1)][m % 2] for m in range(M)], t_on, t_off, B=B,
                             penalty_us=2_000_000_000)
    rows = _rows(5, n, M + 1, seed=M + 1)
    rows[1] = rng.integers(0, 4, n)                                     # deep queues on four replicas
    with GpuWorkload(tr) as g:
        got = g.eval(rows)
        scored, replayed = g.counts()
    assert_same(got, oracle_for(tr).eval_batch(rows, nthreads=8), f"three kernels, long lengths M={M} B={B}")
    assert (scored, replayed) == (5, 5)


@pytest.mark.parametrize("seed", range(160))
def test_random_shapes_against_the_oracle(seed):
    """Shapes, loads and replica tables drawn at random within the documented limits: whichever kernels the
    library's plan picks for them, every record must equal the oracle's."""
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.choice([1, 7, 63, 64, 65, 500, 511, 513, 1023, 1025, 3000, 4097, 9000]))
    M = int(rng.choice([1, 2, 3, 5, 8, 13, 20, 33, 64, 100, 128, 257, 600, 1024]))
    B = int(rng.choice([1, 2, 3, 7, 8, 16, 31, 32, 33, 48, 64]))
    gap = int(10 ** rng.uniform(0.5, 4.7))                      # 3 us .. 50 ms between arrivals
    homogeneous = bool(rng.integers(0, 2))
    windows = (not homogeneous) and bool(rng.integers(0, 2))
    t_on = t_off = None
    if windows:
        span = max(1, n * gap // 2)
        xy = rng.integers(0, span + 1, size=(M, 2)) + 1_000_000_007
        t_on, t_off = xy.min(1).astype(np.uint64), xy.max(1).astype(np.uint64)
    tr = _mk(n, M, B, gap, seed=seed, coef=[FAST] * M if homogeneous else None, t_on=t_on, t_off=t_off,
             ties=bool(rng.integers(0, 2)), penalty_us=int(rng.choice([1, 5_000_000, 3_600_000_000])),
             slo_ttft_us=int(rng.choice([3_000, 500_000])), slo_tpot_us=int(rng.choice([20, 50_000])))
    C = int(rng.integers(1, 7))
    rows = _rows(C, n, M + int(rng.integers(0, 3)), seed=seed + 7)       # sometimes a few unknown ids
    if C > 1:
        rows[1] = np.arange(n) % M                                      # the most even candidate
    both(tr, rows, f"random shape n={n} M={M} B={B} gap={gap} homogeneous={homogeneous} windows={windows}")


def test_all_requests_on_one_replica_and_empty_replicas():
    tr = _mk(5000, 9, 16, 200, seed=3)
    rows = np.zeros((4, 5000), np.uint16)
    rows[1] = 8
    rows[2, ::2] = 4
    rows[3] = np.random.default_rng(0).integers(0, 2, 5000) * 7
    both(tr, rows, "one replica")


def test_invalid_replica_ids_are_rejected():
    tr = _mk(3000, 5, 4, 400, seed=9, penalty_us=12_345_678)
    rows = _rows(6, 3000, 9, seed=4)                  # ids 5..8 do not exist
    rows[5] = 65535
    got = both(tr, rows, "invalid ids")
    assert int(got["n_rejected"][5]) == 3000 and int(got["makespan_us"][5]) == 0


def test_availability_windows():
    n, M = 6000, 12
    base = _mk(n, M, 8, 300, seed=21)
    span = int(base.arrival_us[-1] - base.arrival_us[0])
    a0 = int(base.arrival_us[0])
    rng = np.random.default_rng(8)
    xy = rng.integers(0, span + 1, size=(M, 2)) + a0
    t_on, t_off = xy.min(1).astype(np.uint64), xy.max(1).astype(np.uint64)
    t_on[0], t_off[0] = 0, a0                                      # closed before the trace starts
    t_on[1], t_off[1] = a0 + span + 5, U64MAX                      # opens after the last arrival: all wait
    t_on[2], t_off[2] = a0 + span // 2, a0 + span // 2             # empty window
    t_on[3], t_off[3] = 0, U64MAX
    t_on[4], t_off[4] = a0 + 10, a0 + 11                           # one microsecond
    tr = _mk(n, M, 8, 300, seed=21, t_on=t_on, t_off=t_off, penalty_us=900_000_000)
    both(tr, _rows(10, n, M, seed=5), "windows")
    both(tr, _rows(4, n, M, seed=6), "windows B=64", B=64)


def test_slo_variants_and_small_penalty():
    tr = _mk(4000, 4, 6, 900, seed=33)
    rows = _rows(6, 4000, 5, seed=2)
    both(tr, rows, "tight tpot", slo_tpot_us=30)
    both(tr, rows, "tight ttft", slo_ttft_us=2500)
    both(tr, rows, "huge slo", slo_ttft_us=2**40, slo_tpot_us=2**40)
    both(tr, rows, "zero slo", slo_ttft_us=0, slo_tpot_us=0)
    both(tr, rows, "small penalty", penalty_us=5)
    both(tr, rows, "huge penalty", penalty_us=2**40 + 12345)


def test_results_do_not_depend_on_batch_composition():
    tr = traces.make_trace(1, C=40, R=4096, rate_scale=60.0)
    rows = tr.assignment_rows(0, 40)
    with GpuWorkload(tr, B=4) as g:
        whole = g.eval(rows)
        perm = np.random.default_rng(0).permutation(40)
        assert_same(g.eval(rows[perm]), whole[perm], "permuted batch")
        assert_same(g.eval(rows[7:8]), whole[7:8], "single row")
        assert_same(g.eval(rows), whole, "second call on the same workload")
    assert_same(whole, oracle_for(tr, B=4).eval_batch(rows, nthreads=8), "cfg1 saturated")


def test_cost_model_can_be_replaced():
    tr = _mk(3000, 3, 4, 500, seed=77)
    rows = _rows(5, 3000, 3, seed=1)
    with GpuWorkload(tr) as g:
        first = g.eval(rows)
        binding.ap_costmodel_set(g.handle, binding.make_replicas([SLOW, SLOW, FAST], [0] * 3, [U64MAX] * 3), 2,
                                 400_000, 40, 1_000_000)
        second = g.eval(rows)
    assert_same(first, oracle_for(tr).eval_batch(rows), "before swap")
    assert_same(second, oracle_for(tr, coef=[SLOW, SLOW, FAST], B=2, slo_ttft_us=400_000, slo_tpot_us=40,
                                   penalty_us=1_000_000).eval_batch(rows), "after swap")


def test_error_paths():
    tr = _mk(100, 2, 2, 100, seed=1)
    with pytest.raises(binding.ApError) as e:
        binding.ap_workload_create(tr.arrival_us[::-1].copy(), tr.prompt_len, tr.out_len)      # unsorted
    assert e.value.status == binding.AP_ERR_INVALID
    with pytest.raises(binding.ApError) as e:
        binding.ap_workload_create(tr.arrival_us, np.zeros(100, np.int32), tr.out_len)         # prompt 0
    assert e.value.status == binding.AP_ERR_INVALID
    h = binding.ap_workload_create(tr.arrival_us, tr.prompt_len, tr.out_len)
    try:
        d = torch.zeros((1, 100), dtype=torch.int16, device="cuda")
        o = torch.zeros((1, 8), dtype=torch.int64, device="cuda")
        with pytest.raises(binding.ApError) as e:
            binding.ap_eval_candidates(h, d.data_ptr(), 1, o.data_ptr(), 0)                    # no cost model yet
        assert e.value.status == binding.AP_ERR_STATE
        rep = binding.make_replicas([STD, STD], [0, 0], [U64MAX, U64MAX])
        for bad_B in (0, 65):
            with pytest.raises(binding.ApError):
                binding.ap_costmodel_set(h, rep, bad_B, 1, 1, 1)
        with pytest.raises(binding.ApError) as e:                                              # t_on > t_off
            binding.ap_costmodel_set(h, binding.make_replicas([STD], [5], [4]), 2, 1, 1, 1)
        assert e.value.status == binding.AP_ERR_INVALID
        with pytest.raises(binding.ApError) as e:                                              # 32-bit horizon
            binding.ap_costmodel_set(h, binding.make_replicas([(4_000_000_000, 3, 25, 5)], [0], [U64MAX]), 2, 1, 1, 1)
        assert e.value.status == binding.AP_ERR_RANGE
        with pytest.raises(binding.ApError) as e:                                              # more replicas than supported
            binding.ap_costmodel_set(h, binding.make_replicas([STD] * 1025, [0] * 1025, [U64MAX] * 1025), 64, 1, 1, 1)
        assert e.value.status == binding.AP_ERR_RANGE
        binding.ap_costmodel_set(h, rep, 2, 500_000, 50_000, 1_000_000)
        binding.ap_eval_candidates(h, d.data_ptr(), 0, o.data_ptr(), 0)                        # C == 0: no-op
        with pytest.raises(binding.ApError) as e:
            binding.ap_eval_candidates(h, 0, 1, o.data_ptr(), 0)
        assert e.value.status == binding.AP_ERR_INVALID
        binding.ap_eval_candidates(h, d.data_ptr(), 1, o.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert_same(to_records(o), oracle_for(tr).eval_batch(np.zeros((1, 100), np.uint16)), "after errors")
    finally:
        binding.ap_workload_destroy(h)


# ------------------------------------------------------------------ stream capture
@pytest.mark.parametrize("name,n,M,B,gap,homogeneous", [
    ("screen_then_replay", 8192, 16, 8, 1500, True),      # some candidates pass the screen, the others are replayed
    ("replay", 5000, 12, 8, 300, False),
    ("three_kernels", 20000, 1024, 64, 20, False),        # the large-table path: several launches per call
])
def test_eval_captured_in_a_graph_and_replayed(name, n, M, B, gap, homogeneous):
    """ap_eval_candidates allocates nothing and only launches kernels on the caller's stream, so a caller may
    capture it in a graph.  The graph is replayed several times with new assignments written into the same
    buffers in between (ordinary eager copies and synchronisations); every replay must equal the oracle."""
    tr = _mk(n, M, B, gap, seed=n + 3, coef=[STD] * M if homogeneous else None)
    C = 10
    orc = oracle_for(tr)
    with GpuWorkload(tr) as g:
        d_assign = torch.zeros((C, n), dtype=torch.int16, device="cuda")
        d_out = torch.full((C, 8), -1, dtype=torch.int64, device="cuda")
        g.eval_device(d_assign, d_out)                                   # eager warm-up call
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):                                    # capture on torch's capture stream
            g.eval_device(d_assign, d_out)
        for it in range(4):
            rows = _rows(C, n, M + (it % 2), seed=100 * it + M)          # odd rounds carry a few unknown ids
            rows[0] = np.arange(n) % M
            d_assign.copy_(torch.from_numpy(rows.view(np.int16)).cuda())
            d_out.fill_(-1)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert_same(to_records(d_out), orc.eval_batch(rows, nthreads=8), f"{name}: replay {it}")
            assert_same(g.eval(rows), to_records(d_out), f"{name}: eager call after replay {it}")


# ------------------------------------------------------------------ the five configurations
@pytest.mark.parametrize("cfg", [0, 1])
def test_small_configurations_every_row(cfg):
    tr = traces.make_trace(cfg)
    rows = tr.assignment_rows(0, tr.C)
    both(tr, rows, tr.spec.name)


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_full_size_configurations_every_row(cfg):
    """All C rows run on the GPU at full size, in the launch configuration the benchmark times (one call over
    the whole batch; rows drawn and uploaded in slabs), and the oracle scores every one of them (sixteen threads,
    slab by slab: configs[4] is 2.1e9 request simulations, about twenty seconds of host time)."""
    tr = traces.make_trace(cfg)
    C, R = tr.C, tr.R
    orc = oracle_for(tr)
    d_assign = torch.empty((C, R), dtype=torch.int16, device="cuda")
    want = np.empty(C, dtype=binding.METRICS_DTYPE)
    slab = 512
    for lo in range(0, C, slab):
        hi = min(C, lo + slab)
        rows = tr.assignment_rows(lo, hi)
        d_assign[lo:hi] = torch.from_numpy(rows.view(np.int16)).cuda()
        want[lo:hi] = orc.eval_batch(rows, nthreads=16)
    with GpuWorkload(tr) as g:
        d_out = g.eval_device(d_assign)
        torch.cuda.synchronize()
        got = to_records(d_out)
    assert_same(got, want, tr.spec.name)
    if cfg != 3:
        assert (got["n_rejected"] == 0).all()


@pytest.mark.parametrize("cfg", [3, 4])
def test_saturated_variants_reduced(cfg):
    """Arrival rate x100 on a reduced number of candidates: queues really form."""
    tr = traces.make_trace(cfg, C=24, rate_scale=100.0)
    rows = tr.assignment_rows(0, 24)
    got = both(tr, rows, tr.spec.name + " x100")
    nominal = oracle_for(tr, B=64).eval_batch(rows[:1])            # sanity: the variant does queue
    assert int(got["sum_ttft_us"][0]) >= int(nominal["sum_ttft_us"][0])
