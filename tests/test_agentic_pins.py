"""Pins for the agentic-workflow oracle (no GPU needed): hand-worked schedules, closed forms for the
uncontended and the fully serialised cases, sweep-line invariants of the per-call record, and the metrics
recomputed from that record with numpy."""
import numpy as np
import pytest

from oracle.agentic import AgenticOracle
from paper_2604_07144_amd import traces


def tiny(P=1, cap=300):
    """One workflow: call 0, then calls 1 and 2 which both wait for call 0."""
    return AgenticOracle(arrival_us=[0], slo_us=[10000], wf=[0, 0, 0], in_len=[100, 200, 50], out_len=[10, 5, 20],
                         pred_first=[0, 0, 1, 2], pred=[0, 0], pa=[100] * P, pb=[1] * P, qc=[10], qd=[0], cap=[cap],
                         penalty_permille=77_000)


def test_hand_worked_one_prefill_instance():
    """Call 0: prefill 0-200 (100 + 100), decode 200-300 (10 * 10).  Calls 1 and 2 are released at 300; call 2
    has the smaller key: prefill 300-450, decode 450-650 (20 * 10); call 1: prefill 450-750, decode 750-800."""
    m, d = tiny().eval([0, 0, 0], [0, 0, 0], [0, 1, 0], detail=True)
    assert d["release_us"].tolist() == [0, 300, 300]
    assert d["pre_start_us"].tolist() == [0, 450, 300] and d["pre_end_us"].tolist() == [200, 750, 450]
    assert d["dec_start_us"].tolist() == [200, 750, 450] and d["done_us"].tolist() == [300, 800, 650]
    assert (int(m["sum_ratio_permille"]), int(m["p95_permille"]), int(m["p99_permille"]), int(m["makespan_us"]),
            int(m["n_late"]), int(m["n_failed"])) == (80, 80, 80, 800, 0, 0)
    # equal keys: the lower call index goes first
    _, d = tiny().eval([0, 0, 0], [0, 0, 0], [5, 5, 5], detail=True)
    assert d["pre_start_us"].tolist() == [0, 300, 600]


def test_hand_worked_token_budget_blocks_admission():
    """Two prefill instances: call 1 prefills 300-600, call 2 300-450.  Budget 250 tokens: call 2 (70 tokens)
    decodes 450-650; call 1 (205 tokens) does not fit beside it at 600 and is admitted at 650, done at 700."""
    m, d = tiny(P=2, cap=250).eval([0, 0, 1], [0, 0, 0], [0, 0, 0], detail=True)
    assert d["pre_end_us"].tolist() == [200, 600, 450]
    assert d["dec_start_us"].tolist() == [200, 650, 450] and d["done_us"].tolist() == [300, 700, 650]
    assert int(m["makespan_us"]) == 700
    # a call that can never fit fails when its prefill completes; its workflow gets the penalty ratio
    m, d = tiny(P=2, cap=150).eval([0, 0, 1], [0, 0, 0], [0, 0, 0], detail=True)
    assert d["failed"].tolist() == [False, True, False] and int(d["done_us"][1]) == 600
    assert (int(m["sum_ratio_permille"]), int(m["n_failed"]), int(m["n_late"])) == (77_000, 1, 1)
    # unknown instances: prefill id fails at release (successors go on at once), decode id at the end of prefill
    m, d = tiny(P=2).eval([9, 0, 1], [0, 0, 9], [0, 0, 0], detail=True)
    assert d["failed"].tolist() == [True, False, True] and d["release_us"].tolist() == [0, 0, 0]
    assert d["done_us"].tolist() == [0, 350, 150]


def _workload(seed, **kw):
    wl = traces.make_agentic(seed, **kw)
    return wl, AgenticOracle.from_workload(wl), len(wl["wf"])


def test_uncontended_schedule_is_the_critical_path():
    """Every call on instances of its own, unlimited budget: done = release + prefill + decode, and a
    workflow completes at the end of its longest dependency chain (textbook longest-path recursion)."""
    wl, _, K = _workload(3, W=20)
    big = dict(pa=[700] * K, pb=[2] * K, qc=[30] * K, qd=[4] * K, cap=[1 << 30] * K)
    orc = AgenticOracle.from_workload(wl, **big)
    ids = np.arange(K, dtype=np.uint16)
    m, d = orc.eval(ids, ids, np.zeros(K, np.uint32), detail=True)
    dur = 700 + 2 * wl["in_len"].astype(np.int64) + wl["out_len"].astype(np.int64) * (30 + 4 * ((wl["in_len"].astype(np.int64) + 1023) // 1024))
    done = np.zeros(K, dtype=np.int64)
    for k in range(K):
        preds = wl["pred"][wl["pred_first"][k]:wl["pred_first"][k + 1]]
        start = max([int(wl["arrival_us"][wl["wf"][k]])] + [int(done[j]) for j in preds])
        done[k] = start + dur[k]
    assert d["done_us"].astype(np.int64).tolist() == done.tolist()
    assert int(m["n_failed"]) == 0


def test_single_prefill_instance_serves_in_key_order():
    """Independent calls, all there at time 0, one prefill instance, decode uncontended: prefill end times
    are the running sums of the prefill times in (key, index) order."""
    K = 40
    rng = np.random.default_rng(4)
    in_len = rng.integers(1, 3000, K)
    orc = AgenticOracle(arrival_us=[0] * K, slo_us=[10**9] * K, wf=np.arange(K), in_len=in_len, out_len=[1] * K,
                        pred_first=[0] * (K + 1), pred=[], pa=[50], pb=[3], qc=[1] * K, qd=[0] * K, cap=[1 << 30] * K,
                        penalty_permille=1)
    key = rng.integers(0, 10, K).astype(np.uint32)                       # many ties
    _, d = orc.eval(np.zeros(K, np.uint16), np.arange(K, dtype=np.uint16), key, detail=True)
    order = np.lexsort((np.arange(K), key))
    ends = np.cumsum(50 + 3 * in_len[order])
    assert d["pre_end_us"][order].astype(np.int64).tolist() == ends.tolist()


def test_full_budget_calls_decode_one_after_the_other():
    """Each call needs the whole budget of the one decode instance; prefill is uncontended and equally long, so
    all wait for decode together and are admitted one at a time in key order."""
    K = 12
    orc = AgenticOracle(arrival_us=[0] * K, slo_us=[10**9] * K, wf=np.arange(K), in_len=[60] * K, out_len=[40] * K,
                        pred_first=[0] * (K + 1), pred=[], pa=[10] * K, pb=[0] * K, qc=[7], qd=[0], cap=[100],
                        penalty_permille=1)
    key = np.array([5, 3, 9, 1, 1, 8, 0, 2, 7, 4, 6, 3], dtype=np.uint32)
    _, d = orc.eval(np.arange(K, dtype=np.uint16), np.zeros(K, np.uint16), key, detail=True)
    order = np.lexsort((np.arange(K), key))
    assert d["dec_start_us"][order].astype(np.int64).tolist() == [10 + 280 * i for i in range(K)]


@pytest.mark.parametrize("seed,P,Q,capacity,rate", [(0, 4, 4, 16384, 20.0), (1, 2, 2, 3000, 200.0), (2, 1, 3, 9000, 80.0),
                                                     (3, 3, 1, 12000, 500.0)])
def test_invariants_and_metrics_on_random_workloads(seed, P, Q, capacity, rate):
    wl, orc, K = _workload(seed, P=P, Q=Q, capacity=capacity, rate=rate)
    pre, dec, key = traces.draw_agentic_candidates(seed, 6, K, P, Q, key_range=50, bad_ids=seed == 1)
    in_len, out_len, wf = wl["in_len"].astype(np.int64), wl["out_len"].astype(np.int64), wl["wf"]
    for c in range(6):
        m, d = orc.eval(pre[c], dec[c], key[c], detail=True)
        rel, ps, pe, ds, done = (d[n].astype(np.int64) for n in ("release_us", "pre_start_us", "pre_end_us", "dec_start_us", "done_us"))
        ok = ~d["failed"]
        served_pre = pre[c] < P                                          # these went through prefill
        for k in range(K):
            preds = wl["pred"][wl["pred_first"][k]:wl["pred_first"][k + 1]]
            assert rel[k] == max([int(wl["arrival_us"][wf[k]])] + [int(done[j]) for j in preds])      # precedence
        p_ids, q_ids = pre[c].astype(np.int64), dec[c].astype(np.int64)
        assert (pe[served_pre] - ps[served_pre] == wl["pa"][p_ids[served_pre]] + wl["pb"][p_ids[served_pre]] * in_len[served_pre]).all()
        assert (ps[served_pre] >= rel[served_pre]).all() and (ds[ok] >= pe[ok]).all()
        assert (done[ok] - ds[ok] == out_len[ok] * (wl["qc"][q_ids[ok]] + wl["qd"][q_ids[ok]] * ((in_len[ok] + 1023) // 1024))).all()
        for p in range(P):                                               # one prefill at a time, never idle while a call waits
            mine = np.nonzero(served_pre & (p_ids == p))[0]
            mine = mine[np.argsort(ps[mine], kind="stable")]
            assert (ps[mine][1:] >= pe[mine][:-1]).all()
            for j in mine:
                busy = sum(min(pe[i], ps[j]) - max(ps[i], rel[j]) for i in mine if pe[i] > rel[j] and ps[i] < ps[j])
                assert busy == ps[j] - rel[j]                            # the instance was busy for all of j's wait
                for i in mine:                                           # whoever started while j waited had the better key
                    if i != j and rel[j] <= ps[i] < ps[j] and rel[i] <= ps[i]:
                        assert (key[c][i], i) < (key[c][j], j)
        for q in range(Q):                                               # the token budget is never exceeded
            mine = np.nonzero(ok & (q_ids == q))[0]
            events = sorted([(int(ds[k]), 1, int(in_len[k] + out_len[k])) for k in mine] +
                            [(int(done[k]), 0, -int(in_len[k] + out_len[k])) for k in mine])
            level = 0
            for _, _, delta in events:
                level += delta
                assert level <= capacity
            waiting = mine[np.argsort(pe[mine], kind="stable")]
            for j in waiting:                                            # no overtaking in the decode queue
                for i in waiting:
                    if i != j and pe[j] <= ds[i] < ds[j] and pe[i] <= ds[i]:
                        assert (key[c][i], i) < (key[c][j], j)
        W = len(wl["arrival_us"])
        wf_failed = np.bincount(wf[d["failed"]], minlength=W) > 0
        comp = np.array([max([int(done[k]) for k in np.nonzero(wf == w)[0]] + [int(wl["arrival_us"][w])]) for w in range(W)])
        c_w = comp - wl["arrival_us"].astype(np.int64)
        ratio = np.where(wf_failed, wl["penalty_permille"], c_w * 1000 // wl["slo_us"].astype(np.int64))
        srt = np.sort(ratio)
        assert int(m["sum_ratio_permille"]) == int(ratio.sum())
        assert int(m["p95_permille"]) == int(srt[-(-95 * W // 100) - 1]) and int(m["p99_permille"]) == int(srt[-(-99 * W // 100) - 1])
        assert int(m["n_late"]) == int((wf_failed | (c_w > wl["slo_us"].astype(np.int64))).sum())
        assert int(m["n_failed"]) == int(wf_failed.sum())
        assert int(m["makespan_us"]) == int(done.max() - wl["arrival_us"].min())
