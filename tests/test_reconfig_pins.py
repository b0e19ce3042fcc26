"""Pins for the reconfiguration-cost / trace-time oracle (no GPU needed): worked numbers the paper prints
(system prompt Examples A-C, Table 1), equal plans, brute force."""
import itertools

import numpy as np

from oracle import reconfig as rc
from oracle import roofline as rf

# a model of exactly 13e9 bytes: one layer, no MLP/attention weight beyond what the equation needs is not
# possible in general, so take the transfer-time equation on a stand-in whose weight size is computed first
SMALL = rf.Model(layers=40, hidden=5120, intermediate=13824, vocab=32000, heads=40, kv_heads=40, weight_bits=8)


def gpu(pcie):
    return rf.Gpu(80e9, 1e15, 3e12, pcie, 4e11, 5e10, 8)


def test_example_c_small_model_moves_between_gpu_types():
    """Appendix "System Prompts", Example C: a 13 GB model, loading over 64 GB/s takes 13 / 64 = 0.20 s,
    terminating on the 32 GB/s side 13 / 32 = 0.41 s, together 0.61 s (coefficient 1)."""
    w = rf.weight_bytes(SMALL)
    coef = 13e9 / w                                        # scale the stand-in to 13 GB exactly
    tau = rc.transfer_ns([SMALL], [coef], [gpu(32e9), gpu(64e9)])
    assert [round(int(t) / 1e9, 2) for t in tau[0]] == [0.41, 0.20]
    prev = [[(1, 1), (0, 0)]]                              # on the 32 GB/s type ...
    new = [[(0, 0), (1, 1)]]                               # ... moved to the 64 GB/s type
    term, load = rc.reconfig_ns(tau, prev, new)
    assert (round(term / 1e9, 2), round(load / 1e9, 2), round((term + load) / 1e9, 2)) == (0.41, 0.20, 0.61)


def test_examples_a_and_b_reconfiguration_is_termination_plus_loading():
    """Examples A and B: 0.25 s + 0.25 s = 0.50 s, and 0.51 s + 0.25 s = 0.76 s."""
    for t_load, t_term, want in ((0.25, 0.25, 0.50), (0.51, 0.25, 0.76)):
        tau = np.array([[int(t_term * 1e9), int(t_load * 1e9)]], dtype=np.uint64)
        term, load = rc.reconfig_ns(tau, [[(8, 1), (0, 0)]], [[(0, 0), (4, 2)]])
        assert round((term + load) / 1e9, 2) == want


def test_table_1_rows():
    """Section 5.3, Table 1: T_total of the parent and its two children from their cost breakdowns
    (N = 2, 5, 1 rescheduling intervals; sums of stale / reconfiguration / serving time in seconds)."""
    rows = ((2, 7.6, 12.0, 25.2, 44.8), (5, 5.5, 4.0, 24.0, 33.5), (1, 10.0, 17.0, 23.0, 50.0))
    for n_resched, stale, reconfig, serve, total in rows:
        # spread each sum evenly over the rescheduling intervals; interval 1 is the cold start
        n = n_resched + 1
        tau = np.array([[int(reconfig / n_resched * 1e9 / 2)]], dtype=np.uint64)     # term + load = twice tau
        plans = [[[(1 + (i % 2), 1)]] for i in range(n)]                                # the TP degree flips every interval
        stale_ns = [0] + [int(round(stale / n_resched * 1e9))] * n_resched
        serve_ns = [int(round(serve / n * 1e9))] * n
        got = rc.trace_time(tau, plans, n, 0, stale_ns, serve_ns)
        assert got[0] == n
        assert [round(x / 1e9, 1) for x in got[1:]] == [stale, reconfig, serve, total]


def test_loading_cost_ranges_over_every_deployed_model_hand_worked():
    """Appendix "Serving Simulator", Reconfiguration Cost, worked by hand for two models on one GPU type.
    tau(0, g) = 3 s, tau(1, g) = 8 s.  Model 0 changes its TP degree, model 1 stays as it is (and has the larger
    transfer time).  Delta M = {0}.  Termination cost: max over the changed models the previous plan deploys:
    tau(0, g) = 3 s.  Loading cost as printed: T_load(sigma_i) = max over g, max over EVERY z that sigma_i
    deploys on g = max(3, 8) = 8 s, so Reconfig-Cost = 3 + 8 = 11 s.  Restricted to the changed models (the
    alternative scope) the loading cost is 3 s and the sum 6 s."""
    tau = np.array([[3_000_000_000], [8_000_000_000]], dtype=np.uint64)
    prev = [[(2, 1)], [(4, 1)]]
    new = [[(4, 1)], [(4, 1)]]
    assert rc.reconfig_ns(tau, prev, new) == (3_000_000_000, 8_000_000_000)
    assert rc.reconfig_ns(tau, prev, new, "deployed") == (3_000_000_000, 8_000_000_000)
    assert rc.reconfig_ns(tau, prev, new, "changed") == (3_000_000_000, 3_000_000_000)
    # the same through the execution model: one rescheduling, T_total = 1 + 2 + (0.5 + 11 + 4) s
    plans = [prev, new]
    got = rc.trace_time(tau, plans, 2, 10**9, [0, 5 * 10**8], [2 * 10**9, 4 * 10**9])
    assert got == (2, 5 * 10**8, 11 * 10**9, 6 * 10**9, 185 * 10**8)
    got = rc.trace_time(tau, plans, 2, 10**9, [0, 5 * 10**8], [2 * 10**9, 4 * 10**9], "changed")
    assert got == (2, 5 * 10**8, 6 * 10**9, 6 * 10**9, 135 * 10**8)


def test_equal_plans_cost_nothing_and_termination_counts_changed_models_only():
    tau = np.array([[5, 7], [11, 13], [17, 19]], dtype=np.uint64)
    plan = [[(2, 1), (0, 0)], [(0, 0), (4, 2)], [(1, 3), (1, 1)]]
    for scope in ("deployed", "changed"):
        assert rc.reconfig_ns(tau, plan, plan, scope) == (0, 0)
        # a TP degree written on a GPU type the model is not deployed on is not a change
        ghost = [[(2, 1), (9, 0)], [(0, 0), (4, 2)], [(1, 3), (1, 1)]]
        assert rc.reconfig_ns(tau, plan, ghost, scope) == (0, 0)
    moved = [[(2, 1), (0, 0)], [(0, 0), (4, 3)], [(1, 3), (1, 1)]]          # model 1: one more replica
    assert rc.reconfig_ns(tau, plan, moved, "changed") == (13, 13)
    assert rc.reconfig_ns(tau, plan, moved) == (13, 19)                     # model 2, unchanged, loads slowest
    retp = [[(4, 1), (0, 0)], [(0, 0), (4, 2)], [(1, 3), (1, 1)]]           # model 0: another TP degree
    assert rc.reconfig_ns(tau, plan, retp, "changed") == (5, 5)
    assert rc.reconfig_ns(tau, plan, retp) == (5, 19)
    gone = [[(2, 1), (0, 0)], [(0, 0), (4, 2)], [(0, 0), (0, 0)]]           # model 2 removed: terminated, not loaded
    assert rc.reconfig_ns(tau, plan, gone, "changed") == (19, 0)
    assert rc.reconfig_ns(tau, plan, gone) == (19, 13)                      # what the new plan still deploys


def test_brute_force_over_tiny_plan_pairs():
    """Two models, two GPU types, placements from a small set: the cost against the definition written as
    set comprehensions."""
    tau = np.array([[3, 10], [7, 2]], dtype=np.uint64)
    options = [(0, 0), (1, 1), (2, 1), (1, 2)]
    for prev in itertools.product(options, repeat=4):
        for new in itertools.product(options, repeat=4):
            p = np.array(prev).reshape(2, 2, 2)
            q = np.array(new).reshape(2, 2, 2)
            key = lambda a, z: {(g, int(a[z, g, 0]), int(a[z, g, 1])) for g in range(2) if a[z, g, 1]}
            changed = [z for z in range(2) if key(p, z) != key(q, z)]
            term = max([int(tau[z, g]) for z in changed for g in range(2) if p[z, g, 1]], default=0)
            load = max([int(tau[z, g]) for z in changed for g in range(2) if q[z, g, 1]], default=0)
            assert rc.reconfig_ns(tau, p, q, "changed") == (term, load)
            every = max([int(tau[z, g]) for z in range(2) for g in range(2) if q[z, g, 1]], default=0)
            assert rc.reconfig_ns(tau, p, q) == ((term, every) if changed else (0, 0))
