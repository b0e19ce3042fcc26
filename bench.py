#!/usr/bin/env python3
"""Benchmark: candidate-request simulations per second on one MI355X.

One step = one ap_eval_candidates call over the whole candidate batch of the chosen
configuration (all stages of the path), with trace, cost model and assignments already
resident in HBM.  Prints ONE JSON line with the throughput, the HBM roofline of the
evaluation kernel (algorithmic bytes / measured kernel time) and the CPU oracle timed on
this host on a bounded sample of the same workload.  Where the configuration is a mutation
sweep the same candidates are also scored from their edit lists (ap_eval_children) and
reported in a `sparse_children` object beside the dense figures.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 0..4] [--rate-scale S]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
TABLE_BYTES_PER_REQUEST = 16   # arrival + prefill/decode/tpot-class inputs, per replica type

KERNEL_SOURCE_DIR = os.path.join(ROOT, "paper_2604_07144_amd", "csrc")
# HBM bytes per ap_eval_candidates call from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch, summed over
# the call's kernels, scaled by what the same counters read for a device copy of known size; see profiles/).
# Keyed by configuration; valid only for the library source (all of csrc/) whose hash is recorded with it.
MEASURED_TRAFFIC = {
    # cfg: (sha256 of the kernel source when measured, bytes per call)
    4: ("1a42a8b4fa7181bd5050da52d4d30baea2d61460da69886659d22c0978f43fe2", 4305337611),
    3: ("1a42a8b4fa7181bd5050da52d4d30baea2d61460da69886659d22c0978f43fe2", 2049930752),
}
# Wave-instructions per candidate-request of one ap_eval_candidates call (all its kernels), from rocprofv3 --pmc
# SQ_INSTS_VALU / SQ_INSTS_SALU / SQ_INSTS_LDS; same validity rule.  The chip issues at most 256 CUs x 4 SIMDs x
# 2.4 GHz / 4 cycles = 6.1e11 64-lane vector instructions per second.
VALU_PEAK_PER_S = 256 * 4 * 2.4e9 / 4
MEASURED_ALU = {
    4: ("1a42a8b4fa7181bd5050da52d4d30baea2d61460da69886659d22c0978f43fe2", {"valu": 0.1381, "salu": 0.0796, "lds": 0.0353}),
    3: ("1a42a8b4fa7181bd5050da52d4d30baea2d61460da69886659d22c0978f43fe2", {"valu": 1.6043, "salu": 0.4891, "lds": 0.1236}),
}
# the same for one ap_eval_children call on the sparse form of configs[4]
MEASURED_TRAFFIC_CHILDREN = {4: ("1a42a8b4fa7181bd5050da52d4d30baea2d61460da69886659d22c0978f43fe2", 131102012)}


def kernel_source_hash() -> str:
    """sha256 over every file of the library's source directory, in name order."""
    import hashlib
    h = hashlib.sha256()
    for name in sorted(os.listdir(KERNEL_SOURCE_DIR)):
        with open(os.path.join(KERNEL_SOURCE_DIR, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()


def measured_traffic(cfg: int, table=None):
    """Recorded HBM traffic for this configuration, or None once the kernels have changed since."""
    rec = (MEASURED_TRAFFIC if table is None else table).get(cfg)
    if rec is None or rec[0] != kernel_source_hash():
        return None
    return rec[1]


def copy_calibration(n_bytes: int = 1 << 30, repeats: int = 5) -> int:
    """A plain device-to-device copy of known size, for scaling the FETCH_SIZE / WRITE_SIZE counters."""
    import torch
    src = torch.empty(n_bytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(repeats):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_calibration_bytes": n_bytes, "repeats": repeats}))
    return 0


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def algorithmic_bytes(C: int, R: int, n_types: int) -> int:
    """Bytes the method itself must move per call: every uint16 assignment once, one 64-byte
    record per candidate, the per-request tables once."""
    return 2 * C * R + 64 * C + TABLE_BYTES_PER_REQUEST * n_types * R


def time_calls(step, stream, steps: int, warmup: int, settle_ms: float = 60.0):
    """`warmup` untimed calls - and as many more as it takes to keep the device busy for `settle_ms`, so that the
    clocks have settled however short a call is - then exactly `steps` timed calls, each between two HIP events on
    the stream the kernels are launched on.  Returns (wall seconds of the timed calls, device ms per call)."""
    import torch
    t0 = time.perf_counter()
    done = 0
    while done < warmup or (time.perf_counter() - t0) * 1e3 < settle_ms:
        step()
        done += 1
        if done % 8 == 0 or done >= warmup:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record(stream)
        step()
        b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, [a.elapsed_time(b) for a, b in ev]


def upload_rows(tr, C: int):
    """Candidate rows 0..C of a trace, drawn and uploaded in slabs; returns the device tensor [C][R] (2-byte elements)."""
    import torch
    d_assign = torch.empty((C, tr.R), dtype=torch.int16, device="cuda")
    slab = max(1, (256 << 20) // (2 * tr.R))
    for lo in range(0, C, slab):
        hi = min(C, lo + slab)
        d_assign[lo:hi] = torch.from_numpy(tr.assignment_rows(lo, hi).view(np.int16)).cuda()
    return d_assign


def tables_of(tr):
    """The trace's linear cost model evaluated once per replica type and request: the inputs of ap_costtable_set."""
    kinds = sorted({tuple(int(x) for x in row) for row in tr.coef})
    rep_type = np.array([kinds.index(tuple(int(x) for x in row)) for row in tr.coef], dtype=np.uint32)
    prompt = tr.prompt_len.astype(np.int64)
    prefill = np.stack([a + b * prompt for a, b, _, _ in kinds]).astype(np.uint32)
    tpot = np.stack([c + d * ((prompt + 1023) // 1024) for _, _, c, d in kinds]).astype(np.uint32)
    return rep_type, prefill, tpot


def side_workload(cfg: int, rate_scale: float, C: int, d_assign, steps: int, warmup: int, label: str,
                  cost_tables: bool = False) -> dict:
    """One more workload timed the same way as the main one (same protocol, fewer words): device time per
    ap_eval_candidates call, throughput, roofline fraction on its own algorithmic bytes, how many candidates went
    through the exact replay.  `d_assign` may be shared with another workload whose rows are drawn the same way."""
    import torch
    from paper_2604_07144_amd import binding, traces
    tr = traces.make_trace(cfg, rate_scale=rate_scale)
    n_types = len({tuple(int(x) for x in row) for row in tr.coef})
    if d_assign is None:
        d_assign = upload_rows(tr, C)
    d_out = torch.zeros((C, 8), dtype=torch.int64, device="cuda")
    stream = torch.cuda.current_stream()
    h = binding.ap_workload_create(tr.arrival_us, tr.prompt_len, tr.out_len)
    try:
        if cost_tables:
            rep_type, prefill, tpot = tables_of(tr)
            binding.ap_costtable_set(h, rep_type, tr.t_on_us, tr.t_off_us, tr.B, tr.slo_ttft_us, tr.slo_tpot_us,
                                     tr.penalty_us, prefill, tpot)
        else:
            binding.ap_costmodel_set(h, binding.make_replicas(tr.coef, tr.t_on_us, tr.t_off_us), tr.B,
                                     tr.slo_ttft_us, tr.slo_tpot_us, tr.penalty_us)

        def step():
            binding.ap_eval_candidates(h, d_assign.data_ptr(), C, d_out.data_ptr(), stream.cuda_stream)

        wall, ms = time_calls(step, stream, steps, warmup)
        scored, replayed = binding.ap_eval_counts_get(h)
    finally:
        binding.ap_workload_destroy(h)
    alg = algorithmic_bytes(C, tr.R, n_types)
    avg_s = float(np.mean(ms)) * 1e-3
    full = C == tr.C and rate_scale == 1.0
    return {"workload": f"configs[{cfg}] {tr.spec.name}: C={C} R={tr.R} M={tr.M} B={tr.B}"
                        + (f" arrival rate x{rate_scale:g}" if rate_scale != 1.0 else "") + label,
            "value": C * tr.R / (wall / steps), "unit": "sims/s", "ms_per_step": wall * 1e3 / steps,
            "kernel_ms_avg": avg_s * 1e3, "kernel_ms_min": float(np.min(ms)),
            "roofline": {"bound": "hbm", "achieved": alg / avg_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": alg / avg_s / 1e9 / HBM_PEAK_GBS,
                         "traffic": measured_traffic(cfg) if full and not cost_tables else None,
                         "algorithmic_bytes": alg},
            "replayed_fraction": replayed / max(1, scored)}, d_assign


def agentic_bench(args) -> int:
    """Candidate plans per second for one 64-workflow slice (Section 8.3 uses two such slices), plans resident in HBM."""
    import torch
    from paper_2604_07144_amd import binding, traces
    torch.cuda.set_device(0)
    fields = ("arrival_us", "slo_us", "wf", "in_len", "out_len", "pred_first", "pred", "pa", "pb", "qc", "qd", "cap",
              "penalty_permille")
    wl = traces.make_agentic(0, 64, P=4, Q=4, capacity=6000, rate=60.0)
    K, C = len(wl["wf"]), args.rows if args.rows else 8192
    pre, dec, key = traces.draw_agentic_candidates(0, C, K, 4, 4)
    d_pre = torch.from_numpy(pre.view(np.int16)).cuda()
    d_dec = torch.from_numpy(dec.view(np.int16)).cuda()
    d_key = torch.from_numpy(key.view(np.int32)).cuda()
    d_out = torch.zeros((C, 5), dtype=torch.int64, device="cuda")
    h = binding.ap_agentic_create(*(wl[f] for f in fields))
    stream = torch.cuda.current_stream()
    try:
        def step():
            binding.ap_agentic_eval(h, d_pre.data_ptr(), d_dec.data_ptr(), d_key.data_ptr(), C, d_out.data_ptr(), stream.cuda_stream)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        t0 = time.perf_counter()
        for a, b in ev:
            a.record(stream)
            step()
            b.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms = [a.elapsed_time(b) for a, b in ev]
        got = d_out.cpu().numpy().view(binding.AGENTIC_METRICS_DTYPE).reshape(-1)
    finally:
        binding.ap_agentic_destroy(h)
    result = {"metric": "candidate plans/s (agentic workflows)", "value": C / (wall / args.steps), "unit": "plans/s",
              "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps,
              "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32", "data": "synthetic",
              "config": {"workload": f"one 64-workflow slice: K={K} calls, 4 prefill + 4 decode instances, C={C} plans"},
              "kernel_ms_avg": float(np.mean(ms)), "kernel_ms_min": float(np.min(ms)),
              "call_stages_per_s": 2 * K * C / (float(np.mean(ms)) * 1e-3)}
    if not args.no_cpu:
        from oracle.agentic import AgenticOracle
        orc = AgenticOracle.from_workload(wl)
        n = min(C, 512)
        t0 = time.perf_counter()
        want = orc.eval_batch(pre[:n], dec[:n], key[:n])
        cpu_s = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": n / cpu_s, "unit": "plans/s", "cores": 1, "kind": "oracle",
                                  "sample": f"the first {n} plans, {cpu_s:.2f} s on one thread",
                                  "matches_gpu": bool(all(got[c].tolist() == want[c].tolist() for c in range(n)))}
    print(json.dumps(result))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # a call is under a millisecond: enough of them for the clocks to settle before and while timing
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload configuration 0..4 (default: the largest)")
    ap.add_argument("--rate-scale", type=float, default=1.0, help=">1 compresses arrivals (saturated variant)")
    ap.add_argument("--rows", type=int, default=0, help="use only the first ROWS candidates (0 = all)")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows of the oracle sample (0 = auto)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-children", action="store_true", help="skip the sparse (edit-list) leg of a mutation sweep")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the side workloads of the default run (configs[3], configs[2], the saturated variants)")
    ap.add_argument("--cost-tables", action="store_true",
                    help="pass the configuration's cost model as per-type tables (ap_costtable_set) instead of coefficients")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a 1 GiB device copy (reference dispatch for the HBM byte counters)")
    ap.add_argument("--agentic", action="store_true",
                    help="time the agentic-workflow evaluator instead (64-workflow slice, 8192 candidate plans); "
                         "prints its own JSON line")
    args = ap.parse_args()
    if args.calibrate_copy:
        return copy_calibration()
    if args.agentic:
        return agentic_bench(args)
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU; candidates are independent, so more GPUs would only "
              "split the rows. Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2604_07144_amd import binding, traces

    torch.cuda.set_device(0)
    tr = traces.make_trace(args.config, rate_scale=args.rate_scale)
    C = args.rows if args.rows else tr.C
    R, M = tr.R, tr.M
    n_types = len({tuple(int(x) for x in row) for row in tr.coef})

    # inputs resident in HBM before anything is timed (rows drawn and uploaded in slabs)
    d_assign = upload_rows(tr, C)
    slab = max(1, (256 << 20) // (2 * R))
    d_out = torch.zeros((C, 8), dtype=torch.int64, device="cuda")

    h = binding.ap_workload_create(tr.arrival_us, tr.prompt_len, tr.out_len)
    try:
        if args.cost_tables:
            # the same cost model, evaluated here once per replica type and request and handed over as tables
            rep_type, prefill, tpot = tables_of(tr)
            binding.ap_costtable_set(h, rep_type, tr.t_on_us, tr.t_off_us, tr.B, tr.slo_ttft_us, tr.slo_tpot_us,
                                     tr.penalty_us, prefill, tpot)
        else:
            binding.ap_costmodel_set(h, binding.make_replicas(tr.coef, tr.t_on_us, tr.t_off_us), tr.B,
                                     tr.slo_ttft_us, tr.slo_tpot_us, tr.penalty_us)
        stream = torch.cuda.current_stream()

        def step():
            binding.ap_eval_candidates(h, d_assign.data_ptr(), C, d_out.data_ptr(), stream.cuda_stream)

        # HIP events on the stream the kernels are launched on: per-launch device time
        before = binding.ap_eval_counts_get(h)
        wall, kernel_ms = time_calls(step, stream, args.steps, args.warmup)
        after = binding.ap_eval_counts_get(h)
        got = d_out.cpu().numpy().view(binding.METRICS_DTYPE).reshape(-1)

        # The same candidates in their sparse form, where the configuration is a mutation sweep: every row is
        # the join-shortest-queue parent plus a short list of reassignments, so a caller that holds the parent
        # passes the lists instead of the rows (ap_parent_set + ap_eval_children).  Reported beside `value`,
        # never as `value`: the metric above is defined on dense rows.
        children = None
        if not args.no_children and all(tr.is_mutated_row(c) for c in (0, C // 2, C - 1)):
            parent = tr.jsq_base()
            d_parent = torch.from_numpy(parent.view(np.int16)).cuda()
            counts, reqs, reps = [], [], []
            for lo in range(0, C, slab):                      # the lists: where a row differs from the parent
                hi = min(C, lo + slab)
                differs = d_assign[lo:hi] != d_parent[None, :]
                counts.append(differs.sum(dim=1))
                where = differs.nonzero()                     # row-major: per row, requests in increasing order
                reqs.append(where[:, 1].to(torch.int32))
                reps.append(d_assign[lo:hi][where[:, 0], where[:, 1]])
                del differs, where
            d_first = torch.zeros(C + 1, dtype=torch.int64, device="cuda")
            d_first[1:] = torch.cat(counts).cumsum(0)
            n_edits = int(d_first[-1])
            d_first = d_first.to(torch.int32)
            d_request = torch.cat(reqs + [torch.zeros(1, dtype=torch.int32, device="cuda")])
            d_replica = torch.cat(reps + [torch.zeros(1, dtype=torch.int16, device="cuda")])
            d_out2 = torch.zeros((C, 8), dtype=torch.int64, device="cuda")
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            binding.ap_parent_set(h, parent, C)                # the first call also allocates the rows
            parent_first_ms = (time.perf_counter() - t0) * 1e3
            t0 = time.perf_counter()
            for _ in range(5):
                binding.ap_parent_set(h, parent, C)
            parent_set_ms = (time.perf_counter() - t0) * 1e3 / 5

            def child_step():
                binding.ap_eval_children(h, d_first.data_ptr(), d_request.data_ptr(), d_replica.data_ptr(), C,
                                         d_out2.data_ptr(), stream.cuda_stream)

            child_wall, child_ms = time_calls(child_step, stream, args.steps, args.warmup)
            got2 = d_out2.cpu().numpy().view(binding.METRICS_DTYPE).reshape(-1)
            # bytes this form must move: the lists (4 + 2 per edit, 4 per child), one record per child,
            # the parent row and the per-request tables once
            child_alg = 6 * n_edits + 4 * (C + 1) + 64 * C + 2 * R + TABLE_BYTES_PER_REQUEST * n_types * R
            child_s = float(np.mean(child_ms)) * 1e-3
            children = {"value": C * R / (child_wall / args.steps), "unit": "sims/s (same candidates, passed as edit lists)",
                        "ms_per_step": child_wall * 1e3 / args.steps, "kernel_ms_avg": child_s * 1e3,
                        "kernel_ms_median": float(np.median(child_ms)), "kernel_ms_min": float(np.min(child_ms)),
                        "edits": n_edits, "algorithmic_bytes": child_alg,
                        "roofline": {"bound": "hbm", "achieved": child_alg / child_s / 1e9, "peak": HBM_PEAK_GBS,
                                     "unit": "GB/s", "frac": child_alg / child_s / 1e9 / HBM_PEAK_GBS,
                                     "traffic": measured_traffic(args.config, MEASURED_TRAFFIC_CHILDREN)
                                     if C == tr.C and args.rate_scale == 1.0 else None},
                        "ap_parent_set_ms": parent_set_ms, "ap_parent_set_first_ms": parent_first_ms,
                        "matches_dense": bool(got2.tobytes() == got.tobytes())}
    finally:
        binding.ap_workload_destroy(h)

    sims = C * R
    full_batch = (C == tr.C and args.rate_scale == 1.0 and not args.cost_tables)
    ms_per_step = wall * 1e3 / args.steps
    avg_kernel_s = float(np.mean(kernel_ms)) * 1e-3
    alg = algorithmic_bytes(C, R, n_types)
    achieved = alg / avg_kernel_s / 1e9

    result = {
        "metric": "candidate-request simulations/s",
        "value": sims / (wall / args.steps),
        "unit": "sims/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {tr.spec.name}: C={C} R={R} M={M} B={tr.B}"
                               + (f" arrival rate x{args.rate_scale:g}" if args.rate_scale != 1.0 else "")
                               + (" (cost model passed as tables)" if args.cost_tables else ""),
                   "candidates": C, "requests": R, "replicas": M, "slots": tr.B, "replica_types": n_types},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(args.config) if full_batch else None,
                     "kernel": "one ap_eval_candidates call (screening kernel + replay of pending candidates)",
                     "kernel_ms_avg": avg_kernel_s * 1e3, "kernel_ms_median": float(np.median(kernel_ms)),
                     "kernel_ms_min": float(np.min(kernel_ms)), "algorithmic_bytes": alg},
        "mean_ttft_us_row0": int(got["sum_ttft_us"][0]) / R,
        "rejected_row0": int(got["n_rejected"][0]),
        # of the candidates scored by the calls above: how many the exact shortcuts settled, how many went through
        # the request-by-request replay
        "screened": {"candidates": after[0] - before[0], "replayed": after[1] - before[1],
                     "settled_by_shortcut": (after[0] - before[0]) - (after[1] - before[1])},
    }
    alu = MEASURED_ALU.get(args.config)
    if full_batch and alu is not None and alu[0] == kernel_source_hash():
        result["alu"] = dict(alu[1], unit="wave-instructions per candidate-request, rocprofv3 SQ_INSTS_* (see profiles/)",
                             valu_peak_per_s=VALU_PEAK_PER_S,
                             valu_per_s=alu[1]["valu"] * sims / avg_kernel_s,
                             valu_frac=alu[1]["valu"] * sims / avg_kernel_s / VALU_PEAK_PER_S)

    # Side workloads of the default run, each timed like the main one: configs[3] (the other configuration the
    # target names), configs[2] (the one-wavefront screening kernel at its stated size) and the saturated variants
    # (arrival rate x100; NOT part of the benchmark spec: the stated traces are lightly loaded).
    if args.config == 4 and full_batch and not args.no_extras:
        side = {}
        side["configs3"], d_rows3 = side_workload(3, 1.0, traces.SPECS[3].C, None, args.steps, args.warmup, "")
        alu3 = MEASURED_ALU.get(3)
        if alu3 is not None and alu3[0] == kernel_source_hash():
            side["configs3"]["alu"] = alu3[1]
        # the same workload with its cost model handed over as tables, the form in which the paper's roofline cost
        # model reaches the replay
        side["configs3_cost_tables"], _ = side_workload(3, 1.0, traces.SPECS[3].C, d_rows3, args.steps, args.warmup,
                                                        " cost model as tables", cost_tables=True)
        sat3, _ = side_workload(3, 100.0, traces.SPECS[3].C, d_rows3, args.steps, args.warmup, " (outside BASELINE.json)")
        del d_rows3
        side["configs2"], _ = side_workload(2, 1.0, traces.SPECS[2].C, None, args.steps, args.warmup, "")
        sat4, _ = side_workload(4, 100.0, 2048, d_assign[:2048], max(3, args.steps // 4), min(args.warmup, 2),
                                " first 2048 rows (outside BASELINE.json)")
        side["saturated"] = {"configs3_x100": sat3, "configs4_x100": sat4}
        result.update(side)

    if children is not None:
        result["sparse_children"] = children

    if not args.no_cpu:
        import oracle
        threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")), 16)
        orc = oracle.Oracle.from_trace(tr)
        if args.cpu_rows:
            n_cpu = args.cpu_rows
        else:
            # size the sample for about 15 s of CPU work: time one row per thread first
            probe = np.stack([tr.assignment_row(int(c)) for c in range(min(C, threads))])
            t0 = time.perf_counter()
            orc.eval_batch(probe, nthreads=threads)
            per_row_cpu_s = max(1e-6, (time.perf_counter() - t0) * threads / probe.shape[0])
            n_cpu = int(min(C, max(1024, 15.0 / per_row_cpu_s)))     # at least 1024 rows whenever a subset is timed
        pick = np.unique(np.linspace(0, C - 1, n_cpu).astype(np.int64))
        rows = np.stack([tr.assignment_row(int(c)) for c in pick])
        t0 = time.perf_counter()
        want = orc.eval_batch(rows, nthreads=threads)
        cpu_s = time.perf_counter() - t0
        same = got[pick].tobytes() == want.tobytes()
        # the same oracle on one thread, on a few of those rows
        one = rows[:: max(1, len(rows) // 8)][:8]
        t0 = time.perf_counter()
        orc.eval_batch(one, nthreads=1)
        one_s = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": len(pick) * R / cpu_s, "unit": "sims/s", "cores": threads,
                                  "kind": "oracle",
                                  "sample": f"{len(pick)} of {C} candidate rows (evenly spaced), all {R} requests, "
                                            f"{cpu_s:.2f} s wall on {threads} threads",
                                  "matches_gpu": bool(same),
                                  "value_one_thread": one.shape[0] * R / one_s, "cpu_model": cpu_model()}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
