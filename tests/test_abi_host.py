"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and its host helpers agree with the oracle's histogram map."""
import os
import re
import subprocess

import numpy as np

import oracle
from paper_2604_07144_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in os.listdir(inc):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names.update(re.findall(r"\b(ap_[a-z0-9_]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    names = declared_functions()
    assert {"ap_workload_create", "ap_costmodel_set", "ap_eval_candidates", "ap_workload_destroy",
            "ap_status_str", "ap_hist_bin", "ap_hist_lower"} <= names
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    seen = {binding.ap_status_str(s) for s in range(6)}
    assert len(seen) == 6 and "ok" in seen


def test_struct_sizes_match_header():
    assert binding.METRICS_DTYPE.itemsize == 64
    assert binding.REPLICA_DTYPE.itemsize == 32
    assert binding.METRICS_DTYPE == oracle.METRICS_DTYPE      # same record layout on both sides


def test_host_histogram_helpers_match_oracle():
    rng = np.random.default_rng(0)
    vals = np.concatenate([np.arange(0, 4096), (2 ** rng.uniform(7, 64, 20000)).astype(np.float64)])
    vals = [min(int(v), 2**64 - 1) for v in vals] + [2**38 - 2**30 - 1, 2**38 - 2**30, 2**38, 2**64 - 1]
    for v in vals:
        assert binding.ap_hist_bin(v) == oracle.hist_bin(v), v
    for b in range(4096):
        assert binding.ap_hist_lower(b) == oracle.hist_lower(b), b


def test_struct_layouts_match_the_header_as_gcc_sees_it(tmp_path):
    """Every struct of the header, compiled by gcc: sizes and field offsets must be the ones the binding's numpy
    dtypes (and, for the two shared records, the oracle's) assume."""
    structs = {"ap_replica": binding.REPLICA_DTYPE, "ap_metrics": binding.METRICS_DTYPE,
               "ap_typed_replica": binding.TYPED_REPLICA_DTYPE, "ap_model": binding.MODEL_DTYPE, "ap_gpu": binding.GPU_DTYPE,
               "ap_group": binding.GROUP_DTYPE, "ap_placement": binding.PLACEMENT_DTYPE, "ap_breakdown": binding.BREAKDOWN_DTYPE,
               "ap_agentic_metrics": binding.AGENTIC_METRICS_DTYPE}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "autopoiesis_eval.h"', 'int main(void) {']
    for name, dt in structs.items():
        lines.append(f'printf("{name} size %zu\\n", sizeof({name}));')
        for field in dt.names:
            lines.append(f'printf("{name} {field} %zu\\n", offsetof({name}, {field}));')
    lines += ['printf("ap_slo size %zu\\n", sizeof(ap_slo));', 'printf("ap_prefill_instance size %zu\\n", sizeof(ap_prefill_instance));',
              'printf("ap_decode_instance size %zu\\n", sizeof(ap_decode_instance));', 'return 0; }']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c11", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    seen = {}
    for line in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines():
        name, what, value = line.split()
        seen[(name, what)] = int(value)
    for name, dt in structs.items():
        assert seen[(name, "size")] == dt.itemsize, name
        for field in dt.names:
            assert seen[(name, field)] == dt.fields[field][1], (name, field)
    assert seen[("ap_slo", "size")] == 24 and seen[("ap_prefill_instance", "size")] == 8
    assert seen[("ap_decode_instance", "size")] == 12
    from oracle import agentic
    assert agentic.METRICS_DTYPE == binding.AGENTIC_METRICS_DTYPE


def test_generators_produce_well_formed_inputs():
    """The seeded generators shared by both sides hold no method arithmetic, but what they draw must be
    well-formed: sorted arrivals, positive lengths, edit ranges that tile the arrays, DAGs in topological order."""
    from paper_2604_07144_amd import traces
    for cfg in (0, 1):
        tr = traces.make_trace(cfg)
        assert (np.diff(tr.arrival_us.astype(np.int64)) >= 0).all() and tr.prompt_len.min() >= 1 and tr.out_len.min() >= 1
        assert tr.assignment_rows(0, 4).shape == (4, tr.R) and int(tr.assignment_rows(0, 4).max()) < tr.M
    tr = traces.make_trace(1)
    assert not tr.is_mutated_row(0) and tr.is_mutated_row(tr.C - 1)
    first, request, replica = tr.mutation_lists(tr.C // 2, tr.C // 2 + 5)
    assert first[0] == 0 and first[-1] == len(request) == len(replica) and (np.diff(first.astype(np.int64)) > 0).all()
    first, request, replica = traces.draw_edit_lists(3, 50, 1000, 7, 4.0, request_range=1003, replica_range=8, sorted_lists=True)
    assert first[-1] == len(request) and int(request.max()) < 1003 and int(replica.max()) < 8
    assert all((np.diff(request[first[c]:first[c + 1]].astype(np.int64)) >= 0).all() for c in range(50))
    wl = traces.make_agentic(5, 40)
    K = len(wl["wf"])
    assert wl["pred_first"][0] == 0 and wl["pred_first"][-1] == len(wl["pred"]) and len(wl["pred_first"]) == K + 1
    for k in range(K):
        for j in wl["pred"][wl["pred_first"][k]:wl["pred_first"][k + 1]]:
            assert j < k and wl["wf"][j] == wl["wf"][k]
    assert (np.diff(wl["arrival_us"].astype(np.int64)) >= 0).all() and wl["slo_us"].min() >= 1
    pre, dec, key = traces.draw_agentic_candidates(5, 3, K, 4, 4)
    assert pre.shape == dec.shape == key.shape == (3, K) and int(pre.max()) < 4 and int(dec.max()) < 4 and (key[1] == 0).all()
