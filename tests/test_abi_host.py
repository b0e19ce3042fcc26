"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and its host helpers agree with the oracle's histogram map."""
import os
import re

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
