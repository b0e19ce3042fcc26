"""Seeded synthetic request traces and candidate request-to-replica assignments.

This module only *draws inputs*: arrival times, prompt/output lengths, the replica
table (cost coefficients and availability windows) and batches of candidate
assignments.  It contains none of the evaluator's arithmetic (no cost model, no
queue, no metric), so both the CPU oracle's tests and the GPU path's tests can use
it without sharing any of the method between them.

The traces stand in for the production traces the paper replays (ShareGPT /
LongBench derived request traces and Azure-Functions derived cluster membership,
Section 7 "System Evaluation", Experimental setup): they keep their structure
(Poisson or bursty arrivals, heavy-tailed lengths, elastic replica membership) with
every parameter fixed and seeded here.

Randomness: numpy ``Generator(PCG64(SeedSequence([seed, stream, row])))``.  Every
array has a stream of its own and every assignment row a generator of its own, so a
single candidate row can be regenerated without materialising the whole batch.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

UINT64_MAX = np.uint64(0xFFFFFFFFFFFFFFFF)

# (prefill_base_us, prefill_per_tok_us, decode_base_us, decode_per_kctx_us)
COEF_STANDARD = (2000, 3, 25, 5)
COEF_FAST = (1200, 2, 15, 3)
COEF_SLOW = (3500, 5, 40, 8)

_STREAM_ARRIVAL, _STREAM_PROMPT, _STREAM_OUT, _STREAM_REPLICA, _STREAM_ASSIGN, _STREAM_EDITS, _STREAM_AGENTIC = 1, 2, 3, 4, 5, 6, 7


def _rng(seed: int, stream: int, row: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream, row])))


@dataclass(frozen=True)
class TraceSpec:
    name: str
    seed: int
    C: int
    R: int
    M: int
    B: int
    arrivals: str          # "poisson" | "gamma_cv4" | "diurnal"
    rate: float            # mean requests per second
    lengths: str           # "lognormal" | "bimodal"
    replicas: str          # "homogeneous" | "hetero_elastic"
    assign: str            # "uniform" | "half_jsq5" | "jsq1"


SPECS = (
    TraceSpec("cfg0_tiny", 0, 64, 256, 4, 8, "poisson", 20.0, "lognormal", "homogeneous", "uniform"),
    TraceSpec("cfg1_jsq_mix", 1, 1024, 4096, 8, 32, "poisson", 200.0, "lognormal", "homogeneous", "half_jsq5"),
    TraceSpec("cfg2_bursty", 2, 4096, 16384, 32, 32, "gamma_cv4", 800.0, "bimodal", "homogeneous", "uniform"),
    TraceSpec("cfg3_hetero_elastic", 3, 8192, 32768, 64, 64, "poisson", 1500.0, "lognormal",
              "hetero_elastic", "uniform"),
    TraceSpec("cfg4_mutation_sweep", 4, 16384, 131072, 128, 64, "diurnal", 3000.0, "bimodal",
              "homogeneous", "jsq1"),
)


@dataclass
class Trace:
    """One observed request trace plus the recipe for its candidate assignments."""
    spec: TraceSpec
    arrival_us: np.ndarray      # uint64[R], non-decreasing
    prompt_len: np.ndarray      # int32[R]
    out_len: np.ndarray         # int32[R]
    coef: np.ndarray            # uint32[M, 4]
    t_on_us: np.ndarray         # uint64[M]
    t_off_us: np.ndarray        # uint64[M]
    B: int
    slo_ttft_us: int = 500_000
    slo_tpot_us: int = 50_000
    penalty_us: int = 3_600_000_000
    _jsq_base: Optional[np.ndarray] = field(default=None, repr=False)

    @property
    def R(self) -> int:
        return int(self.arrival_us.shape[0])

    @property
    def M(self) -> int:
        return int(self.coef.shape[0])

    @property
    def C(self) -> int:
        return self.spec.C

    # ---- candidate assignments -------------------------------------------------
    def jsq_base(self) -> np.ndarray:
        """Greedy join-shortest-queue by accumulated prompt tokens (ties: lowest id)."""
        if self._jsq_base is None:
            load = np.zeros(self.M, dtype=np.int64)
            base = np.empty(self.R, dtype=np.uint16)
            prompts = self.prompt_len.tolist()
            for r, p in enumerate(prompts):
                m = int(np.argmin(load))
                base[r] = m
                load[m] += p
            self._jsq_base = base
        return self._jsq_base

    def assignment_row(self, c: int) -> np.ndarray:
        """Candidate row ``c`` as uint16[R]; depends only on (seed, c)."""
        spec, R, M = self.spec, self.R, self.M
        rng = _rng(spec.seed, _STREAM_ASSIGN, c)
        if spec.assign == "uniform" or (spec.assign == "half_jsq5" and c < spec.C // 2):
            return rng.integers(0, M, size=R, dtype=np.uint16)
        row = self.jsq_base().copy()
        pos, val = self._mutation_draws(rng)
        row[pos] = val
        return row

    def _mutation_draws(self, rng: np.random.Generator):
        """The (request, replica) pairs a mutated row draws, in draw order (requests may repeat)."""
        frac = 0.05 if self.spec.assign == "half_jsq5" else 0.01
        n = max(1, int(round(frac * self.R)))
        pos = rng.integers(0, self.R, size=n)
        return pos, rng.integers(0, self.M, size=n, dtype=np.uint16)

    def is_mutated_row(self, c: int) -> bool:
        """True when row ``c`` is the join-shortest-queue parent plus a list of reassignments."""
        return self.spec.assign == "jsq1" or (self.spec.assign == "half_jsq5" and c >= self.spec.C // 2)

    def mutation_lists(self, lo: int, hi: int, *, tidy: bool = False):
        """Rows ``lo..hi`` of a mutation sweep as edit lists against ``jsq_base()``.

        Returns ``(edit_first uint32[hi-lo+1], edit_request uint32[E], edit_replica uint16[E])``: the very
        pairs ``assignment_row`` draws, in draw order, so a request can occur more than once in a list.
        ``tidy=True`` lists every request once, in increasing order, keeping the pair drawn last.
        """
        first, reqs, reps = [0], [], []
        for c in range(lo, hi):
            if not self.is_mutated_row(c):
                raise ValueError(f"row {c} of {self.spec.name} is not drawn as a mutation of the parent")
            pos, val = self._mutation_draws(_rng(self.spec.seed, _STREAM_ASSIGN, c))
            if tidy:
                # last occurrence of every request: first occurrence in the reversed list
                uniq, idx = np.unique(pos[::-1], return_index=True)
                pos, val = uniq, val[::-1][idx]
            reqs.append(pos.astype(np.uint32))
            reps.append(val.astype(np.uint16))
            first.append(first[-1] + pos.shape[0])
        return (np.asarray(first, dtype=np.uint32), np.concatenate(reqs) if reqs else np.zeros(0, np.uint32),
                np.concatenate(reps) if reps else np.zeros(0, np.uint16))

    def assignment_rows(self, lo: int, hi: int) -> np.ndarray:
        out = np.empty((hi - lo, self.R), dtype=np.uint16)
        for i, c in enumerate(range(lo, hi)):
            out[i] = self.assignment_row(c)
        return out


def draw_edit_lists(seed: int, n_children: int, R: int, M: int, mean_edits: float, *,
                    request_range: Optional[int] = None, replica_range: Optional[int] = None,
                    sorted_lists: bool = False):
    """Edit lists for ``n_children`` children of some parent row: per child a Poisson(``mean_edits``) number
    of (request, replica) pairs (so some lists are empty), requests uniform below ``request_range``
    (default R; larger values produce edits that name no request), replicas uniform below ``replica_range``
    (default M; larger values produce unknown replica ids).  ``sorted_lists`` orders each list by request
    (stable: equal requests keep their draw order).  Returns ``(edit_first, edit_request, edit_replica)``."""
    rng = _rng(seed, _STREAM_EDITS)
    counts = rng.poisson(mean_edits, size=n_children)
    first = np.zeros(n_children + 1, dtype=np.uint32)
    np.cumsum(counts, out=first[1:])
    total = int(first[-1])
    request = rng.integers(0, request_range or R, size=total).astype(np.uint32)
    replica = rng.integers(0, replica_range or M, size=total).astype(np.uint16)
    if sorted_lists:
        for c in range(n_children):
            lo, hi = int(first[c]), int(first[c + 1])
            order = np.argsort(request[lo:hi], kind="stable")
            request[lo:hi], replica[lo:hi] = request[lo:hi][order], replica[lo:hi][order]
    return first, request, replica


def make_agentic(seed: int, W: int = 64, *, P: int = 4, Q: int = 4, mean_calls: float = 5.0, rate: float = 20.0,
                 capacity: int = 16384) -> dict:
    """A slice of multi-call agentic workflows (stands in for the 64-workflow ShareGPT slices of Section 8.3):
    ``W`` workflows arriving as a Poisson process of ``rate`` per second; each a DAG of 1 + Poisson(mean_calls - 1)
    calls in which call j depends on call j - 1 with probability 0.7 and on one or two earlier calls otherwise
    (fan-out / fan-in), lengths log-normal like the request traces; ``P`` prefill and ``Q`` decode instances of three
    speeds in turn; a committed horizon per workflow proportional to its total token count.  Inputs only: nothing
    here schedules anything."""
    rng = _rng(seed, _STREAM_AGENTIC)
    arrival = np.floor(np.cumsum(rng.exponential(1.0 / rate, size=W)) * 1e6).astype(np.uint64)
    wf, in_len, out_len, pred_first, pred = [], [], [], [0], []
    for w in range(W):
        n = 1 + int(rng.poisson(max(0.0, mean_calls - 1.0)))
        base = len(wf)
        for j in range(n):
            wf.append(w)
            in_len.append(int(np.clip(np.floor(rng.lognormal(6.0, 1.0)), 16, 8192)))
            out_len.append(int(np.clip(np.floor(rng.lognormal(5.0, 1.0)), 1, 2048)))
            if j > 0:
                if rng.random() < 0.7:
                    mine = {base + j - 1}
                else:
                    mine = {base + int(x) for x in rng.integers(0, j, size=int(rng.integers(1, 3)))}
                pred.extend(sorted(mine))
            pred_first.append(len(pred))
    wf = np.asarray(wf, dtype=np.uint32)
    in_len, out_len = np.asarray(in_len, dtype=np.uint32), np.asarray(out_len, dtype=np.uint32)
    tokens = np.bincount(wf, weights=(in_len + out_len).astype(np.float64), minlength=W)
    slo = np.maximum(1, np.floor(tokens * rng.uniform(20.0, 120.0, size=W))).astype(np.uint64)
    kinds_p = ((1500, 2), (2500, 3), (900, 1))
    kinds_q = ((25, 5), (40, 8), (15, 3))
    return dict(arrival_us=arrival, slo_us=slo, wf=wf, in_len=in_len, out_len=out_len,
                pred_first=np.asarray(pred_first, dtype=np.uint32), pred=np.asarray(pred, dtype=np.uint32),
                pa=np.array([kinds_p[i % 3][0] for i in range(P)], dtype=np.uint32),
                pb=np.array([kinds_p[i % 3][1] for i in range(P)], dtype=np.uint32),
                qc=np.array([kinds_q[i % 3][0] for i in range(Q)], dtype=np.uint32),
                qd=np.array([kinds_q[i % 3][1] for i in range(Q)], dtype=np.uint32),
                cap=np.full(Q, capacity, dtype=np.uint32), penalty_permille=100_000)


def draw_agentic_candidates(seed: int, n_candidates: int, K: int, P: int, Q: int, *, key_range: int = 1 << 20,
                            bad_ids: bool = False):
    """Candidate plans for ``K`` calls: a prefill instance, a decode instance and a queue key per call, uniform;
    row 1 (if present) orders every queue by call index.  ``bad_ids`` lets a few ids fall outside the cluster."""
    rng = _rng(seed, _STREAM_AGENTIC, 1)
    pre = rng.integers(0, P + (1 if bad_ids else 0), size=(n_candidates, K)).astype(np.uint16)
    dec = rng.integers(0, Q + (1 if bad_ids else 0), size=(n_candidates, K)).astype(np.uint16)
    key = rng.integers(0, key_range, size=(n_candidates, K)).astype(np.uint32)
    if n_candidates > 1:
        key[1] = 0                                            # all keys equal: ties go to the lower call index
    return pre, dec, key


def _arrivals(spec: TraceSpec, R: int, rate_scale: float) -> np.ndarray:
    rng = _rng(spec.seed, _STREAM_ARRIVAL)
    rate = spec.rate
    if spec.arrivals == "poisson":
        t = np.cumsum(rng.exponential(1.0 / rate, size=R))
    elif spec.arrivals == "gamma_cv4":
        # renewal process with squared CV 16: shape 1/16, mean gap 1/rate
        t = np.cumsum(rng.gamma(1.0 / 16.0, 16.0 / rate, size=R))
    elif spec.arrivals == "diurnal":
        # rate(t) = rate * (1 + 0.5 sin(2 pi t / 600 s)), by thinning a 1.5*rate process
        lam_max = 1.5 * rate
        n = int(2.5 * R) + 4096
        cand = np.cumsum(rng.exponential(1.0 / lam_max, size=n))
        keep = rng.random(n) * lam_max < rate * (1.0 + 0.5 * np.sin(2.0 * np.pi * cand / 600.0))
        t = cand[keep]
        if t.shape[0] < R:
            raise RuntimeError("thinning produced too few arrivals")
        t = t[:R]
    else:
        raise ValueError(spec.arrivals)
    t = t / rate_scale
    return np.floor(t * 1e6).astype(np.uint64)


def _lengths(spec: TraceSpec, R: int):
    rp, ro = _rng(spec.seed, _STREAM_PROMPT), _rng(spec.seed, _STREAM_OUT)
    if spec.lengths == "lognormal":
        prompt = np.clip(np.floor(rp.lognormal(6.0, 1.0, size=R)), 16, 4096)
        out = np.clip(np.floor(ro.lognormal(5.0, 1.0, size=R)), 1, 1024)
    elif spec.lengths == "bimodal":
        short = rp.lognormal(5.0, 0.8, size=R)
        long_ = rp.lognormal(8.0, 0.5, size=R)
        pick_long = rp.random(R) >= 0.7
        prompt = np.clip(np.floor(np.where(pick_long, long_, short)), 16, 32768)
        out = np.clip(np.floor(ro.lognormal(5.5, 1.2, size=R)), 1, 2048)
    else:
        raise ValueError(spec.lengths)
    return prompt.astype(np.int32), out.astype(np.int32)


def _replicas(spec: TraceSpec, M: int, arrival_us: np.ndarray):
    coef = np.empty((M, 4), dtype=np.uint32)
    t_on = np.zeros(M, dtype=np.uint64)
    t_off = np.full(M, UINT64_MAX, dtype=np.uint64)
    if spec.replicas == "homogeneous":
        coef[:] = COEF_STANDARD
    elif spec.replicas == "hetero_elastic":
        kinds = (COEF_STANDARD, COEF_FAST, COEF_SLOW)
        for m in range(M):
            coef[m] = kinds[m % 3]
        rng = _rng(spec.seed, _STREAM_REPLICA)
        last = int(arrival_us[-1])
        xy = rng.integers(0, last + 1, size=(M, 2), dtype=np.uint64)
        t_on = xy.min(axis=1).astype(np.uint64)
        t_off = xy.max(axis=1).astype(np.uint64)
    else:
        raise ValueError(spec.replicas)
    return coef, t_on, t_off


def make_trace(cfg: int, *, C: Optional[int] = None, R: Optional[int] = None, M: Optional[int] = None,
               B: Optional[int] = None, rate_scale: float = 1.0) -> Trace:
    """Build configuration ``cfg`` (0..4).  ``C``/``R``/``M``/``B`` shrink or reshape it for
    tests; ``rate_scale`` > 1 compresses arrivals to make a saturated variant."""
    base = SPECS[cfg]
    spec = TraceSpec(base.name, base.seed, C or base.C, R or base.R, M or base.M, B or base.B,
                     base.arrivals, base.rate, base.lengths, base.replicas, base.assign)
    arrival = _arrivals(spec, spec.R, rate_scale)
    prompt, out = _lengths(spec, spec.R)
    coef, t_on, t_off = _replicas(spec, spec.M, arrival)
    return Trace(spec, arrival, prompt, out, coef, t_on, t_off, spec.B)


def custom_trace(arrival_us, prompt_len, out_len, coef, t_on_us=None, t_off_us=None, *, B: int,
                 slo_ttft_us: int = 500_000, slo_tpot_us: int = 50_000,
                 penalty_us: int = 3_600_000_000, name: str = "custom") -> Trace:
    """Wrap hand-made arrays (edge-case tests) in a Trace."""
    arrival = np.asarray(arrival_us, dtype=np.uint64)
    coef = np.asarray(coef, dtype=np.uint32).reshape(-1, 4)
    M = coef.shape[0]
    t_on = np.zeros(M, dtype=np.uint64) if t_on_us is None else np.asarray(t_on_us, dtype=np.uint64)
    t_off = np.full(M, UINT64_MAX, dtype=np.uint64) if t_off_us is None else np.asarray(t_off_us, dtype=np.uint64)
    spec = TraceSpec(name, 0, 0, int(arrival.shape[0]), M, B, "custom", 0.0, "custom", "custom", "uniform")
    return Trace(spec, arrival, np.asarray(prompt_len, dtype=np.int32), np.asarray(out_len, dtype=np.int32),
                 coef, t_on, t_off, B, slo_ttft_us, slo_tpot_us, penalty_us)
