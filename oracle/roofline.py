"""CPU oracle for the roofline cost tables (numpy, float64).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``; the product never imports it and it shares no code
with the HIP path.

What is computed, and which passage of the paper each step follows (Appendix "Serving Simulator"):

* ``weight_bytes``: the model-weight-size equation,
  ``W_z = [L (3 H I + 2 A H d + 2 K H d) + 2 H V] * eta / 8`` with ``d = H / A``.
* ``op_time``: the roofline equations, ``pi = min(F / A * B_g, F_g)`` and ``T_op = F / pi`` for an
  operation of ``F`` FLOPs touching ``A`` bytes.
* ``comm_time``: the ring all-reduce equation,
  ``T_comm = 2 (t - 1) / t * 2 L * H * b * s * eta / 8 / R_{g,t}``, with the intra-node bandwidth when
  ``t <= nu_g`` and the cross-node one otherwise.
* ``prefill_time`` / ``decode_time``: "apply the roofline equations to each sublayer and add the
  all-reduce time", and the serve-latency equation ``Lambda = T_prefill(s_p) + sum_{k = s_p}^{s_p + s_d - 1}
  T_decode(k)`` (the prefix table of ``tables`` and the difference taken in ``request_costs``).
* ``feasible``: the memory-feasibility test, ``W_z / t <= theta * m_g`` with ``theta = 0.8``.

Readings where the paper is silent (it names the sublayers' weights in the weight equation but prints no
FLOP or byte counts for them).  Per transformer layer, for ``n`` new tokens per sequence attending to a
context of ``c`` tokens, batch ``b``, tensor-parallel degree ``t`` (FLOPs, weights and head-sharded
activations divide by ``t``), ``e = eta / 8`` bytes per element:

    QKV projection     F = 2 b n H (A + 2K) d / t    bytes = e [H (A + 2K) d / t + b n H + b n (A + 2K) d / t]
    attention          F = 4 b n c A d / t           bytes = e [2 b n A d / t + 2 b c K d / t]
    output projection  F = 2 b n A d H / t           bytes = e [A d H / t + b n A d / t + b n H]
    MLP (3 matrices)   F = 6 b n H I / t             bytes = e [3 H I / t + 2 b n H + 3 b n I / t]

and once per forward pass the output head on the last position,

    LM head            F = 2 b H V / t               bytes = e [H V / t + b H + b V / t].

The weights these read add up to the weight equation's terms (3HI, 2AHd, 2KHd, and one of the two HV).
Prefill is ``n = c = s_p`` (no causal halving); a decode step at context ``k`` is ``n = 1, c = k``.
Every time is quantised to integer nanoseconds (round half to even) before anything is summed, so sums
over decode steps are exact integers; a request's table entries are
``prefill_us = (T_prefill_ns(s_p) + 500) // 1000`` and
``tpot_us = (decode_ns + 500 s_d) // (1000 s_d)`` (rounded time per output token).

Pins (tests/test_roofline_pins.py): published parameter counts of two public model families for the
weight equation; the compute-bound and memory-bound closed forms and the ridge point for the roofline;
hand-computed values for the all-reduce term; brute-force summation for the prefix table.  The sublayer
counts are a reading of "each sublayer" with no printed value to be checked against; what fixes them
from outside: every FLOP coefficient by the rule of 2 FLOPs per matrix parameter and token (with the
published parameter counts) plus 4 s c H per layer for attention, on a device where every operation is
compute-bound; the weight bytes through the weight equation; the key/value bytes by the linear growth
of a memory-bound decode step with its context (2 K d e bytes per layer and token).  The bytes of the
activations read and written per sublayer have no such anchor: parity unpinned for those terms.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

THETA = 0.8


@dataclass(frozen=True)
class Model:
    layers: int
    hidden: int
    intermediate: int
    vocab: int
    heads: int
    kv_heads: int
    weight_bits: int


@dataclass(frozen=True)
class Gpu:
    mem_bytes: float
    flops: float
    hbm_bytes_per_s: float
    pcie_bytes_per_s: float
    link_intra_bytes_per_s: float
    link_inter_bytes_per_s: float
    gpus_per_node: int


@dataclass(frozen=True)
class Group:
    model: int
    gpu: int
    tp: int
    batch: int


def weight_bytes(m: Model) -> float:
    d = m.hidden / m.heads
    per_layer = 3.0 * m.hidden * m.intermediate + 2.0 * m.heads * m.hidden * d + 2.0 * m.kv_heads * m.hidden * d
    return (m.layers * per_layer + 2.0 * m.hidden * m.vocab) * (m.weight_bits / 8.0)


def feasible(m: Model, g: Gpu, tp: int) -> bool:
    return not (weight_bytes(m) / tp > THETA * g.mem_bytes)


def op_time(flops, nbytes, g: Gpu):
    """Roofline: achieved performance min(F / A * B_g, F_g); time F / that."""
    flops = np.asarray(flops, dtype=np.float64)
    nbytes = np.asarray(nbytes, dtype=np.float64)
    perf = np.minimum(flops / nbytes * g.hbm_bytes_per_s, g.flops)
    return flops / perf


def comm_time(m: Model, g: Gpu, tp: int, batch: int, s):
    s = np.asarray(s, dtype=np.float64)
    if tp == 1:
        return np.zeros_like(s)
    link = g.link_intra_bytes_per_s if tp <= g.gpus_per_node else g.link_inter_bytes_per_s
    return 2.0 * (tp - 1.0) / tp * (2.0 * m.layers) * m.hidden * batch * s * (m.weight_bits / 8.0) / link


def phase_time(m: Model, g: Gpu, tp: int, batch: int, n, c):
    """Seconds for one forward pass of ``n`` new tokens per sequence over a context of ``c`` tokens."""
    n = np.asarray(n, dtype=np.float64)
    c = np.asarray(c, dtype=np.float64)
    e = m.weight_bits / 8.0
    H, I, V, A, K = float(m.hidden), float(m.intermediate), float(m.vocab), float(m.heads), float(m.kv_heads)
    d = H / A
    b, t = float(batch), float(tp)
    qkv = op_time(2.0 * b * n * H * (A + 2.0 * K) * d / t,
                  e * (H * (A + 2.0 * K) * d / t + b * n * H + b * n * (A + 2.0 * K) * d / t), g)
    att = op_time(4.0 * b * n * c * A * d / t,
                  e * (2.0 * b * n * A * d / t + 2.0 * b * c * K * d / t), g)
    proj = op_time(2.0 * b * n * A * d * H / t,
                   e * (A * d * H / t + b * n * A * d / t + b * n * H), g)
    mlp = op_time(6.0 * b * n * H * I / t,
                  e * (3.0 * H * I / t + 2.0 * b * n * H + 3.0 * b * n * I / t), g)
    head = op_time(2.0 * b * H * V / t, e * (H * V / t + b * H + b * V / t), g)
    return m.layers * (((qkv + att) + proj) + mlp) + head + comm_time(m, g, tp, batch, n)


def prefill_time(m: Model, g: Gpu, tp: int, batch: int, s_p):
    return phase_time(m, g, tp, batch, s_p, s_p)


def decode_time(m: Model, g: Gpu, tp: int, batch: int, k):
    return phase_time(m, g, tp, batch, np.ones_like(np.asarray(k, dtype=np.float64)), k)


def to_ns(seconds) -> np.ndarray:
    return np.rint(np.asarray(seconds, dtype=np.float64) * 1e9).astype(np.uint64)


def tables(models, gpus, groups, max_seq: int):
    """``prefill_ns[G][max_seq + 1]`` (entry 0 is 0) and ``decode_prefix_ns[G][max_seq + 2]`` with
    ``decode_prefix_ns[k] = sum_{1 <= j < k} T_decode_ns(j)`` (entries 0 and 1 are 0: a context holds at least
    one token, and the attention operation of an empty context would be 0 FLOPs over a non-zero number of bytes,
    for which the roofline equations give 0 / 0)."""
    G = len(groups)
    prefill_ns = np.zeros((G, max_seq + 1), dtype=np.uint64)
    prefix_ns = np.zeros((G, max_seq + 2), dtype=np.uint64)
    seq = np.arange(max_seq + 1, dtype=np.float64)
    for i, grp in enumerate(groups):
        m, g = models[grp.model], gpus[grp.gpu]
        prefill_ns[i, 1:] = to_ns(prefill_time(m, g, grp.tp, grp.batch, seq[1:]))
        step_ns = np.zeros(max_seq + 1, dtype=np.uint64)                    # contexts 0 .. max_seq; a context is >= 1
        step_ns[1:] = to_ns(decode_time(m, g, grp.tp, grp.batch, seq[1:]))
        prefix_ns[i, 1:] = np.cumsum(step_ns, dtype=np.uint64)
    return prefill_ns, prefix_ns


def request_costs(models, gpus, groups, prompt_len, out_len):
    """Per group and request: ``prefill_us`` and ``tpot_us`` (uint32 [G][R]), from the tables."""
    prompt = np.asarray(prompt_len, dtype=np.int64)
    out = np.asarray(out_len, dtype=np.int64)
    max_seq = int((prompt + out).max())
    prefill_ns, prefix_ns = tables(models, gpus, groups, max_seq)
    decode_ns = prefix_ns[:, prompt + out] - prefix_ns[:, prompt]           # sum over k = s_p .. s_p + s_d - 1
    prefill_us = (prefill_ns[:, prompt] + np.uint64(500)) // np.uint64(1000)
    tpot_us = (decode_ns + (500 * out).astype(np.uint64)) // (1000 * out).astype(np.uint64)
    return prefill_us.astype(np.uint32), tpot_us.astype(np.uint32)
