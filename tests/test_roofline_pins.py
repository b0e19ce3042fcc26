"""Pins for the roofline cost-table oracle (no GPU needed): each ties ``oracle/roofline.py`` to something
other than itself - published parameter counts, the closed forms of the roofline model, hand-computed values
of the printed all-reduce equation, brute-force sums."""
import numpy as np
import pytest

from oracle import roofline as rf

LLAMA2_7B = rf.Model(layers=32, hidden=4096, intermediate=11008, vocab=32000, heads=32, kv_heads=32, weight_bits=16)
LLAMA3_8B = rf.Model(layers=32, hidden=4096, intermediate=14336, vocab=128256, heads=32, kv_heads=8, weight_bits=16)
# a GPU in round numbers: 1e15 FLOP/s, 4e12 B/s HBM -> ridge point at 250 FLOP/byte
GPU = rf.Gpu(mem_bytes=80e9, flops=1e15, hbm_bytes_per_s=4e12, pcie_bytes_per_s=64e9,
             link_intra_bytes_per_s=450e9, link_inter_bytes_per_s=50e9, gpus_per_node=8)


def test_weight_equation_against_published_parameter_counts():
    """Appendix "Serving Simulator", model weight size.  The equation counts the projection, MLP, embedding
    and output matrices; the published totals of these two public models add the 65 norm vectors of length H
    (two per layer and a final one): 6,738,415,616 and 8,030,261,248 parameters."""
    for model, published in ((LLAMA2_7B, 6_738_415_616), (LLAMA3_8B, 8_030_261_248)):
        params = rf.weight_bytes(model) / (model.weight_bits / 8)
        assert params + (2 * model.layers + 1) * model.hidden == published
    assert rf.weight_bytes(LLAMA2_7B) == 2 * 6_738_149_376          # 16-bit weights: two bytes each


def test_memory_feasibility():
    """W_z / t > theta * m_g is infeasible, theta = 0.8."""
    small = rf.Gpu(16e9, 1e14, 1e12, 32e9, 1e11, 1e10, 8)
    assert not rf.feasible(LLAMA2_7B, small, 1)                      # 13.5 GB of weights > 12.8 GB
    assert rf.feasible(LLAMA2_7B, small, 2)
    assert rf.feasible(LLAMA2_7B, GPU, 1)
    exact = rf.Gpu(rf.weight_bytes(LLAMA2_7B) / 0.8, 1e14, 1e12, 32e9, 1e11, 1e10, 8)
    assert rf.feasible(LLAMA2_7B, exact, 1)                          # equality is still feasible (strict ">")


def test_roofline_closed_forms():
    """pi = min(F / A * B, F_g), T = F / pi: compute-bound operations take F / F_g, memory-bound ones A / B,
    and the two meet at the ridge point F_g / B."""
    flops = np.array([1e12, 1e12, 1e12, 5e9])
    nbytes = np.array([1e9, 4e9, 1e10, 1e9])                         # intensities 1000, 250 (ridge), 100, 5
    got = rf.op_time(flops, nbytes, GPU)
    want = np.array([1e12 / 1e15, 1e12 / 1e15, 1e10 / 4e12, 1e9 / 4e12])
    assert np.allclose(got, want, rtol=1e-15, atol=0)
    assert np.all(rf.op_time(flops, nbytes, GPU) >= np.maximum(flops / GPU.flops, nbytes / GPU.hbm_bytes_per_s) * (1 - 1e-15))


def test_allreduce_equation_by_hand():
    """T_comm = 2 (t - 1) / t * 2 L * H * b * s * eta / 8 / R: for t = 4, L = 32, H = 4096, b = 2, s = 1000,
    16-bit, R = 450e9: 1.5 * 64 * 4096 * 2 * 1000 * 2 / 450e9 seconds."""
    got = float(rf.comm_time(LLAMA2_7B, GPU, 4, 2, 1000))
    assert got == pytest.approx(1.5 * 64 * 4096 * 2 * 1000 * 2 / 450e9, rel=1e-15)
    assert float(rf.comm_time(LLAMA2_7B, GPU, 1, 2, 1000)) == 0.0                      # no partner, no all-reduce
    cross = float(rf.comm_time(LLAMA2_7B, GPU, 16, 2, 1000))                           # t > nu_g: cross-node links
    assert cross == pytest.approx(2 * 15 / 16 * 64 * 4096 * 2 * 1000 * 2 / 50e9, rel=1e-15)


def test_decode_step_is_linear_in_context_when_memory_bound():
    """At batch 1 every sublayer of a decode step sits far below the ridge point, so the step costs its bytes
    over the HBM bandwidth, and only the key/value read grows with the context: by 2 K d e bytes per layer and
    token."""
    k = np.arange(1, 4000, dtype=np.float64)
    t = rf.decode_time(LLAMA3_8B, GPU, 1, 1, k)
    slope = np.diff(t)
    want = LLAMA3_8B.layers * 2 * LLAMA3_8B.kv_heads * 128 * 2 / GPU.hbm_bytes_per_s
    assert np.allclose(slope, want, rtol=1e-6)
    weights_once = rf.weight_bytes(LLAMA3_8B) - 2 * 4096 * 128256          # every matrix but the embedding is read
    assert t[0] >= weights_once / GPU.hbm_bytes_per_s                        # at least the weights cross the bus


def test_prefill_is_compute_bound_for_long_prompts_and_scales_with_tp():
    s = np.array([4096.0])
    t1 = float(rf.prefill_time(LLAMA2_7B, GPU, 1, 1, s)[0])
    m = LLAMA2_7B
    flops = m.layers * (2 * s * m.hidden * 3 * m.hidden + 4 * s * s * m.hidden + 2 * s * m.hidden * m.hidden
                        + 6 * s * m.hidden * m.intermediate)[0]
    assert t1 == pytest.approx(flops / GPU.flops, rel=2e-3)          # the head and rounding aside: F / F_g
    t4 = float(rf.prefill_time(LLAMA2_7B, GPU, 4, 1, s)[0])
    comm = float(rf.comm_time(LLAMA2_7B, GPU, 4, 1, s)[0])
    assert t4 - comm == pytest.approx(t1 / 4, rel=2e-2)              # a quarter of the work per GPU, plus the all-reduce


@pytest.mark.parametrize("model,published_params", [(LLAMA2_7B, 6.74e9), (LLAMA3_8B, 8.03e9)], ids=["llama2_7b", "llama3_8b"])
def test_flop_counts_follow_two_flops_per_parameter_and_token(model, published_params):
    """On a device that is compute-bound for every operation the time of a pass is its FLOPs over F_g.  A dense
    transformer spends 2 FLOPs per matrix parameter and token (one multiply-add per weight), the output head once
    per pass, plus 4 s c H per layer for the attention scores and their product with the values: with the published
    parameter counts of the two model families this fixes every FLOP coefficient of the sublayers."""
    slow = rf.Gpu(mem_bytes=80e9, flops=1e9, hbm_bytes_per_s=1e30, pcie_bytes_per_s=64e9,
                  link_intra_bytes_per_s=450e9, link_inter_bytes_per_s=50e9, gpus_per_node=8)
    head = model.hidden * model.vocab
    per_token = published_params - 2 * head                 # the matrices of the layers (norms are ~1e-4 of them)
    for s, c in [(1.0, 1.0), (1.0, 700.0), (512.0, 512.0), (3000.0, 3000.0)]:
        flops = float(rf.phase_time(model, slow, 1, 1, np.array([s]), np.array([c]))[0]) * slow.flops
        want = 2 * s * per_token + 2 * head + 4 * model.layers * s * c * model.hidden
        assert flops == pytest.approx(want, rel=5e-3), (s, c)       # the published counts are rounded to 3 digits
    # batch multiplies everything; tensor parallelism divides it (the all-reduce aside)
    one = float(rf.phase_time(model, slow, 1, 1, np.array([64.0]), np.array([64.0]))[0])
    assert float(rf.phase_time(model, slow, 1, 8, np.array([64.0]), np.array([64.0]))[0]) == pytest.approx(8 * one, rel=1e-12)
    tp4 = float(rf.phase_time(model, slow, 4, 1, np.array([64.0]), np.array([64.0]))[0])
    assert tp4 - float(rf.comm_time(model, slow, 4, 1, np.array([64.0]))[0]) == pytest.approx(one / 4, rel=1e-12)


def test_tables_and_request_costs_against_brute_force():
    models, gpus = [LLAMA2_7B, LLAMA3_8B], [GPU]
    groups = [rf.Group(0, 0, 1, 1), rf.Group(1, 0, 2, 4)]
    prefill_ns, prefix_ns = rf.tables(models, gpus, groups, 300)
    assert prefill_ns[:, 0].tolist() == [0, 0] and prefix_ns[:, :2].tolist() == [[0, 0], [0, 0]]
    prompt, out = np.array([1, 17, 200, 64]), np.array([1, 100, 100, 3])
    pre_us, tpot_us = rf.request_costs(models, gpus, groups, prompt, out)
    for gi, grp in enumerate(groups):
        m = models[grp.model]
        for r in range(4):
            steps = [int(rf.to_ns(rf.decode_time(m, GPU, grp.tp, grp.batch, np.array([float(k)])))[0])
                     for k in range(int(prompt[r]), int(prompt[r] + out[r]))]          # the serve-latency sum, step by step
            assert int(prefix_ns[gi, prompt[r] + out[r]] - prefix_ns[gi, prompt[r]]) == sum(steps)
            assert int(tpot_us[gi, r]) == (sum(steps) + 500 * int(out[r])) // (1000 * int(out[r]))
            pre = int(rf.to_ns(rf.prefill_time(m, GPU, grp.tp, grp.batch, np.array([float(prompt[r])])))[0])
            assert int(pre_us[gi, r]) == (pre + 500) // 1000
    assert (np.diff(prefill_ns[:, 1:].astype(np.int64), axis=1) >= 0).all()         # longer prompts never cost less
