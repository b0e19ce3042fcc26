"""The entry point that allocates nothing (``ap_trace_time_static``) against the one it is a variant of
(``ap_trace_time``), through the C ABI: integer nanoseconds, so every field of every record must be equal.  Two calls in a
row on the same GPU, the second with a smaller input (fewer models, GPU types, intervals and candidates), so that
whatever the first call left in the library's fixed array would show if the second call looked at it."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import roofline as rf                          # noqa: E402
from paper_2604_07144_amd import binding                  # noqa: E402
from tests.test_gpu_roofline import GPUS, MODELS, _pack    # noqa: E402


def _inputs(seed, C, N, models, gpus):
    rng = np.random.default_rng(seed)
    Z, G = len(models), len(gpus)
    options = np.array([(0, 0), (0, 0), (1, 1), (2, 1), (2, 2), (8, 1), (16, 4), (3, 0)], dtype=np.uint32)
    plans = options[rng.integers(0, len(options), size=(C, N, Z, G))]
    keep = rng.random((C, N)) < 0.35
    for i in range(1, N):
        plans[:, i][keep[:, i]] = plans[:, i - 1][keep[:, i]]
    m, g, _ = _pack(models, gpus, [rf.Group(0, 0, 1, 1)])
    dev = lambda a, t: torch.from_numpy(np.ascontiguousarray(a).view(t)).cuda()
    return dict(models=m, gpus=g, coef=list(rng.uniform(5.3, 11.5, Z)), C=C, N=N,
                plans=dev(plans, np.int32), n=dev(rng.integers(0, N + 2, size=C).astype(np.uint32), np.int32),
                sched=dev(rng.integers(0, 10**10, size=C).astype(np.uint64), np.int64),
                stale=dev(rng.integers(0, 10**10, size=(C, N)).astype(np.uint64), np.int64),
                serve=dev(rng.integers(0, 10**11, size=(C, N)).astype(np.uint64), np.int64))


def _call(fn, x, scope, out):
    fn(x["models"], x["coef"], x["gpus"], x["plans"].data_ptr(), x["n"].data_ptr(), x["sched"].data_ptr(),
       x["stale"].data_ptr(), x["serve"].data_ptr(), x["C"], x["N"], out.data_ptr(), scope,
       torch.cuda.current_stream().cuda_stream)


def test_static_variant_equals_the_allocating_one_on_two_calls_in_a_row():
    big = _inputs(1, 900, 6, MODELS, GPUS)
    small = _inputs(2, 70, 3, MODELS[1:3], GPUS[:1])
    for scope in (binding.AP_LOAD_DEPLOYED, binding.AP_LOAD_CHANGED):
        outs = []
        for x in (big, small):                                          # the second call has the smaller input
            out = torch.full((x["C"], 6), -1, dtype=torch.int64, device="cuda")
            _call(binding.ap_trace_time_static, x, scope, out)
            outs.append(out)
        torch.cuda.synchronize()
        for x, out in zip((big, small), outs):
            want = torch.full((x["C"], 6), -2, dtype=torch.int64, device="cuda")
            _call(binding.ap_trace_time, x, scope, want)
            assert torch.equal(out, want), scope
        assert int((outs[0][:, 2] > 0).sum()) > 0                       # reconfiguration happened somewhere


def test_static_variant_refuses_what_does_not_fit_its_array():
    x = _inputs(3, 4, 2, MODELS[:1], GPUS[:1])
    out = torch.zeros((4, 6), dtype=torch.int64, device="cuda")
    many_models = np.repeat(x["models"], 65)
    with pytest.raises(binding.ApError) as e:
        binding.ap_trace_time_static(many_models, [6.0] * 65, x["gpus"], x["plans"].data_ptr(), x["n"].data_ptr(),
                                     x["sched"].data_ptr(), x["stale"].data_ptr(), x["serve"].data_ptr(), 4, 2, out.data_ptr())
    assert e.value.status == binding.AP_ERR_RANGE
    many_gpus = np.repeat(x["gpus"], 17)
    with pytest.raises(binding.ApError) as e:
        binding.ap_trace_time_static(x["models"], x["coef"], many_gpus, x["plans"].data_ptr(), x["n"].data_ptr(),
                                     x["sched"].data_ptr(), x["stale"].data_ptr(), x["serve"].data_ptr(), 4, 2, out.data_ptr())
    assert e.value.status == binding.AP_ERR_RANGE
