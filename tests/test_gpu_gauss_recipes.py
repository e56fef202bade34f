"""The Gaussian kernels on every way the three policies' parameters can relate to each other.

The continuous workloads draw each policy's log standard deviations on their own, uniformly in the stated
range, with the target's and the worker's means a small offset from the learner's (the default recipe).  Here
the same kernels also meet (a) all three policies drawn fully on their own, means included: log-probabilities
of magnitude up to about two thousand and importance weights over hundreds of orders of magnitude, and (b) the
three policies a few small offsets apart in both means and log-stds, where the weights sit near one and both
branches of every min and clip are taken.  Time-major and fused, fp32 and bf16 ring, bf16 learner tensor,
cached log-probabilities, specialised and generic kernels, every output element against the oracle."""
from dataclasses import replace

import numpy as np
import pytest

import oracle
import workloads
from gpu_common import check_against_oracle, gpu_loss, say, shape_workload, to_device
from test_gpu_buffer import _fused_case

pytestmark = pytest.mark.gpu

RECIPES = {
    "per_policy_logstd": dict(logstd_mode="per_policy", mean_mode="offsets"),       # the workloads' own recipe
    "all_per_policy": dict(logstd_mode="per_policy", mean_mode="per_policy"),
    "offsets": dict(logstd_mode="offsets", mean_mode="offsets"),
}
SHAPES = {
    "C3": dict(T=64, B=1024, num_slots=2048),           # D = 6, the workload's own shape
    "C5": dict(T=128, B=256, num_slots=512),            # D = 17, full trajectory length, several tiles
    "C5-ragged": dict(T=37, B=36, num_slots=64),        # ragged tile and ragged first chunk
    "D3": dict(T=50, B=64, A=3, num_slots=128),
}


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_1912_00167_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()
    return torch, binding


def _workload(shape, recipe, **kw):
    base = workloads.C5 if shape.startswith("C5") else workloads.C3
    if shape == "D3":
        base = workloads.C5
    return shape_workload(base, **{**SHAPES[shape], **RECIPES[recipe], **kw})


@pytest.mark.parametrize("recipe", list(RECIPES))
@pytest.mark.parametrize("shape", list(SHAPES))
@pytest.mark.parametrize("flags", [0, 1], ids=["specialised", "generic"])
def test_time_major(env, shape, recipe, flags):
    torch, binding = env
    wl = _workload(shape, recipe, storage="f32")
    say(f"case gauss recipes time-major {shape} {recipe} flags={flags}")
    x = workloads.make_batch(wl, stream=70)
    got = gpu_loss(torch, binding, wl, x, flags=flags)
    check_against_oracle(wl, x, got, label=f"time-major {shape} {recipe} flags={flags}")


@pytest.mark.parametrize("recipe", list(RECIPES))
@pytest.mark.parametrize("shape", list(SHAPES))
@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_fused(env, shape, recipe, storage):
    torch, binding = env
    wl = _workload(shape, recipe, storage=storage)
    say(f"case gauss recipes fused {shape} {recipe} {storage}")
    for flags in (0, 1):
        _fused_case(torch, binding, wl, wl.num_slots, wl.B, flags, seed=71, label=f"fused {shape} {recipe} {storage} flags={flags}")


@pytest.mark.parametrize("recipe", list(RECIPES))
@pytest.mark.parametrize("shape", ["C3", "C5", "C5-ragged"])
@pytest.mark.parametrize("keep_target", [True, False], ids=["with_target", "no_target"])
def test_cached(env, shape, recipe, keep_target):
    torch, binding = env
    wl = _workload(shape, recipe, storage="bf16" if shape.startswith("C5") else "f32")
    h = wl.hyper if keep_target else replace(wl.hyper, kl_coeff=0.0)
    flags = binding.IMPACT_BUFFER_CACHE_LOGP | (0 if keep_target else binding.IMPACT_BUFFER_NO_TARGET_DIST)
    say(f"case gauss recipes cached {shape} {recipe} keep_target={keep_target}")
    n = wl.num_slots
    buf = binding.Buffer(wl.dist, wl.T, wl.A, n, wl.K, wl.storage, flags=flags)
    x = workloads.make_trajectories(wl, n, stream=72)
    binding.impact_buffer_insert(buf, to_device(x, torch))
    slots = np.ascontiguousarray(np.random.default_rng(7).permutation(n)[: wl.B].astype(np.int32))
    xb = workloads.take_trajectories(x, slots)
    learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
    cached = "with_target" if keep_target else "no_target"
    for flag_bits in (0, 1):
        out = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots).cuda(), learner, values, boot,
                                                      binding.config_from_hyper(h, flag_bits))
        torch.cuda.synchronize()
        check_against_oracle(wl, xb, {k: v.cpu().numpy() for k, v in out.items()}, hyper=h, cached=cached,
                             label=f"cached {shape} {recipe} flags={flag_bits}")
    buf.close()


@pytest.mark.parametrize("recipe", list(RECIPES))
@pytest.mark.parametrize("shape", ["C5", "C5-ragged"])
def test_learner_in_bf16(env, shape, recipe):
    torch, binding = env
    wl = _workload(shape, recipe, storage="bf16")
    say(f"case gauss recipes bf16 learner {shape} {recipe}")
    n = wl.num_slots
    buf = binding.Buffer(wl.dist, wl.T, wl.A, n, wl.K, "bf16")
    x = dict(workloads.make_trajectories(wl, n, stream=73))
    x["learner"] = oracle.quantize_bf16(x["learner"])[1]
    binding.impact_buffer_insert(buf, to_device(x, torch))
    slots = np.ascontiguousarray(np.random.default_rng(8).permutation(n)[: wl.B].astype(np.int32))
    xb = workloads.take_trajectories(x, slots)
    learner = torch.from_numpy(xb["learner"]).cuda().to(torch.bfloat16)
    values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("values", "bootstrap"))
    for flags in (0, 1):
        out = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots).cuda(), learner, values, boot,
                                                      binding.config_from_hyper(wl.hyper, flags))
        torch.cuda.synchronize()
        check_against_oracle(wl, xb, {k: v.cpu().numpy() for k, v in out.items()}, label=f"bf16 learner {shape} {recipe} flags={flags}")
    buf.close()


@pytest.mark.parametrize("recipe", ["all_per_policy", "offsets"])
def test_full_size_c5_time_major(env, recipe):
    """The largest workload's shape at full size on the two recipes that are not its default (which
    test_gpu_loss and test_gpu_buffer run at full size)."""
    torch, binding = env
    wl = replace(workloads.C5, **RECIPES[recipe])
    say(f"case gauss recipes full C5 {recipe}: generating")
    x = workloads.make_batch(wl, stream=74)
    d = to_device(x, torch)
    # through the storage dtype of the workload: a pre-gathered bf16 batch, as the buffer would hand it out
    for k in ("worker", "target", "rewards", "actions"):
        d[k] = d[k].to(torch.bfloat16)
    out = binding.impact_loss_fwd_bwd(wl.dist, d["learner"], d["values"], d["bootstrap"], d, binding.config_from_hyper(wl.hyper))
    torch.cuda.synchronize()
    say("  oracle")
    check_against_oracle(wl, x, {k: v.cpu().numpy() for k, v in out.items()}, label=f"C5 full {recipe}")
