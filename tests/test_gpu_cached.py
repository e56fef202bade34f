"""GPU parity for buffers that keep log pi_worker(a) and log pi_target(a) per step in place of the worker's
distribution (and optionally of the target's): the stored numbers, and the loss computed from them, against
the oracle's cached path."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_common import check_against_oracle, oracle_inputs, say, shape_workload, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_1912_00167_amd import binding
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.load()
    return torch, binding


CASES = [
    ("C1", dict(num_slots=64), "f32"), ("C2", dict(T=21, B=64, num_slots=128), "bf16"),
    ("C3", dict(T=17, B=64, num_slots=128), "f32"), ("C5", dict(T=24, B=64, num_slots=128), "bf16"),
    ("C2", dict(T=9, B=21, A=7, num_slots=40), "f32"),                     # ragged batch, generic kernels
    ("C2", dict(T=50, B=10, num_slots=40), "f32"), ("C5", dict(T=30, B=20, num_slots=64), "bf16"),   # ragged tile
    ("C3", dict(T=512, B=16, num_slots=32), "f32"), ("C2", dict(T=300, B=10, num_slots=32), "bf16"), # time segments
    # batches large enough for single-wavefront tiles (2048 of them) and for two wavefronts per tile
    ("C5", dict(T=22, B=16384, num_slots=16384), "bf16"), ("C4", dict(T=21, B=8192, num_slots=8192), "f32"),
    ("C3", dict(T=13, B=16384, num_slots=16384), "f32"), ("C4", dict(T=50, A=9, B=16384, num_slots=16384), "bf16"),
]


@pytest.mark.parametrize("ci", range(len(CASES)))
@pytest.mark.parametrize("keep_target", [True, False], ids=["with_target", "no_target"])
def test_cached_buffer_stores_the_log_probabilities_and_the_loss_uses_them(env, ci, keep_target):
    torch, binding = env
    name, kw, storage = CASES[ci]
    wl = shape_workload(workloads.WORKLOADS[name], storage=storage, **kw)
    h = wl.hyper if keep_target else shape_workload(wl.hyper, kl_coeff=0.0)
    flags = binding.IMPACT_BUFFER_CACHE_LOGP | (0 if keep_target else binding.IMPACT_BUFFER_NO_TARGET_DIST)
    say(f"case cached {name} {kw} {storage} keep_target={keep_target}")
    n = wl.num_slots
    buf = binding.Buffer(wl.dist, wl.T, wl.A, n, wl.K, storage, flags=flags)
    x = workloads.make_trajectories(wl, n, stream=40 + ci)
    d = to_device(x, torch)
    half = n // 2
    # first half with the target's outputs at hand, second half appended later (k = 0 in Algorithm 1)
    first = {k: v[:, :half].contiguous() if v.dim() > 1 else v[:half].contiguous() for k, v in d.items()}
    second = {k: v[:, half:].contiguous() if v.dim() > 1 else v[half:].contiguous() for k, v in d.items() if k != "target"}
    s1 = binding.impact_buffer_insert(buf, first)
    s2 = binding.impact_buffer_insert(buf, second)
    binding.impact_buffer_put_target(buf, s2, d["target"][:, half:].contiguous())
    assert list(s1) + list(s2) == list(range(n))

    slots, _ = binding.impact_buffer_sample(buf, wl.B)
    slots = np.ascontiguousarray(slots[np.random.default_rng(ci).permutation(wl.B)])
    xb = workloads.take_trajectories(x, slots)
    dev_slots = torch.from_numpy(slots).cuda()

    # the stored pair, through gather
    g = binding.impact_buffer_gather(buf, dev_slots)
    torch.cuda.synchronize()
    assert "worker" not in g and ("target" in g) == keep_target
    stored_actions = oracle_inputs(xb, storage)["actions"]
    want_lp = oracle.behaviour_logp(wl.dist, xb["target"], xb["worker"], stored_actions)
    np.testing.assert_allclose(g["logp"].cpu().numpy(), want_lp, rtol=1e-12, atol=1e-12)

    learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
    cached = "with_target" if keep_target else "no_target"
    for flag_bits, tag in ((0, "specialised"), (1, "generic")):
        cfg = binding.config_from_hyper(h, flag_bits)
        fused = binding.impact_loss_fwd_bwd_from_buffer(buf, dev_slots, learner, values, boot, cfg)
        torch.cuda.synchronize()
        check_against_oracle(wl, xb, {k: v.cpu().numpy() for k, v in fused.items()}, hyper=h, cached=cached,
                             label=f"cached fused {tag} {name}")
        unfused = binding.impact_loss_fwd_bwd(wl.dist, learner, values, boot, g, cfg)
        torch.cuda.synchronize()
        check_against_oracle(wl, xb, {k: v.cpu().numpy() for k, v in unfused.items()}, hyper=h, cached=cached,
                             label=f"cached gathered {tag} {name}")
    if not keep_target:
        with pytest.raises(binding.ImpactError):          # a KL term needs the target's distribution
            binding.impact_loss_fwd_bwd_from_buffer(buf, dev_slots, learner, values, boot,
                                                    binding.config_from_hyper(shape_workload(h, kl_coeff=0.5)))
    buf.close()
