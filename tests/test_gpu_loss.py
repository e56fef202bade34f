"""GPU parity of the loss kernels against the CPU oracle, through the C ABI."""
import math
from dataclasses import replace

import numpy as np
import pytest

import workloads
from gpu_common import check_against_oracle, gpu_loss, say, shape_workload, to_device, wide_range_inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_1912_00167_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()                       # fails loudly when libimpact.so is not built
    return torch, binding


FORCE_GENERIC = 1


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
@pytest.mark.parametrize("flags", [0, FORCE_GENERIC], ids=["specialised", "generic"])
def test_workloads_small(env, name, flags):
    torch, binding = env
    wl = replace(workloads.WORKLOADS[name], storage="f32")
    say(f"case {name} flags={flags} T={wl.T} B={wl.B} A={wl.A}")
    x = workloads.make_batch(wl, stream=0)
    got = gpu_loss(torch, binding, wl, x, flags=flags)
    check_against_oracle(wl, x, got, label=f"{name}/{'generic' if flags else 'specialised'}")


RAGGED = [
    ("categorical", 1, 1, 2), ("categorical", 33, 37, 5), ("categorical", 70, 9, 7), ("categorical", 31, 64, 33),
    ("categorical", 64, 8, 18), ("categorical", 45, 24, 18), ("categorical", 7, 16, 4), ("categorical", 100, 40, 9),
    ("gaussian", 1, 1, 1), ("gaussian", 33, 37, 2), ("gaussian", 65, 9, 5), ("gaussian", 40, 24, 17),
    ("gaussian", 96, 16, 3), ("gaussian", 50, 8, 6),
    # many actions / dimensions: no specialised kernel
    ("categorical", 6, 16, 300), ("gaussian", 5, 8, 40),
    ("categorical", 3, 4, 20000), ("gaussian", 2, 3, 5000),     # ... thousands of them
    # batches that end in a ragged tile of the specialised kernels (rows and ragged segment whole 16-byte vectors)
    ("categorical", 50, 10, 18), ("categorical", 21, 500, 18), ("categorical", 9, 4, 4), ("categorical", 30, 20, 6),
    ("gaussian", 40, 12, 6), ("gaussian", 19, 36, 17), ("gaussian", 5, 2, 6), ("gaussian", 70, 100, 3),
    # shortest trajectories on the specialised kernels (a single, ragged chunk)
    ("categorical", 1, 8, 6), ("categorical", 2, 16, 18), ("gaussian", 1, 8, 17), ("gaussian", 3, 8, 6), ("gaussian", 5, 16, 17),
]


@pytest.mark.parametrize("dist,T,Bn,A", RAGGED)
def test_ragged_and_odd_shapes(env, dist, T, Bn, A):
    torch, binding = env
    base = workloads.C2 if dist == "categorical" else workloads.C3
    wl = shape_workload(base, T=T, B=Bn, A=A, storage="f32")
    say(f"case ragged {dist} T={T} B={Bn} A={A}")
    x = workloads.make_batch(wl, stream=T * 1000 + Bn)
    got = gpu_loss(torch, binding, wl, x)
    check_against_oracle(wl, x, got, label=f"{dist} T{T} B{Bn} A{A}")


HYPERS = [
    dict(lam=0.995), dict(lam=0.9, gamma=0.9), dict(rho_clip=math.inf), dict(eps=math.inf),
    dict(kl_coeff=0.7, ent_coeff=0.05), dict(rho_bar=1.5, c_bar=0.7), dict(rho_bar=0.0), dict(c_bar=0.0),
    dict(vf_coeff=0.5, ent_coeff=0.0, kl_coeff=0.0), dict(eps=0.0), dict(rho_clip=1.0),
    dict(ratio_mode=1), dict(ratio_mode=1, kl_coeff=0.5, eps=0.1),      # the ablation's ratio pi_theta / pi_worker
    dict(gamma=0.0), dict(lam=0.0), dict(gamma=1.0, lam=1.0, rho_bar=3.0, c_bar=3.0),
]


@pytest.mark.parametrize("dist", ["categorical", "gaussian"])
@pytest.mark.parametrize("hi", range(len(HYPERS)))
def test_hyper_parameter_variants(env, dist, hi):
    torch, binding = env
    base = workloads.C4 if dist == "categorical" else workloads.C3
    wl = shape_workload(base, T=40, B=64, storage="f32")
    h = replace(wl.hyper, **HYPERS[hi])
    say(f"case hyper {dist} {HYPERS[hi]}")
    x = workloads.make_batch(wl, stream=50 + hi)
    for flags in (0, FORCE_GENERIC):
        got = gpu_loss(torch, binding, wl, x, hyper=h, flags=flags)
        check_against_oracle(wl, x, got, hyper=h, label=f"{dist} {HYPERS[hi]} flags={flags}")


@pytest.mark.parametrize("name", ["C2", "C3"])
@pytest.mark.parametrize("flags", [0, FORCE_GENERIC], ids=["specialised", "generic"])
def test_impala_objective_with_the_learner_in_the_targets_place(env, name, flags):
    """V-trace with learner-over-worker weights and the importance-sampled policy gradient (Section 2.3) come
    out of the same kernels when the learner's own distribution is handed over as the target's, with no ratio
    clipping and equal truncation levels."""
    torch, binding = env
    wl = shape_workload(workloads.WORKLOADS[name], B=64, num_slots=64)
    x = dict(workloads.make_trajectories(wl, 64, stream=17))
    x["target"] = x["learner"].copy()
    h = replace(wl.hyper, rho_clip=math.inf, eps=math.inf, rho_bar=1.3, c_bar=1.3, kl_coeff=0.0)
    say(f"case impala objective {name} flags={flags}")
    got = gpu_loss(torch, binding, wl, x, hyper=h, flags=flags)
    check_against_oracle(wl, x, got, hyper=h, label=f"impala objective {name}")


@pytest.mark.parametrize("name", ["C2", "C3"])
@pytest.mark.parametrize("flags", [0, FORCE_GENERIC], ids=["specialised", "generic"])
def test_ppo_with_gae_with_the_worker_in_the_targets_place(env, name, flags):
    """The on-policy baseline (Section 2.1's clipped surrogate on GAE(lambda) advantages) from the same kernels:
    with the worker's distribution handed over as the target's every weight of the scan is one and the ratio
    is pi_theta / pi_worker."""
    torch, binding = env
    wl = shape_workload(workloads.WORKLOADS[name], B=64, num_slots=64)
    x = dict(workloads.make_trajectories(wl, 64, stream=19))
    x["target"] = x["worker"].copy()
    h = replace(wl.hyper, lam=0.95, rho_bar=1.0, c_bar=1.0, eps=0.2, kl_coeff=0.0)
    say(f"case ppo+gae {name} flags={flags}")
    got = gpu_loss(torch, binding, wl, x, hyper=h, flags=flags)
    check_against_oracle(wl, x, got, hyper=h, label=f"ppo+gae {name}")


@pytest.mark.parametrize("name,kw", [("C1", {}), ("C3", dict(B=64)), ("C2", dict(T=50, B=10)), ("C2", dict(T=33, B=37, A=5)),
                                     ("C5", dict(T=40, B=2048))])
def test_per_step_scalars_as_packed_records(env, name, kw):
    """grad_values, vs and adv as one record {dL/dV, vs, adv, 0} per step: the same numbers, bit for bit, as in
    the three separate tensors, and the oracle's within tolerance."""
    torch, binding = env
    wl = shape_workload(workloads.WORKLOADS[name], storage="f32", **kw)
    x = workloads.make_batch(wl, stream=23)
    say(f"case packed records {name} {kw}")
    d = {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in x.items()}
    cfg = binding.config_from_hyper(wl.hyper)
    plain = binding.impact_loss_fwd_bwd(wl.dist, d["learner"], d["values"], d["bootstrap"], d, cfg)
    packed = binding.impact_loss_fwd_bwd(wl.dist, d["learner"], d["values"], d["bootstrap"], d, cfg,
                                         out=binding.alloc_loss_out(wl.T, wl.B, wl.W, packed=True))
    torch.cuda.synchronize()
    for k in ("grad_dist", "grad_values", "vs", "adv", "loss5"):
        assert torch.equal(plain[k], packed[k].contiguous()), k
    assert torch.all(packed["step_outputs"][..., 3] == 0)
    got = {k: packed[k].contiguous().cpu().numpy() for k in ("grad_dist", "grad_values", "vs", "adv", "loss5")}
    check_against_oracle(wl, x, got, label=f"packed records {name}")


LONG = [
    ("gaussian", 1024, 32, 6, {}), ("gaussian", 1024, 32, 17, dict(lam=0.97, c_bar=0.8)),      # the MuJoCo table's shape
    ("categorical", 600, 16, 18, {}), ("categorical", 333, 10, 18, dict(lam=0.9)),             # ragged tile as well
    ("gaussian", 257, 8, 3, dict(rho_bar=2.0, c_bar=1.5)), ("categorical", 2000, 64, 6, dict(ratio_mode=1)),
    ("categorical", 129, 8, 4, {}),
]


@pytest.mark.parametrize("dist,T,Bn,A,hyper", LONG)
@pytest.mark.parametrize("packed", [False, True], ids=["separate", "packed"])
def test_long_trajectories_of_a_small_batch(env, dist, T, Bn, A, hyper, packed):
    """Few tiles and many chunks: the time axis is cut into segments that run side by side, each started from
    the carry its successors compose to (the scan is affine in the carry).  Same results as ever."""
    torch, binding = env
    base = workloads.C2 if dist == "categorical" else workloads.C3
    wl = shape_workload(base, T=T, B=Bn, A=A, storage="f32")
    h = replace(wl.hyper, **hyper)
    x = workloads.make_batch(wl, stream=T + Bn)
    # some episode ends, so that the carry is cut inside segments and at their borders
    x["dones"][::97] = 1
    say(f"case long {dist} T={T} B={Bn} A={A} {hyper} packed={packed}")
    d = {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in x.items()}
    out = binding.impact_loss_fwd_bwd(wl.dist, d["learner"], d["values"], d["bootstrap"], d, binding.config_from_hyper(h),
                                      out=binding.alloc_loss_out(T, Bn, wl.W, packed=packed))
    torch.cuda.synchronize()
    got = {k: out[k].contiguous().cpu().numpy() for k in ("grad_dist", "grad_values", "vs", "adv", "loss5")}
    check_against_oracle(wl, x, got, hyper=h, label=f"long {dist} T{T} B{Bn} A{A}")


def test_optional_outputs_may_be_null(env):
    torch, binding = env
    wl = shape_workload(workloads.C2, B=16)
    x = workloads.make_batch(wl, stream=3)
    say("case null vs/adv")
    a = gpu_loss(torch, binding, wl, x, want_targets=True)
    b = gpu_loss(torch, binding, wl, x, want_targets=False)
    assert "vs" not in b
    for k in ("grad_dist", "grad_values", "loss5"):
        np.testing.assert_array_equal(a[k], b[k])      # same launch shape: bit-identical


def test_results_are_deterministic(env):
    torch, binding = env
    wl = shape_workload(workloads.C3, B=64)
    x = workloads.make_batch(wl, stream=4)
    say("case determinism")
    a = gpu_loss(torch, binding, wl, x)
    b = gpu_loss(torch, binding, wl, x)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])


def test_out_of_range_action_is_flagged_not_dereferenced(env):
    torch, binding = env
    wl = shape_workload(workloads.C1, B=8)
    x = workloads.make_batch(wl, stream=5)
    x["actions"][3, 2] = 99
    x["actions"][0, 0] = -4
    say("case bad action")
    for flags in (0, FORCE_GENERIC):
        got = gpu_loss(torch, binding, wl, x, flags=flags)
        assert np.all(np.isnan(got["loss5"]))
        assert np.all(np.isfinite(got["grad_dist"]))


@pytest.mark.parametrize("name", ["C4", "C5"])
def test_full_size_workloads_time_major(env, name):
    """The two large workloads at full size, every output element against the oracle."""
    torch, binding = env
    wl = replace(workloads.WORKLOADS[name], storage="f32")
    say(f"case full {name} T={wl.T} B={wl.B} A={wl.A}: generating")
    x = workloads.make_batch(wl, stream=0)
    say("  gpu")
    got = gpu_loss(torch, binding, wl, x)
    say("  oracle")
    check_against_oracle(wl, x, got, label=f"{name} full")


@pytest.mark.parametrize("dist", ["categorical", "gaussian"])
@pytest.mark.parametrize("flags", [0, FORCE_GENERIC], ids=["specialised", "generic"])
def test_wide_range_inputs(env, dist, flags):
    """Peaked and nearly flat policies far apart from each other: logits of magnitude up to 40 (softmax
    probabilities down to e^-80), standard deviations from e^-4 to e^1.5 with actions out to four of them, importance
    weights over many orders of magnitude (all truncated or clipped in the end).  The shifts and the fp64 parts of
    the kernels have to hold."""
    torch, binding = env
    base = workloads.C4 if dist == "categorical" else workloads.C5
    wl = shape_workload(base, T=24, B=64, storage="f32")
    x = wide_range_inputs(wl, workloads.make_batch(wl, stream=31), seed=9)
    say(f"case wide range {dist} flags={flags}")
    got = gpu_loss(torch, binding, wl, x, flags=flags)
    for k, v in got.items():
        assert np.all(np.isfinite(v)), k
    check_against_oracle(wl, x, got, label=f"wide range {dist}")


@pytest.mark.parametrize("dist", ["categorical", "gaussian"])
@pytest.mark.parametrize("pattern", ["every step", "none", "last step only", "first step only"])
def test_episode_end_patterns(env, dist, pattern):
    """The flag cuts the bootstrap and the carry at its own step: all steps terminal (every advantage is its own
    delta), none, and a single flag at either end of the trajectory, on both kernel families."""
    torch, binding = env
    base = workloads.C4 if dist == "categorical" else workloads.C5
    wl = shape_workload(base, T=37, B=24, storage="f32")
    x = dict(workloads.make_batch(wl, stream=41))
    d = np.zeros_like(x["dones"])
    if pattern == "every step":
        d[:] = 1
    elif pattern == "last step only":
        d[-1] = 1
    elif pattern == "first step only":
        d[0] = 1
    x["dones"] = d
    say(f"case episode ends {dist} {pattern}")
    for flags in (0, FORCE_GENERIC):
        got = gpu_loss(torch, binding, wl, x, flags=flags)
        check_against_oracle(wl, x, got, label=f"episode ends {pattern} {dist} flags={flags}")


@pytest.mark.parametrize("name,kw", [("C1", {}), ("C2", dict(T=50, B=40)), ("C3", dict(T=33, B=24)), ("C5", dict(T=40, B=21, storage="f32")),
                                     ("C4", dict(T=100, B=256))])
@pytest.mark.parametrize("packed", [False, True], ids=["separate", "packed"])
def test_batch_major_learner_tensors(env, name, kw, packed):
    """The learner's distribution, the values and every per-step output handed over trajectory by trajectory
    ([B][T][..], as a network that runs over whole trajectories produces them): the same numbers as time-major,
    element for element, and the oracle's within tolerance."""
    torch, binding = env
    wl = shape_workload(workloads.WORKLOADS[name], **{"storage": "f32", **kw})
    x = workloads.make_batch(wl, stream=29)
    say(f"case batch-major {name} {kw} packed={packed}")
    d = {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in x.items()}
    cfg_bm = binding.config_from_hyper(wl.hyper, binding.IMPACT_FLAG_BATCH_MAJOR)
    out = binding.impact_loss_fwd_bwd(wl.dist, d["learner"].transpose(0, 1).contiguous(), d["values"].t().contiguous(),
                                      d["bootstrap"], d, cfg_bm,
                                      out=binding.alloc_loss_out(wl.B, wl.T, wl.W, packed=packed))
    torch.cuda.synchronize()
    assert out["grad_dist"].shape == (wl.B, wl.T, wl.W) and out["vs"].shape == (wl.B, wl.T)
    got = {k: out[k].transpose(0, 1).contiguous().cpu().numpy() for k in ("grad_dist", "grad_values", "vs", "adv")}
    got.update(loss5=out["loss5"].cpu().numpy(), fractions=out["fractions"].cpu().numpy())
    check_against_oracle(wl, x, got, label=f"batch-major {name}")
    tm = gpu_loss(torch, binding, wl, x, flags=FORCE_GENERIC)          # the same kernels on time-major tensors
    for k in got:
        np.testing.assert_array_equal(got[k], tm[k], err_msg=k)


def test_calls_without_a_buffer_on_one_and_on_two_streams(env):
    """impact_loss_fwd_bwd takes its completion counter from the library's per-stream table: calls in a row on one
    stream, and calls that overlap on two streams (a workspace and outputs each), must give the same bits as a call
    on its own, every time."""
    torch, binding = env
    for name, kw in (("C2", dict(T=50, B=512)), ("C5", dict(T=40, B=2048, storage="f32")), ("C3", dict(T=700, B=24))):
        wl = shape_workload(workloads.WORKLOADS[name], **kw)
        say(f"case time-major calls on one and two streams {name} {kw}")
        xs = [workloads.make_batch(wl, stream=60 + i) for i in range(2)]
        ds = [to_device(x, torch) for x in xs]
        cfg = binding.config_from_hyper(wl.hyper)
        call = lambda d, out, ws, stream=None: binding.impact_loss_fwd_bwd(wl.dist, d["learner"], d["values"], d["bootstrap"], d, cfg,
                                                                          out=out, workspace=ws, stream=stream)
        nbytes = binding.impact_loss_workspace_bytes(wl.dist, wl.T, wl.B, wl.A)
        want = []
        for x, d in zip(xs, ds):
            out = call(d, binding.alloc_loss_out(wl.T, wl.B, wl.W), torch.empty(nbytes, dtype=torch.uint8, device="cuda"))
            torch.cuda.synchronize()
            check_against_oracle(wl, x, {k: v.cpu().numpy() for k, v in out.items()}, label=f"{name} alone")
            want.append({k: v.clone() for k, v in out.items()})
        # in a row on the current stream, alternating the two batches
        out, ws = binding.alloc_loss_out(wl.T, wl.B, wl.W), torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        for i in range(12):
            call(ds[i % 2], out, ws)
            if i % 5 == 4:
                torch.cuda.synchronize()
                for k in out:
                    assert torch.equal(out[k], want[i % 2][k]), (name, "in a row", i, k)
        torch.cuda.synchronize()
        # overlapping on two streams
        lanes = [dict(stream=torch.cuda.Stream(), out=binding.alloc_loss_out(wl.T, wl.B, wl.W),
                      ws=torch.empty(nbytes, dtype=torch.uint8, device="cuda")) for _ in range(2)]
        for rnd in range(6):
            for n, ln in enumerate(lanes):
                which = (rnd + n) % 2
                with torch.cuda.stream(ln["stream"]):
                    for v in ln["out"].values():
                        v.fill_(float("nan"))
                call(ds[which], ln["out"], ln["ws"], stream=ln["stream"])
            torch.cuda.synchronize()
            for n, ln in enumerate(lanes):
                for k in ln["out"]:
                    assert torch.equal(ln["out"][k], want[(rnd + n) % 2][k]), (name, "two streams", rnd, n, k)


def test_a_call_without_a_buffer_replays_in_a_captured_graph(env):
    """While its stream is being captured the call does not use the per-stream counter (a replay may run beside other
    work of that stream): it records its loss kernel and the small launch that sums the loss terms.  Every replay,
    with eager calls on the same stream in between, gives the eager result."""
    torch, binding = env
    wl = shape_workload(workloads.C2, T=50, B=256)
    say("case time-major call in a graph")
    x = workloads.make_batch(wl, stream=77)
    d = to_device(x, torch)
    cfg = binding.config_from_hyper(wl.hyper)
    out = binding.alloc_loss_out(wl.T, wl.B, wl.W)
    ws = torch.empty(binding.impact_loss_workspace_bytes(wl.dist, wl.T, wl.B, wl.A), dtype=torch.uint8, device="cuda")
    step = lambda: binding.impact_loss_fwd_bwd(wl.dist, d["learner"], d["values"], d["bootstrap"], d, cfg, out=out, workspace=ws)
    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    for rep in range(4):
        d["learner"].copy_(torch.from_numpy((x["learner"] + 0.1 * rep * rng.standard_normal(x["learner"].shape)).astype(np.float32)))
        step()                                           # eager, with the stream's counter
        torch.cuda.synchronize()
        eager = {k: v.clone() for k, v in out.items()}
        for v in out.values():
            v.fill_(float("nan"))
        junk = (torch.randn(1 << 16, device="cuda") * 2).sum()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(junk)
        for k in eager:
            assert torch.equal(out[k], eager[k]), (rep, k)
