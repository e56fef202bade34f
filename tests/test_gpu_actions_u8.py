"""GPU parity for buffers that keep the index of the action taken as one byte (a storage variant for
categorical policies with at most 256 actions): the buffer round trip bit for bit, and the loss read in
place from such a buffer, or from its gathered batch, against the oracle."""
import numpy as np
import pytest

import workloads
from gpu_common import check_against_oracle, say, shape_workload, to_device
from oracle.buffer import BufferOracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_1912_00167_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()
    return torch, binding


def _bytes_of(t, torch):
    return (t.view(torch.int16) if t.dtype == torch.bfloat16 else t).cpu().numpy().tobytes()


def _with_byte_actions(d, torch):
    d = dict(d)
    d["actions"] = d["actions"].to(torch.uint8)
    return d


@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_round_trip_bit_exact(env, storage):
    torch, binding = env
    wl = shape_workload(workloads.C1, T=13, A=5, num_slots=24, K=2, storage=storage)
    say(f"case byte actions round trip {storage}")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, storage, flags=binding.IMPACT_BUFFER_ACTIONS_U8)
    ob = BufferOracle(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, storage, actions_u8=True)
    rng = np.random.default_rng(3)
    for step in range(6):
        n = int(rng.integers(3, 9))
        if ob.num_empty() < n:
            binding.impact_buffer_release_discarded(buf)
            ob.release()
        if ob.num_empty() >= n:
            x = workloads.make_trajectories(wl, n, stream=step)
            slots = binding.impact_buffer_insert(buf, _with_byte_actions(to_device(x, torch), torch))
            assert slots.tolist() == ob.insert_records(x["worker"], x["actions"], x["rewards"], x["dones"], target=x["target"])
        Bn = int(rng.integers(1, ob.num_live() + 1))
        slots, counts = binding.impact_buffer_sample(buf, Bn)
        ws, wc = ob.sample(Bn)
        assert slots.tolist() == ws and counts.tolist() == wc
        got = binding.impact_buffer_gather(buf, torch.from_numpy(slots).cuda())
        torch.cuda.synchronize()
        want = ob.gather(ws)
        assert got["actions"].dtype == torch.uint8 and want["actions"].dtype == np.uint8
        for k in ("worker", "target", "actions", "rewards", "dones"):
            assert _bytes_of(got[k], torch) == want[k].tobytes(), f"{k} step {step}"
    with pytest.raises(TypeError):                     # the binding refuses int32 indices for such a buffer
        binding.impact_buffer_insert(buf, to_device(workloads.make_trajectories(wl, 1, stream=99), torch))
    buf.close()


# (name, shape, storage, buffer flags beyond ACTIONS_U8 as names)
CASES = [
    ("C2", dict(T=21, B=64, A=18, num_slots=128), "f32", ()),                 # A = 18: specialised, four wavefronts per tile
    ("C2", dict(T=50, B=10, A=18, num_slots=40), "f32", ()),                  # ragged tile; 50 bytes per slot, padded to 64
    ("C4", dict(T=23, B=1028, num_slots=2048), "bf16", ()),                   # ragged, bf16 ring
    ("C4", dict(T=100, B=8192, num_slots=8192), "f32", ()),                   # the benchmark's shape: three wavefronts per tile
    ("C4", dict(T=37, B=12288, num_slots=12288), "bf16", ()),                 # two wavefronts per tile
    ("C4", dict(T=19, B=16384, num_slots=16384), "bf16", ()),                 # single-wavefront tiles, rewards and indices preloaded
    ("C2", dict(T=400, B=24, A=18, num_slots=32), "f32", ()),                 # time segments (two launches)
    ("C4", dict(T=21, B=8192, num_slots=8192), "f32", ("CACHE_LOGP",)),
    ("C4", dict(T=30, B=256, num_slots=256), "bf16", ("CACHE_LOGP", "NO_TARGET_DIST")),
    ("C2", dict(T=37, B=21, A=7, num_slots=40), "f32", ()),                   # no specialised kernel: shape-generic
    ("C2", dict(T=9, B=64, A=6, num_slots=64), "bf16", ("CACHE_LOGP",)),      # shape-generic, cached
    ("C2", dict(T=5, B=16, A=256, num_slots=16), "f32", ()),                  # every byte value is a valid index
]


@pytest.mark.parametrize("ci", range(len(CASES)))
def test_loss_on_byte_actions(env, ci):
    torch, binding = env
    name, kw, storage, extra = CASES[ci]
    wl = shape_workload(workloads.WORKLOADS[name], storage=storage, **kw)
    keep_target = "NO_TARGET_DIST" not in extra
    cached = None if "CACHE_LOGP" not in extra else ("with_target" if keep_target else "no_target")
    h = wl.hyper if keep_target else shape_workload(wl.hyper, kl_coeff=0.0)
    flags = binding.IMPACT_BUFFER_ACTIONS_U8
    for f in extra:
        flags |= getattr(binding, "IMPACT_BUFFER_" + f)
    say(f"case byte actions {name} {kw} {storage} {extra}")
    n = wl.num_slots
    buf = binding.Buffer(wl.dist, wl.T, wl.A, n, wl.K, storage, flags=flags)
    x = workloads.make_trajectories(wl, n, stream=70 + ci)
    if wl.A == 256:
        x["actions"][0, :] = np.arange(wl.B, dtype=np.int32) * 17 % 256      # includes 255
        x["actions"][1, 0] = 255
    assert x["actions"].min() >= 0 and x["actions"].max() < wl.A
    slots_in = binding.impact_buffer_insert(buf, _with_byte_actions(to_device(x, torch), torch))
    assert slots_in.tolist() == list(range(n))
    slots, _ = binding.impact_buffer_sample(buf, wl.B)
    slots = np.ascontiguousarray(slots[np.random.default_rng(ci).permutation(wl.B)])
    xb = workloads.take_trajectories(x, slots)
    dev_slots = torch.from_numpy(slots).cuda()
    learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
    g = binding.impact_buffer_gather(buf, dev_slots)
    torch.cuda.synchronize()
    assert g["actions"].dtype == torch.uint8
    np.testing.assert_array_equal(g["actions"].cpu().numpy(), xb["actions"].astype(np.uint8))
    for flag_bits, tag in ((0, "specialised"), (binding.IMPACT_FLAG_FORCE_GENERIC, "generic")):
        cfg = binding.config_from_hyper(h, flag_bits)
        fused = binding.impact_loss_fwd_bwd_from_buffer(buf, dev_slots, learner, values, boot, cfg)
        torch.cuda.synchronize()
        check_against_oracle(wl, xb, {k: v.cpu().numpy() for k, v in fused.items()}, hyper=h, cached=cached,
                             label=f"byte actions fused {tag} {name} {kw}")
        # the gathered batch, whose indices are bytes as well
        cfg_tm = binding.config_from_hyper(h, flag_bits | binding.IMPACT_FLAG_ACTIONS_U8)
        unfused = binding.impact_loss_fwd_bwd(wl.dist, learner, values, boot, g, cfg_tm)
        torch.cuda.synchronize()
        check_against_oracle(wl, xb, {k: v.cpu().numpy() for k, v in unfused.items()}, hyper=h, cached=cached,
                             label=f"byte actions gathered {tag} {name} {kw}")
    buf.close()


def test_a_byte_index_out_of_range_is_flagged(env):
    torch, binding = env
    for A, Bn in ((18, 64), (7, 24)):
        wl = shape_workload(workloads.C2, T=12, B=Bn, A=A, num_slots=Bn)
        say(f"case byte actions out of range A={A}")
        buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, "f32", flags=binding.IMPACT_BUFFER_ACTIONS_U8)
        x = workloads.make_trajectories(wl, Bn, stream=5)
        d = _with_byte_actions(to_device(x, torch), torch)
        d["actions"][3, 5] = A            # one index past the last action
        binding.impact_buffer_insert(buf, d)
        slots, _ = binding.impact_buffer_sample(buf, Bn)
        xb = workloads.take_trajectories(x, slots)
        learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
        out = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots).cuda(), learner, values, boot,
                                                      binding.config_from_hyper(wl.hyper))
        torch.cuda.synchronize()
        assert np.isnan(out["loss5"].cpu().numpy()).all()
        assert np.isfinite(out["grad_dist"].cpu().numpy()).all()
        buf.close()


def test_the_flags_are_refused_where_they_make_no_sense(env):
    torch, binding = env
    with pytest.raises(binding.ImpactError):
        binding.Buffer("gaussian", 8, 3, 16, 1, "f32", flags=binding.IMPACT_BUFFER_ACTIONS_U8)
    with pytest.raises(binding.ImpactError):
        binding.Buffer("categorical", 8, 257, 16, 1, "f32", flags=binding.IMPACT_BUFFER_ACTIONS_U8)
    wl = shape_workload(workloads.C3, T=8, B=16, num_slots=16)
    x = workloads.make_trajectories(wl, 16, stream=1)
    d = to_device(x, torch)
    learner, values, boot = d["learner"], d["values"], d["bootstrap"]
    with pytest.raises(binding.ImpactError):           # a Gaussian policy's action is no index
        binding.impact_loss_fwd_bwd(wl.dist, learner, values, boot, d,
                                    binding.config_from_hyper(wl.hyper, binding.IMPACT_FLAG_ACTIONS_U8))
