"""GPU parity of the circular buffer (insert, put_target, gather: bit-exact) and of the loss
with the gather fused in, against the CPU oracles, through the C ABI."""
from dataclasses import replace

import numpy as np
import pytest

import workloads
from gpu_common import check_against_oracle, say, shape_workload, to_device, wide_range_inputs
from oracle.buffer import BufferOracle, bf16_bits_to_f32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_1912_00167_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()
    return torch, binding


def _bits(t, torch):
    """Raw bytes of a device tensor as a numpy array (bf16 -> uint16 patterns)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def _assert_same_bytes(a, b, what):
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    assert a.shape == b.shape and a.dtype.itemsize == b.dtype.itemsize, what
    assert a.tobytes() == b.tobytes(), what


def _fill(torch, binding, buf, ob, wl, n, stream, with_target=True):
    x = workloads.make_trajectories(wl, n, stream=stream)
    d = to_device(x, torch)
    src = {k: d[k] for k in ("worker", "actions", "rewards", "dones")}
    if with_target:
        src["target"] = d["target"]
    slots = binding.impact_buffer_insert(buf, src)
    want = ob.insert_records(x["worker"], x["actions"], x["rewards"], x["dones"],
                             target=x["target"] if with_target else None)
    assert slots.tolist() == want
    return x, slots


@pytest.mark.parametrize("dist", ["categorical", "gaussian"])
@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_insert_sample_gather_bit_exact(env, dist, storage):
    torch, binding = env
    base = workloads.C1 if dist == "categorical" else workloads.C3
    wl = shape_workload(base, T=13, A=5, num_slots=24, K=2, storage=storage)
    say(f"case buffer round trip {dist} {storage}")
    buf = binding.Buffer(dist, wl.T, wl.A, wl.num_slots, wl.K, storage)
    ob = BufferOracle(dist, wl.T, wl.A, wl.num_slots, wl.K, storage)
    _fill(torch, binding, buf, ob, wl, 10, 1)
    # target appended later for the next group (Algorithm 1: evaluate on target when k = 0)
    x2, slots2 = _fill(torch, binding, buf, ob, wl, 7, 2, with_target=False)
    binding.impact_buffer_put_target(buf, slots2, to_device({"t": x2["target"]}, torch)["t"])
    ob.put_target(slots2.tolist(), x2["target"])
    rng = np.random.default_rng(0)
    for step in range(12):
        Bn = int(rng.integers(1, 9))
        if binding.impact_buffer_num_live(buf) < Bn:
            binding.impact_buffer_release_discarded(buf)
            ob.release()
            assert binding.impact_buffer_num_empty(buf) == ob.num_empty()
            n = int(rng.integers(max(1, Bn - ob.num_live()), ob.num_empty() + 1))
            _fill(torch, binding, buf, ob, wl, n, 10 + step)      # lands in fragmented free slots
        slots, counts = binding.impact_buffer_sample(buf, Bn)
        ws, wc = ob.sample(Bn)
        assert slots.tolist() == ws and counts.tolist() == wc
        got = binding.impact_buffer_gather(buf, torch.from_numpy(slots).cuda())
        torch.cuda.synchronize()
        want = ob.gather(ws)
        for k in ("worker", "target", "actions", "rewards", "dones"):
            _assert_same_bytes(_bits(got[k], torch), want[k], f"{k} step {step}")
    buf.close()


def test_gather_long_records_and_ragged_tiles(env):
    """Records longer than the gather kernel's tile (element-wise copy) and shapes that leave partial tiles."""
    torch, binding = env
    for A, T, n, storage in ((700, 5, 11, "f32"), (33, 70, 19, "bf16"), (3, 257, 9, "bf16")):
        wl = shape_workload(workloads.C1, T=T, A=A, num_slots=24, K=1, storage=storage)
        say(f"case gather A={A} T={T} n={n} {storage}")
        buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, storage)
        ob = BufferOracle(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, storage)
        _fill(torch, binding, buf, ob, wl, 24, 4)
        perm = np.random.default_rng(A).permutation(24)[:n].astype(np.int32)
        got = binding.impact_buffer_gather(buf, torch.from_numpy(perm).cuda())
        torch.cuda.synchronize()
        want = ob.gather(perm.tolist())
        for k in ("worker", "target", "actions", "rewards", "dones"):
            _assert_same_bytes(_bits(got[k], torch), want[k], f"{k} A={A}")
        buf.close()


@pytest.mark.parametrize("case", [("categorical", 18, 64, "f32"), ("gaussian", 17, 128, "bf16"), ("gaussian", 6, 100, "f32")])
def test_gather_large_planes(env, case):
    """Planes of several MB take the tiled gather kernel (vector and word paths, ragged batch)."""
    torch, binding = env
    dist, A, T, storage = case
    base = workloads.C4 if dist == "categorical" else workloads.C5
    wl = shape_workload(base, T=T, A=A, num_slots=1200, K=1, storage=storage)
    say(f"case gather large {case}")
    buf = binding.Buffer(dist, T, A, wl.num_slots, wl.K, storage)
    ob = BufferOracle(dist, T, A, wl.num_slots, wl.K, storage)
    _fill(torch, binding, buf, ob, wl, 1200, 6)
    perm = np.random.default_rng(2).permutation(1200)[:1157].astype(np.int32)
    got = binding.impact_buffer_gather(buf, torch.from_numpy(perm).cuda())
    torch.cuda.synchronize()
    want = ob.gather(perm.tolist())
    for k in ("worker", "target", "actions", "rewards", "dones"):
        _assert_same_bytes(_bits(got[k], torch), want[k], k)
    buf.close()


def test_gather_full_ring_large(env):
    torch, binding = env
    wl = shape_workload(workloads.C2, B=512, num_slots=1024, K=1)
    say("case gather C2-sized")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, "f32")
    ob = BufferOracle(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, "f32")
    _fill(torch, binding, buf, ob, wl, 1024, 0)
    perm = np.random.default_rng(1).permutation(1024)[:512].astype(np.int32)
    got = binding.impact_buffer_gather(buf, torch.from_numpy(perm).cuda())
    torch.cuda.synchronize()
    want = ob.gather(perm.tolist())
    for k in ("worker", "target", "actions", "rewards", "dones"):
        _assert_same_bytes(_bits(got[k], torch), want[k], k)
    buf.close()


def _fused_case(torch, binding, wl, n_fill, Bn, flags, seed, label):
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    x = workloads.make_trajectories(wl, n_fill, stream=seed)
    d = to_device(x, torch)
    slots_in = binding.impact_buffer_insert(buf, d)
    assert slots_in.tolist() == list(range(n_fill))
    # take a non-trivial subset in a shuffled order so that slot != batch index
    slots, _ = binding.impact_buffer_sample(buf, Bn)
    order = np.random.default_rng(seed).permutation(Bn)
    slots = np.ascontiguousarray(slots[order])
    xb = workloads.take_trajectories(x, slots)              # the batch those slots hold, time-major
    dev_slots = torch.from_numpy(slots).cuda()
    learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
    cfg = binding.config_from_hyper(wl.hyper, flags)
    out = binding.impact_loss_fwd_bwd_from_buffer(buf, dev_slots, learner, values, boot, cfg)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in out.items()}
    check_against_oracle(replace(wl, B=Bn), xb, got, label=label)
    # the same call with the per-step scalars as packed records: the same bits
    packed = binding.impact_loss_fwd_bwd_from_buffer(buf, dev_slots, learner, values, boot, cfg,
                                                     out=binding.alloc_loss_out(wl.T, Bn, wl.W, packed=True))
    torch.cuda.synchronize()
    for k in ("vs", "adv", "grad_values", "grad_dist", "loss5"):
        np.testing.assert_array_equal(packed[k].contiguous().cpu().numpy(), got[k], err_msg=f"{label}: packed {k}")
    # The unfused route (gather, then the time-major loss) must agree with the fused one.  The two may run
    # different kernels (the fused specialised ones need 16-byte aligned trajectories in the planes), so the
    # comparison is to the parity tolerance, on gradients scaled by M like the comparison with the oracle.
    g = binding.impact_buffer_gather(buf, dev_slots)
    out2 = binding.impact_loss_fwd_bwd(wl.dist, learner, values, boot, g, cfg)
    torch.cuda.synchronize()
    M = wl.T * Bn
    for k in ("vs", "adv", "grad_values", "grad_dist", "loss5"):
        scale = M if k.startswith("grad") else 1
        np.testing.assert_allclose(got[k] * scale, out2[k].cpu().numpy() * scale, rtol=1e-5, atol=1e-6,
                                   err_msg=f"{label}: fused vs gather+loss {k}")
    buf.close()


FUSED = [
    ("C1", dict(), 64, 32), ("C2", dict(B=128, num_slots=256), 256, 128),
    ("C3", dict(B=128, num_slots=256), 256, 128),
    ("C5", dict(B=64, num_slots=128), 128, 64),                       # bf16 storage, D = 17
    ("C4", dict(B=64, num_slots=128, storage="bf16"), 128, 64),       # bf16 storage, categorical
    # trajectory lengths whose bytes per slot are no multiple of 16: the planes pad each slot
    ("C4", dict(T=50, B=64, num_slots=128, storage="bf16"), 128, 64),  # A = 18 bf16: 1800 bytes per slot
    ("C2", dict(T=7, B=64, A=9, num_slots=128), 128, 64),             # A = 9 fp32: 252 bytes; actions 28
    ("C3", dict(T=13, B=64, A=3, num_slots=128, storage="bf16"), 128, 64),   # D = 3 bf16: 156 and 78 bytes
    ("C5", dict(T=50, B=64, num_slots=128), 128, 64),                 # D = 17 bf16: 3400 and 1700 bytes
    ("C5", dict(T=33, B=64, num_slots=128, storage="f32"), 128, 64),  # D = 17 fp32: 4488 and 2244 bytes
    ("C2", dict(T=1000, B=64, A=6, num_slots=64), 64, 64),            # a long trajectory: 32 chunks and more
    # long trajectories of a small batch: time segments (two launches), fused
    ("C3", dict(T=1024, B=32, num_slots=64), 64, 32),
    ("C5", dict(T=700, B=20, num_slots=32), 32, 20),
    ("C2", dict(T=400, B=24, num_slots=32, storage="bf16"), 32, 24),
    # batches that end in a ragged tile of the specialised kernels
    ("C2", dict(T=50, B=10, num_slots=40), 40, 10),                   # fragments of 50 steps, 500 steps per batch
    ("C4", dict(T=23, B=1028, num_slots=2048, storage="bf16"), 2048, 1028),
    ("C5", dict(T=40, B=36, num_slots=64), 64, 36),
    ("C3", dict(T=64, B=2, num_slots=16), 16, 2),
    ("C2", dict(T=37, B=21, A=7, num_slots=40), 40, 21),              # generic kernels, ragged
    ("C5", dict(T=45, B=19, A=4, num_slots=32), 32, 19),              # generic kernels, bf16, ragged
]


@pytest.mark.parametrize("ci", range(len(FUSED)))
@pytest.mark.parametrize("flags", [0, 1], ids=["specialised", "generic"])
def test_loss_from_buffer(env, ci, flags):
    torch, binding = env
    name, kw, n_fill, Bn = FUSED[ci]
    wl = shape_workload(workloads.WORKLOADS[name], **kw)
    say(f"case fused {name} {kw} flags={flags}")
    _fused_case(torch, binding, wl, n_fill, Bn, flags, seed=ci, label=f"fused {name} {kw} flags={flags}")


@pytest.mark.parametrize("case", [("C5", dict(T=24, B=64, num_slots=128), "bf16"), ("C4", dict(T=21, B=64, num_slots=128), "bf16"),
                                  ("C2", dict(T=17, B=24, num_slots=64), "f32"), ("C5", dict(T=40, B=16384, num_slots=16384), "bf16"),
                                  ("C4", dict(T=30, B=8192, num_slots=8192), "bf16"), ("C3", dict(T=300, B=16, num_slots=32), "bf16")])
def test_learner_distribution_in_bf16(env, case):
    """The learner's distribution tensor as a network under mixed precision hands it over (bf16); gradients in
    fp32.  The oracle sees the same, already rounded, values."""
    import oracle
    torch, binding = env
    name, kw, storage = case
    wl = shape_workload(workloads.WORKLOADS[name], storage=storage, **kw)
    say(f"case bf16 learner {name} {kw} {storage}")
    n = wl.num_slots
    buf = binding.Buffer(wl.dist, wl.T, wl.A, n, wl.K, storage)
    x = dict(workloads.make_trajectories(wl, n, stream=61))
    x["learner"] = oracle.quantize_bf16(x["learner"])[1]
    binding.impact_buffer_insert(buf, to_device(x, torch))
    slots = np.random.default_rng(8).permutation(n)[: wl.B].astype(np.int32)
    xb = workloads.take_trajectories(x, slots)
    learner = torch.from_numpy(xb["learner"]).cuda().to(torch.bfloat16)
    assert torch.equal(learner.float().cpu(), torch.from_numpy(xb["learner"]))           # exactly the rounded values
    values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("values", "bootstrap"))
    for flags in (0, 1):
        out = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots).cuda(), learner, values, boot,
                                                      binding.config_from_hyper(wl.hyper, flags))
        torch.cuda.synchronize()
        check_against_oracle(wl, xb, {k: v.cpu().numpy() for k, v in out.items()}, label=f"bf16 learner {name} flags={flags}")
    buf.close()


def test_fused_calls_in_a_row_on_one_handle(env):
    """The last workgroup to finish sums the loss terms with a counter kept in the buffer's storage, which
    every call must leave at zero: calls of different sizes (many tiles, one tile, a ragged batch on the
    generic kernels) follow each other on one handle, each checked against the oracle."""
    torch, binding = env
    wl = shape_workload(workloads.C5, B=512, num_slots=1024)
    say("case fused calls in a row")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    x = workloads.make_trajectories(wl, 1024, stream=11)
    binding.impact_buffer_insert(buf, to_device(x, torch))
    cfg = binding.config_from_hyper(wl.hyper)
    rng = np.random.default_rng(5)
    for Bn in (512, 8, 264, 19, 512, 1024):
        slots = rng.permutation(1024)[:Bn].astype(np.int32)
        xb = workloads.take_trajectories(x, slots)
        learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
        out = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots).cuda(), learner, values, boot, cfg)
        torch.cuda.synchronize()
        check_against_oracle(replace(wl, B=Bn), xb, {k: v.cpu().numpy() for k, v in out.items()},
                             label=f"call with B={Bn}")
    buf.close()


def test_calls_of_different_lanes_run_side_by_side_on_two_streams(env):
    """Each lane has a completion counter of its own in the buffer's storage, so the steps of successive
    batches may alternate between two streams (one launch starts while the other drains).  The results
    are those of the same calls made one after the other: checked against the oracle once, then bit for bit."""
    torch, binding = env
    wl = shape_workload(workloads.C5, T=64, B=4096, num_slots=8192)
    say("case lanes on two streams")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    x = workloads.make_trajectories(wl, 2048, stream=12)
    d = to_device(x, torch)
    for _ in range(4):                              # the ring holds the 2048 trajectories four times over
        binding.impact_buffer_insert(buf, d)
    rng = np.random.default_rng(6)
    batches = []
    for q in range(4):
        slots = rng.permutation(8192)[: wl.B].astype(np.int32)
        xb = workloads.take_trajectories(x, slots % 2048)
        batches.append((torch.from_numpy(slots).cuda(), xb,
                        [torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap")]))
    cfg0 = binding.config_from_hyper(wl.hyper)
    serial = []
    for slots, xb, (learner, values, boot) in batches:
        out = binding.impact_loss_fwd_bwd_from_buffer(buf, slots, learner, values, boot, cfg0)
        torch.cuda.synchronize()
        serial.append({k: v.clone() for k, v in out.items()})
    check_against_oracle(wl, batches[0][1], {k: v.cpu().numpy() for k, v in serial[0].items()}, label="lane 0, alone")

    lanes = (3, 15)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    cfgs = [binding.config_from_hyper(wl.hyper, binding.IMPACT_FLAG_LANE(n)) for n in lanes]
    ws = [torch.empty(binding.impact_loss_workspace_bytes(wl.dist, wl.T, wl.B, wl.A), dtype=torch.uint8, device="cuda")
          for _ in lanes]
    outs = [binding.alloc_loss_out(wl.T, wl.B, wl.W) for _ in range(8)]
    torch.cuda.synchronize()
    for rnd in range(5):
        for i in range(8):                          # eight launches in flight over the two streams, then a look at each
            slots, _, (learner, values, boot) = batches[i % 4]
            binding.impact_loss_fwd_bwd_from_buffer(buf, slots, learner, values, boot, cfgs[i % 2], out=outs[i],
                                                    workspace=ws[i % 2], stream=streams[i % 2])
        torch.cuda.synchronize()
        for i in range(8):
            for k, v in serial[i % 4].items():
                assert torch.equal(outs[i][k], v), (rnd, i, k)
            outs[i]["loss5"].fill_(float("nan"))
        torch.cuda.synchronize()
    buf.close()


def test_fused_full_size_c5(env):
    """The headline configuration as the benchmark launches it: a full ring of 65536 bf16 slots, 16384
    sampled trajectories of 128 steps, D = 17; every output element against the oracle.  (The ring holds
    16384 distinct trajectories four times over, which keeps the host-side generation short.)"""
    torch, binding = env
    wl = workloads.C5
    distinct, block = 16384, 4096
    say(f"case fused full C5 T={wl.T} B={wl.B} A={wl.A} slots={wl.num_slots}: generating")
    parts = [workloads.make_trajectories(wl, block, stream=500 + i) for i in range(distinct // block)]
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    say("  filling the ring")
    for rnd in range(wl.num_slots // distinct):
        for i, part in enumerate(parts):
            slots_in = binding.impact_buffer_insert(buf, to_device(part, torch))
            assert int(slots_in[0]) == rnd * distinct + i * block
    x = {k: np.concatenate([p_[k] for p_ in parts], axis=0 if k == "bootstrap" else 1) for k in parts[0]}
    del parts
    # one traversal of the whole ring, then a shuffled quarter of it: the batch's slots lie scattered
    ring = np.concatenate([binding.impact_buffer_sample(buf, wl.B)[0].copy() for _ in range(wl.num_slots // wl.B)])
    assert sorted(ring.tolist()) == list(range(wl.num_slots))
    slots = np.ascontiguousarray(np.random.default_rng(5).permutation(ring)[: wl.B].astype(np.int32))
    xb = workloads.take_trajectories(x, slots % distinct)
    del x
    learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
    say("  gpu")
    out = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(np.ascontiguousarray(slots)).cuda(), learner, values,
                                                  boot, binding.config_from_hyper(wl.hyper))
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in out.items()}
    # the same batch as the benchmark's two-stream variant issues it: four launches over two lanes and two streams,
    # in flight together, each with the bits of the launch above
    say("  two lanes")
    dev_slots = torch.from_numpy(np.ascontiguousarray(slots)).cuda()
    lanes = [dict(stream=torch.cuda.Stream(), cfg=binding.config_from_hyper(wl.hyper, binding.IMPACT_FLAG_LANE(n + 1)),
                  ws=torch.empty(binding.impact_loss_workspace_bytes(wl.dist, wl.T, wl.B, wl.A), dtype=torch.uint8, device="cuda"),
                  outs=[binding.alloc_loss_out(wl.T, wl.B, wl.W) for _ in range(2)]) for n in range(2)]
    torch.cuda.synchronize()
    for i in range(4):
        ln = lanes[i % 2]
        binding.impact_loss_fwd_bwd_from_buffer(buf, dev_slots, learner, values, boot, ln["cfg"], out=ln["outs"][i // 2],
                                                workspace=ln["ws"], stream=ln["stream"])
    torch.cuda.synchronize()
    for ln in lanes:
        for o in ln["outs"]:
            for k in out:
                assert torch.equal(o[k], out[k]), k
    del lanes
    buf.close()
    say("  oracle")
    check_against_oracle(wl, xb, got, label="fused C5 full")


def test_fused_full_size_c4(env):
    """The large discrete workload as the benchmark launches it: fp32 ring of 32768 slots, 8192 sampled
    trajectories of 100 steps, 18 actions, the slots scattered over the ring; every output element against
    the oracle.  (This is the three-wavefronts-per-tile form of the fused categorical kernel.)"""
    torch, binding = env
    wl = workloads.C4
    distinct, block = 8192, 4096
    say(f"case fused full C4 T={wl.T} B={wl.B} A={wl.A} slots={wl.num_slots}: generating")
    parts = [workloads.make_trajectories(wl, block, stream=600 + i) for i in range(distinct // block)]
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    for rnd in range(wl.num_slots // distinct):
        for i, part in enumerate(parts):
            slots_in = binding.impact_buffer_insert(buf, to_device(part, torch))
            assert int(slots_in[0]) == rnd * distinct + i * block
    x = {k: np.concatenate([p_[k] for p_ in parts], axis=0 if k == "bootstrap" else 1) for k in parts[0]}
    del parts
    ring = np.concatenate([binding.impact_buffer_sample(buf, wl.B)[0].copy() for _ in range(wl.num_slots // wl.B)])
    assert sorted(ring.tolist()) == list(range(wl.num_slots))
    slots = np.ascontiguousarray(np.random.default_rng(6).permutation(ring)[: wl.B].astype(np.int32))
    xb = workloads.take_trajectories(x, slots % distinct)
    learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
    say("  gpu")
    out = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots).cuda(), learner, values, boot,
                                                  binding.config_from_hyper(wl.hyper))
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in out.items()}
    # a run of consecutive slots across the ring's end, in page-locked memory: what the benchmark's sampling
    # yields (the kernel is then given the first slot and reads no index array)
    run = ((wl.num_slots - 3000 + np.arange(wl.B)) % wl.num_slots).astype(np.int32)
    xr = workloads.take_trajectories(x, run % distinct)
    del x
    lr, vr, br = (torch.from_numpy(xr[k]).cuda() for k in ("learner", "values", "bootstrap"))
    out_r = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(run).pin_memory(), lr, vr, br,
                                                    binding.config_from_hyper(wl.hyper))
    torch.cuda.synchronize()
    got_r = {k: v.cpu().numpy() for k, v in out_r.items()}
    buf.close()
    say("  oracle")
    check_against_oracle(wl, xr, got_r, label="fused C4 full, consecutive slots")
    check_against_oracle(wl, xb, got, label="fused C4 full")


@pytest.mark.parametrize("case", [("C2", dict(T=22, A=6, B=16384, num_slots=16384), "f32"),
                                  ("C2", dict(T=24, A=18, B=16384, num_slots=16384), "bf16"),
                                  ("C2", dict(T=13, A=18, B=16384, num_slots=16384), "bf16"),
                                  ("C3", dict(T=50, A=6, B=16384, num_slots=16384), "bf16"),
                                  ("C4", dict(T=21, A=9, B=8192, num_slots=8192), "f32"),
                                  # longer than the single-wavefront tiles' preload arrays: two wavefronts per tile
                                  ("C3", dict(T=130, A=6, B=16384, num_slots=16384), "bf16")])
def test_fused_large_batch_short_ragged_trajectories(env, case):
    """Batches large enough for one- and two-wavefront tiles, with trajectory lengths that leave a ragged
    first chunk: every output element against the oracle, and the fused form against gather + loss."""
    torch, binding = env
    name, kw, storage = case
    wl = shape_workload(workloads.WORKLOADS[name], storage=storage, **kw)
    say(f"case fused large ragged {name} {kw} {storage}")
    _fused_case(torch, binding, wl, wl.num_slots, wl.B, 0, seed=9, label=f"fused large {name} {kw}")


def test_slot_indices_in_host_memory(env):
    """Page-locked host memory is read in place (same bits as a device copy); pageable memory is refused."""
    torch, binding = env
    wl = shape_workload(workloads.C3, B=64, num_slots=128)
    say("case slots in host memory")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    x = workloads.make_trajectories(wl, 128, stream=3)
    binding.impact_buffer_insert(buf, to_device(x, torch))
    slots = np.random.default_rng(1).permutation(128)[:64].astype(np.int32)
    xb = workloads.take_trajectories(x, slots)
    learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
    cfg = binding.config_from_hyper(wl.hyper)
    on_device = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots).cuda(), learner, values, boot, cfg)
    pinned = torch.from_numpy(slots).pin_memory()
    in_place = binding.impact_loss_fwd_bwd_from_buffer(buf, pinned, learner, values, boot, cfg)
    torch.cuda.synchronize()
    for k in on_device:
        np.testing.assert_array_equal(on_device[k].cpu().numpy(), in_place[k].cpu().numpy(), err_msg=k)
    with pytest.raises(binding.ImpactError):
        binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots.copy()), learner, values, boot, cfg)
    # A run of consecutive slots (the usual outcome of sampling in ring order), also across the ring's end:
    # seen in host memory, it is passed to the kernel as its first slot.  Same bits as with an index array.
    for first in (0, 37, 100):
        run = ((first + np.arange(64)) % 128).astype(np.int32)
        xr = workloads.take_trajectories(x, run)
        lr, vr, br = (torch.from_numpy(xr[k]).cuda() for k in ("learner", "values", "bootstrap"))
        as_array = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(run).cuda(), lr, vr, br, cfg)
        as_run = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(run).pin_memory(), lr, vr, br, cfg)
        torch.cuda.synchronize()
        for k in as_array:
            np.testing.assert_array_equal(as_array[k].cpu().numpy(), as_run[k].cpu().numpy(), err_msg=f"{first} {k}")
        check_against_oracle(wl, xr, {k: v.cpu().numpy() for k, v in as_run.items()}, label=f"run from slot {first}")
    buf.close()


def test_fused_step_replays_in_a_captured_graph(env):
    """A launch-bound learner loop can capture the step once and replay it: the call records nothing but its
    kernel launch.  Every replay, with eager work and new inputs in between, must give the eager result."""
    torch, binding = env
    wl = shape_workload(workloads.C3, B=64, num_slots=128)
    say("case fused step in a graph")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    x = workloads.make_trajectories(wl, 128, stream=21)
    binding.impact_buffer_insert(buf, to_device(x, torch))
    slots_np = np.random.default_rng(2).permutation(128)[:64].astype(np.int32)
    dev_slots = torch.from_numpy(slots_np).cuda()
    xb = workloads.take_trajectories(x, slots_np)
    learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
    cfg = binding.config_from_hyper(wl.hyper)
    out = binding.alloc_loss_out(wl.T, 64, wl.W)
    ws = torch.empty(binding.impact_loss_workspace_bytes(wl.dist, wl.T, 64, wl.A), dtype=torch.uint8, device="cuda")
    step = lambda: binding.impact_loss_fwd_bwd_from_buffer(buf, dev_slots, learner, values, boot, cfg, out=out, workspace=ws)
    step()                                               # the handle's first call (it clears the counter)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    rng = np.random.default_rng(4)
    for rep in range(4):
        # new inputs in the captured tensors, the eager result for them, then unrelated eager work
        learner.copy_(torch.from_numpy((xb["learner"] + 0.1 * rep * rng.standard_normal(xb["learner"].shape)).astype(np.float32)))
        dev_slots.copy_(torch.from_numpy(np.roll(slots_np, rep)))
        step()
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
    buf.close()


def test_a_lane_first_used_inside_a_graph_capture(env):
    """The first call of a lane clears its completion counter; a call that is only recorded into a graph has
    cleared nothing yet.  The buffer's storage starts out as garbage here, the first call ever made on the
    handle is a captured one, and both the replays and the eager calls that follow have to be right."""
    torch, binding = env
    wl = shape_workload(workloads.C3, B=64, num_slots=128)
    say("case lane first used under capture")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    buf.storage[-256:] = 0x5A                            # the block of completion counters at the end of the storage
    x = workloads.make_trajectories(wl, 128, stream=22)
    binding.impact_buffer_insert(buf, to_device(x, torch))
    slots_np = np.random.default_rng(3).permutation(128)[:64].astype(np.int32)
    dev_slots = torch.from_numpy(slots_np).cuda()
    xb = workloads.take_trajectories(x, slots_np)
    learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
    out = binding.alloc_loss_out(wl.T, 64, wl.W)
    ws = torch.empty(binding.impact_loss_workspace_bytes(wl.dist, wl.T, 64, wl.A), dtype=torch.uint8, device="cuda")
    call = lambda lane: binding.impact_loss_fwd_bwd_from_buffer(
        buf, dev_slots, learner, values, boot, binding.config_from_hyper(wl.hyper, binding.IMPACT_FLAG_LANE(lane)), out=out, workspace=ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(5)
    torch.cuda.synchronize()

    def result(run):
        for v in out.values():
            v.fill_(float("nan"))
        run()
        torch.cuda.synchronize()
        return {k: v.clone() for k, v in out.items()}
    first = result(graph.replay)
    check_against_oracle(replace(wl, B=64), xb, {k: v.cpu().numpy() for k, v in first.items()}, label="first replay")
    for run in (lambda: call(0), lambda: call(5), graph.replay, lambda: call(5), graph.replay):
        again = result(run)
        for k in first:
            assert torch.equal(again[k], first[k]), k
    buf.close()


@pytest.mark.parametrize("name,storage", [("C4", "f32"), ("C4", "bf16"), ("C5", "bf16"), ("C5", "f32")])
@pytest.mark.parametrize("cached", [False, True], ids=["full", "cached"])
def test_fused_wide_range_inputs(env, name, storage, cached):
    """Peaked and nearly flat policies, ratios over fifty orders of magnitude, through the ring (rounded to bf16
    where it stores bf16) and, with cached log-probabilities, through the stored fp64 pair."""
    torch, binding = env
    wl = shape_workload(workloads.WORKLOADS[name], T=24, B=64, num_slots=64, storage=storage)
    x = wide_range_inputs(wl, workloads.make_trajectories(wl, 64, stream=33), seed=10)
    say(f"case fused wide range {name} {storage} cached={cached}")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, 64, wl.K, storage, flags=binding.IMPACT_BUFFER_CACHE_LOGP if cached else 0)
    binding.impact_buffer_insert(buf, to_device(x, torch))
    slots = np.random.default_rng(3).permutation(64).astype(np.int32)
    xb = workloads.take_trajectories(x, slots)
    learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
    for flag_bits in (0, 1):
        out = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots).cuda(), learner, values, boot,
                                                      binding.config_from_hyper(wl.hyper, flag_bits))
        torch.cuda.synchronize()
        got = {k: v.cpu().numpy() for k, v in out.items()}
        for k, v in got.items():
            assert np.all(np.isfinite(v)), k
        check_against_oracle(wl, xb, got, cached="with_target" if cached else None, label=f"fused wide range {name} {storage}")
    buf.close()


def test_out_of_range_slot_is_flagged_not_dereferenced(env):
    torch, binding = env
    wl = shape_workload(workloads.C1, num_slots=16)
    say("case bad slot")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, "f32")
    x = workloads.make_trajectories(wl, 16, stream=0)
    binding.impact_buffer_insert(buf, to_device(x, torch))
    slots = np.arange(8, dtype=np.int32)
    slots[3] = 1_000_000
    slots[5] = -2
    xb = workloads.take_trajectories(x, np.clip(slots, 0, 15))
    learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
    for flags in (0, 1):
        out = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots).cuda(), learner, values, boot,
                                                      binding.config_from_hyper(wl.hyper, flags))
        torch.cuda.synchronize()
        assert torch.isnan(out["loss5"]).all()
        assert torch.isfinite(out["grad_dist"]).all()
    g = binding.impact_buffer_gather(buf, torch.from_numpy(slots).cuda())
    torch.cuda.synchronize()
    assert torch.isfinite(g["worker"]).all()
    buf.close()


def test_errors_from_the_device_side_calls(env):
    torch, binding = env
    buf = binding.Buffer("categorical", 4, 3, 4, 1, "f32")
    wl = shape_workload(workloads.C1, T=4, A=3, num_slots=4)
    x = to_device(workloads.make_trajectories(wl, 3, stream=0), torch)
    say("case device-side errors")
    binding.impact_buffer_insert(buf, x)
    with pytest.raises(binding.ImpactError) as e:
        binding.impact_buffer_insert(buf, x)                 # 3 more do not fit in 1 free slot
    assert e.value.status == binding.IMPACT_ERR_BUFFER_FULL
    assert binding.impact_buffer_num_live(buf) == 3
    with pytest.raises(binding.ImpactError) as e:
        binding.impact_buffer_sample(buf, 4)
    assert e.value.status == binding.IMPACT_ERR_NOT_ENOUGH_LIVE
    slots, counts = binding.impact_buffer_sample(buf, 3)
    assert slots.tolist() == [0, 1, 2] and counts.tolist() == [0, 0, 0]
    assert binding.impact_buffer_num_live(buf) == 0          # K = 1: discarded after one traversal
    buf.close()


def test_learner_loop_of_algorithm_1_through_the_library(env):
    """Algorithm 1's learner loop with the library keeping its books: workers insert batches without the
    target's output; the learner samples, asks which trajectories still lack the target's output (those handed
    out for the first time), appends it, computes loss and gradients, releases what was handed out for the K-th
    time, counts the step and is told when the target update is due (every N K steps, Section 4.1.1).  Every
    step's results against the oracle; the bookkeeping against the oracle's ring."""
    torch, binding = env
    wl = shape_workload(workloads.C3, T=16, B=16, num_slots=48, K=2)
    say("case learner loop")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    ob = BufferOracle(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    period = binding.impact_target_period(wl.num_slots, wl.B, wl.K)
    assert period == 6
    held = {}                                        # slot -> index of its trajectory in `pool`
    pool, n_pool, n_blocks = None, 0, 0
    cfg = binding.config_from_hyper(wl.hyper)
    syncs = []
    for step in range(1, 15):
        while binding.impact_buffer_num_empty(buf) >= wl.B:          # the workers send what fits
            x = workloads.make_trajectories(wl, wl.B, stream=300 + n_blocks)
            d = to_device(x, torch)
            slots_in = binding.impact_buffer_insert(buf, {k: d[k] for k in ("worker", "actions", "rewards", "dones")})
            assert slots_in.tolist() == ob.insert_records(x["worker"], x["actions"], x["rewards"], x["dones"])
            for i, s in enumerate(slots_in):
                held[int(s)] = n_pool + i
            pool = x if pool is None else {k: np.concatenate([pool[k], x[k]], axis=0 if x[k].ndim == 1 else 1) for k in x}
            n_pool += wl.B
            n_blocks += 1
        slots, counts = binding.impact_buffer_sample(buf, wl.B)
        ws, wc = ob.sample(wl.B)
        assert slots.tolist() == ws and counts.tolist() == wc
        xb = workloads.take_trajectories(pool, np.asarray([held[int(s)] for s in slots]))
        need = binding.impact_buffer_missing_targets(buf, slots)
        assert need.tolist() == ob.missing_targets(ws) == [i for i, k in enumerate(wc) if k == 0]
        if len(need):                                                # "if k = 0, evaluate B on target, append"
            tgt = np.ascontiguousarray(xb["target"][:, need])
            binding.impact_buffer_put_target(buf, slots[need], torch.from_numpy(tgt).cuda())
            ob.put_target([ws[i] for i in need], tgt)
        assert len(binding.impact_buffer_missing_targets(buf, slots)) == 0
        learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
        out = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots).cuda(), learner, values, boot, cfg)
        # a full ring cannot take the workers' next batch before the loss above has been enqueued and the discards released
        if binding.impact_buffer_num_empty(buf) < wl.B and binding.impact_buffer_num_live(buf) + wl.B <= wl.num_slots:
            with pytest.raises(binding.ImpactError) as e:
                binding.impact_buffer_reserve(buf, wl.num_slots - binding.impact_buffer_num_live(buf))
            assert e.value.status == binding.IMPACT_ERR_BUFFER_FULL
        binding.impact_buffer_release_discarded(buf)                 # "if k = K, discard"
        ob.release()
        t, due = binding.impact_buffer_learner_step(buf, period)     # "if t = 0 (mod t_target), update target"
        assert t == step and due == ob.learner_step(period) == (step % period == 0)
        syncs.append(due)
        torch.cuda.synchronize()
        check_against_oracle(wl, xb, {k: v.cpu().numpy() for k, v in out.items()}, label=f"learner loop step {step}")
        assert binding.impact_buffer_num_live(buf) == ob.num_live() and binding.impact_buffer_num_empty(buf) == ob.num_empty()
    assert syncs.count(True) == 2
    buf.close()


def test_records_of_the_last_traversal_survive_until_their_loss(env):
    """A slot handed out for the K-th time stays out of the workers' reach until it is released: an insert
    issued between that sample and the loss finds the ring full instead of overwriting what the loss reads."""
    torch, binding = env
    wl = shape_workload(workloads.C2, T=20, B=32, num_slots=32, K=1)
    say("case last traversal, then insert, then loss")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    x = workloads.make_trajectories(wl, 32, stream=90)
    y = workloads.make_trajectories(wl, 32, stream=91)
    binding.impact_buffer_insert(buf, to_device(x, torch))
    slots, counts = binding.impact_buffer_sample(buf, 32)              # K = 1: this is every slot's last traversal
    assert binding.impact_buffer_num_live(buf) == 0 and binding.impact_buffer_num_empty(buf) == 0
    with pytest.raises(binding.ImpactError) as e:
        binding.impact_buffer_insert(buf, to_device(y, torch))          # the workers' next batch: not yet
    assert e.value.status == binding.IMPACT_ERR_BUFFER_FULL
    cfg = binding.config_from_hyper(wl.hyper)
    dev = to_device(x, torch)
    out = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots).cuda(), dev["learner"], dev["values"],
                                                  dev["bootstrap"], cfg)
    binding.impact_buffer_release_discarded(buf)
    binding.impact_buffer_insert(buf, to_device(y, torch))              # same stream: ordered after the loss
    torch.cuda.synchronize()
    check_against_oracle(wl, x, {k: v.cpu().numpy() for k, v in out.items()}, label="loss of the last traversal")
    slots2, _ = binding.impact_buffer_sample(buf, 32)
    devy = to_device(y, torch)
    out2 = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots2).cuda(), devy["learner"], devy["values"],
                                                   devy["bootstrap"], cfg)
    torch.cuda.synchronize()
    check_against_oracle(wl, y, {k: v.cpu().numpy() for k, v in out2.items()}, label="loss of the batch that replaced it")
    buf.close()


def test_an_invalid_fused_call_enqueues_nothing_and_a_valid_one_follows(env):
    """Arguments are checked before the completion counter is cleared or anything else touches the stream; a
    counter left non-zero by a failed launch is recovered with impact_buffer_reset_lanes."""
    torch, binding = env
    wl = shape_workload(workloads.C3, B=64, num_slots=64)
    say("case invalid fused call, then valid")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    buf.storage[-256:] = 0x5A                            # garbage in the block of completion counters
    x = workloads.make_trajectories(wl, 64, stream=92)
    binding.impact_buffer_insert(buf, to_device(x, torch))
    slots, _ = binding.impact_buffer_sample(buf, 64)
    dev = to_device(x, torch)
    args = (buf, torch.from_numpy(slots).cuda(), dev["learner"], dev["values"], dev["bootstrap"])
    with pytest.raises(binding.ImpactError) as e:
        binding.impact_loss_fwd_bwd_from_buffer(*args, binding.make_config(gamma=float("nan")))
    assert e.value.status == binding.IMPACT_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert int(buf.storage[-256:].min()) == 0x5A and int(buf.storage[-256:].max()) == 0x5A     # nothing ran on the storage
    cfg = binding.config_from_hyper(wl.hyper)
    out = binding.impact_loss_fwd_bwd_from_buffer(*args, cfg)
    torch.cuda.synchronize()
    check_against_oracle(wl, x, {k: v.cpu().numpy() for k, v in out.items()}, label="valid call after an invalid one")
    # a counter that a launch left behind non-zero (planted here from the host) makes the next launch skip the final
    # sum; after impact_buffer_reset_lanes the lane is cleared again before its next launch
    buf.storage[-256:-252] = 1
    binding.impact_buffer_reset_lanes(buf)
    out["loss5"].fill_(float("nan"))
    out2 = binding.impact_loss_fwd_bwd_from_buffer(*args, cfg, out=out)
    torch.cuda.synchronize()
    check_against_oracle(wl, x, {k: v.cpu().numpy() for k, v in out2.items()}, label="after reset_lanes")
    buf.close()


@pytest.mark.parametrize("name,kw", [("C2", dict(T=50, B=64, num_slots=128)), ("C5", dict(T=64, B=40, num_slots=64))])
def test_batch_major_learner_tensors_with_the_gather_fused(env, name, kw):
    """Slot-major buffer fields and batch-major learner tensors: every tensor of the call is then laid out
    trajectory by trajectory."""
    torch, binding = env
    wl = shape_workload(workloads.WORKLOADS[name], **kw)
    say(f"case batch-major fused {name} {kw}")
    buf = binding.Buffer(wl.dist, wl.T, wl.A, wl.num_slots, wl.K, wl.storage)
    x = workloads.make_trajectories(wl, wl.num_slots, stream=93)
    binding.impact_buffer_insert(buf, to_device(x, torch))
    slots = np.ascontiguousarray(np.random.default_rng(9).permutation(wl.num_slots)[: wl.B].astype(np.int32))
    xb = workloads.take_trajectories(x, slots)
    learner, values, boot = (torch.from_numpy(xb[k]).cuda() for k in ("learner", "values", "bootstrap"))
    out = binding.impact_loss_fwd_bwd_from_buffer(buf, torch.from_numpy(slots).cuda(), learner.transpose(0, 1).contiguous(),
                                                  values.t().contiguous(), boot,
                                                  binding.config_from_hyper(wl.hyper, binding.IMPACT_FLAG_BATCH_MAJOR))
    torch.cuda.synchronize()
    got = {k: out[k].transpose(0, 1).contiguous().cpu().numpy() for k in ("grad_dist", "grad_values", "vs", "adv")}
    got.update(loss5=out["loss5"].cpu().numpy(), fractions=out["fractions"].cpu().numpy())
    check_against_oracle(wl, xb, got, label=f"batch-major fused {name}")
    buf.close()
