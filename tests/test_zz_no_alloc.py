"""impact_loss_fwd_bwd_static (the entry point that allocates nothing: its workspace is a device array inside
the library) against impact_loss_fwd_bwd on the same inputs, through the C ABI; two calls in a row, the
second on a smaller batch, so that what the first left in the array is there when the second runs."""
import numpy as np
import pytest

import workloads
from gpu_common import check_against_oracle, say, shape_workload, to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_1912_00167_amd import binding
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    binding.load()
    return torch, binding


CASES = [
    # (workload, T, first batch, second batch)
    (workloads.C5, 128, 2048, 520),       # D = 17: 256 tiles, then 65
    (workloads.C2, 50, 1024, 136),        # categorical: 128 tiles, then 17
    (workloads.C3, 1024, 64, 24),         # long trajectories of a small batch: both calls run in time segments (their pairs
                                          # live in the workspace next to the partial sums)
]


@pytest.mark.parametrize("base,T,B1,B2", CASES, ids=lambda v: getattr(v, "name", str(v)))
def test_static_workspace_matches_caller_workspace(env, base, T, B1, B2):
    torch, binding = env
    for call, Bn in enumerate((B1, B2)):
        wl = shape_workload(base, T=T, B=Bn, storage="f32")
        x = workloads.make_trajectories(wl, Bn, stream=900 + call)
        d = to_device(x, torch)
        cfg = binding.config_from_hyper(wl.hyper)
        say(f"static workspace: {wl.name} T={T} B={Bn} (call {call + 1})")
        ref = binding.impact_loss_fwd_bwd(wl.dist, d["learner"], d["values"], d["bootstrap"], d, cfg)
        out = binding.alloc_loss_out(T, Bn, wl.W)
        for v in out.values():
            v.fill_(float("nan"))
        torch.cuda.synchronize()
        binding.impact_loss_fwd_bwd_static(wl.dist, d["learner"], d["values"], d["bootstrap"], d, cfg, out)
        torch.cuda.synchronize()
        got = {k: v.cpu().numpy() for k, v in out.items()}
        for k, v in ref.items():
            # the same kernels on the same inputs, only the workspace's address differs: identical results
            assert np.array_equal(got[k], v.cpu().numpy()), f"{k} differs (call {call + 1})"
        check_against_oracle(wl, x, got, label=f"static {wl.name} B={Bn}")


def test_static_workspace_limit_is_an_error(env):
    torch, binding = env
    # more tiles than the array holds partial sums for: refused before anything is enqueued (no tensor is touched)
    B_big = (binding.IMPACT_STATIC_WORKSPACE_BYTES // 32 + 1) * 8
    assert binding.impact_loss_workspace_bytes("categorical", 1, B_big, 2) > binding.IMPACT_STATIC_WORKSPACE_BYTES
    wl = shape_workload(workloads.C1, T=2, B=16)
    d = to_device(workloads.make_trajectories(wl, 16, stream=1), torch)
    out = binding.alloc_loss_out(2, 16, wl.W)
    lib = binding.load()
    import ctypes
    b, o = binding._batch_struct(d), binding._out_struct(out)
    cfg = binding.config_from_hyper(wl.hyper)
    rc = lib.impact_loss_fwd_bwd_static(0, 0, 1, B_big, 2, binding._ptr(d["learner"]), binding._ptr(d["values"]),
                                        binding._ptr(d["bootstrap"]), ctypes.byref(b), ctypes.byref(cfg), ctypes.byref(o), None)
    assert rc == binding.IMPACT_ERR_TOO_LARGE
    assert "static workspace" in binding.status_string(rc)
