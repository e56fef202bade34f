"""The CPU-side code under AddressSanitizer and UndefinedBehaviorSanitizer: the C oracle with its pins, and
the library's host logic (argument checks, ring bookkeeping, state export and import) with its CPU tests.
Each runs in a child process, because the sanitizer runtime has to be loaded before the interpreter starts."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_1912_00167_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True, check=True).stdout.strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        pytest.skip(f"{name} not found")
    return path


def _child_env(**extra):
    env = dict(os.environ)
    env["LD_PRELOAD"] = _runtime("libasan.so") + ":" + _runtime("libubsan.so")
    # the interpreter itself is not instrumented: its own allocations at exit are not ours to report
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra)
    return env


def _pytest_child(env, args):
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-s", "-p", "no:cacheprovider", "-m", "not gpu"] + args   # -s: a sanitizer report must reach our pipe, not pytest's capture file
    run = subprocess.run(cmd, env=env, cwd=ROOT, capture_output=True, text=True)
    tail = (run.stdout + run.stderr)[-3000:]
    assert run.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    return run.stdout


@pytest.mark.timeout(300)
def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    lib = str(tmp_path / "liboracle_san.so")
    subprocess.run(["gcc", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra"] + SAN +
                   ["-o", lib, os.path.join(ROOT, "oracle", "impact_oracle.c"), "-lm"], check=True)
    pins = ["test_oracle_policy.py", "test_oracle_vtrace.py", "test_oracle_surrogate.py", "test_oracle_gradients.py",
            "test_oracle_cached.py", "test_oracle_bf16.py", "test_oracle_impala.py", "test_oracle_ppo.py"]
    out = _pytest_child(_child_env(ORACLE_LIB_OVERRIDE=lib), [os.path.join(HERE, p) for p in pins])
    assert " passed" in out


# The launchers of the device code, which the host logic calls and a CPU-only build cannot link: no-ops here
# (no test without a GPU gets as far as a launch that matters).
STUBS = r"""
#include "impact_internal.h"
namespace impact {
bool launch_loss_cat_static(int, bool, LossArgs &, hipStream_t) { return true; }
bool launch_loss_gauss_static(int, bool, LossArgs &, hipStream_t) { return true; }
bool launch_loss_cat_cached(int, bool, LossArgs &, hipStream_t) { return true; }
bool launch_loss_gauss_cached(int, bool, LossArgs &, hipStream_t) { return true; }
void launch_loss_generic(int, int, bool, const LossArgs &, hipStream_t) {}
void launch_reduce(const ReduceArgs &, hipStream_t) {}
void launch_zero_words(unsigned *, int, hipStream_t) {}
void launch_insert_plane(PlaneKind, const PlaneCopyArgs &, hipStream_t) {}
void launch_gather_plane(const GatherArgs &, hipStream_t) {}
void launch_cache_logp(const LogpArgs &, hipStream_t) {}
unsigned *done_counter_of_stream(hipStream_t) { return nullptr; }
}
extern "C" impact_status_t impact_loss_fwd_bwd_static(int32_t, int32_t, int32_t, int32_t, int32_t, const void *, const float *,
                                                      const float *, const impact_batch_t *, const impact_loss_config_t *,
                                                      const impact_loss_out_t *, impact_stream_t) { return IMPACT_ERR_UNSUPPORTED; }
"""


@pytest.mark.timeout(300)
def test_host_logic_under_asan_and_ubsan(tmp_path):
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    if not os.path.exists(os.path.join(rocm, "include", "hip", "hip_runtime.h")):
        pytest.skip("no HIP headers")
    stubs = tmp_path / "stubs.cpp"
    stubs.write_text(STUBS)
    lib = str(tmp_path / "libimpact_host_san.so")
    subprocess.run(["g++", "-std=c++17", "-shared", "-fPIC", "-Wall", "-D__HIP_PLATFORM_AMD__"] + SAN +
                   ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", os.path.join(rocm, "include"),
                    "-o", lib, os.path.join(CSRC, "api.cpp"), str(stubs),
                    "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath," + os.path.join(rocm, "lib")], check=True)
    out = _pytest_child(_child_env(IMPACT_LIB_PATH=lib), [os.path.join(HERE, "test_abi_cpu.py")])
    assert " passed" in out
