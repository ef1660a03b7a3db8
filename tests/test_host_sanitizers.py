"""The library's host code under the host sanitizers: tests/host/plan_stress.cpp drives a
plan-only pool (no HIP call, no GPU) from several threads through the C ABI - swaps, reuse
map, eviction, both allocators, swap manager - and is built once with AddressSanitizer +
UndefinedBehaviorSanitizer and once with ThreadSanitizer (host pass only; device code is
compiled as usual)."""

import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2411_18424_amd", "csrc")
SOURCES = [os.path.join(ROOT, "tests", "host", "plan_stress.cpp")] + [
    os.path.join(CSRC, f) for f in ("kv_kernels.hip", "kv_engine.cpp", "kv_reuse.cpp", "kvswap.cpp",
                                    "kv_probe.cpp", "kv_manager.cpp")]
FLAGS = ["-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-pthread",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
SANITIZERS = {
    "address_undefined": ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                          "-Xarch_host", "-fno-sanitize-recover=undefined"],
    "thread": ["-Xarch_host", "-fsanitize=thread"],
}


@pytest.mark.parametrize("kind", sorted(SANITIZERS))
def test_host_logic_is_clean_under(kind, tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / ("plan_stress_" + kind))
    build = subprocess.run([hipcc] + FLAGS + SANITIZERS[kind] + SOURCES + ["-o", exe],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert build.returncode == 0, build.stdout[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", TSAN_OPTIONS="halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1")
    iters = "20000" if kind == "address_undefined" else "6000"
    run = subprocess.run([exe, iters], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                         timeout=300, env=env)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "plan_stress: 0 failures" in run.stdout, run.stdout[-2000:]
    assert "Sanitizer" not in run.stdout, run.stdout[-4000:]


def test_polling_never_harvests_an_op_that_is_still_being_enqueued(tmp_path):
    """tests/host/reap_unissued.cpp: the engine's completion polling against an op whose events
    are not recorded yet (the runtime reports such events as complete).  Host only."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "reap_unissued")
    srcs = [os.path.join(ROOT, "tests", "host", "reap_unissued.cpp")] + SOURCES[1:]
    build = subprocess.run([hipcc] + FLAGS + SANITIZERS["address_undefined"] + srcs + ["-o", exe],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert build.returncode == 0, build.stdout[-4000:]
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=60,
                         env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"))
    assert run.returncode == 0 and "reap_unissued: 0 failures" in run.stdout, run.stdout[-4000:]


def test_copy_plans_move_exactly_the_moved_records(tmp_path):
    """tests/host/copy_plan.cpp: move lists reordered for strided copies and cut into contiguous
    and 2-D copies, applied to byte arrays on the CPU in both directions.  Host only."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "copy_plan")
    srcs = [os.path.join(ROOT, "tests", "host", "copy_plan.cpp")] + SOURCES[1:]
    build = subprocess.run([hipcc] + FLAGS + SANITIZERS["address_undefined"] + srcs + ["-o", exe],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert build.returncode == 0, build.stdout[-4000:]
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120,
                         env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"))
    assert run.returncode == 0 and "copy_plan: 0 failures" in run.stdout, run.stdout[-4000:]
