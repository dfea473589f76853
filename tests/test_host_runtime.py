"""Host half of the slot protocol on the CPU, under ThreadSanitizer.

tests/fake_device/fake_gpu.cpp links the library's planner, streaming copies and host threads
(drain / fill / watchdog / crew) for the CPU and drives them against a thread model of the
device half.  Checked here: the switch result equals memcpy, also in place; a plan is reusable;
every failure path (credits withheld, the device gives up, the device never starts) ends with
NIXIE_ETIMEOUT instead of a hang; and ThreadSanitizer sees no data race in any of it."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2601_11743_amd", "csrc")


@pytest.fixture(scope="module")
def fake_gpu(tmp_path_factory):
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    out = str(tmp_path_factory.mktemp("fake") / "fake_gpu_tsan")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-pthread",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
           os.path.join(ROOT, "tests", "fake_device", "fake_gpu.cpp"),
           os.path.join(CSRC, "hostside.cpp"), os.path.join(CSRC, "planner.cpp"), os.path.join(CSRC, "spaces.cpp"), os.path.join(CSRC, "hostcopy.cpp"),
           "-o", out]
    subprocess.check_call(cmd)
    return out


def run(binary, scenario, seed):
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=0 exitcode=66")
    r = subprocess.run([binary, scenario, str(seed)], capture_output=True, text=True, timeout=120, env=env)
    text = r.stdout + r.stderr
    assert "ThreadSanitizer" not in text, text[-3000:]
    assert r.returncode == 0, text[-3000:]
    return text


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_swap_equals_memcpy_and_is_race_free(fake_gpu, seed):
    out = run(fake_gpu, "swap", seed)
    assert "pass 1" in out           # the same plan switched twice


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_in_place_swap(fake_gpu, seed):
    run(fake_gpu, "in_place", seed)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_in_place_swap_between_two_spaces_of_one_pool(fake_gpu, seed):
    """The applications see the shared memory at different addresses (one file mapped twice and
    registered as two spaces): overlap and dependencies must be found through the pool coordinate,
    a plan without NIXIE_IN_PLACE must be refused, and so must a range across the edge of a space."""
    run(fake_gpu, "spaces", seed)


@pytest.mark.parametrize("scenario", ["tier", "tier_in_place"])
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_pinned_tier_allocations_move_directly(fake_gpu, scenario, seed):
    """Host ranges registered as pinned tier: those allocations take no slot and no host thread,
    the others are staged in the same switch; NIXIE_NO_DIRECT turns the tier off."""
    run(fake_gpu, scenario, seed)


@pytest.mark.parametrize("scenario", ["stall", "gpu_quits", "dead_gpu"])
def test_failure_paths_time_out_cleanly(fake_gpu, scenario):
    out = run(fake_gpu, scenario, 1)
    assert "error -5" in out


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_shim_block_allocator_against_a_bitmap(tmp_path_factory, seed):
    """First fit over whole blocks with merging on release (the shim's address space), checked step by
    step against a brute-force bitmap."""
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    out = str(tmp_path_factory.mktemp("runs") / "blockruns_test")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-I" + CSRC,
                           os.path.join(ROOT, "tests", "fake_device", "blockruns_test.cpp"), "-o", out])
    r = subprocess.run([out, str(seed)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "ok seed" in r.stdout, r.stdout + r.stderr


# ---- the transparent shim's logic against a CPU model of the runtime -----------------------------

CLANG = "/opt/rocm/lib/llvm/bin/clang++"      # g++ does not get through the runtime's hip_ext.h


@pytest.fixture(scope="module")
def shim_model(tmp_path_factory):
    """shim.cpp itself, compiled into a test program in front of tests/fake_device/fake_runtime.cpp (a
    CPU stand-in for the HIP calls it forwards to and the libnixie calls it makes), all under
    ThreadSanitizer."""
    if not os.path.exists(CLANG):
        pytest.skip("no clang++ with the HIP headers")
    d = str(tmp_path_factory.mktemp("shim_model"))
    flags = ["-std=c++17", "-O1", "-g", "-fsanitize=thread", "-D__HIP_PLATFORM_AMD__", "-w", "-I/opt/rocm/include",
             "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
    fake = os.path.join(ROOT, "tests", "fake_device")
    subprocess.check_call([CLANG, *flags, "-shared", "-fPIC", os.path.join(fake, "fake_runtime.cpp"),
                           "-o", os.path.join(d, "libfake_runtime.so")])
    out = os.path.join(d, "shim_model_test")
    subprocess.check_call([CLANG, *flags, os.path.join(CSRC, "shim.cpp"), os.path.join(fake, "shim_model_test.cpp"),
                           "-L" + d, "-lfake_runtime", "-Wl,-rpath," + d, "-ldl", "-pthread", "-o", out])
    return out


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_shim_with_three_application_threads_against_constant_evictions(shim_model, seed):
    """Launches, waits, copies, allocations and memory reports of three threads while the main thread evicts
    every 150 us: no update is lost or doubled (a launch past the execution flag would die on unmapped
    memory, a migration before the kernels have finished would be a race), and no data race in the shim."""
    out = run(shim_model, "threads", seed)
    assert "ok" in out.splitlines()[-1], out


@pytest.mark.parametrize("seed", [1, 2])
def test_shim_idleness_rule_with_several_threads(shim_model, seed):
    out = run(shim_model, "idle", seed)
    assert "ok" in out.splitlines()[-1], out


def test_shim_refuses_to_migrate_inside_a_stream_capture(shim_model):
    out = run(shim_model, "capture", 1)
    assert "evict during capture -7" in out
