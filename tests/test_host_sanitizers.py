"""Host code of the library built with g++ under AddressSanitizer and UndefinedBehaviorSanitizer and driven through
the C ABI by small drivers under tests/host/.

The schedule planner (csrc/schedule.cpp): output arrays of exactly the needed size, arrays that are too small,
argument errors, a sweep of (W, N, mini-batches); every plan the driver prints must equal the oracle's simulation.
The stage executor's host logic (csrc/stage.cpp, with the kernel launchers and the three HIP runtime calls it makes
replaced by host stand-ins, tests/host/kernel_stubs.cpp): layout and argument checks on valid, invalid and random
layer lists, then slot and buffer bookkeeping of forward / backward / update on host memory.
Both runs must end without a sanitizer report."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import schedule as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def build(tmp_path_factory, name, sources):
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    exe = str(tmp_path_factory.mktemp("san") / name)
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-pthread"] + [os.path.join(ROOT, s) for s in sources] + ["-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return exe


def run_clean(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)      # the sanitizer runtime has to come first in the process
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    assert "runtime error" not in r.stderr and "Sanitizer" not in r.stderr and "FAILED" not in r.stderr, r.stderr[-2000:]
    return r


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    return build(tmp_path_factory, "sanitize_schedule", ["tests/host/sanitize_schedule.cpp", "paper_2410_14312_amd/csrc/schedule.cpp"])


def test_stage_host_logic_is_clean_under_sanitizers(tmp_path_factory):
    run_clean(build(tmp_path_factory, "sanitize_stage", ["tests/host/sanitize_stage.cpp", "tests/host/kernel_stubs.cpp",
                                                         "paper_2410_14312_amd/csrc/stage.cpp"]))


def test_planner_is_clean_under_sanitizers_and_equals_the_oracle(driver):
    r = run_clean(driver)
    plans = versions = 0
    for line in r.stdout.splitlines():
        f = line.split()
        if f[0] == "plan":
            W, N, n = int(f[1]), int(f[2]), int(f[3])
            got = np.array(f[4:], dtype=np.int64).reshape(-1, 7)
            want = np.array(S.simulate(W, N, n)["ops"], dtype=np.int64)
            assert np.array_equal(got, want), (W, N, n)
            plans += 1
        elif f[0] == "plan1f1b":
            from oracle import baseline
            W, n = int(f[1]), int(f[2])
            got = np.array(f[3:], dtype=np.int64).reshape(-1, 7)
            assert np.array_equal(got, np.array(baseline.simulate_1f1b(W, n), dtype=np.int64)), (W, n)
        elif f[0] == "v":
            W, N = int(f[1]), int(f[2])
            assert int(f[3]) == S.version_difference_simulated(W, N), (W, N)
            need = S.stash_groups_needed(W, N, 3 * W + 4)
            ops = S.simulate(W, N, 4 * W + 4 * N + 8)["ops"]
            for s, pair in enumerate(f[4:]):
                groups, shadow = (int(v) for v in pair.split(":"))
                assert groups == need[s], (W, N, s)
                assert shadow == max([sv - nv for (t, w, kind, b, j, sv, nv) in ops if kind == S.FWD and w == s] + [0]), (W, N, s)
            versions += 1
    assert plans == 9 * 8 and versions == 12 * 9
