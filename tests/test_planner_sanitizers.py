"""The host planner under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU involved).

plan.hip holds no device code, so its host side is compiled alone (--cuda-host-only) together with
tests/planner_sanitizer.cpp, which plans thousands of random shapes and follows every index of every plan.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def fuzz_binary(tmp_path_factory):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc is needed to build the planner with sanitizers")
    out = str(tmp_path_factory.mktemp("planner_san") / "planner_fuzz")
    cmd = [hipcc, "--cuda-host-only", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-fno-sanitize-recover=undefined",
           os.path.join(ROOT, "paper_2503_23294_amd", "csrc", "plan.hip"),
           "-x", "hip", os.path.join(ROOT, "tests", "planner_sanitizer.cpp"), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    return out


@pytest.mark.parametrize("seed", [1, 2])
def test_planner_is_clean_under_asan_and_ubsan(fuzz_binary, seed):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([fuzz_binary, "2500", str(seed)], capture_output=True, text=True, env=env)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "passed" in r.stdout


@pytest.mark.parametrize("env", [{"COCKTAIL_POOL_PERCENT": "100"}, {"COCKTAIL_GROUP_WORKERS": "3", "COCKTAIL_POOL_PERCENT": "50"},
                                 {"COCKTAIL_LAYOUT": "1", "COCKTAIL_PAIR_MODE": "2"}, {"COCKTAIL_MIN_POOL_BLOCKS": "1"}])
def test_planner_tuning_knobs_are_clean_too(fuzz_binary, env):
    e = dict(os.environ, **env)
    r = subprocess.run([fuzz_binary, "600", "7"], capture_output=True, text=True, env=e)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
