"""The CPU side under AddressSanitizer and UndefinedBehaviorSanitizer: the C oracle (its pins and a walk through
extreme shapes) and the host code of the HIP library (its argument checks).  Each runs in a child process with the
matching sanitizer runtime preloaded; any finding aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

ORACLE_MODULES = ["tests/test_oracle_extremes.py", "tests/test_oracle_sampler.py", "tests/test_oracle_groups.py",
                  "tests/test_oracle_pool_all.py", "tests/test_oracle_zones.py", "tests/test_oracle_rounds.py",
                  "tests/test_oracle_tables_dp.py", "tests/test_oracle_replay.py", "tests/test_oracle_weights.py",
                  "tests/test_oracle_moves.py"]


def _child_env(runtime, extra):
    env = dict(os.environ)
    inherited = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = runtime + (":" + inherited if inherited else "")     # the sanitizer runtime has to come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra)
    return env


def _run_pytest(modules, env):
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu", *modules]
    return subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)


def test_oracle_pins_and_extreme_shapes_under_the_sanitizers():
    import oracle
    oracle.build(sanitize=True)
    res = _run_pytest(ORACLE_MODULES, _child_env(oracle.sanitizer_runtime(), {oracle.SANITIZE_ENV: "1"}))
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert " passed" in res.stdout and "failed" not in res.stdout, tail


def test_host_argument_checks_of_the_hip_library_under_the_sanitizers():
    from paper_2403_14097_amd import build as hip_build
    runtime = hip_build.host_sanitizer_runtime()
    if not os.path.exists(runtime):
        pytest.skip("the compiler's sanitizer runtime is not installed")
    hip_build.build_host_sanitized()
    res = _run_pytest(["tests/test_host_boundary.py"], _child_env(runtime, {"PARCAE_HOST_SANITIZE": "1"}))
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert " passed" in res.stdout and "failed" not in res.stdout, tail
