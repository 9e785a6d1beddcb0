"""The library's host code -- descriptor checks, workspace arithmetic, launch plans, error paths -- under the
undefined-behaviour sanitizer (no GPU needed): the sources are built once more with the host side instrumented in
trap mode, and the host-side test file runs again in a child process against that build.  Undefined behaviour
(signed overflow in a size computation, a shift out of range, a misaligned or null access) kills the child."""
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_tests_pass_against_a_build_with_sanitized_host_code(tmp_path):
    spec = importlib.util.spec_from_file_location("lvlm_build", os.path.join(ROOT, "paper_2509_00419_amd", "build.py"))
    build = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(build)
    lib = build.build_host_sanitized(str(tmp_path))
    env = dict(os.environ, LVLM_LIBRARY=lib)
    run = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_abi.py"), "-x", "-q", "-p",
                          "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, timeout=600)
    assert run.returncode == 0, run.stdout[-3000:]
    assert " passed" in run.stdout
