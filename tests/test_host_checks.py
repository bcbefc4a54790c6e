"""Native host-side checks, built with AddressSanitizer and UndefinedBehaviorSanitizer:

* tests/host_checks/partition_check.cpp replays the work decomposition the kernels index with
  (paper_2510_00932_amd/csrc/launch_plan.hpp) and checks that every launch shape touches every
  element exactly once, for small arrays element by element and for element counts up to 2^62
  through the launch arithmetic;
* tests/host_checks/oracle_check.cpp runs the CPU oracle natively on exactly-sized heap arrays
  (edge sizes, whole and ragged tiles) against closed forms.

No GPU involved; the GPU library is not loaded."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CHECKS = os.path.join(ROOT, "tests", "host_checks")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan"]
BASE = ["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-Werror"]


def _build_and_run(tmp_path, name, sources, includes=(), sanitize=True):
    exe = str(tmp_path / name)
    cmd = BASE + (SAN if sanitize else []) + ["-I" + i for i in includes] + list(sources) + ["-o", exe]
    subprocess.run(cmd, check=True, cwd=ROOT)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)


@pytest.fixture(scope="module")
def gxx():
    if shutil.which("g++") is None:
        pytest.fail("g++ is needed for the host checks")


@pytest.mark.parametrize("sanitize", [True, False], ids=["asan_ubsan", "plain"])
def test_every_launch_shape_covers_every_element_once(tmp_path, gxx, sanitize):
    r = _build_and_run(tmp_path, "partition_check", [os.path.join(CHECKS, "partition_check.cpp")],
                       includes=[os.path.join(ROOT, "paper_2510_00932_amd", "csrc")], sanitize=sanitize)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert "partition ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_oracle_under_sanitizers(tmp_path, gxx):
    r = _build_and_run(tmp_path, "oracle_check", [os.path.join(CHECKS, "oracle_check.cpp"),
                                                  os.path.join(ROOT, "oracle", "oracle.cpp")])
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert "oracle ok" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_a_planted_indexing_mistake_is_caught(tmp_path, gxx):
    """The partition check must be able to fail: shift one index function by one run."""
    src = open(os.path.join(ROOT, "paper_2510_00932_amd", "csrc", "launch_plan.hpp")).read()
    needle = "return chunk * p.chunk_runs + index + (size_t)k * (p.waves / 2);"
    assert needle in src
    mutant_dir = tmp_path / "mutant"
    mutant_dir.mkdir()
    (mutant_dir / "launch_plan.hpp").write_text(src.replace(needle, needle[:-1] + " + 1;"))
    r = _build_and_run(tmp_path, "partition_mutant", [os.path.join(CHECKS, "partition_check.cpp")],
                       includes=[str(mutant_dir)], sanitize=False)
    assert r.returncode == 1 and "FAIL" in r.stdout
