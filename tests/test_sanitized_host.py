"""The host side of the library (trace loading, evolution-strategy arithmetic, argument and option checks, workspace
planning) and the CPU oracle, each built for the CPU with AddressSanitizer and UndefinedBehaviorSanitizer and run on
seeded inputs: a mutation fuzz of the JSON-lines loader followed by a walk over the host-side entry points, and the
oracle's replays on small traces in awkward shapes.  The GPU kernels are not part of these builds (GPU sanitizers are
not available to this project): the library's device operations are replaced by stubs that fail."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2602_11688_amd", "csrc")
SAN = os.path.join(ROOT, "tests", "sanitize")
FLAGS = ["-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
# (sanitized programs must not inherit a preloaded library that interposes before the sanitizer's runtime)
ENV.pop("LD_PRELOAD", None)

pytestmark = pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")


def _build(out, sources, includes):
    cmd = ["g++", *FLAGS, *[f"-I{i}" for i in includes], *sources, "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True, env=ENV, timeout=600)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-6000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-6000:]
    return r.stdout


@pytest.fixture(scope="module")
def host_fuzz(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("san") / "host_fuzz")
    _build(out, [os.path.join(CSRC, f) for f in ("trace.cpp", "es.cpp", "api.cpp")] +
           [os.path.join(SAN, "host_stubs.cpp"), os.path.join(SAN, "host_fuzz.cpp")],
           [os.path.join(ROOT, "include"), CSRC])
    return out


@pytest.mark.parametrize("seed", [1, 20260211, 11688])
def test_host_side_survives_a_mutation_fuzz_under_asan_and_ubsan(host_fuzz, tmp_path, seed):
    out = _run([host_fuzz, str(seed), "700", str(tmp_path / "fuzz.jsonl")])
    assert "700 iterations" in out


def test_oracle_replays_run_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _build(exe, [os.path.join(ROOT, "oracle", "gorgo_oracle.cpp"), os.path.join(SAN, "oracle_san.cpp")], [])
    out = _run([exe, "7", "60"])
    assert "60 rounds" in out
