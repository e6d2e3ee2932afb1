"""Host sanitizer tier (no GPU): the C oracle and the host side of the C ABI are built with
AddressSanitizer and UndefinedBehaviorSanitizer and run over fixed cases.

* tests/sanitize/oracle_san_driver.c includes oracle/gqa_oracle.c and runs contiguous (both
  layouts), paged and append cases; the sanitized build must print exactly what the plain build
  prints and report nothing.  A third build, in which the driver hands the oracle a cache that is
  one row too short, must be caught: that shows the tier would see an out-of-bounds read.
* tests/sanitize/abi_san_driver.cpp calls every validating entry point of libgqa_decode with bad
  arguments; the library sources are compiled with hipcc and the sanitizers on the host side."""
import glob
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
           OMP_NUM_THREADS="3")


def build(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-4000:]


def run(exe):
    return subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=300)


@pytest.fixture(scope="module")
def oracle_builds(tmp_path_factory):
    d = tmp_path_factory.mktemp("oracle_san")
    src = os.path.join(SAN, "oracle_san_driver.c")
    common = ["gcc", "-std=c11", "-fopenmp", "-ffp-contract=off", "-g", src, "-lm"]
    plain, san, planted = (str(d / n) for n in ("plain", "san", "planted"))
    build(common + ["-O2", "-o", plain])
    flags = ["-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
    build(common + flags + ["-o", san])
    build(common + flags + ["-DPLANT_OVERRUN", "-o", planted])
    return plain, san, planted


def test_oracle_is_clean_under_asan_and_ubsan(oracle_builds):
    plain, san, _ = oracle_builds
    a, b = run(plain), run(san)
    assert a.returncode == 0 and a.stderr == "", a.stderr[-2000:]
    assert b.returncode == 0 and b.stderr == "", b.stderr[-2000:]
    lines = a.stdout.strip().splitlines()
    assert len(lines) == 7 and all(" rc=1 " in ln or "_append rc=0 " in ln for ln in lines), a.stdout
    assert a.stdout == b.stdout           # same arithmetic, same digests, with every access checked


def test_sanitized_oracle_build_catches_a_short_cache(oracle_builds):
    r = run(oracle_builds[2])
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr and "heap-buffer-overflow" in r.stderr


def test_abi_validation_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "abi_san")
    sources = sorted(glob.glob(os.path.join(ROOT, "paper_2510_07356_amd", "csrc", "*.hip")))
    build(["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "-O1", "-std=c++17", "-g",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer",
           "-x", "hip", *sources, os.path.join(SAN, "abi_san_driver.cpp"), "-o", exe])
    r = run(exe)
    assert r.returncode == 0 and r.stdout.strip().endswith("abi ok"), (r.stdout[-2000:], r.stderr[-4000:])
    assert "Sanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
