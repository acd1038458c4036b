"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU): the C oracle on small random
problems, and the library's host side (descriptor handling and the static work partition, through its debug
hook) on random batches.  The device code is compiled as usual and never runs here."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
# the environment is passed through untouched except for the sanitizers' own options (a preloaded
# library ahead of the ASan runtime is tolerated instead of being removed)
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_fuzz")
    r = run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
             "-o", exe, os.path.join(SAN, "oracle_fuzz.c"), os.path.join(ROOT, "oracle", "rl_decode_attn_ref.c"), "-lm"])
    assert r.returncode == 0, r.stderr
    plain = str(tmp_path / "oracle_plain")
    r2 = run(["gcc", "-O2", "-std=c11", "-fopenmp", "-o", plain, os.path.join(SAN, "oracle_fuzz.c"),
              os.path.join(ROOT, "oracle", "rl_decode_attn_ref.c"), "-lm"])
    assert r2.returncode == 0, r2.stderr
    a, b = run([exe], env=ENV), run([plain], env=ENV)
    assert a.returncode == 0 and "runtime error" not in a.stderr and "AddressSanitizer" not in a.stderr, a.stderr[-2000:]
    assert a.stdout.startswith("ok ") and a.stdout == b.stdout            # and the sanitised build computes the same numbers


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_library_host_side_under_asan_and_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    exe = str(tmp_path / "partition_fuzz")
    csrc = os.path.join(ROOT, "paper_2512_21450_amd", "csrc")
    r = run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
             "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
             "-o", exe, os.path.join(SAN, "partition_fuzz.cpp")] +
            [os.path.join(csrc, f) for f in ("rlda_api.hip", "rlda_simple.hip", "rlda_shared.hip")])
    assert r.returncode == 0, r.stderr[-3000:]
    a = run([exe], env=ENV)
    assert a.returncode == 0 and a.stdout.startswith("ok "), (a.stdout, a.stderr[-2000:])
    assert "runtime error" not in a.stderr and "AddressSanitizer" not in a.stderr, a.stderr[-2000:]
