"""The oracle and the host-only code of the library under AddressSanitizer and
UndefinedBehaviorSanitizer (CPU only).

Both are rebuilt with the sanitizers and the existing CPU pins run through them in a child
process whose dynamic loader preloads the sanitizer runtime (an instrumented shared library
cannot be loaded into an uninstrumented python otherwise).  A heap overrun, a use after free or
undefined arithmetic anywhere on the paths those tests walk aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TESTS = os.path.join(ROOT, "tests")


def _runtime(compiler, name):
    path = subprocess.run([compiler, f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def _run_pytest(files, env_extra, preload):
    env = dict(os.environ)
    env.update(env_extra)
    env["LD_PRELOAD"] = ":".join([preload] + [p for p in env.get("LD_PRELOAD", "").split(":") if p])
    # python itself is not instrumented: its interned objects look like leaks, and something else
    # may already sit first in the loader's list
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + \
          [os.path.join(TESTS, f) for f in files]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-4000:]
    assert res.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    return res.stdout


def test_oracle_pins_pass_under_asan_and_ubsan():
    asan = _runtime("gcc", "libasan.so")
    if asan is None:
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    out = _run_pytest(["test_oracle_sampling.py", "test_oracle_attention.py", "test_oracle_prefill.py",
                       "test_oracle_philox.py", "test_oracle_policy_loss.py"],
                      {"ROLL_ORACLE_SANITIZE": "1"}, asan)
    assert " passed" in out
    assert os.path.exists(os.path.join(ROOT, "oracle", "libroll_oracle_san.so"))


def test_host_code_of_the_library_passes_under_asan_and_ubsan(tmp_path):
    # allocator, SampleBuffer, the dealing arithmetic and every argument check are host code in
    # the HIP sources; only the host pass is instrumented (the GPU pass has no sanitizer here)
    from paper_2510_11345_amd import build as hip_build
    asan = _runtime(os.path.join(os.path.dirname(hip_build.hipcc_path()), "..", "lib", "llvm", "bin", "clang"),
                    "libclang_rt.asan-x86_64.so") or _runtime("/opt/rocm/lib/llvm/bin/clang", "libclang_rt.asan-x86_64.so")
    if asan is None:
        pytest.skip("clang's AddressSanitizer runtime is not installed")
    lib = str(tmp_path / "libroll_decode_san.so")
    hip_build.build(out=lib, sanitize_host=True)
    out = _run_pytest(["test_abi_and_allocator.py", "test_sample_buffer.py", "test_attn_ranges.py",
                       "test_scheduler_bound.py"], {"ROLL_DECODE_LIB": lib}, asan)
    assert " passed" in out
