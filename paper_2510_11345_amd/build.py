"""Build libroll_decode.so for gfx950 with hipcc (in-tree, no JIT cache)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libroll_decode.so")
SOURCES = ["api.hip", "kv_pool.hip", "decode_attn.hip", "prefill_attn.hip", "sample_logprob.hip", "policy_loss.hip",
           "sample_buffer.hip", "prof_probe.hip"]


def hipcc_path() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


TIMELINE_LIB = os.path.join(HERE, "libroll_decode_timeline.so")


def build(verbose: bool = False, out: str = LIB, sanitize_host: bool = False, timeline: bool = False) -> str:
    """Compile the library to `out`.  sanitize_host instruments the HOST pass only with
    AddressSanitizer and UndefinedBehaviorSanitizer (allocator, SampleBuffer, dealing arithmetic,
    argument checks); the CPU test suite runs its host-only tests through such a build."""
    cmd = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-function",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", out]
    if timeline:  # per-wave timestamps in the attention kernel (bench.py --attn-timeline)
        cmd += ["-DROLL_ATTN_TIMELINE"]
    if sanitize_host:
        cmd += ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer",
                "-shared-libsan", "-g"]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines()
                    if "packed-fp32-ops" not in l)  # the host pass does not know the GPU feature
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if err.strip() and verbose:
        print(err, file=sys.stderr)
    return out


if __name__ == "__main__":
    if "--timeline" in sys.argv[1:]:
        print(build(verbose=True, out=TIMELINE_LIB, timeline=True))
    else:
        print(build(verbose=True))
