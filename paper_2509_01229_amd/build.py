"""Build the C-ABI library paper_2509_01229_amd/libliquidgemm.so with hipcc for gfx950.

`python -m paper_2509_01229_amd.build` compiles csrc/*.hip and csrc/*.cpp in-tree.
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libliquidgemm.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SOURCES = ["liquidgemm.hip", "actquant.hip", "calib.hip", "lqq_pack.cpp"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep hipcc from forming packed-FP32 instructions out of ordinary float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-pragmas",
    # per-kernel register / scratch report on stderr, checked below
    "-Rpass-analysis=kernel-resource-usage",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    "-lpthread",
]


# The kernels that load straight into LDS and the one-wave-per-SIMD kernels count their loads in
# flight by hand (s_waitcnt vmcnt(N) in assembly) and rely on the order in which this compiler
# emits the statements between scheduling barriers; the GPU parity tests are what validates a
# compiler.  Another compiler must be validated the same way before its library is used.
VALIDATED_COMPILERS = ("roc-7.2.0",)


def check_compiler() -> None:
    res = subprocess.run([HIPCC, "--version"], capture_output=True, text=True)
    text = res.stdout + res.stderr
    if any(tag in text for tag in VALIDATED_COMPILERS) or os.environ.get("LIQUIDGEMM_UNVALIDATED_COMPILER") == "1":
        return
    raise RuntimeError(
        "hipcc is not a compiler this library's hand-counted waits were validated with "
        f"({', '.join(VALIDATED_COMPILERS)}):\n{text}\nRun the GPU parity tests "
        "(pytest tests -m gpu) on a build made with LIQUIDGEMM_UNVALIDATED_COMPILER=1, then add its tag to "
        "VALIDATED_COMPILERS in paper_2509_01229_amd/build.py.")


def build_library(verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    check_compiler()
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = [HIPCC, *FLAGS, *extra_flags, "-o", out, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed building libliquidgemm.so")
    usage = kernel_resource_usage(res.stderr)
    spilling = {k: v for k, v in usage.items() if v.get("ScratchSize [bytes/lane]", 0) > 0}
    if spilling:
        os.remove(out)  # never leave a library behind that must not be run
        raise RuntimeError("kernels must not use scratch memory, but these do: "
                           + ", ".join(f"{k} ({v['ScratchSize [bytes/lane]']} B/lane)" for k, v in spilling.items()))
    if verbose:
        other = "\n".join(l for l in res.stderr.splitlines() if "kernel-resource-usage" not in l
                          and not l.lstrip().startswith(("|", "^")) and l.strip())
        if other:
            sys.stderr.write(other + "\n")
        print(f"{len(usage)} kernels, max VGPRs {max(v.get('VGPRs', 0) for v in usage.values())}, no scratch")
    return out


def kernel_resource_usage(stderr_text: str) -> dict:
    """Parse hipcc's -Rpass-analysis=kernel-resource-usage remarks: {kernel: {field: int}}."""
    import re

    usage, cur = {}, None
    for line in stderr_text.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = usage.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z][^:]*): (\d+) \[-Rpass-analysis", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return usage


if __name__ == "__main__":
    print(build_library(verbose=True))
