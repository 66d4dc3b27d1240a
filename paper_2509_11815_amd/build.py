"""Builds libspecvlm.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libspecvlm.so")
SOURCES = ["api.hip", "sample_kernels.hip", "accept_sample.hip", "draft_tree.hip", "head_argmax.hip", "compress.hip", "attn_valu.hip", "attn_mfma.hip"]


def hipcc_command(out: str = LIB) -> list[str]:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
            "-I" + INCLUDE, "-I" + CSRC,
            # compiler-generated packed fp32 ops are switched off on the test machines
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            # keep MFMA accumulators in architectural VGPRs: the attention kernel rescales and
            # converts them with VALU ops, and AGPR copies would dominate its inner loop
            "-mllvm", "-amdgpu-mfma-vgpr-form",
            "-o", out] + [os.path.join(CSRC, s) for s in SOURCES]


def build(verbose: bool = False) -> str:
    """Compile every kernel for gfx950 (cross-compiles without a GPU).  Always rebuilds."""
    proc = subprocess.run(hipcc_command(), capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
    if verbose:
        print(proc.stderr)
    return LIB


def kernel_resource_usage(source: str) -> dict:
    """Per-kernel VGPR count, scratch bytes per lane and LDS bytes of one source file, from the
    compiler's own kernel-resource-usage remarks (device code only, nothing is linked)."""
    import re
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE, "-I" + CSRC,
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-mllvm", "-amdgpu-mfma-vgpr-form",
               "-Rpass-analysis=kernel-resource-usage", "--cuda-device-only", "-c", "-o", os.path.join(tmp, "k.o"),
               os.path.join(CSRC, source)]
        proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stderr)
    out, name = {}, None
    for line in proc.stderr.splitlines():
        m = re.search(r"remark: Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            out[name] = {}
        for key, pat in (("vgprs", r"\bVGPRs: (\d+)"), ("scratch", r"ScratchSize \[bytes/lane\]: (\d+)"),
                         ("lds", r"LDS Size \[bytes/block\]: (\d+)")):
            m = re.search(pat, line)
            if m and name:
                out[name][key] = int(m.group(1))
    return out


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(INCLUDE, "specvlm.h")]
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    print(build(verbose=True))
