"""Builds libqfc.so (HIP, gfx950 only) in-tree with hipcc.

Usage: python -m paper_2505_00232_amd.build [--force]
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libqfc.so")
SOURCES = ["api.hip", "pack.hip", "gemv.hip", "gemv_q8.hip", "actquant.hip", "rmsnorm.hip", "attention.hip", "gemm_i8.hip", "gemm_f16.hip", "probe.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed-fp32 code generation is switched off on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# Kernels that load MFMA operands into registers with hand-written asynchronous loads and place the
# waits themselves: the compiler takes a destination register to be valid right after the load
# instruction, so if it spilled one it would save the stale value.  The build refuses any spill
# in these kernels (mangled-name fragments per source file).
NO_SPILL = {"gemm_i8.hip": ("gemm_i8_dw_kernel", "gemm_i8_dw4_kernel")}


def _spilling_kernels(remarks: list[str], fragments: tuple[str, ...]) -> list[str]:
    """Names of the kernels matching `fragments` whose resource-usage remarks report scratch memory."""
    import re
    bad, name = [], None
    for line in remarks:
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            continue
        m = re.search(r"(ScratchSize \[bytes/lane\]|VGPRs Spill|SGPRs Spill): (\d+)", line)
        if m and name and any(f in name for f in fragments) and int(m.group(2)) != 0 and name not in bad:
            bad.append(name)
    return bad


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def _deps_newer(target: str) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "qfc.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    if not force and not _deps_newer(LIB):
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    cc = _hipcc()

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        cmd = [cc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if src in NO_SPILL:
            cmd.append("-Rpass-analysis=kernel-resource-usage")
        r = subprocess.run(cmd, capture_output=True, text=True)
        lines = r.stderr.splitlines()
        if src in NO_SPILL:
            spilled = _spilling_kernels(lines, NO_SPILL[src])
            lines = [l for l in lines if "-Rpass-analysis=kernel-resource-usage" not in l]
            if r.returncode == 0 and spilled:
                raise RuntimeError(f"{src}: register spills in {', '.join(spilled)} (their loads complete behind the compiler's back)")
        err = "\n".join(l for l in lines if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err)
        return obj

    with ThreadPoolExecutor(max_workers=7) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    r = subprocess.run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
