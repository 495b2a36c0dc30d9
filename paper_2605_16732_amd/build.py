"""Build libdirotq.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2605_16732_amd.build`."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdirotq.so")
PROBE_LIB = os.path.join(HERE, "libdirotq_probe.so")     # matrix-pipe rate probes used by bench.py only
SOURCES = ["dirotq_abi.hip", "rotate_quantize.hip", "w4a4_gemm.hip", "w4a4_gemm_ws.hip", "w4a4_gemm_skinny.hip", "w4a8_gemm.hip", "w4a16_gemm.hip", "prepare.hip"]

# packed-fp32 VALU instructions are switched off on purpose (they have produced wrong
# results on the test machines); no fast-math: the quantizer relies on IEEE division.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True, extra_flags: list[str] | None = None) -> str:
    """Compile every HIP source and link the shared library.  Always recompiles."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    cc = hipcc()
    flags = HIPCC_FLAGS + (extra_flags or []) + ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [cc, *flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        keep = [ln for ln in out.splitlines() if "packed-fp32-ops" not in ln or "error" in ln]
        if p.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n" + out, file=sys.stderr)
        elif verbose and keep:
            print("\n".join(keep))
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    cmd = [cc, *flags, "-shared", os.path.join(CSRC, "bench_probe.hip"), "-o", PROBE_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    return LIB


if __name__ == "__main__":
    build()
