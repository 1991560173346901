"""Build libfastar.so (hand-written HIP for gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfastar.so")
SOURCES = ["api.hip", "encode.hip", "select.hip", "tempcache.hip", "attention.hip", "attention_d128.hip",
           "attention_d128_pp.hip", "attention_fp8.hip", "buckets.hip"]
ASM_CHECKED = ["attention_d128.hip", "attention_d128_pp.hip"]  # kernels that read LDS through inline assembly
# Integer matrix-core results that feed plain ALU epilogues (arg-max, top-k scores): keep them in ordinary vector
# registers, not accumulation registers that every ALU instruction would first have to copy from.
PER_SOURCE_FLAGS = {src: ["-mllvm", "-amdgpu-mfma-vgpr-form"] for src in ("tempcache.hip", "select.hip", "encode.hip", "buckets.hip")}
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-fast-math", "-ffp-contract=on",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def verify_asm_reads(hipcc: str, extra: list[str] | None = None) -> None:
    """The tuned attention kernel reads LDS through inline assembly; check on the generated ISA that the
    compiler kept its hands off those registers until the explicit wait (see asmcheck.py)."""
    try:
        from . import asmcheck
    except ImportError:  # run as a script
        import asmcheck
    for src in ASM_CHECKED:
        asm = os.path.join(CSRC, src.replace(".hip", ".s"))
        cmd = [hipcc, *FLAGS, *(extra or []), "-S", "--cuda-device-only", os.path.join(CSRC, src), "-o", asm]
        subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        bad = asmcheck.check(asm, verbose=False)
        os.remove(asm)
        if bad:
            raise RuntimeError(f"{src}: {bad} instruction(s) touch registers of an in-flight inline-asm LDS read")


def build(verbose: bool = False, extra: list[str] | None = None) -> str:
    """Compile every kernel source and link the shared library.  Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *PER_SOURCE_FLAGS.get(src, []), *(extra or []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n{out}", file=sys.stderr)
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    verify_asm_reads(hipcc, extra)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
