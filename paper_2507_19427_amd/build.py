"""Compile the HIP sources under csrc/ into paper_2507_19427_amd/libmfa.so for gfx950, and check the machine
code of the attention kernels (asm_check.py) before the library is put in place."""
import glob
import os
import shutil
import subprocess
import sys
import tempfile

from . import asm_check

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmfa.so")
HEADER = os.path.join(os.path.dirname(HERE), "include", "mfa.h")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
    "-Wall", "-Wno-unused-command-line-argument",
    # packed fp32 VALU forms are kept off for this device
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.hpp")) + [HEADER]
    return any(os.path.getmtime(p) > t for p in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not _stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = tempfile.mkdtemp(prefix="mfa_build_")
    try:
        # -save-temps leaves the device assembly of every source in the working directory: the check below
        # reads the very code that goes into the library
        out_lib = os.path.join(tmp, "libmfa.so")
        cmd = [hipcc] + HIPCC_FLAGS + ["-save-temps", "-o", out_lib] + sources()
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, cwd=tmp)
        out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out)
        if verbose and out.strip():
            print(out)
        asm = glob.glob(os.path.join(tmp, "mfa_attn-hip-amdgcn-amd-amdhsa-gfx950.s"))
        if len(asm) != 1:
            raise RuntimeError("the device assembly of mfa_attn.hip was not produced; cannot check it")
        try:
            with open(asm[0]) as f:
                asm_check.check_attention_asm(f.read())
        except AssertionError as e:
            raise RuntimeError(f"the compiled attention kernels fail the machine-code check, library not installed: {e}")
        shutil.move(out_lib, LIB + ".tmp")
        os.replace(LIB + ".tmp", LIB)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
    sys.exit(0)
