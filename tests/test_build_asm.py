"""Host-side check of the compiled attention kernels for the 8-bit and 4-bit caches.

Its register pipeline loads cache data with inline-assembly loads and waits for them with an
inline-assembly s_waitcnt; between the two the compiler does not know that the destination registers are
still in flight.  The code is written so that it has no reason to touch them (one loading statement and one
waiting statement per register set inside the loop), but nothing in the language forbids the register
allocator from copying such a register to another one before the wait, which would copy a value that has
not arrived.  This test compiles the kernel to assembly (no GPU needed) and verifies, for every step of the
pipeline loop, that no register written by one of those loads is read by a move before the next explicit
wait, and that the loop's explicit waits are the partial ones the pipeline counts on."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2507_19427_amd", "csrc", "mfa_attn.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def asm_text(tmp_path_factory):
    if not (os.path.exists(HIPCC) or shutil.which(HIPCC)):
        pytest.skip("hipcc not available")
    out = tmp_path_factory.mktemp("asm") / "mfa_attn.s"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "--cuda-device-only", "-S", "-o", str(out), SRC]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    return out.read_text()


def _kernel_body(text, mangled):
    start = text.index("\n" + mangled + ":")
    end = text.index(".size\t" + mangled, start)
    return text[start:end].split("\n")


def _regs(token):
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", token)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"v(\d+)", token)
    return {int(m.group(1))} if m else set()


def _check_pipeline(lines, ops_per_step=5):
    in_asm = False
    queue = []                 # vector-memory operations in issue order: the registers each one writes
                               # (empty for direct-to-LDS loads, stores and compiler-made loads)
    partial_waits = 0

    def in_flight():
        regs = set()
        for r in queue:
            regs |= r
        return regs

    for ln in lines:
        t = ln.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not t or t.startswith(";") or t.startswith("."):
            continue
        op, _, rest = t.partition(" ")
        operands = [o.strip() for o in rest.split(",")] if rest else []
        if op.startswith("global_load") or op.startswith("global_store") or op.startswith("buffer_"):
            tracked = in_asm and op in ("global_load_dwordx4", "global_load_dword")
            queue.append(_regs(operands[0]) if tracked else set())
            continue
        if op == "s_waitcnt" and "vmcnt" in rest:
            left = int(re.search(r"vmcnt\((\d+)\)", rest).group(1))
            if in_asm and left == ops_per_step:
                partial_waits += 1
            if not in_asm and partial_waits > 0:
                # a compiler-made vector-memory wait inside the pipeline loop: it must not reach the
                # pipeline's own loads (the compiler does not count them, so its number is too small)
                assert not in_flight(), f"compiler-inserted wait drains the pipeline: {t}"
            queue = queue[max(0, len(queue) - left):] if left else []
            continue
        if op.startswith("v_mov") or op.startswith("v_pk_mov") or op.startswith("v_accvgpr"):
            sources = set()
            for o in operands[1:]:
                sources |= _regs(o)
            assert not (sources & in_flight()), f"in-flight register copied before its wait: {t}"
    assert partial_waits >= 2, "the two steps of the unrolled loop each wait for all but the youngest step's loads"


@pytest.mark.parametrize("bits,ops_per_step", [(8, 5), (4, 3)])
@pytest.mark.parametrize("q_len", [1, 2])
@pytest.mark.parametrize("paged", [0, 1])
def test_lowbit_pipeline_registers_stay_untouched_between_load_and_wait(asm_text, paged, q_len, bits, ops_per_step):
    name = f"_ZN3mfa20decode_lowbit_kernelILb{paged}ELi{q_len}ELi{bits}EEEvNS_8AttnArgsE"
    _check_pipeline(_kernel_body(asm_text, name), ops_per_step)


def _snippet(between):
    load = [";;#ASMSTART", "global_load_dwordx4 v[10:13], v[2:3], off", ";;#ASMEND"]
    wait = [";;#ASMSTART", "s_waitcnt vmcnt(5)", ";;#ASMEND"]
    filler = [";;#ASMSTART"] + ["global_load_lds_dwordx4 v[4:5], off"] * 5 + [";;#ASMEND"]
    return wait + load + filler + wait + load + filler + between + wait + ["v_mov_b32_e32 v20, v11"]


def test_the_checker_itself_catches_a_copy_and_a_drain():
    _check_pipeline(_snippet([]))                                   # clean: the copy comes after the wait
    with pytest.raises(AssertionError, match="copied before its wait"):
        _check_pipeline(_snippet(["v_mov_b32_e32 v20, v11"]))
    with pytest.raises(AssertionError, match="drains the pipeline"):
        _check_pipeline(_snippet(["s_waitcnt vmcnt(0)"]))
