"""Host-side checks of the compiled attention kernels (no GPU needed).

The kernels for the 8-bit and 4-bit caches load cache data with inline-assembly loads and wait for them with
an inline-assembly s_waitcnt (a counted wait that leaves the youngest step's loads in flight; left to the
compiler the wait would drain the pipeline every tile).  Between the two statements the compiler does not
know that the destination registers are still in flight.  The code gives it no reason to touch them, but
nothing in the language forbids the register allocator from copying, spilling or reusing such a register
before the wait, which would silently use a value that has not arrived.  So the build checks the machine
code it has just produced:

  * between a pipeline load and the explicit wait that covers it, no instruction of any kind names one of
    the load's destination registers (as a source or as a destination);
  * no compiler-made vector-memory wait inside the pipeline loop reaches the pipeline's own loads;
  * the kernels use no scratch memory (a spill of an in-flight register would go there) -- for every
    attention kernel, since scratch also costs every wave its set-up.

build.py runs check_attention_asm() on the assembly of every build and fails the build on a violation;
tests/test_build_asm.py runs the same functions, and the checker itself against planted mistakes.
"""
import re

PIPELINE_KERNELS = [(paged, q_len, bits) for bits in (8, 4) for q_len in (1, 2) for paged in (0, 1)]
OPS_PER_STEP = {8: 5, 4: 3}

_REG = re.compile(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b")


def lowbit_kernel_name(paged, q_len, bits):
    return f"_ZN3mfa20decode_lowbit_kernelILb{paged}ELi{q_len}ELi{bits}EEEvNS_8AttnArgsE"


def kernel_body(text, mangled):
    start = text.index("\n" + mangled + ":")
    end = text.index(".size\t" + mangled, start)
    return text[start:end].split("\n")


def registers_named(operand_text):
    regs = set()
    for m in _REG.finditer(operand_text):
        if m.group(3) is not None:
            regs.add(int(m.group(3)))
        else:
            regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
    return regs


def check_pipeline(lines, ops_per_step=5):
    """Raises AssertionError when the register pipeline of a kernel body (lines of assembly) is disturbed."""
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
        t = t.split(";")[0].strip()                    # drop trailing comments
        op, _, rest = t.partition(" ")
        if op.startswith("global_load") or op.startswith("global_store") or op.startswith("buffer_") or \
                op.startswith("scratch_") or op.startswith("flat_"):
            operands = [o.strip() for o in rest.split(",")] if rest else []
            tracked = in_asm and op in ("global_load_dwordx4", "global_load_dword")
            touched = registers_named(rest)
            if tracked:
                dest = registers_named(operands[0])
                assert not (dest & in_flight()), f"a pipeline load overwrites a register still in flight: {t}"
                assert not ((touched - dest) & in_flight()), f"in-flight register used as an address: {t}"
                queue.append(dest)
            else:
                assert not (touched & in_flight()), f"in-flight register touched by a memory instruction before its wait: {t}"
                queue.append(set())
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
        touched = registers_named(rest)
        assert not (touched & in_flight()), f"in-flight register touched before its wait: {t}"
    assert partial_waits >= 2, "the two steps of the unrolled loop each wait for all but the youngest step's loads"


def scratch_bytes(text):
    """{kernel name: bytes of scratch per lane} from the .amdhsa_private_segment_fixed_size directives."""
    out = {}
    name = None
    for ln in text.split("\n"):
        t = ln.strip()
        if t.startswith(".amdhsa_kernel "):
            name = t.split()[1]
        elif t.startswith(".amdhsa_private_segment_fixed_size") and name is not None:
            out[name] = int(t.split()[1])
        elif t.startswith(".end_amdhsa_kernel"):
            name = None
    return out


def check_attention_asm(text):
    """All checks on the assembly text of mfa_attn.hip.  Raises AssertionError naming the first violation."""
    for paged, q_len, bits in PIPELINE_KERNELS:
        name = lowbit_kernel_name(paged, q_len, bits)
        try:
            check_pipeline(kernel_body(text, name), OPS_PER_STEP[bits])
        except AssertionError as e:
            raise AssertionError(f"{name}: {e}") from None
    scratch = scratch_bytes(text)
    decode = {k: v for k, v in scratch.items() if "decode_" in k}
    assert len(decode) == 16, f"expected 16 attention kernels, found {sorted(decode)}"
    for name, nbytes in decode.items():
        assert nbytes == 0, f"{name} uses {nbytes} bytes of scratch per lane (register spills)"
