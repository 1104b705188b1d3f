"""Host-side check of the compiled attention kernels (the checker is paper_2507_19427_amd/asm_check.py, which
the build itself runs on every library it produces).  Here: the same checks on a fresh compilation of
mfa_attn.hip, kernel by kernel, and the checker against planted mistakes."""
import os
import shutil
import subprocess

import pytest

from paper_2507_19427_amd import asm_check as A

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


@pytest.mark.parametrize("paged,q_len,bits", A.PIPELINE_KERNELS)
def test_lowbit_pipeline_registers_stay_untouched_between_load_and_wait(asm_text, paged, q_len, bits):
    A.check_pipeline(A.kernel_body(asm_text, A.lowbit_kernel_name(paged, q_len, bits)), A.OPS_PER_STEP[bits])


def test_no_attention_kernel_uses_scratch_memory(asm_text):
    scratch = {k: v for k, v in A.scratch_bytes(asm_text).items() if "decode_" in k}
    assert len(scratch) == 16        # bf16 / 8 bit / 4 bit x paged or not x one or two query tokens; bf16 x paged or not x three or four
    assert all(v == 0 for v in scratch.values()), scratch


def test_everything_the_build_checks(asm_text):
    A.check_attention_asm(asm_text)


def _snippet(between):
    load = [";;#ASMSTART", "global_load_dwordx4 v[10:13], v[2:3], off", ";;#ASMEND"]
    wait = [";;#ASMSTART", "s_waitcnt vmcnt(5)", ";;#ASMEND"]
    filler = [";;#ASMSTART"] + ["global_load_lds_dwordx4 v[4:5], off"] * 5 + [";;#ASMEND"]
    return wait + load + filler + wait + load + filler + between + wait + ["v_mov_b32_e32 v20, v11"]


def test_the_checker_itself_catches_planted_mistakes():
    A.check_pipeline(_snippet([]))                                   # clean: the copy comes after the wait
    A.check_pipeline(_snippet(["v_add_f32_e32 v21, v14, v15"]))      # clean: other registers
    for bad in ("v_mov_b32_e32 v20, v11",                            # copied
                "v_add_f32_e32 v21, v10, v15",                       # read by arithmetic
                "v_mov_b32_e32 v12, v30",                            # overwritten
                "v_pk_mul_f32 v[40:41], v[12:13], v[2:3]",           # read as part of a register range
                "ds_write_b128 v7, v[10:13]"):                       # stored to LDS
        with pytest.raises(AssertionError, match="touched before its wait"):
            A.check_pipeline(_snippet([bad]))
    with pytest.raises(AssertionError, match="touched by a memory instruction"):
        A.check_pipeline(_snippet(["scratch_store_dwordx4 off, v[10:13], off offset:16"]))   # spilled
    with pytest.raises(AssertionError, match="drains the pipeline"):
        A.check_pipeline(_snippet(["s_waitcnt vmcnt(0)"]))


def test_scratch_directive_parser():
    text = "\n".join(["\t.amdhsa_kernel _ZN3mfa18decode_x", "\t\t.amdhsa_private_segment_fixed_size 24", "\t.end_amdhsa_kernel",
                      "\t.amdhsa_kernel other", "\t\t.amdhsa_private_segment_fixed_size 0", "\t.end_amdhsa_kernel"])
    assert A.scratch_bytes(text) == {"_ZN3mfa18decode_x": 24, "other": 0}
