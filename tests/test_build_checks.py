"""Host-only tests of the build's checks on generated assembly (paper_2603_15619_amd/build.py):
each check is run on small hand-written assembly texts, one that must pass and ones that carry
exactly the mistake the check exists for."""
import pytest

from paper_2603_15619_amd import build as B

GOOD_ACC = """\
_Z6kernelv:
\tv_accvgpr_write_b32 a3, v1
\t;;#ASMSTART
\t; MODA_ACC_REGISTERS_ACQUIRED
\t;;#ASMEND
.LBB0_1:
\t;;#ASMSTART
\tv_mfma_f32_32x32x16_bf16 a[64:79], a[32:35], v[0:3], a[64:79]
\t;;#ASMEND
\tv_add_f32_e32 v1, v2, v3
\ts_cbranch_scc1 .LBB0_1
\t;;#ASMSTART
\t; MODA_ACC_REGISTERS_RELEASED
\t;;#ASMEND
\tv_accvgpr_read_b32 v5, a7
\ts_endpgm
.Lfunc_end0:
"""


def check(tmp_path, text):
    f = tmp_path / "k.s"
    f.write_text(text)
    for name, body in B._kernel_bodies(str(f)):
        B._check_kernel(str(f), name, body)


def test_named_register_region_accepts_clean_code(tmp_path):
    check(tmp_path, GOOD_ACC)


def test_compiler_use_inside_owned_region_is_rejected(tmp_path):
    bad = GOOD_ACC.replace("\tv_add_f32_e32 v1, v2, v3\n", "\tv_accvgpr_write_b32 a9, v1\n")
    with pytest.raises(RuntimeError, match="compiler-allocated accumulation register"):
        check(tmp_path, bad)


def test_named_use_after_release_is_rejected(tmp_path):
    bad = GOOD_ACC.replace("\tv_accvgpr_read_b32 v5, a7\n",
                           "\t;;#ASMSTART\n\tv_accvgpr_read_b32 v5, a7\n\t;;#ASMEND\n")
    with pytest.raises(RuntimeError, match="outside the owned region"):
        check(tmp_path, bad)


def test_missing_marker_is_rejected(tmp_path):
    bad = GOOD_ACC.replace("\t; MODA_ACC_REGISTERS_RELEASED\n", "\t; nothing\n")
    with pytest.raises(RuntimeError, match="expected exactly one"):
        check(tmp_path, bad)


SCRATCH = """\
_Z9my_kernelv:
\tscratch_store_dword off, v1, off
.LBB0_1:                                ; =>This Inner Loop Header: Depth=1
\tv_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], v[20:23], v[0:15]
%s
\ts_cbranch_scc1 .LBB0_1
; %%bb.2:
\tscratch_load_dword v1, off, off
.LBB0_3:                                ; =>This Inner Loop Header: Depth=1
\tscratch_load_dword v2, off, off
\ts_cbranch_scc1 .LBB0_3
\ts_endpgm
.Lfunc_end0:
"""


def test_scratch_outside_key_loops_is_accepted(tmp_path):
    f = tmp_path / "s.s"
    f.write_text(SCRATCH % "\tv_add_f32_e32 v1, v2, v3")
    B.scan_scratch_in_key_loops(str(f), "my_kernel")


def test_scratch_inside_a_key_loop_is_rejected(tmp_path):
    f = tmp_path / "s.s"
    f.write_text(SCRATCH % "\tscratch_load_dword v3, off, off offset:4")
    with pytest.raises(RuntimeError, match="inside a key loop"):
        B.scan_scratch_in_key_loops(str(f), "my_kernel")
    with pytest.raises(RuntimeError, match="no kernel named"):
        B.scan_scratch_in_key_loops(str(f), "other_kernel")
