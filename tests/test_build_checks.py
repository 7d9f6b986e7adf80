"""Host-side checks the build applies to the generated code (CPU only)."""
from paper_2604_26666_amd import build

KERNEL = """
_ZN4fact4attn15attn_fwd_kernelILi128ELi4EEEvNS0_8AttnArgsE: ; @x
\tv_add_f32_e32 v40, v1, v2
{first}
\t;;#ASMSTART
\tv_mfma_f32_16x16x32_bf16 a[0:3], v[4:7], v[8:11], a[0:3]
\t;;#ASMEND
{second}
\ts_endpgm
"""


def findings(first="\ts_nop 0", second="\ts_nop 0"):
    return build.check_asm_mfma_hazards(KERNEL.format(first=first, second=second))


def test_clean_code_has_no_findings():
    assert findings("\tv_add_f32_e32 v20, v1, v2\n\tv_add_f32_e32 v21, v1, v2") == []


def test_vector_write_right_before_an_asm_mfma_operand_is_found():
    assert len(findings("\tv_mov_b32_e32 v5, 0")) == 1                       # one instruction before
    assert len(findings("\tv_mov_b64_e32 v[10:11], v[0:1]\n\ts_nop 0")) == 1   # two before
    assert findings("\tv_mov_b32_e32 v5, 0\n\ts_nop 0\n\ts_nop 0") == []     # three before: accepted


def test_vector_read_of_a_fresh_mfma_result_is_found():
    assert len(findings(second="\tv_accvgpr_read_b32 v30, a1")) == 1
    assert findings(second="\ts_nop 15\n\ts_nop 15\n\tv_accvgpr_read_b32 v30, a1") == []


def test_a_missing_kernel_is_reported():
    assert build.check_asm_mfma_hazards("_ZN4fact11gemm_kernelE: ; @y\n\ts_endpgm\n") != []


def test_wide_store_data_hazard_scan():
    bad = ("\tbuffer_store_dwordx4 v[18:21], v52, s[20:23], s5 offen\n"
           "\tv_add_u32_e32 v19, v1, v2\n")
    assert len(build.check_wide_store_hazards(bad)) == 1
    # a constant scalar offset: the compiler's own hazard pass covers it
    assert build.check_wide_store_hazards(bad.replace(", s5 offen", ", 0 offen")) == []
    # a wait state, a write to other registers, or a narrow store in between: nothing to report
    assert build.check_wide_store_hazards(bad.replace("\tv_add", "\ts_nop 0\n\tv_add")) == []
    assert build.check_wide_store_hazards(bad.replace("v19, v1", "v22, v1")) == []
    assert build.check_wide_store_hazards(bad.replace("dwordx4 v[18:21]", "dwordx2 v[18:19]")) == []
    # the product's generated code, as built, is clean
    import glob, os
    files = glob.glob(os.path.join(os.path.dirname(build.__file__), "_build", "inst*.s"))
    if files:
        for f in files:
            assert build.check_wide_store_hazards(open(f).read()) == [], f


def test_accumulator_register_scan():
    kern = ("_ZN4fact11gemm_kernelE: ; @x\n"
            "\t;;#ASMSTART\n\tv_mfma_f32_16x16x32_bf16 a[0:3], v[2:5], v[6:9], a[0:3]\n\t;;#ASMEND\n"
            "{extra}"
            "\ts_endpgm\n")
    assert build.check_accumulators_untouched(kern.format(extra="\tv_add_f32_e32 v1, v2, v3\n")) == []
    assert len(build.check_accumulators_untouched(kern.format(extra="\tv_accvgpr_write_b32 a5, v1\n"))) == 1
    assert len(build.check_accumulators_untouched(kern.format(extra="\tscratch_load_dwordx4 a[8:11], off, off\n"))) == 1
    assert len(build.check_accumulators_untouched(kern.format(extra="\tv_accvgpr_read_b32 v7, a12\n"))) == 1
