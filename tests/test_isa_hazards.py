"""The compiled kernels hold no hazard around their hand-written instructions (see paper_2505_23949_amd/isa_check.py).
CPU only: hipcc cross-compiles the listings; nothing runs."""
from paper_2505_23949_amd import isa_check

PLANTED_H1 = """
kernel:
\tv_add_f32_e32 v40, v40, v42
\tv_rcp_f32_e32 v40, v40
\tv_min_f32 v40, v40, v85
\ts_nop 0
\tv_mul_f32_e32 v41, v41, v40
"""
CLEAN_H1 = PLANTED_H1.replace("\tv_min_f32 v40, v40, v85\n\ts_nop 0\n", "\ts_nop 0\n\tv_min_f32 v40, v40, v85\n")
PLANTED_H2 = """
kernel:
\tv_min_f64 v[2:3], v[2:3], -v[6:7]
\tv_add_f32_e32 v9, v9, v10
\tv_mov_b32_dpp v4, v3 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf bound_ctrl:1
"""
CLEAN_H2 = PLANTED_H2.replace("\tv_add_f32_e32 v9, v9, v10\n", "\tv_add_f32_e32 v9, v9, v10\n\ts_nop 0\n")


def test_scanner_finds_planted_hazards_and_only_those():
    assert len(isa_check.hazards(PLANTED_H1)) == 1 and isa_check.hazards(PLANTED_H1)[0].startswith("H1")
    assert isa_check.hazards(CLEAN_H1) == []
    assert len(isa_check.hazards(PLANTED_H2)) == 1 and isa_check.hazards(PLANTED_H2)[0].startswith("H2")
    assert isa_check.hazards(CLEAN_H2) == []
    # the compiler's own instructions (printed with their encoding suffix) are its business
    assert isa_check.hazards(PLANTED_H1.replace("v_min_f32 ", "v_min_f32_e32 ")) == []


def test_no_hazard_in_the_library():
    problems = isa_check.check_all()
    assert problems == [], "\n".join(problems)
