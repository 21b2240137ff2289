"""The build's scan of the GEMM assembly: accumulation-register accesses too close behind an MFMA are reported."""
from paper_2503_12668_amd.build import scan_mfma_hazards, kMfmaDistance

HEAD = "_ZN3zo24kernEv:\n"
MFMA = "\tv_mfma_f32_16x16x32_bf16 a[0:3], v[0:3], v[4:7], a[0:3]\n"


def test_read_right_behind_an_mfma_is_reported():
    bad = scan_mfma_hazards(HEAD + MFMA + "\tv_accvgpr_read_b32 v9, a1\n")
    assert len(bad) == 1 and bad[0][0] == "_ZN3zo24kernEv" and bad[0][3] == 0
    # a store straight from an accumulation register counts as well
    assert scan_mfma_hazards(HEAD + MFMA + "\tds_write_b128 v1, a[0:3]\n")


def test_distance_by_nops_or_instructions_clears_it():
    assert not scan_mfma_hazards(HEAD + MFMA + "\ts_nop 15\n\ts_nop 15\n\tv_accvgpr_read_b32 v9, a1\n")
    filler = "\tv_add_u32_e32 v1, v2, v3\n" * kMfmaDistance
    assert not scan_mfma_hazards(HEAD + MFMA + filler + "\tv_accvgpr_read_b32 v9, a1\n")
    assert scan_mfma_hazards(HEAD + MFMA + "\tv_add_u32_e32 v1, v2, v3\n" * (kMfmaDistance - 1) + "\tv_accvgpr_mov_b32 a7, a1\n")


def test_mfma_chains_and_plain_vector_code_are_fine():
    assert not scan_mfma_hazards(HEAD + MFMA * 8 + "\tds_read_b128 v[0:3], v9 offset:2048\n\ts_waitcnt lgkmcnt(0)\n" + MFMA)
