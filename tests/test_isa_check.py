"""The build-time assembly scan (host logic): a consumer of a matrix-core result that sits too close on ANY path is
reported, padded or same-block-late consumers and dependent matrix instructions are not."""
from paper_2505_11157_amd import isa_check

HEAD = "_Z6kernelv:\n"
MFMA = "\tv_mfma_f32_16x16x32_bf16 v[130:133], v[166:169], v[18:21], v[158:161]\n"


def test_consumer_behind_taken_branch_is_found():
    asm = (HEAD + MFMA + "\ts_cbranch_scc1 .LBB0_2\n" + "".join(f"\tv_add_u32_e32 v{i}, 1, v{i}\n" for i in range(1, 12)) +
           ".LBB0_2:\n\tv_mul_f32_e32 v157, v38, v130\n\ts_endpgm\n")
    found = isa_check.scan(asm)
    assert len(found) == 1 and "after 1 of 8" in found[0] and "v_mul_f32_e32 v157" in found[0]


def test_padded_and_late_consumers_pass():
    late = HEAD + MFMA + "\ts_nop 6\n\tv_mov_b32_e32 v1, v2\n\tv_mul_f32_e32 v157, v38, v130\n\ts_endpgm\n"
    assert isa_check.scan(late) == []
    both = (HEAD + MFMA + "\ts_nop 3\n\ts_cbranch_scc1 .LBB0_2\n\tv_mov_b32_e32 v1, v2\n.LBB0_2:\n\ts_nop 2\n"
            "\tv_mul_f32_e32 v157, v38, v131\n\ts_endpgm\n")
    assert isa_check.scan(both) == []


def test_one_state_short_is_found_and_chained_mfma_is_not():
    short = HEAD + MFMA + "\ts_nop 5\n\tds_write_b32 v16, v133\n\ts_endpgm\n"
    assert len(isa_check.scan(short)) == 1
    chain = HEAD + MFMA + "\tv_mfma_f32_16x16x32_bf16 v[130:133], v[166:169], v[22:25], v[130:133]\n\ts_nop 7\n\tv_mov_b32_e32 v1, v130\n\ts_endpgm\n"
    assert isa_check.scan(chain) == []


def test_wait_states_by_shape():
    f32 = HEAD + "\tv_mfma_f32_32x32x2_f32 v[0:15], v35, v21, v[0:15]\n\ts_nop 7\n\ts_nop 7\n\tv_mov_b32_e32 v20, v15\n\ts_endpgm\n"
    assert len(isa_check.scan(f32)) == 1            # 16 of 18
    f32ok = HEAD + "\tv_mfma_f32_32x32x2_f32 v[0:15], v35, v21, v[0:15]\n\ts_nop 7\n\ts_nop 7\n\ts_nop 1\n\tv_mov_b32_e32 v20, v15\n\ts_endpgm\n"
    assert isa_check.scan(f32ok) == []
