"""The kernels issue some loads and stores from inline assembly with a scalar base address.  The compiler
pads the wait states a vector-memory instruction needs after a VECTOR instruction wrote one of its
scalar operands only for its own instructions, not inside an asm block: these tests pin the checker that
looks for such places in the generated gfx950 assembly, and run it over the kernel sources."""
import pytest

from paper_2504_04704_amd import isa_check

HEAD = "_ZN5lagkv6kernelEv:\n"


def _sites(body):
    return isa_check.scan(HEAD + body)


def test_checker_finds_a_store_behind_a_lane_read_of_its_base():
    # the sequence that once sent a score store to a stale address: base re-read from a vector register, 0 wait states
    s = _sites("\tv_readlane_b32 s8, v127, 6\n\tv_readlane_b32 s9, v127, 7\n\t;;#ASMSTART\n"
               "\tglobal_store_dword v95, v0, s[8:9]\n\t;;#ASMEND\n")
    assert len(s) == 1 and s[0].wait_states == 0 and s[0].function == "_ZN5lagkv6kernelEv"
    # four instructions in between are still one wait state short
    s = _sites("\tv_readfirstlane_b32 s4, v1\n" + "\tv_add_f32_e32 v2, v2, v3\n" * 4 + "\t;;#ASMSTART\n"
               "\tglobal_load_lds_dwordx4 v9, s[4:5] nt\n\t;;#ASMEND\n")
    assert len(s) == 1 and s[0].wait_states == 4
    # a compare in the short encoding writes vcc
    s = _sites("\tv_cmp_gt_u32_e32 vcc, v1, v2\n\t;;#ASMSTART\n\tglobal_store_dword v1, v0, vcc\n\t;;#ASMEND\n")
    assert len(s) == 1


def test_checker_accepts_padded_and_scalar_written_bases():
    ok = ["\tv_readlane_b32 s9, v127, 7\n\t;;#ASMSTART\n\ts_nop 4\n\tglobal_store_dword v95, v0, s[8:9]\n\t;;#ASMEND\n",
          "\tv_readlane_b32 s9, v127, 7\n" + "\tv_add_f32_e32 v2, v2, v3\n" * 5 +
          "\t;;#ASMSTART\n\tglobal_store_dword v95, v0, s[8:9]\n\t;;#ASMEND\n",
          # the base copied by a scalar move inside the block: the store reads registers no vector instruction wrote
          "\tv_readlane_b32 s11, v127, 0\n\t;;#ASMSTART\n\ts_mov_b64 s[8:9], s[10:11]\n"
          "\tglobal_store_dword v96, v1, s[8:9]\n\t;;#ASMEND\n",
          "\ts_add_u32 s8, s8, s20\n\ts_addc_u32 s9, s9, 0\n\t;;#ASMSTART\n\tglobal_store_dwordx4 v1, v[2:5], s[8:9] sc0 nt\n\t;;#ASMEND\n",
          # the compiler's own instructions are its business
          "\tv_readlane_b32 s9, v127, 7\n\tglobal_store_dword v95, v0, s[8:9]\n",
          # vector operands only
          "\tv_mov_b32_e32 v1, s3\n\t;;#ASMSTART\n\tglobal_store_dwordx4 v[0:1], v[2:5], off sc0 nt\n\t;;#ASMEND\n"]
    for body in ok:
        assert _sites(body) == []
    # a scalar move that rewrites a register a vector instruction wrote just before does not end the search
    s = _sites("\tv_readlane_b32 s3, v127, 51\n\t;;#ASMSTART\n\ts_mov_b64 s[2:3], s[10:11]\n"
               "\tglobal_store_dword v79, v0, s[2:3]\n\t;;#ASMEND\n")
    assert len(s) == 1 and s[0].wait_states == 1


def test_checker_finds_a_vector_write_of_the_data_of_a_wide_store():
    store = "\t;;#ASMSTART\n\tglobal_store_dwordx4 v130, v[30:33], s[10:11] sc0 nt\n\t;;#ASMEND\n"
    find = lambda body: isa_check.scan_store_data(HEAD + body)
    assert len(find(store + "\tv_mov_b32_e32 v31, v2\n")) == 1
    assert len(find(store + "\ts_or_b64 exec, exec, s[8:9]\n\tv_lshlrev_b32_e32 v33, 2, v1\n")) == 1
    assert find(store + "\ts_or_b64 exec, exec, s[8:9]\n\tv_cmp_lt_i32_e32 vcc, -1, v131\n\tv_mov_b32_e32 v31, v2\n") == []
    assert find(store + "\ts_nop 1\n\tv_mov_b32_e32 v31, v2\n") == []
    assert find(store + "\tv_mov_b32_e32 v34, v2\n\tv_mov_b32_e32 v29, v2\n") == []          # other registers
    assert find(store + "\tds_read_b128 v[30:33], v5\n") == []                                   # not a vector-ALU write
    assert find("\t;;#ASMSTART\n\tglobal_store_dword v95, v0, s[8:9]\n\t;;#ASMEND\n\tv_mov_b32_e32 v0, v2\n") == []   # 32 bits


def test_kernel_sources_have_no_such_place():
    found = isa_check.check_sources()
    assert set(found) == set(isa_check.KERNEL_SOURCES)
    for src, sites in found.items():
        assert sites == [], f"{src}: {sites[:3]}"
