"""The build's two nets under the hand-scheduled kernels, on hand-written listings: kernels that use private
memory are refused, and a register of a load issued from inline assembly may not be written or used as an
address before the wait that covers it."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _load(name):
    spec = importlib.util.spec_from_file_location(name, os.path.join(ROOT, "paper_2504_05897_amd", name + ".py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def listing(body):
    return "_Z6kernelv:\n" + body + ".Lfunc_end0:\n"


HAND = "\t;;#ASMSTART\n\tglobal_load_dwordx4 v[10:13], v[2:3], off nt\n\t;;#ASMEND\n"


def test_register_of_a_load_in_flight():
    check = _load("asm_check").find_inflight_hazards
    # the destination rebuilt as the next address, then loaded into again: both reported
    bad = listing(HAND + "\tv_lshl_add_u64 v[10:11], v[4:5], 0, s[2:3]\n"
                  "\t;;#ASMSTART\n\tglobal_load_dwordx4 v[10:13], v[10:11], off nt\n\t;;#ASMEND\n\ts_waitcnt vmcnt(0)\n")
    found = check(bad)
    assert len(found) == 3 and "v_lshl_add_u64 writes v[10, 11]" in found[0] and "reads v[10, 11]" in found[2]
    # the same after a wait that covers the first load: clean
    good = listing(HAND + "\ts_waitcnt vmcnt(0)\n\tv_lshl_add_u64 v[10:11], v[4:5], 0, s[2:3]\n"
                   "\t;;#ASMSTART\n\tglobal_load_dwordx4 v[10:13], v[10:11], off nt\n\t;;#ASMEND\n\ts_waitcnt vmcnt(0)\n")
    assert check(good) == []
    # vmcnt(1) retires all but the youngest: the first load has landed, the second has not
    two = listing(HAND + "\t;;#ASMSTART\n\tglobal_load_dwordx4 v[20:23], v[2:3], off\n\t;;#ASMEND\n\ts_waitcnt vmcnt(1)\n"
                  "\tv_mov_b32_e32 v10, 0\n\tv_mov_b32_e32 v21, 0\n")
    found = check(two)
    assert len(found) == 1 and "v_mov_b32_e32 writes v[21]" in found[0]
    # a load the compiler issued itself is its own business; reads by matrix instructions are not checked; other
    # registers are free
    own = listing("\tglobal_load_dwordx4 v[10:13], v[2:3], off\n\tv_mov_b32_e32 v10, 0\n" + HAND.replace("v[10:13]", "v[30:33]")
                  + "\tv_mfma_f32_32x32x16_bf16 v[50:65], v[30:33], v[44:47], v[50:65]\n\tds_read_b128 v[40:43], v7\n"
                  "\ts_waitcnt vmcnt(0)\n")
    assert check(own) == []
    # a copy of a destination into the accumulation registers before the wait: reported
    copy = listing(HAND + "\tv_accvgpr_write_b32 a4, v11\n\ts_waitcnt vmcnt(0)\n")
    assert len(check(copy)) == 1 and "v_accvgpr_write_b32 reads v[11]" in check(copy)[0]
    # an LDS read landing in the destination, a store of it: reported
    lds = listing(HAND + "\tds_read_b128 v[12:15], v7\n\tglobal_store_dword v[4:5], v11, off\n")
    assert len(check(lds)) == 2


def test_labels_without_fall_through():
    check = _load("asm_check").find_inflight_hazards
    tail = "\tv_mov_b32_e32 v10, 0\n\ts_waitcnt vmcnt(0)\n"
    # the text behind an unconditional branch is another path's start: the load above it is not in flight there
    assert check(listing(HAND + "\ts_branch .LBB0_9\n.LBB0_3:\n" + tail + ".LBB0_9:\n\ts_waitcnt vmcnt(0)\n")) == []
    # ... unless a branch seen earlier jumps to it with the load in flight
    found = check(listing(HAND + "\ts_cbranch_scc1 .LBB0_3\n\ts_waitcnt vmcnt(0)\n\ts_branch .LBB0_9\n.LBB0_3:\n" + tail
                          + ".LBB0_9:\n\ts_waitcnt vmcnt(0)\n"))
    assert len(found) == 1 and "v_mov_b32_e32 writes v[10]" in found[0]
    # a label that execution falls into keeps the queue
    assert len(check(listing(HAND + ".LBB0_3:\n" + tail))) == 1
    # behind a conditional branch execution falls through
    assert len(check(listing(HAND + "\ts_cbranch_scc1 .LBB0_9\n" + tail + ".LBB0_9:\n\ts_waitcnt vmcnt(0)\n"))) == 1


def test_private_memory_remarks():
    build = _load("build")
    remarks = ("a.hip:5:0: remark: Function Name: _Z1av [-Rpass-analysis=kernel-resource-usage]\n"
               "a.hip:5:0: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n"
               "a.hip:9:0: remark: Function Name: _Z1bv [-Rpass-analysis=kernel-resource-usage]\n"
               "a.hip:9:0: remark:     VGPRs: 256 [-Rpass-analysis=kernel-resource-usage]\n"
               "a.hip:9:0: remark:     ScratchSize [bytes/lane]: 64 [-Rpass-analysis=kernel-resource-usage]\n")
    assert build.kernels_with_scratch(remarks) == ["_Z1bv"]
    assert build.kernels_with_scratch(remarks.replace(": 64", ": 0")) == []
