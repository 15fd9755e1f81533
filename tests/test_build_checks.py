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
    # an LDS read landing in the destination, a store of it: reported (the store also as a memory instruction of the
    # compiler's own under a hand-issued load)
    lds = listing(HAND + "\tds_read_b128 v[12:15], v7\n\tglobal_store_dword v[4:5], v11, off\n")
    assert len(check(lds)) == 3


def test_load_from_a_scalar_base_with_a_lane_offset():
    """The form the walking blocks issue their weight loads in (address in scalar registers, a 32-bit offset per lane):
    its destination is tracked like the other form's, and its offset register is an address like any other."""
    check = _load("asm_check").find_inflight_hazards
    hand = "\t;;#ASMSTART\n\tglobal_load_dwordx4 v[10:13], v5, s[2:3]\n\t;;#ASMEND\n"
    assert len(check(listing(hand + "\tv_mov_b32_e32 v12, 0\n\ts_waitcnt vmcnt(0)\n"))) == 1
    assert check(listing(hand + "\ts_waitcnt vmcnt(0)\n\tv_mov_b32_e32 v12, 0\n")) == []
    # the offset of a second load taken from the first one's destination while that is in flight
    found = check(listing(hand + "\t;;#ASMSTART\n\tglobal_load_dwordx4 v[20:23], v11, s[2:3] nt\n\t;;#ASMEND\n\ts_waitcnt vmcnt(0)\n"))
    assert len(found) == 1 and "reads v[11]" in found[0]


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


def test_compiler_emitted_memory_instruction_under_hand_issued_loads():
    """A vector-memory instruction the compiler emitted itself while a hand-issued one is in flight would be one more
    'younger operation' than the hand-counted waits allow for: reported.  Before the first hand-issued operation and
    after the wait that retires the last one, the compiler's own loads and stores are fine."""
    check = _load("asm_check").find_inflight_hazards
    own = "\tglobal_load_dword v9, v[2:3], off\n"
    assert check(listing(own + "\ts_waitcnt vmcnt(0)\n" + HAND + "\ts_waitcnt vmcnt(0)\n\tglobal_store_dwordx4 v[4:5], v[10:13], off\n")) == []
    found = check(listing(HAND + own + "\ts_waitcnt vmcnt(0)\n"))
    assert len(found) == 1 and "global_load_dword was emitted by the compiler" in found[0]
    # a copy into LDS issued by hand counts as in flight too; a store under it is reported
    lds = "\t;;#ASMSTART\n\ts_mov_b32 m0, s31\n\ts_nop 0\n\tglobal_load_lds_dwordx4 v[128:129], off\n\t;;#ASMEND\n"
    found = check(listing(lds + "\tglobal_store_dword v[4:5], v9, off\n\ts_waitcnt vmcnt(0)\n"))
    assert len(found) == 1 and "global_store_dword was emitted by the compiler" in found[0]
    # the compiler's load is older than the hand-issued one: every wait that covers the latter covers it as well
    assert check(listing(own + HAND + "\ts_waitcnt vmcnt(0)\n")) == []


def _loop(body):
    return listing("\ts_mov_b32 s0, 0\n.LBB0_1:\n" + body + "\ts_cbranch_scc1 .LBB0_1\n\ts_endpgm\n")


def _hand(text):
    return "\t;;#ASMSTART\n\t" + text + "\n\t;;#ASMEND\n"


def test_wait_recount_ring_of_weight_tiles():
    """Main loop with a ring of two weight registers, each reloaded right after its use: the tile multiplied in a
    substep was requested two substeps earlier, one younger load may stay in flight -> vmcnt(1).  vmcnt(2) lets
    the matrix instruction read a register whose load may not have landed."""
    check = _load("asm_check").find_wait_count_errors

    def body(n):
        return (_hand("s_waitcnt vmcnt(%d)" % n) + "\tv_mfma_f32_32x32x16_bf16 v[50:65], v[30:33], v[10:13], v[50:65]\n"
                + _hand("global_load_dwordx4 v[10:13], v[2:3], off nt")
                + _hand("s_waitcnt vmcnt(%d)" % n) + "\tv_mfma_f32_32x32x16_bf16 v[50:65], v[30:33], v[14:17], v[50:65]\n"
                + _hand("global_load_dwordx4 v[14:17], v[4:5], off nt"))
    assert check(_loop(body(1))) == []
    assert check(_loop(body(0))) == []           # waits for more than needed: slow, not wrong
    found = check(_loop(body(2)))
    assert found and "reads v[10, 11, 12, 13] before a wait has retired the hand-issued load" in found[0]


def test_wait_recount_activation_stages():
    """Main loop of one K step per walk: a weight load, two copies into LDS that make up a stage (closed by the
    'activation stage issued' mark), and the wait that opens a stage.  With a ring of 4 the stage to open was closed
    two marks before the last one at that point: at the wait the youngest operations are the 3 of the previous step and
    the weight load of this one, so vmcnt(4) is exact, vmcnt(5) leaves one of the stage's copies in flight; with a
    ring of 3 the stage to open is the one closed last and vmcnt(1) is the most that is allowed."""
    check = _load("asm_check").find_wait_count_errors
    copy = _hand("s_mov_b32 m0, s31\n\ts_nop 0\n\tglobal_load_lds_dwordx4 v[128:129], off")

    def body(n, ring):
        return (_hand("global_load_dwordx4 v[10:13], v[2:3], off nt")
                + _hand("s_waitcnt vmcnt(%d) ; hmoe: opens an activation stage, ring of %d" % (n, ring)) + "\ts_barrier\n"
                + copy + copy + _hand("; hmoe: activation stage issued"))
    assert check(_loop(body(4, 4))) == []
    found = check(_loop(body(5, 4)))
    assert len(found) == 1 and "opens an activation stage while 1 of its copies into LDS" in found[0]
    assert check(_loop(body(1, 3))) == []
    assert check(_loop(body(2, 3))) != []
    # a loop without hand-issued operations is not looked at
    assert check(_loop("\tglobal_load_dword v9, v[2:3], off\n\ts_waitcnt vmcnt(0)\n")) == []


def test_load_in_flight_where_paths_merge():
    """What faulted once: a block that issues its next tile's loads before its epilogue.  Where the path with the
    loads in flight met one without, the compiler copied the ring registers and reused them for a store address."""
    check = _load("asm_check").find_inflight_hazards
    copy = "\tv_mov_b64_e32 v[20:21], v[10:11]\n\tv_lshl_add_u64 v[10:11], v[4:5], 0, s[2:3]\n\ts_waitcnt vmcnt(0)\n"
    # a clean path falls into the label, a branch brings the load: the copy and the reuse behind the label are reported
    merged = listing(HAND + "\ts_branch .LBB0_3\n.LBB0_2:\n\ts_nop 0\n.LBB0_3:\n" + copy)
    found = check(merged)
    assert len(found) == 2 and "v_mov_b64_e32 reads v[10, 11]" in found[0] and "writes v[10, 11]" in found[1]
    # the same with the wait first: clean
    assert check(listing(HAND + "\ts_branch .LBB0_3\n.LBB0_2:\n\ts_nop 0\n.LBB0_3:\n\ts_waitcnt vmcnt(0)\n" + copy)) == []
    # a branch back to text that was scanned without the load: reported, whatever that text does ...
    back = listing(".LBB0_1:\n\tv_mov_b32_e32 v30, 0\n\ts_branch .LBB0_3\n.LBB0_2:\n" + HAND + "\ts_branch .LBB0_1\n"
                   ".LBB0_3:\n\ts_waitcnt vmcnt(0)\n")
    found = check(back)
    assert len(found) == 1 and "goes back to .LBB0_1" in found[0]
    # ... unless that text starts by waiting for everything (the shared tail of several paths)
    tail = listing(".LBB0_1:\n\ts_or_b64 exec, exec, s[0:1]\n\ts_waitcnt lgkmcnt(0)\n\ts_waitcnt vmcnt(0)\n\ts_branch .LBB0_3\n.LBB0_2:\n"
                   + HAND + "\ts_branch .LBB0_1\n.LBB0_3:\n\ts_endpgm\n")
    assert check(tail) == []
    # the closing branch of a main loop is where loads are meant to be in flight
    loop = listing(".LBB0_1:\n\ts_waitcnt vmcnt(0)\n\tv_mfma_f32_32x32x16_bf16 v[50:65], v[10:13], v[44:47], v[50:65]\n" + HAND
                   + "\ts_cbranch_scc1 .LBB0_1\n\ts_waitcnt vmcnt(0)\n")
    assert check(loop) == []


def test_wait_recount_skips_what_is_not_a_loop():
    """A stretch from a label to a later branch back to it is walked as a loop only if it holds no other such stretch
    and no unconditional branch: a block that works through several tiles has its K loops inside a tile loop, and the
    compiler lays single K steps out in front of code that jumps back to them once."""
    check = _load("asm_check").find_wait_count_errors
    step = ("\ts_waitcnt vmcnt(1)\n\tv_mfma_f32_32x32x16_bf16 v[50:65], v[10:13], v[44:47], v[50:65]\n" + HAND)
    # one K step per walk with a ring of two would need vmcnt(1) to retire the load it reads: as a loop it is wrong ...
    assert check(listing(".LBB0_1:\n" + step + "\ts_cbranch_scc1 .LBB0_1\n")) != []
    # ... but not if the stretch leaves through an unconditional branch before its end (a step laid out on its own)
    assert check(listing(".LBB0_1:\n" + step + "\ts_branch .LBB0_3\n.LBB0_2:\n\ts_nop 0\n\ts_cbranch_scc1 .LBB0_1\n.LBB0_3:\n")) == []
    # ... and an outer loop around a correct inner one is not walked as one body
    good = ("\ts_waitcnt vmcnt(0)\n\tv_mfma_f32_32x32x16_bf16 v[50:65], v[10:13], v[44:47], v[50:65]\n" + HAND)
    nested = listing(".LBB0_0:\n" + HAND.replace("v[10:13]", "v[30:33]") + ".LBB0_1:\n" + good + "\ts_cbranch_scc1 .LBB0_1\n"
                     "\tv_mfma_f32_32x32x16_bf16 v[50:65], v[30:33], v[44:47], v[50:65]\n\ts_cbranch_scc1 .LBB0_0\n")
    assert check(nested) == []
