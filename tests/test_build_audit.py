"""The build-time audit of asynchronous loads (paper_2409_17066_amd/check_async.py) on hand-written assembly snippets:
it must flag a register that is read, copied or overwritten while an inline-assembly load into it is pending, and
accept the same code once a counted wait has retired the load."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, os.path.join(ROOT, "paper_2409_17066_amd"))
import check_async  # noqa: E402

HEAD = "_Z6kernelv:\n"
TAIL = "\ts_endpgm\n"


def _asm(body):
    return HEAD + "".join("\t%s\n" % line for line in body) + TAIL


def test_use_before_wait_is_flagged():
    bad = _asm(["#ASMSTART", "buffer_load_dwordx3 v[4:6], v1, s[8:11], 0 offen", "#ASMEND", "v_mov_b32_e32 v9, v5"])
    found = check_async.audit(bad)
    assert len(found) == 1 and found[0][3] == [5]


def test_counted_wait_retires_the_oldest_loads_only():
    body = ["#ASMSTART", "buffer_load_dwordx3 v[4:6], v1, s[8:11], 0 offen", "#ASMEND",
            "#ASMSTART", "buffer_load_dwordx4 v[10:13], v1, s[8:11], 0 offen offset:16", "#ASMEND",
            "#ASMSTART", "s_waitcnt vmcnt(1)", "#ASMEND",
            "v_add_u32_e32 v20, v4, v6"]
    assert check_async.audit(_asm(body)) == []                       # the first load has landed
    assert len(check_async.audit(_asm(body + ["v_mov_b32_e32 v21, v12"]))) == 1   # the second has not
    assert check_async.audit(_asm(body + ["#ASMSTART", "s_waitcnt vmcnt(0)", "#ASMEND", "v_mov_b32_e32 v21, v12"])) == []


def test_compiler_loads_count_in_the_queue_but_are_not_tracked():
    body = ["#ASMSTART", "buffer_load_dwordx2 v[2:3], v1, s[8:11], 0 offen", "#ASMEND",
            "buffer_load_dword v30, v1, s[8:11], 0 offen",            # the compiler's own: it waits for it itself
            "#ASMSTART", "s_waitcnt vmcnt(1)", "#ASMEND",
            "v_mov_b32_e32 v7, v2", "v_mov_b32_e32 v8, v30"]
    assert check_async.audit(_asm(body)) == []


def test_lds_reads_from_assembly_follow_lgkmcnt():
    body = ["#ASMSTART", "ds_read_b128 v[40:43], v1", "#ASMEND", "v_mov_b32_e32 v7, v41"]
    assert len(check_async.audit(_asm(body))) == 1
    ok = ["#ASMSTART", "ds_read_b128 v[40:43], v1", "#ASMEND", "#ASMSTART", "s_waitcnt lgkmcnt(0)", "#ASMEND", "v_mov_b32_e32 v7, v41"]
    assert check_async.audit(_asm(ok)) == []


def test_overwriting_a_pending_register_is_flagged_and_pending_loads_cross_labels():
    bad = _asm(["#ASMSTART", "buffer_load_dword v4, v1, s[8:11], 0 offen", "#ASMEND", "v_mov_b32_e32 v4, 0"])
    assert len(check_async.audit(bad)) == 1
    # a label does not retire anything: the queue is carried into the next block (the single-block pass starts afresh)
    split = _asm(["#ASMSTART", "buffer_load_dword v4, v1, s[8:11], 0 offen", "#ASMEND", ".LBB0_1:", "v_mov_b32_e32 v9, v4"])
    assert len(check_async.audit(split)) == 1 and check_async.audit_blocks(split) == []


def test_a_copy_at_a_loop_back_edge_is_found():
    """The mistake seen in practice: a ring slot refilled at the end of the loop body, copied by the compiler at the top of
    the next round before the counted wait."""
    loop = ["#ASMSTART", "buffer_load_dword v4, v1, s[8:11], 0 offen", "#ASMEND",
            ".LBB0_1:",
            "v_mov_b32_e32 v9, v4",                                    # second trip through the loop and later: v4 was refilled below
            "#ASMSTART", "s_waitcnt vmcnt(0)", "#ASMEND",
            "v_add_u32_e32 v10, v4, v10",
            "#ASMSTART", "buffer_load_dword v4, v1, s[8:11], 0 offen", "#ASMEND",
            "s_cbranch_scc1 .LBB0_1"]
    found = check_async.audit(_asm(loop))
    assert [f[2] for f in found] == ["v_mov_b32_e32 v9, v4"]
    fixed = [l for l in loop if l != "v_mov_b32_e32 v9, v4"]
    assert check_async.audit(_asm(fixed)) == []


def test_a_branch_around_the_wait_is_found():
    body = ["#ASMSTART", "ds_read_b128 v[40:43], v1", "#ASMEND",
            "s_cbranch_scc1 .LBB0_2",
            "#ASMSTART", "s_waitcnt lgkmcnt(0)", "#ASMEND",
            "v_mov_b32_e32 v7, v41",
            ".LBB0_2:",
            "v_mov_b32_e32 v40, 0"]                                    # on the taken path the read is still on its way
    found = check_async.audit(_asm(body))
    assert [f[2] for f in found] == ["v_mov_b32_e32 v40, 0"]


def test_a_younger_load_of_the_same_queue_may_reuse_the_destination():
    same = ["#ASMSTART", "ds_read_b128 v[40:43], v1", "#ASMEND", "#ASMSTART", "ds_read_b128 v[40:43], v2", "#ASMEND"]
    assert check_async.audit(_asm(same)) == []                         # LDS reads land in order: the younger value stays
    other = ["#ASMSTART", "ds_read_b128 v[40:43], v1", "#ASMEND", "buffer_load_dwordx4 v[40:43], v2, s[8:11], 0 offen"]
    assert len(check_async.audit(_asm(other))) == 1                    # another queue: no order between the two
    addr = ["#ASMSTART", "ds_read_b32 v40, v1", "#ASMEND", "#ASMSTART", "ds_read_b32 v41, v40", "#ASMEND"]
    assert len(check_async.audit(_asm(addr))) == 1                     # an address register must have landed
