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


def test_overwriting_a_pending_register_is_flagged_and_blocks_are_separate():
    bad = _asm(["#ASMSTART", "buffer_load_dword v4, v1, s[8:11], 0 offen", "#ASMEND", "v_mov_b32_e32 v4, 0"])
    assert len(check_async.audit(bad)) == 1
    # the audit is block-local by design: a label starts with a clean slate
    split = _asm(["#ASMSTART", "buffer_load_dword v4, v1, s[8:11], 0 offen", "#ASMEND", ".LBB0_1:", "v_mov_b32_e32 v9, v4"])
    assert check_async.audit(split) == []
