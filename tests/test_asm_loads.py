"""The attention kernels issue some loads from inline assembly, which the compiler keeps no count for: every wait for
them is placed by hand in the source.  This test compiles the kernels to assembly (no GPU needed) and checks, on every
path through each kernel, that no register is read or written while such a load into it may still be in flight.  The
checker itself is first shown to flag planted mistakes in small hand-written listings."""
import os
import subprocess
import tempfile

import pytest

from asm_wait_check import check, split_kernels
from paper_2601_01298_amd import build as ws_build


def listing(text):
    return [(i, "\t" + t if not t.endswith(":") else t) for i, t in enumerate(text.strip().split("\n"), 1)]


ASM_LOAD = ";;#ASMSTART\nglobal_load_dword v5, v1, s[2:3]\n;;#ASMEND"


def test_checker_accepts_a_waited_load():
    v, n = check(listing(f"{ASM_LOAD}\nv_add_u32_e32 v2, 1, v2\ns_waitcnt vmcnt(0)\nv_add_u32_e32 v6, v5, v2\ns_endpgm"))
    assert v == [] and n == 1


def test_checker_flags_a_read_before_the_wait():
    v, _ = check(listing(f"{ASM_LOAD}\nv_add_u32_e32 v6, v5, v2\ns_waitcnt vmcnt(0)\ns_endpgm"))
    assert [x[:2] for x in v] == [(2, 4)]


def test_checker_flags_a_register_reused_while_the_load_is_in_flight():
    # the situation after a loop whose last iteration asked for data nobody reads: the register is given to another value
    v, _ = check(listing(f"{ASM_LOAD}\ns_waitcnt lgkmcnt(0)\ns_barrier\nv_lshl_or_b32 v5, v70, 2, s2\nds_write_b32 v5, v9\ns_endpgm"))
    assert (2, 7) in [x[:2] for x in v]


def test_checker_counts_newer_operations_behind_a_partial_wait():
    ok = f"{ASM_LOAD}\nglobal_load_lds_dwordx4 v7, s[4:5]\nglobal_load_lds_dwordx4 v8, s[4:5]\ns_waitcnt vmcnt(2)\nv_mov_b32_e32 v9, v5\ns_endpgm"
    bad = ok.replace("vmcnt(2)", "vmcnt(3)")
    assert check(listing(ok))[0] == [] and check(listing(bad))[0] != []
    # a store between the load and a partial wait: loads and stores retire in no fixed order, so nothing is retired
    mixed = f"{ASM_LOAD}\nglobal_store_dword v1, v2, s[4:5]\ns_waitcnt vmcnt(1)\nv_mov_b32_e32 v9, v5\ns_endpgm"
    assert check(listing(mixed))[0] != []


def test_checker_follows_the_back_edge_of_a_loop():
    # the load is waited for inside the loop on the way round, but the loop's exit path touches the register unwaited
    text = f""".LBB0_1:
v_add_u32_e32 v2, 1, v2
s_waitcnt vmcnt(0)
v_mov_b32_e32 v9, v5
{ASM_LOAD}
s_cmp_lt_i32 s4, s5
s_cbranch_scc1 .LBB0_1
v_mov_b32_e32 v5, 0
s_endpgm"""
    v, _ = check(listing(text))
    assert len(v) == 1 and v[0][2].startswith("v_mov_b32_e32 v5")


@pytest.fixture(scope="module")
def attend_assembly():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not installed")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "attend.s")
        cmd = [hipcc] + ws_build.FLAGS + ["-S", "--cuda-device-only", os.path.join(ws_build.CSRC, "attend.hip"), "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return open(out).read()


def test_attention_kernels_wait_for_their_assembly_loads(attend_assembly):
    kernels = split_kernels(attend_assembly)
    names = [k for k in kernels if "attend_bf16" in k]
    assert len(names) == 4, names                          # d = 64 / 128, with and without the index stage
    loads = {}
    for k in names:
        violations, loads[k] = check(kernels[k])
        assert violations == [], f"{k}: {violations[:5]}"
    # the query rows come by such loads in every instance, the landmark indices in the two one-pass instances
    assert all(n > 0 for n in loads.values())
    for k in names:
        if "ELb1E" in k:
            assert loads[k] > loads[k.replace("ELb1E", "ELb0E")]
