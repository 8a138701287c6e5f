"""Host-only checks of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ws_synapse.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2601_01298_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.lib()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ws_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_symbols()
    assert {"ws_synapse_density", "ws_synapse_select", "ws_synapse_gather", "ws_synapse_attend",
            "ws_synapse_workspace_bytes", "ws_status_string"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_has_the_same_names():
    from paper_2601_01298_amd import binding
    for n in declared_symbols():
        if n.startswith("ws_synapse_"):
            assert callable(getattr(binding, n)), n


def test_status_strings(lib):
    from paper_2601_01298_amd import binding
    seen = {binding.status_string(s) for s in range(6)}
    assert len(seen) == 6 and "ok" in seen


def test_workspace_query(lib):
    from paper_2601_01298_amd import binding as b
    assert b.ws_synapse_workspace_bytes(b.WS_OP_GATHER, b.WS_BF16, 4, 100, 64) == 0
    assert b.ws_synapse_workspace_bytes(b.WS_OP_ATTEND, b.WS_BF16, 384, 1, 64, k=655, N=100, Hq=384) == 0
    # few heads, many landmarks: partial rows of a split landmark range (4 splits x 8192 rows x (128 + 4) floats)
    assert b.ws_synapse_workspace_bytes(b.WS_OP_ATTEND, b.WS_BF16, 8, 1, 128, k=2621, N=256, Hq=32) == 4 * 8192 * 132 * 4
    assert b.ws_synapse_workspace_bytes(b.WS_OP_ATTEND, b.WS_F32, 8, 1, 128, k=2621, N=256, Hq=32) == 0
    with pytest.raises(b.WsError):
        b.ws_synapse_workspace_bytes(b.WS_OP_ATTEND, b.WS_BF16, 4, 1, 64, k=10, N=4, Hq=6)
    n1 = b.ws_synapse_workspace_bytes(b.WS_OP_DENSITY, b.WS_BF16, 4, 1000, 64)
    n2 = b.ws_synapse_workspace_bytes(b.WS_OP_DENSITY, b.WS_BF16, 8, 1000, 64)
    assert 0 < n1 < n2 and n1 >= 4 * 1000 * 16
    assert b.ws_synapse_workspace_bytes(b.WS_OP_SELECT, b.WS_F32, 1, 512, 64) > 0
    with pytest.raises(b.WsError):
        b.ws_synapse_workspace_bytes(b.WS_OP_DENSITY, b.WS_BF16, 4, 1000, 96)      # d not in {64,128}
    with pytest.raises(b.WsError):
        b.ws_synapse_workspace_bytes(b.WS_OP_SELECT, b.WS_BF16, 4, 1 << 24, 64)    # L too large


def test_bad_arguments_are_rejected_on_the_host(lib):
    from paper_2601_01298_amd import binding as b
    vp = ctypes.c_void_p
    fake = vp(0x1000)            # aligned, never dereferenced: validation fails first
    odd = vp(0x1004)
    sig = (ctypes.c_float * 2)(1.0, 1.0)
    bad_sig = (ctypes.c_float * 2)(1.0, 0.0)
    nan_sig = (ctypes.c_float * 2)(1.0, float("nan"))
    D = lib.ws_synapse_density
    assert D(None, b.WS_BF16, 2, 100, 64, sig, fake, fake, 1 << 30, None) == b.WS_ERR_INVALID_ARG
    assert D(fake, b.WS_BF16, 2, 100, 96, sig, fake, fake, 1 << 30, None) == b.WS_ERR_UNSUPPORTED
    assert D(fake, 7, 2, 100, 64, sig, fake, fake, 1 << 30, None) == b.WS_ERR_UNSUPPORTED
    assert D(fake, b.WS_BF16, 0, 100, 64, sig, fake, fake, 1 << 30, None) == b.WS_ERR_INVALID_ARG
    assert D(odd, b.WS_BF16, 2, 100, 64, sig, fake, fake, 1 << 30, None) == b.WS_ERR_INVALID_ARG
    assert D(fake, b.WS_BF16, 2, 100, 64, sig, fake, None, 0, None) == b.WS_ERR_WORKSPACE
    assert D(fake, b.WS_BF16, 2, 100, 64, sig, fake, fake, 16, None) == b.WS_ERR_WORKSPACE
    assert D(fake, b.WS_BF16, 2, 100, 64, bad_sig, fake, fake, 1 << 30, None) == b.WS_ERR_INVALID_ARG
    assert D(fake, b.WS_BF16, 2, 100, 64, nan_sig, fake, fake, 1 << 30, None) == b.WS_ERR_INVALID_ARG
    huge_sig = (ctypes.c_float * 2)(1.0, 1e15)       # the padding sentinel would no longer underflow
    assert D(fake, b.WS_BF16, 2, 100, 64, huge_sig, fake, fake, 1 << 30, None) == b.WS_ERR_UNSUPPORTED
    S = lib.ws_synapse_select
    assert S(fake, b.WS_BF16, 2, 100, 64, fake, 101, 0.5, fake, None, fake, 1 << 30, None) == b.WS_ERR_INVALID_ARG
    assert S(fake, b.WS_BF16, 2, 100, 64, fake, 0, 0.5, fake, None, fake, 1 << 30, None) == b.WS_ERR_INVALID_ARG
    assert S(fake, b.WS_BF16, 2, 100, 64, fake, 10, 1.5, fake, None, fake, 1 << 30, None) == b.WS_ERR_INVALID_ARG
    assert S(fake, b.WS_BF16, 2, 100, 64, fake, 10, float("nan"), fake, None, fake, 1 << 30, None) == b.WS_ERR_INVALID_ARG
    assert S(fake, b.WS_BF16, 2, 100, 64, fake, 10, 0.5, None, None, fake, 1 << 30, None) == b.WS_ERR_INVALID_ARG
    assert S(fake, b.WS_BF16, 2, 100, 64, fake, 10, 0.5, fake, None, fake, 8, None) == b.WS_ERR_WORKSPACE
    W = lib.ws_synapse_select_with
    assert W(3, fake, b.WS_BF16, 2, 100, 64, fake, 10, 0.5, fake, None, fake, 1 << 30, None) == b.WS_ERR_INVALID_ARG
    assert W(b.WS_SELECT_STREAMING, fake, b.WS_BF16, 2, 100, 64, fake, 101, 0.5, fake, None, fake, 1 << 30, None) \
        == b.WS_ERR_INVALID_ARG
    assert W(b.WS_SELECT_RESIDENT, fake, b.WS_F32, 2, 100, 64, fake, 10, 0.5, fake, None, fake, 1 << 30, None) \
        == b.WS_ERR_UNSUPPORTED                                               # fp32 keys have no on-chip kernel
    assert W(b.WS_SELECT_RESIDENT, fake, b.WS_BF16, 2, 100, 64, fake, 10, 0.5, fake, None, fake, 8, None) == b.WS_ERR_WORKSPACE
    out = ctypes.c_int(7)
    assert lib.ws_synapse_select_failed(fake, None, None) == b.WS_ERR_INVALID_ARG
    T = lib.ws_synapse_select_static
    assert T(fake, b.WS_BF16, 2, 100, 64, fake, 101, 0.5, fake, None, None) == b.WS_ERR_INVALID_ARG
    assert T(fake, b.WS_BF16, 2, 100, 96, fake, 10, 0.5, fake, None, None) == b.WS_ERR_UNSUPPORTED
    assert T(None, b.WS_BF16, 2, 100, 64, fake, 10, 0.5, fake, None, None) == b.WS_ERR_INVALID_ARG
    # one head of the streaming kernel needs 8 bytes per key of slabs: more than the fixed 4 MiB
    assert T(fake, b.WS_F32, 2, 600_000, 64, fake, 10, 0.5, fake, None, None) == b.WS_ERR_TOO_LARGE
    assert T(fake, b.WS_BF16, 2, 1_000_000, 128, fake, 10, 0.5, fake, None, None) == b.WS_ERR_TOO_LARGE
    plan = b.SelectPlan()
    P = lib.ws_synapse_select_plan
    assert P(0, b.WS_BF16, 2, 100, 64, 0, 0, None) == b.WS_ERR_INVALID_ARG
    assert P(0, b.WS_BF16, 0, 100, 64, 0, 0, ctypes.byref(plan)) == b.WS_ERR_INVALID_ARG
    assert P(0, b.WS_BF16, 2, 100, 64, -1, 0, ctypes.byref(plan)) == b.WS_ERR_INVALID_ARG
    assert P(9, b.WS_BF16, 2, 100, 64, 0, 0, ctypes.byref(plan)) == b.WS_ERR_INVALID_ARG
    assert P(0, b.WS_BF16, 2, 100, 48, 0, 0, ctypes.byref(plan)) == b.WS_ERR_UNSUPPORTED
    assert P(0, b.WS_BF16, 2, 100, 64, 0, 0, ctypes.byref(plan)) == b.WS_OK and plan.compute_units == 256
    G = lib.ws_synapse_gather
    assert G(fake, None, b.WS_BF16, 2, 100, 64, fake, 10, fake, fake, None) == b.WS_ERR_INVALID_ARG
    assert G(fake, fake, b.WS_BF16, 2, 100, 32, fake, 10, fake, fake, None) == b.WS_ERR_UNSUPPORTED
    A = lib.ws_synapse_attend
    assert A(fake, fake, fake, b.WS_BF16, 4, 6, 4, 10, 64, 0.0, fake, None, 0, None) == b.WS_ERR_INVALID_ARG   # 6 % 4
    assert A(fake, fake, fake, b.WS_BF16, 0, 4, 4, 10, 64, 0.0, fake, None, 0, None) == b.WS_ERR_INVALID_ARG
    assert A(fake, fake, fake, b.WS_BF16, 4, 4, 4, 10, 64, float("inf"), fake, None, 0, None) == b.WS_ERR_INVALID_ARG
    assert A(fake, fake, None, b.WS_BF16, 4, 4, 4, 10, 64, 0.0, fake, None, 0, None) == b.WS_ERR_INVALID_ARG
    assert A(fake, fake, fake, b.WS_BF16, 256, 32, 8, 2621, 128, 0.0, fake, None, 0, None) == b.WS_ERR_WORKSPACE   # split range
    AI = lib.ws_synapse_attend_indexed
    assert AI(fake, fake, fake, None, b.WS_BF16, 4, 4, 4, 100, 10, 64, 0.0, fake, None, 0, None) == b.WS_ERR_INVALID_ARG
    assert AI(fake, fake, fake, fake, b.WS_BF16, 4, 6, 4, 100, 10, 64, 0.0, fake, None, 0, None) == b.WS_ERR_INVALID_ARG   # 6 % 4
    assert AI(fake, fake, fake, fake, b.WS_BF16, 4, 4, 4, 0, 10, 64, 0.0, fake, None, 0, None) == b.WS_ERR_INVALID_ARG
    assert AI(fake, fake, fake, fake, b.WS_F32, 4, 4, 4, 1 << 23, 10, 128, 0.0, fake, None, 0, None) == b.WS_ERR_UNSUPPORTED
    assert AI(fake, fake, fake, fake, b.WS_BF16, 256, 32, 8, 131072, 2621, 128, 0.0, fake, None, 0, None) == b.WS_ERR_WORKSPACE


def test_bad_arguments_of_the_next_steps_are_rejected_on_the_host(lib):
    from paper_2601_01298_amd import binding as b
    vp = ctypes.c_void_p
    fake, odd = vp(0x1000), vp(0x1004)
    big = 1 << 40
    sig = (ctypes.c_float * 2)(1.0, 1.0)
    bad_sig = (ctypes.c_float * 2)(1.0, -1.0)
    M = lib.ws_synapse_attention_mass
    assert M(fake, fake, b.WS_BF16, 2, 4, 6, 100, 64, 0.0, 1, fake, fake, big, None) == b.WS_ERR_INVALID_ARG     # 6 % 4
    assert M(fake, None, b.WS_BF16, 2, 4, 4, 100, 64, 0.0, 1, fake, fake, big, None) == b.WS_ERR_INVALID_ARG
    assert M(fake, odd, b.WS_BF16, 2, 4, 4, 100, 64, 0.0, 1, fake, fake, big, None) == b.WS_ERR_INVALID_ARG
    assert M(fake, fake, b.WS_BF16, 2, 4, 64, 100, 64, 0.0, 1, fake, fake, big, None) == b.WS_ERR_UNSUPPORTED    # 16 per KV head
    assert M(fake, fake, b.WS_BF16, 2, 4, 4, 100, 80, 0.0, 1, fake, fake, big, None) == b.WS_ERR_UNSUPPORTED
    assert M(fake, fake, b.WS_BF16, 2, 4, 4, 100, 64, 0.0, 1, fake, fake, 64, None) == b.WS_ERR_WORKSPACE
    A = lib.ws_synapse_density_append
    assert A(fake, b.WS_BF16, 2, 100, 64, 0, sig, fake, fake, fake, big, None) == b.WS_ERR_INVALID_ARG
    assert A(fake, b.WS_BF16, 2, 100, 64, 100, sig, fake, fake, fake, big, None) == b.WS_ERR_INVALID_ARG          # no old rows
    assert A(fake, b.WS_BF16, 2, 100, 64, 33, sig, fake, fake, fake, big, None) == b.WS_ERR_UNSUPPORTED
    assert A(fake, b.WS_BF16, 2, 100, 64, 4, bad_sig, fake, fake, fake, big, None) == b.WS_ERR_INVALID_ARG
    assert A(fake, b.WS_BF16, 2, 100, 64, 4, sig, None, fake, fake, big, None) == b.WS_ERR_INVALID_ARG
    assert A(fake, b.WS_BF16, 2, 100, 64, 4, sig, fake, fake, None, 0, None) == b.WS_ERR_WORKSPACE
    G = lib.ws_synapse_gate
    assert G(fake, fake, b.WS_BF16, 0, 896, 0.5, fake, fake, None) == b.WS_ERR_INVALID_ARG
    assert G(fake, None, b.WS_BF16, 4, 896, 0.5, fake, fake, None) == b.WS_ERR_INVALID_ARG
    assert G(fake, fake, b.WS_BF16, 4, 896, float("nan"), fake, fake, None) == b.WS_ERR_INVALID_ARG
    assert G(fake, fake, 5, 4, 896, 0.5, fake, fake, None) == b.WS_ERR_UNSUPPORTED
    I = lib.ws_synapse_inject
    assert I(fake, fake, b.WS_BF16, 2, 100, 64, 98, fake, fake, 3, fake, 1e4, fake, big, None) == b.WS_ERR_INVALID_ARG   # no room
    assert I(fake, fake, b.WS_BF16, 2, 100, 64, 10, fake, fake, 3, fake, 0.0, fake, big, None) == b.WS_ERR_INVALID_ARG
    assert I(fake, fake, b.WS_BF16, 2, 100, 64, 10, fake, fake, 3, None, 1e4, fake, big, None) == b.WS_ERR_INVALID_ARG
    assert I(fake, odd, b.WS_BF16, 2, 100, 64, 10, fake, fake, 3, fake, 1e4, fake, big, None) == b.WS_ERR_INVALID_ARG
    assert I(fake, fake, b.WS_BF16, 2, 100, 96, 10, fake, fake, 3, fake, 1e4, fake, big, None) == b.WS_ERR_UNSUPPORTED
    assert I(fake, fake, b.WS_BF16, 2, 100, 64, 10, fake, fake, 3, fake, 1e4, None, 0, None) == b.WS_ERR_WORKSPACE
    assert b.ws_synapse_workspace_bytes(b.WS_OP_INJECT, b.WS_BF16, 2, 100, 64, k=3) >= 3 * 32 * 8
    assert b.ws_synapse_workspace_bytes(b.WS_OP_ATTENTION_MASS, b.WS_BF16, 8, 4096, 64, Hq=8) >= 8 * 4096 * 4
    assert b.ws_synapse_workspace_bytes(b.WS_OP_DENSITY_APPEND, b.WS_BF16, 8, 4096, 64) > 0


def test_selection_kernel_choice_is_host_logic(lib):
    """Which selection kernel a shape gets is decided on the host from the sizes and the device's shape: heads
    whose keys fit the chip's registers and LDS (32 headline heads at a time) stay on chip, fp32 keys and
    heads beyond 128 workgroups' worth of registers and LDS stream.  No environment variable takes part."""
    import subprocess
    import sys
    from paper_2601_01298_amd import binding as b
    from paper_2601_01298_amd import synthetic as syn
    expect = {1: False, 2: True, 3: True, 4: True, 5: True}
    for cfg, w in syn.WORKLOADS.items():
        dt = b.WS_BF16 if w.dtype == "bf16" else b.WS_F32
        assert b.ws_synapse_select_is_resident(dt, w.H, w.L, w.d) == expect[cfg], w.name
        assert b.ws_synapse_workspace_bytes(b.WS_OP_SELECT, dt, w.H, w.L, w.d, w.k) > 0
    assert not b.ws_synapse_select_plan("stream", b.WS_BF16, 384, 32768, 64).resident
    with pytest.raises(b.WsError):
        b.ws_synapse_select_plan("resident", b.WS_F32, 1, 512, 64)          # fp32 keys never sit on chip
    p5 = b.ws_synapse_select_plan("resident", b.WS_BF16, 8, 131072, 128)    # a 32 MiB head: 128 workgroups on two dies
    assert (p5.heads_in_flight, p5.workgroups_per_head, p5.rows_in_registers, p5.rows_in_lds) == (4, 128, 3, 1)
    with pytest.raises(b.WsError):
        b.ws_synapse_select_plan("resident", b.WS_BF16, 8, 300000, 128)     # a head larger than 128 workgroups hold
    code = ("import os; os.environ['WS_SYNAPSE_SELECT']='stream'; from paper_2601_01298_amd import binding as b; "
            "print(int(b.ws_synapse_select_is_resident(b.WS_BF16, 384, 32768, 64)))")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, cwd=ROOT, timeout=120)
    assert r.stdout.strip() == "1", r.stderr                                # the old switch is gone
    assert "getenv" not in "".join(open(os.path.join(ROOT, "paper_2601_01298_amd", "csrc", f)).read()
                                   for f in os.listdir(os.path.join(ROOT, "paper_2601_01298_amd", "csrc")))


@pytest.mark.parametrize("cus", [32, 64, 128, 256, 304])
@pytest.mark.parametrize("per_cu", [1, 2])
def test_selection_grid_fits_the_device(lib, cus, per_cu):
    """The selection kernels' workgroups wait on each other, so a launch must never exceed what the device
    keeps resident at once (compute units x workgroups per unit), whatever the device's shape; and a head
    needs all its keys covered: workgroups_per_head x rows x 256 >= L for the on-chip kernel."""
    from paper_2601_01298_amd import binding as b
    shapes = [(384, 32768, 64), (16, 4096, 64), (32, 8192, 128), (8, 131072, 128), (1, 512, 64), (1, 100, 128),
              (1000, 2048, 64), (3, 70000, 64), (40, 4096, 64), (136, 4096, 64), (72, 4096, 128), (5, 16_000_000, 64)]
    for kernel in ("auto", "stream", "resident"):
        for dt in (b.WS_BF16, b.WS_F32):
            for H, L, d in shapes:
                try:
                    p = b.ws_synapse_select_plan(kernel, dt, H, L, d, cus, per_cu)
                except b.WsError as e:
                    assert kernel == "resident" and e.status == b.WS_ERR_UNSUPPORTED
                    continue
                assert p.compute_units == cus
                assert 1 <= p.heads_in_flight <= H and p.workgroups_per_head >= 1
                assert p.heads_in_flight * p.workgroups_per_head <= cus * per_cu, (kernel, dt, H, L, d)
                if p.resident:
                    assert dt == b.WS_BF16 and kernel != "stream" and p.threads == 256
                    assert p.workgroups_per_head * 256 * (p.rows_in_registers + p.rows_in_lds) >= L
                    assert p.workgroups_per_head <= 128
                    if p.workgroups_per_head > 32:
                        assert p.heads_in_flight in (1, 2, 4, 8, 16)      # whole dies per head
                else:
                    assert kernel != "resident" and p.threads == 512 and p.workgroups_per_head <= 64
    # the headline on the full chip: 32 heads in flight, 16 workgroups each, 6 + 2 rows per lane
    p = b.ws_synapse_select_plan("auto", b.WS_BF16, 384, 32768, 64, 256, 2)
    assert (p.resident, p.heads_in_flight, p.workgroups_per_head, p.rows_in_registers, p.rows_in_lds) == (1, 32, 16, 6, 2)
    # a quarter of the chip still keeps a 32k-token head on chip, fewer at a time
    p = b.ws_synapse_select_plan("auto", b.WS_BF16, 384, 32768, 64, 64, 2)
    assert p.resident and p.heads_in_flight == 8
    # a device too small for one head's group falls back to streaming
    assert not b.ws_synapse_select_plan("auto", b.WS_BF16, 384, 32768, 64, 4, 2).resident


def test_density_workspace_size(lib):
    from paper_2601_01298_amd import binding as b
    # the density workspace: per key a 16-byte record and room for a translated copy of the row (bf16 keys), and
    # column partial sums capped near 4 GiB however many heads
    per_key = 16 + 64 * 2
    a = b.ws_synapse_workspace_bytes(b.WS_OP_DENSITY, b.WS_BF16, 384, 32768, 64)
    c = b.ws_synapse_workspace_bytes(b.WS_OP_DENSITY, b.WS_BF16, 4096, 32768, 64)
    assert a >= 384 * 32768 * per_key and c - a < (4096 - 384) * 32768 * per_key + (2 << 30)
    assert c < 4096 * 32768 * per_key + (5 << 30)
    f = b.ws_synapse_workspace_bytes(b.WS_OP_DENSITY, b.WS_F32, 4, 1000, 64)     # fp32 keys: no copy
    assert 4 * 1000 * 16 <= f < 4 * 1024 * 16 + (1 << 20)


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: asking for more ends with a message and a non-zero status, before anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr
    assert r.stdout.strip() == ""


C_CONSUMER = r"""
#include <stdio.h>
#include <string.h>
#include "ws_synapse.h"
int main(void)
{
    /* a consumer written in C: only calls that need no device */
    size_t n = ws_synapse_workspace_bytes(WS_OP_SELECT, WS_BF16, 16, 4096, 64, 82, 100, 16);
    if (n == 0) return 1;
    if (strcmp(ws_status_string(WS_OK), "ok") != 0) return 2;
    /* arguments are checked on the host before anything is launched */
    if (ws_synapse_gather(NULL, NULL, WS_BF16, 1, 8, 64, NULL, 4, NULL, NULL, NULL) != WS_ERR_INVALID_ARG) return 3;
    printf("%zu\n", n);
    return 0;
}
"""


@pytest.mark.parametrize("compiler,std,suffix", [("gcc", "-std=c99", ".c"), ("g++", "-std=c++11", ".cpp")])
def test_header_serves_a_plain_c_and_a_cxx_consumer(lib, tmp_path, compiler, std, suffix):
    """The header compiles as strict C99 and as C++ without the HIP headers, and a program built from it links
    against the library and runs on a host without a GPU."""
    import shutil
    import subprocess
    from paper_2601_01298_amd import binding
    if shutil.which(compiler) is None:
        pytest.skip(f"no {compiler}")
    src = tmp_path / ("consumer" + suffix)
    src.write_text(C_CONSUMER)
    exe = tmp_path / "consumer"
    libdir = os.path.dirname(binding.LIB_PATH)
    cmd = [compiler, std, "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.dirname(HEADER), str(src), "-o", str(exe),
           "-L", libdir, "-l:" + os.path.basename(binding.LIB_PATH), "-Wl,-rpath," + libdir]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr[-500:])
    assert int(r.stdout.strip()) == binding.ws_synapse_workspace_bytes(binding.WS_OP_SELECT, binding.WS_BF16, 16, 4096, 64, k=82, N=100, Hq=16)
