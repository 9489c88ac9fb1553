"""Host-only checks of the C-ABI library: it loads, exports what the header declares, and rejects
bad arguments before touching the device (no compute call is made here)."""
import os
import re

import pytest

from paper_2205_10357_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000      # 16-byte aligned, never dereferenced: validation fails first


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sol_block.h")).read()
    return re.findall(r"SOL_API\s+[\w\s\*]+?\b(sol_\w+)\s*\(", text)


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert set(names) == set(B.EXPORTS) and len(names) == len(B.EXPORTS) >= 10
    lib = B.lib()
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings():
    assert B.sol_status_string(0) == "ok"
    for s in range(-7, 0):
        assert B.sol_status_string(s) not in ("ok", "unknown status")
    assert B.sol_status_string(-99) == "unknown status"


def desc(**kw):
    base = dict(N=2, H=8, W=8, C_in=16, C_out=32, KH=3, KW=3, stride=1, pad=1, dtype=B.SOL_BF16, flags=B.SOL_RELU)
    base.update(kw)
    return B.BlockDesc(**base)


@pytest.mark.parametrize("kw,status", [
    (dict(N=0), -2), (dict(C_in=-1), -2), (dict(stride=0), -2), (dict(pad=-1), -2),
    (dict(H=1, W=1, KH=3, KW=3, pad=0), -2),                 # empty output
    (dict(dtype=7), -4), (dict(flags=8), -4),
    (dict(N=70000, H=224, W=224, C_in=64), -4),              # beyond 2^31-1 elements
])
def test_descriptor_validation(kw, status):
    d = desc(**kw)
    assert B.sol_block_fwd(d, FAKE, FAKE, FAKE, FAKE, None, FAKE, None, 0, stream=0, check=False) == status
    assert B.sol_block_bwd(d, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, None, None, FAKE, 1 << 40,
                           stream=0, check=False) == status
    assert B.sol_block_workspace_bytes(d, B.SOL_PASS_BWD) == 0


def test_pointer_validation():
    d = desc()
    assert B.sol_block_fwd(d, None, FAKE, FAKE, FAKE, None, FAKE, None, 0, stream=0, check=False) == -1
    assert B.sol_block_fwd(d, FAKE, FAKE, FAKE, None, None, FAKE, None, 0, stream=0, check=False) == -1
    assert B.sol_block_fwd(d, FAKE + 8, FAKE, FAKE, FAKE, None, FAKE, None, 0, stream=0, check=False) == -3
    assert B.sol_block_fwd(d, FAKE, FAKE, FAKE, FAKE, FAKE + 2, FAKE, None, 0, stream=0, check=False) == -3
    args = [FAKE] * 9
    assert B.sol_block_bwd(d, None, *args[1:], None, None, None, None, FAKE, 1 << 40, stream=0, check=False) == -1
    # ReLU block needs y for the mask; a block without ReLU does not
    assert B.sol_block_bwd(d, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, None, None, None, None, FAKE, 1 << 40,
                           stream=0, check=False) == -1
    # dW, dscale, dshift come together; with none of them some other output must be asked for
    assert B.sol_block_bwd(d, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, None, None, None, None, FAKE, 1 << 40,
                           stream=0, check=False) == -1
    assert B.sol_block_bwd(d, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, None, None, None, None, FAKE, 1 << 40,
                           stream=0, check=False) == -1
    assert B.sol_block_bwd(d, FAKE, FAKE, FAKE, FAKE, None, None, None, None, FAKE, None, None, None, None, FAKE, 1 << 40,
                           stream=0, check=False) == -1
    # addend mask without addend
    assert B.sol_block_bwd(d, *args, None, None, FAKE, None, FAKE, 1 << 40, stream=0, check=False) == -1
    # workspace missing / too small
    need = B.sol_block_workspace_bytes(d, B.SOL_PASS_BWD)
    assert need > 0
    assert B.sol_block_bwd(d, *args, None, None, None, None, None, 0, stream=0, check=False) == -5
    assert B.sol_block_bwd(d, *args, None, None, None, None, FAKE, need - 1, stream=0, check=False) == -5
    # bf16 data gradient supports stride <= 2
    d3 = desc(stride=3)
    assert B.sol_block_bwd(d3, *args, None, None, None, None, FAKE, 1 << 40, stream=0, check=False) == -4
    with pytest.raises(B.SolError):
        B.sol_block_fwd(d, None, FAKE, FAKE, FAKE, None, FAKE, None, 0, stream=0)


def test_workspace_sizes():
    assert B.sol_block_workspace_bytes(desc(), B.SOL_PASS_FWD) == 0
    # few input channels (the stem): forward needs the channel-padded image and the packed weights
    stem = desc(N=2, H=32, W=32, C_in=3, C_out=64, KH=7, KW=7, stride=2, pad=3)
    need = B.sol_block_workspace_bytes(stem, B.SOL_PASS_FWD)
    assert need >= 2 * 32 * 32 * 4 * 2 + 14 * 64 * 32
    assert B.sol_block_fwd(stem, FAKE, FAKE, FAKE, FAKE, None, FAKE, None, 0, stream=0, check=False) == -5
    assert B.sol_block_fwd(stem, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, need - 1, stream=0, check=False) == -5
    d = desc(N=64, H=14, W=14, C_in=256, C_out=256)
    need = B.sol_block_workspace_bytes(d, B.SOL_PASS_BWD)
    k = 9 * 256
    assert need >= 256 * k * 2 + 256 * k * 4           # packed weights + at least one fp32 partial
    assert need < 256 << 20
    f32 = desc(dtype=B.SOL_F32)
    assert B.sol_block_workspace_bytes(f32, B.SOL_PASS_BWD) >= 32 * 9 * 16 * 4 + 32 * 4


def test_glue_validation():
    assert B.sol_l1_loss_grad(B.SOL_BF16, FAKE, FAKE, FAKE, 0, False, stream=0, check=False) == -2
    assert B.sol_l1_loss_grad(5, FAKE, FAKE, FAKE, 16, False, stream=0, check=False) == -4
    assert B.sol_l1_loss_grad(B.SOL_F32, None, FAKE, FAKE, 16, False, stream=0, check=False) == -1
    assert B.sol_maxpool_fwd(B.SOL_BF16, FAKE, FAKE, 1, 8, 8, 8, 3, 2, 3, stream=0, check=False) == -2
    assert B.sol_maxpool_fwd(B.SOL_BF16, FAKE, None, 1, 8, 8, 8, 3, 2, 1, stream=0, check=False) == -1


def test_launch_plans_are_a_host_side_table():
    """Install / read back / remove plans; value ranges; the backward workspace follows the split count."""
    B.sol_clear_plans()
    d = B.BlockDesc(64, 14, 14, 256, 256, 3, 3, 1, 1)
    other = B.BlockDesc(64, 14, 14, 256, 256, 1, 1, 1, 0)
    try:
        assert B.sol_block_get_plan(d, B.SOL_PLAN_FWD) == (-1, 0, 0)
        base = B.sol_block_workspace_bytes(d, B.SOL_PASS_BWD)
        B.sol_block_set_plan(d, B.SOL_PLAN_FWD, (1, 3, 0))
        B.sol_block_set_plan(d, B.SOL_PLAN_WGRAD, (-1, 3, 20))
        assert B.sol_block_get_plan(d, B.SOL_PLAN_FWD) == (1, 3, 0)
        assert B.sol_block_get_plan(d, B.SOL_PLAN_DGRAD) == (-1, 0, 0)              # per kernel
        assert B.sol_block_get_plan(other, B.SOL_PLAN_FWD) == (-1, 0, 0)            # per shape
        relu_off = B.BlockDesc(64, 14, 14, 256, 256, 3, 3, 1, 1, B.SOL_BF16, 0)
        assert B.sol_block_get_plan(relu_off, B.SOL_PLAN_WGRAD) == (-1, 3, 20)      # flags do not matter
        # 20 splits of 128-row granularity over 12544 rows, fp32 partial tiles of 2304 x 256
        more = B.sol_block_workspace_bytes(d, B.SOL_PASS_BWD)
        assert more > base and (more - base) % (2304 * 256 * 4) < 64 * 1024
        for bad in ((5, 2, 0), (-2, 2, 0), (0, 1, 0), (0, 5, 0), (3, 4, 0), (0, 2, -1), (0, 2, 70000)):
            assert B.sol_block_set_plan(d, B.SOL_PLAN_FWD, bad, check=False) == -4, bad
        assert B.sol_block_set_plan(d, 3, (0, 2, 0), check=False) == -4
        assert B.sol_block_set_plan(B.BlockDesc(0, 14, 14, 256, 256, 3, 3, 1, 1), 0, (0, 2, 0), check=False) == -2
        assert B.sol_block_get_plan(d, B.SOL_PLAN_FWD) == (1, 3, 0)                 # failed calls change nothing
        B.sol_block_set_plan(d, B.SOL_PLAN_WGRAD, None)
        assert B.sol_block_workspace_bytes(d, B.SOL_PASS_BWD) == base
        B.sol_clear_plans()
        assert B.sol_block_get_plan(d, B.SOL_PLAN_FWD) == (-1, 0, 0)
    finally:
        B.sol_clear_plans()


def test_prepared_sequence_records_on_the_host_and_reports_the_failing_call():
    """Recording touches no device and validates nothing; running stops at the first call whose own checks
    fail and returns that status (here: before any HIP call, so this runs without a GPU)."""
    q = B.Sequence()
    assert len(q) == 0
    bad = B.BlockDesc(1, 8, 8, 8, 8, 3, 3, 0, 1, B.SOL_BF16, 0)                # stride 0
    ok = B.BlockDesc(1, 8, 8, 8, 8, 3, 3, 1, 1, B.SOL_BF16, 0)
    q.add_fwd(ok, None, 4096, 4096, 4096, None, 4096, None, 0, tag=1)          # x is NULL
    q.add_fwd(bad, 4096, 4096, 4096, 4096, None, 4096, None, 0, tag=2)
    q.add_l1_loss_grad(B.SOL_BF16, 4096, 4096, 4096, 0, False, tag=3)          # numel 0
    q.add_bwd(ok, 4096, 4096, 4096, None, 4096, 4096, 4096, 4096, 4096, ws=None, ws_bytes=0, tag=4)   # no workspace
    assert len(q) == 4
    assert q.run(0, 1, stream=0, check=False) == -1
    assert q.run(1, 1, stream=0, check=False) == -2
    assert q.run(2, 1, stream=0, check=False) == -2
    assert q.run(3, 1, stream=0, check=False) == -5
    assert q.run(0, 4, stream=0, check=False) == -1                            # stops at the first
    assert q.run(0, 0, stream=0, check=False) == 0
    assert q.run(3, 2, stream=0, check=False) == -2                            # range beyond the recorded calls
    assert q.run(-1, 1, stream=0, check=False) == -2


def test_trace_kind_names_and_stop_without_start():
    names = {B.sol_trace_kind_name(k) for k in range(0, 18)}
    assert len(names) == 18 and "unknown" not in names
    assert B.sol_trace_kind_name(99) == "unknown"
    import ctypes as C
    n = C.c_int32(7)
    assert B.lib().sol_trace_stop(None, 0, C.byref(n)) == -4                  # no trace is running
