"""The backward entry point that allocates nothing (its scratch is a buffer inside the library's code object):
same bits as sol_block_bwd with a caller-provided workspace, on two calls in a row, the second on a smaller
problem that finds the first call's leftovers in the buffer."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2205_10357_amd import binding as B                 # noqa: E402
from paper_2205_10357_amd import workloads as wl              # noqa: E402
from tests import parity_util as pu                           # noqa: E402


def run_both(case, seed):
    d = case["d"]
    desc = B.BlockDesc(d.N, d.H, d.W, d.C_in, d.C_out, d.KH, d.KW, d.stride, d.pad, B.SOL_BF16, 0)
    r = np.random.default_rng(seed)
    x, w = pu.to_dev(case["x"], True), pu.to_dev(case["w"], True)
    scale = pu.vec_dev(case["scale"])
    dy = pu.to_dev(wl.snap_to_bf16(r.standard_normal((d.N, d.C_out, d.Ho, d.Wo)).astype(np.float32) * 1e-3), True)
    ad = pu.to_dev(wl.snap_to_bf16(r.standard_normal(case["x"].shape).astype(np.float32)), True)
    dxm = pu.to_dev(wl.snap_to_bf16(np.maximum(r.standard_normal(case["x"].shape), 0).astype(np.float32)), True)
    need = B.sol_block_workspace_bytes(desc, B.SOL_PASS_BWD)
    assert 0 < need <= B.sol_block_bwd_noalloc_limit()
    out = []
    for noalloc in (False, True):
        dx = torch.full_like(x, 5.0)
        dW = torch.full(w.shape, 5.0, dtype=torch.float32, device="cuda")
        ds = torch.full((d.C_out,), 5.0, dtype=torch.float32, device="cuda")
        db = torch.full((d.C_out,), 5.0, dtype=torch.float32, device="cuda")
        if noalloc:
            B.sol_block_bwd_noalloc(desc, dy, x, w, None, dx, dW, ds, db, scale, None, ad, None, dxm)
        else:
            ws = torch.full((need // 4 + 64,), float("nan"), dtype=torch.float32, device="cuda")
            B.sol_block_bwd(desc, dy, x, w, None, dx, dW, ds, db, scale, None, ad, None, dxm, ws, need)
        torch.cuda.synchronize()
        out.append((dx, dW, ds, db))
    return out, need


def test_no_alloc_backward_matches_workspace_backward_twice():
    big = pu.make_case(91, 8, 14, 14, 256, 256, 3, 1, 1, relu=False)          # split weight gradient + re-pack
    small = pu.make_case(92, 2, 9, 7, 64, 72, 3, 2, 1, relu=False)            # smaller, strided, ragged
    needs = []
    for case, seed in ((big, 93), (small, 94)):
        print(f"[no-alloc] {case['d']}", flush=True)
        (ref, got), need = run_both(case, seed)
        needs.append(need)
        for name, a, b in zip(("dx", "dW", "dscale", "dshift"), ref, got):
            assert torch.equal(a, b), name
            assert bool(torch.isfinite(b.float()).all()), name
    assert needs[1] < needs[0]


def test_no_alloc_backward_rejects_what_does_not_fit():
    d = B.BlockDesc(64, 14, 14, 512, 512, 3, 3, 1, 1, B.SOL_BF16, 0)
    assert B.sol_block_workspace_bytes(d, B.SOL_PASS_BWD) > B.sol_block_bwd_noalloc_limit()
    t = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(64, dtype=torch.float32, device="cuda")
    # validation precedes every device access: the (far too small) buffers are never touched
    st = B.sol_block_bwd_noalloc(d, t, t, t, None, t, f, f, f, f, check=False)
    assert st == -7 and "scratch" in B.sol_status_string(st)
