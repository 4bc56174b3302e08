"""lobra_mlora_fwd_static_ws (the forward pass whose scratch is the library's static device array)
against lobra_mlora_plan_fwd with a caller workspace, through the C ABI: same kernels, so y must be bit
for bit the same, and within the layer's tolerance of the fp64 oracle.  Two calls in a row on the
same GPU, the second on a smaller batch (the array keeps the first call's contents).
"""
import numpy as np
import pytest

import oracle
from paper_2509_01193_amd import binding as bd
from paper_2509_01193_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def _run_both(p):
    import torch
    dp = bd.DeviceProblem(p)
    assert 0 < dp.plan.fwd_ws_bytes <= bd.STATIC_WS_BYTES
    dp.y.fill_(7.0)
    bd.lobra_mlora_plan_fwd(dp.plan, dp.x, dp.W, dp.A, dp.B, dp.s, dp.y, None, dp.ws)
    torch.cuda.synchronize()
    y_ref = dp.y.clone()
    dp.y.fill_(-3.0)
    bd.lobra_mlora_fwd_static_ws(dp.plan, dp.x, dp.W, dp.A, dp.B, dp.s, dp.y)
    torch.cuda.synchronize()
    assert torch.equal(dp.y.view(torch.int16 if p.dtype == "bf16" else torch.int32),
                       y_ref.view(torch.int16 if p.dtype == "bf16" else torch.int32)), p.name
    o = oracle.Oracle(p.x, p.W, p.A, p.B, p.s, p.dy, p.rank_off, p.seg_off, p.seg_task)
    ref = o.y()
    err = float(np.abs(dp.host(dp.y) - ref).max() / np.abs(ref).max())
    print("static-ws fwd %s max|err|/max|ref| = %.3e" % (p.name, err), flush=True)
    assert err <= TOL[p.dtype], (p.name, err)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_fwd_static_ws_twice_second_call_smaller(dtype):
    if dtype == "bf16":
        big = wl.make_config(3, "shuffled", d_in=320, d_out=448)       # 32768 tokens, ranks up to 64
        small = wl.make_config(2, "shuffled", d_in=264, d_out=328)     # 16384 tokens, rank 16
    else:
        big = wl.make_config(1)
        small = wl.make_custom("static-ws-small-f32", "f32", 72, 40, [4, 8], [0, 19, 19, 50, 83], [1, 0, -1, 0], 11)
    assert small.T < big.T
    _run_both(big)
    _run_both(small)


def test_fwd_static_ws_rejects_a_batch_beyond_the_array():
    import torch
    # 40000 tokens at rank 128: the projected activations alone are 2 x 10 MB
    T = 40000
    p = wl.make_custom("static-ws-too-big", "bf16", 64, 64, [128], [0, T], [0], 5)
    dp = bd.DeviceProblem(p)
    assert dp.plan.fwd_ws_bytes > bd.STATIC_WS_BYTES
    dp.y.fill_(1.0)
    st = bd.lobra_mlora_fwd_static_ws(dp.plan, dp.x, dp.W, dp.A, dp.B, dp.s, dp.y, check=False)
    torch.cuda.synchronize()
    assert st == -7                                   # LOBRA_ERR_WORKSPACE
    assert bool((dp.y == 1.0).all())                  # nothing was launched


def test_fwd_static_ws_goes_without_the_sliced_projection_when_its_sums_do_not_fit():
    """A long rank-16 batch whose K-sliced projection would need 20 MB of partial sums: the entry point uses the
    one-block-per-workgroup projection instead (5 MB of projected activations), so y agrees with the plan form to
    rounding, not bit for bit, and with the oracle within the layer's tolerance."""
    import torch
    T = 80000
    p = wl.make_custom("static-ws-unsliced", "bf16", 2048, 256, [16, 8], [0, 30000, 30001, T], [0, -1, 1], 9,
                       std_x=1.0, std_w=0.05, std_a=0.05, std_b=0.05)
    dp = bd.DeviceProblem(p)
    assert dp.plan.query(bd.Q_SLICED)[0] == 4
    assert dp.plan.fwd_ws_bytes > bd.STATIC_WS_BYTES >= dp.plan.h_save_bytes
    bd.lobra_mlora_plan_fwd(dp.plan, dp.x, dp.W, dp.A, dp.B, dp.s, dp.y, None, dp.ws)
    torch.cuda.synchronize()
    y_ref = dp.y.float().clone()
    dp.y.fill_(-3.0)
    bd.lobra_mlora_fwd_static_ws(dp.plan, dp.x, dp.W, dp.A, dp.B, dp.s, dp.y)
    torch.cuda.synchronize()
    assert float((dp.y.float() - y_ref).abs().max() / y_ref.abs().max()) <= 1e-2
    rows = np.unique(np.concatenate([np.arange(0, T, 97), [29999, 30000, 30001, T - 1]])).astype(np.int64)
    o = oracle.Oracle(p.x, p.W, p.A, p.B, p.s, p.dy, p.rank_off, p.seg_off, p.seg_task)
    ref = o.y(rows)
    got = dp.host(dp.y.index_select(0, torch.from_numpy(rows).to(dp.dev)))
    err = float(np.abs(got - ref).max() / np.abs(ref).max())
    print("static-ws fwd (unsliced) max|err|/max|ref| = %.3e" % err, flush=True)
    assert err <= TOL["bf16"], err
