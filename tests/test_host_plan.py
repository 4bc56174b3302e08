"""CPU tests of the C-ABI library's host side: exported symbols, argument errors, work lists.

No kernel is launched here.  The work lists are compared bit for bit with a brute-force walk
over the token -> task map that the oracle computes from the same segment table.
"""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2509_01193_amd import binding as bd
from paper_2509_01193_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "lobra_mlora.h")).read()
    declared = set(re.findall(r"\b(lobra_[a-z_]+)\s*\(", hdr))
    assert declared == set(bd.EXPORTS)
    L = bd.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert bd.version() >= 100
    assert bd.status_string(0) == "ok" and "segment" in bd.status_string(-4)


def _desc(**kw):
    base = dict(dtype="f32", T=10, d_in=8, d_out=8, rank_off=[0, 2, 5], seg_off=[0, 4, 10], seg_task=[0, 1])
    base.update(kw)
    return bd.make_desc(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(), 0),
    (dict(dtype=7), -3),
    (dict(T=-1), -2),
    (dict(d_in=0), -2),
    (dict(seg_off=[1, 4, 10]), -4),
    (dict(seg_off=[0, 11, 10]), -4),
    (dict(seg_off=[0, 4, 9]), -4),
    (dict(seg_task=[0, 2]), -5),
    (dict(seg_task=[-2, 1]), -5),
    (dict(rank_off=[0, 0, 5]), -6),
    (dict(rank_off=[1, 2, 5]), -6),
    (dict(rank_off=[0, 2, 2 + 129]), -6),
    (dict(dtype="bf16", d_in=12), -8),
    (dict(dtype="bf16", d_in=16, d_out=24), 0),
    (dict(seg_task=[-1, -1]), 0),
])
def test_validate_status_codes(kw, code):
    d, keep = _desc(**kw)
    assert bd.validate(d) == code


def test_validate_null_tables_and_empty_batch():
    d, _ = bd.make_desc("f32", 0, 8, 8, None, None, None)
    assert bd.validate(d) == 0                       # T = 0, S = 0, no tasks
    d, _ = bd.make_desc("f32", 5, 8, 8, None, None, None)
    assert bd.validate(d) == -4                      # tokens but no segment
    d, keep = _desc()
    d.seg_task = None
    assert bd.validate(d) == -1
    assert bd.lib().lobra_mlora_validate(None) == -1


def test_host_only_plan_cannot_run():
    p = wl.make_config(1, fill=False)
    plan = bd.Plan.for_problem(p, bd.PLAN_HOST_ONLY)
    st = bd.lib().lobra_mlora_plan_fwd(plan.handle, None, None, None, None, None, None, None, None, 0, None)
    assert st == -10
    assert bd.lib().lobra_mlora_plan_fwd(None, None, None, None, None, None, None, None, None, 0, None) == -10
    assert bd.lib().lobra_mlora_plan_destroy(None) == 0


def test_shape_limits_are_reported_before_any_launch():
    """Launch grids and 32-bit tile offsets bound the shapes; the bounds are argument errors of validate /
    plan_create / the one-shot calls, not launch failures in the middle of a call."""
    big = (1 << 20) + 8
    for kw in (dict(dtype="bf16", d_in=big, d_out=16), dict(dtype="bf16", d_in=16, d_out=big),
               dict(dtype="f32", d_in=big)):
        d, keep = _desc(**kw)
        assert bd.validate(d) == -2, kw
    # number of 256 x 256 output tiles
    T = (1 << 31) - 256
    d, keep = bd.make_desc("bf16", T, 1 << 20, 8, None, [0, T], [-1])
    assert bd.validate(d) == -2
    d, keep = bd.make_desc("bf16", T, 1024, 8, None, [0, T], [-1])
    assert bd.validate(d) == 0
    # the plain kernels put 64-token tiles on grid.y: fp32 storage, and bf16 under LOBRA_PLAN_PLAIN_KERNELS
    T = 65535 * 64 + 1
    d, keep = bd.make_desc("f32", T, 8, 8, None, [0, T], [-1])
    assert bd.validate(d) == -2
    d, keep = bd.make_desc("bf16", T, 8, 8, None, [0, T], [-1])
    assert bd.validate(d) == 0
    h = ctypes.c_void_p()
    assert bd.lib().lobra_mlora_plan_create(ctypes.byref(d), bd.PLAN_HOST_ONLY | bd.PLAN_PLAIN_KERNELS, ctypes.byref(h)) == -2
    assert bd.lib().lobra_mlora_plan_create(ctypes.byref(d), bd.PLAN_HOST_ONLY, ctypes.byref(h)) == 0
    assert bd.lib().lobra_mlora_plan_destroy(h) == 0


def test_workspace_bytes_and_one_shot_argument_errors():
    """lobra_mlora_workspace_bytes is host only; the one-shot calls report descriptor and workspace errors
    before they touch the device (so all of this runs without a GPU)."""
    p = wl.make_config(1, fill=False)
    d, keep = bd.make_desc(p.dtype, p.T, p.d_in, p.d_out, p.rank_off, p.seg_off, p.seg_task)
    fwd, bwd = bd.lobra_mlora_workspace_bytes(d)
    plan = bd.Plan.for_problem(p, bd.PLAN_HOST_ONLY)
    img = bd.plan_device_bytes(d)
    assert img > 0 and img % 4 == 0
    img256 = (img + 255) // 256 * 256
    assert fwd == img256 + plan.fwd_ws_bytes and bwd == img256 + plan.bwd_ws_bytes
    L = bd.lib()
    a = ctypes.c_size_t()
    assert L.lobra_mlora_workspace_bytes(None, ctypes.byref(a), None) == -1
    assert L.lobra_mlora_workspace_bytes(ctypes.byref(d), None, None) == 0
    assert L.lobra_mlora_plan_device_bytes(ctypes.byref(d), 0, None) == -1
    bad, keep2 = _desc(seg_off=[0, 4, 9])
    assert L.lobra_mlora_workspace_bytes(ctypes.byref(bad), ctypes.byref(a), None) == -4
    one = ctypes.c_void_p(0x1000)                       # a non-NULL, aligned pointer that is never dereferenced
    # descriptor errors come first
    assert L.lobra_mlora_fwd(ctypes.byref(bad), one, one, one, one, one, one, None, one, 1 << 30, None) == -4
    assert L.lobra_mlora_bwd(ctypes.byref(bad), one, one, one, one, one, one, None, one, one, one, 0, one, 1 << 30, None) == -4
    assert L.lobra_token_task_map(ctypes.byref(bad), one, one, None) == -4
    assert L.lobra_mlora_fwd(None, one, one, one, one, one, one, None, one, 1 << 30, None) == -1
    # then the workspace: missing, too small (one byte short), misaligned
    assert L.lobra_mlora_fwd(ctypes.byref(d), one, one, one, one, one, one, None, None, 0, None) == -7
    assert L.lobra_mlora_fwd(ctypes.byref(d), one, one, one, one, one, one, None, one, fwd - 1, None) == -7
    assert L.lobra_mlora_bwd(ctypes.byref(d), one, one, one, one, one, one, None, one, one, one, 0, one, bwd - 1, None) == -7
    assert L.lobra_mlora_fwd(ctypes.byref(d), one, one, one, one, one, one, None, ctypes.c_void_p(0x1004), fwd, None) == -8
    # then the tensors: a missing one, a misaligned one
    assert L.lobra_mlora_fwd(ctypes.byref(d), None, one, one, one, one, one, None, one, fwd, None) == -1
    assert L.lobra_mlora_fwd(ctypes.byref(d), ctypes.c_void_p(0x1008), one, one, one, one, one, None, one, fwd, None) == -8
    assert L.lobra_mlora_bwd(ctypes.byref(d), one, one, one, one, one, None, None, one, one, one, 0, one, bwd, None) == -1
    # an empty batch is a no-op that needs nothing
    e, keep3 = bd.make_desc("f32", 0, 8, 8, None, None, None)
    assert L.lobra_mlora_fwd(ctypes.byref(e), None, None, None, None, None, None, None, None, 0, None) == 0


def test_plan_init_argument_errors():
    """The errors of lobra_mlora_plan_init that precede its first HIP call."""
    p = wl.make_config(1, fill=False)
    d, keep = bd.make_desc(p.dtype, p.T, p.d_in, p.d_out, p.rank_off, p.seg_off, p.seg_task)
    L = bd.lib()
    h = ctypes.c_void_p()
    n = bd.plan_device_bytes(d)
    one = ctypes.c_void_p(0x1000)
    assert L.lobra_mlora_plan_init(ctypes.byref(d), 0, one, n, None, None) == -1
    assert L.lobra_mlora_plan_init(ctypes.byref(d), bd.PLAN_HOST_ONLY, one, n, None, ctypes.byref(h)) == -10
    assert L.lobra_mlora_plan_init(ctypes.byref(d), 0, None, n, None, ctypes.byref(h)) == -7
    assert L.lobra_mlora_plan_init(ctypes.byref(d), 0, one, n - 1, None, ctypes.byref(h)) == -7
    assert L.lobra_mlora_plan_init(ctypes.byref(d), 0, ctypes.c_void_p(0x1004), n, None, ctypes.byref(h)) == -8
    bad, keep2 = _desc(rank_off=[0, 0, 5])
    assert L.lobra_mlora_plan_init(ctypes.byref(bad), 0, one, 1 << 20, None, ctypes.byref(h)) == -6
    assert not h.value


def brute_force_lists(p):
    tok = oracle.token_task(p.T, p.seg_off, p.seg_task, p.n_tasks)
    # maximal runs of equal task
    segs, i = [], 0
    while i < p.T:
        j = i
        while j < p.T and tok[j] == tok[i]:
            j += 1
        segs.append((i, j, int(tok[i])))
        i = j
    return tok, segs


def check_plan(p):
    plan = bd.Plan.for_problem(p, bd.PLAN_HOST_ONLY)
    tok, segs = brute_force_lists(p)
    got = plan.query(bd.Q_SEGMENTS).reshape(-1, 3)
    assert [tuple(r) for r in got.tolist()] == segs
    rb = plan.query(bd.Q_ROWBLOCK_SEG)
    assert len(rb) == (p.T + 31) // 32
    for b, k in enumerate(rb):
        assert segs[k][0] <= 32 * b < segs[k][1]
    ro = p.rank_off
    # what the first token of every 256-token tile row of the base product belongs to
    tr = plan.query(bd.Q_GEMM_TILE_ROWS).reshape(-1, 8)
    assert len(tr) == (p.T + 255) // 256
    for i, rec in enumerate(tr.tolist()):
        row0 = max(0, min(256 * i, p.T - 256))
        k = rec[0]
        assert segs[k][0] <= row0 < segs[k][1]
        task = segs[k][2]
        want = [k, segs[k][0], segs[k][1], task, int(ro[task]) if task >= 0 else 0,
                int(ro[task + 1] - ro[task]) if task >= 0 else 0, 0, 0]
        assert rec == want, (i, rec, want)
    tb = plan.query(bd.Q_TOKEN_BLOCKS).reshape(-1, 4)
    covered = np.zeros(p.T, np.int32)
    last_task, last_row = -1, -1
    for row0, nrows, task, rr0 in tb.tolist():
        assert 1 <= nrows <= 32 and 0 <= task < p.n_tasks and rr0 == ro[task]
        assert (tok[row0:row0 + nrows] == task).all()
        covered[row0:row0 + nrows] += 1
        assert task > last_task or (task == last_task and row0 > last_row)   # by task, then by token
        last_task, last_row = task, row0
    assert (covered == (tok >= 0)).all()          # every adapter token in exactly one block
    # a block never spans two segments, and only a segment's last block may be short
    starts = {s[0] for s in segs}
    ends = {s[1] for s in segs}
    for row0, nrows, task, _ in tb.tolist():
        assert nrows == 32 or (row0 + nrows) in ends
        assert not any(row0 < s < row0 + nrows for s in starts)
    ch = plan.query(bd.Q_GRAD_CHUNKS).reshape(-1, 4)
    tco = plan.query(bd.Q_TASK_CHUNKS)
    assert len(tco) == p.n_tasks + 1 and tco[0] == 0 and tco[-1] == len(ch)
    nxt, prow = 0, 0
    for c, (b0, b1, task, pr0) in enumerate(ch.tolist()):
        assert b0 == nxt and b1 > b0 and pr0 == prow
        assert (tb[b0:b1, 2] == task).all()
        assert tco[task] <= c < tco[task + 1]
        nxt, prow = b1, prow + int(p.ranks[task])
    assert nxt == len(tb)
    # runs of token blocks projected by one workgroup: a partition of the blocks, one task per run
    runs = plan.query(bd.Q_BLOCK_RUNS)
    assert runs[0] == 0 and runs[-1] == len(tb) and (np.diff(runs) >= 1).all() and (np.diff(runs) <= 4).all()
    for r0, r1 in zip(runs[:-1], runs[1:]):
        assert (tb[r0:r1, 2] == tb[r0, 2]).all()
    # launch order of blocks and runs: by descending rank, ties in stored order; empty = stored order
    ranks = np.asarray(p.ranks)
    for what, tasks in ((bd.Q_BLOCK_ORDER, tb[:, 2]), (bd.Q_RUN_ORDER, tb[runs[:-1], 2] if len(tb) else tb[:0, 2])):
        order = plan.query(what)
        expect = np.argsort(-ranks[tasks], kind="stable") if len(tasks) else np.zeros(0, np.int64)
        if len(order) == 0:
            assert (expect == np.arange(len(tasks))).all()
        else:
            assert (order == expect).all() and not (expect == np.arange(len(tasks))).all()
    a, b, c = plan.h_save_bytes, plan.fwd_ws_bytes, plan.bwd_ws_bytes
    assert c >= prow * max(p.d_in, p.d_out) * 4
    plan.close()
    return len(tb), len(ch)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("order", ["shuffled", "sorted"])
def test_work_lists_of_the_five_workloads(cfg, order):
    check_plan(wl.make_config(cfg, order, fill=False))


def test_work_lists_adversarial_tables():
    rng = np.random.default_rng(0)
    for trial in range(40):
        S = int(rng.integers(1, 40))
        lens = rng.choice([0, 1, 2, 15, 16, 17, 31, 32, 33, 64, 100], S)
        seg_task = rng.integers(-1, 5, S)
        seg_off = np.concatenate([[0], np.cumsum(lens)])
        p = wl.make_custom("adv", "bf16", 64, 128, [8, 16, 3, 64, 128], seg_off, seg_task, trial, fill=False)
        check_plan(p)
    # one-token segments alternating between tasks, and an all-empty table
    # (chunks of at least four token blocks for the MFMA kernels, single blocks allowed on the fp32 path)
    p = wl.make_custom("alt", "bf16", 8, 8, [2, 2], np.arange(0, 101), np.arange(100) % 2, 1, fill=False)
    assert check_plan(p) == (100, 2 * -(-50 // 4))
    p = wl.make_custom("alt", "f32", 8, 8, [2, 2], np.arange(0, 101), np.arange(100) % 2, 1, fill=False)
    assert check_plan(p) == (100, 100)
    p = wl.make_custom("none", "f32", 8, 8, [2, 2], [0, 0, 0], [0, 1], 1, fill=False)
    assert check_plan(p) == (0, 0)


def check_sliced_tables(p):
    """The K-sliced projection's shape rule and, when dB is fused into it, the run tables: compared with a walk
    over every item of every workgroup by the rule the kernel itself follows (the items of an XCD's token blocks,
    slice-major, split evenly over its workgroups)."""
    plan = bd.Plan.for_problem(p, bd.PLAN_HOST_ONLY)
    nsl_in, nsl_out, fused, rows, G = plan.query(bd.Q_SLICED).tolist()
    tb = plan.query(bd.Q_TOKEN_BLOCKS).reshape(-1, 4)
    ntb = len(tb)
    ranks = np.asarray(p.ranks)
    r_pad = (int(ranks.max()) + 15) // 16 * 16 if len(ranks) else 0
    n_proj = getattr(p, "n_proj", 1)
    for nsl, D, ok in ((nsl_in, p.d_in, True), (nsl_out, p.d_out, n_proj == 1)):
        want = D // 512 if (p.dtype == "bf16" and ok and r_pad == 16 and D % 512 == 0 and ntb * (D // 512) >= 3072) else 0
        assert nsl == want, (p.name, nsl, want)
    assert G == 256
    # the workspaces hold the fp32 partial projections [slices][T][16]
    assert plan.fwd_ws_bytes >= plan.h_save_bytes + nsl_in * p.T * 64
    assert plan.bwd_ws_bytes >= max(nsl_in, nsl_out) * p.T * 64
    wg_runs, run_row = plan.query(bd.Q_FUSED_WG_RUNS), plan.query(bd.Q_FUSED_RUN_ROW)
    cnt, task_row = plan.query(bd.Q_FUSED_COUNT), plan.query(bd.Q_FUSED_TASK_ROW)
    if not fused:
        assert rows == 0 and len(wg_runs) == len(run_row) == len(cnt) == len(task_row) == 0
        plan.close()
        return False
    assert nsl_out > 0 and len(wg_runs) == G + 1 and wg_runs[0] == 0 and wg_runs[-1] == len(run_row)
    assert len(cnt) == p.n_tasks * nsl_out and len(task_row) == p.n_tasks
    per, seen, covered = G // 8, {}, 0
    for wg in range(G):
        xcd, idx = wg & 7, wg >> 3
        bx0, bx1 = (ntb * xcd) >> 3, (ntb * (xcd + 1)) >> 3
        nbx = bx1 - bx0
        nit = nbx * nsl_out
        e0, e1 = nit * idx // per, nit * (idx + 1) // per
        covered += e1 - e0
        prev, nruns = None, 0
        for e in range(e0, e1):
            sl, bo = divmod(e, nbx)
            key = (int(tb[bx0 + bo, 2]), sl)
            if key != prev:
                k = seen.get(key, 0)
                seen[key] = k + 1
                assert run_row[wg_runs[wg] + nruns] == task_row[key[0]] + 16 * k, (p.name, wg, e)
                nruns, prev = nruns + 1, key
        assert wg_runs[wg + 1] - wg_runs[wg] == nruns, (p.name, wg)
    assert covered == ntb * nsl_out
    want_cnt = np.zeros((p.n_tasks, nsl_out), np.int64)
    for (t, sl), k in seen.items():
        want_cnt[t, sl] = k
    assert (cnt.reshape(p.n_tasks, nsl_out) == want_cnt).all()
    # a task's runs occupy its own range of rows, 16 per run of its busiest slice
    need = 16 * want_cnt.max(axis=1)
    assert (task_row == np.concatenate([[0], np.cumsum(need)[:-1]])).all() and rows == need.sum()
    assert rows <= p.T // 8 and plan.bwd_ws_bytes >= rows * p.d_out * 4
    plan.close()
    return True


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("order", ["shuffled", "sorted"])
def test_sliced_projection_tables_of_the_five_workloads(cfg, order):
    fused = check_sliced_tables(wl.make_config(cfg, order, fill=False))
    assert fused == (cfg in (2, 4))          # rank 16 on long batches; workload 1 is fp32, 3 and 5 have larger ranks


def test_sliced_projection_tables_adversarial():
    rng = np.random.default_rng(3)
    outcomes = set()
    for trial in range(12):
        n_tasks = int(rng.choice([1, 3, 17, 40]))
        S = int(rng.integers(n_tasks, 6 * n_tasks + 2))
        lens = rng.choice([0, 1, 7, 31, 32, 33, 500, 2000, 6000], S)
        seg_task = rng.integers(-1, n_tasks, S)                    # some tasks get no tokens at all
        seg_off = np.concatenate([[0], np.cumsum(lens)])
        ranks = rng.choice([4, 8, 16], n_tasks)
        d_in, d_out = [(1024, 2048), (4096, 512), (1536, 1000)][trial % 3]
        p = wl.make_custom("adv", "bf16", d_in, d_out, ranks, seg_off, seg_task, trial, fill=False)
        outcomes.add(check_sliced_tables(p))
    # many tiny tasks: more rows of sums than the pass is worth, so dB stays with the reduction kernels
    lens = np.full(3000, 33)
    p = wl.make_custom("tiny-tasks", "bf16", 1024, 1024, [16] * 750, np.concatenate([[0], np.cumsum(lens)]),
                       np.arange(3000) % 750, 0, fill=False)
    outcomes.add(check_sliced_tables(p))
    assert outcomes == {True, False}


def test_fused_projections_descriptor_errors():
    mk = lambda **kw: bd.make_desc(**dict(dict(dtype="bf16", T=64, d_in=64, d_out=96, rank_off=[0, 24], seg_off=[0, 64],
                                               seg_task=[0], n_proj=3), **kw))[0]
    assert bd.validate(mk()) == 0
    assert bd.validate(mk(dtype="f32")) == 0
    assert bd.validate(mk(d_out=104)) == -8          # not a multiple of 8 x 3
    assert bd.validate(mk(rank_off=[0, 16])) == -6   # stacked rank not a multiple of 8 x 3
    assert bd.validate(mk(n_proj=-1)) == -2
    assert bd.validate(mk(n_proj=17)) == -2
    plan = bd.Plan("bf16", 64, 64, 96, [0, 24], [0, 64], [0], flags=bd.PLAN_HOST_ONLY, n_proj=3)
    assert plan.R_tot == 24
    plan.close()
