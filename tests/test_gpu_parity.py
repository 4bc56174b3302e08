"""GPU parity: the HIP library against the fp64 oracle, element by element, through the C ABI.

Tolerances (per output tensor Z in {y, dx, dA, dB}): max|Z_gpu - Z_ref| / max|Z_ref|
  <= 1e-5 on the fp32 path, <= 2e-2 on the bf16 path (bf16 storage, fp32 accumulation);
the token -> task indexing is compared bit for bit.
"""
import numpy as np
import pytest

import oracle
from paper_2509_01193_amd import binding as bd
from paper_2509_01193_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def relerr(got, ref):
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def make_oracle(p):
    if p.n_proj > 1:
        return oracle.FusedProjections(p.n_proj, p.x, p.W, p.A, p.B, p.s, p.dy, p.rank_off, p.seg_off, p.seg_task)
    return oracle.Oracle(p.x, p.W, p.A, p.B, p.s, p.dy, p.rank_off, p.seg_off, p.seg_task)


def sample_rows(p, n_random, seed=0):
    """First and last two rows of every segment, every row of short segments, plus random rows."""
    rows = set()
    for k in range(p.S):
        lo, hi = int(p.seg_off[k]), int(p.seg_off[k + 1])
        if hi - lo <= 64:
            rows.update(range(lo, hi))
        else:
            rows.update((lo, lo + 1, hi - 2, hi - 1))
    rows.update((0, p.T - 1))
    rng = np.random.default_rng(seed)
    rows.update(rng.integers(0, p.T, n_random).tolist())
    return np.asarray(sorted(r for r in rows if 0 <= r < p.T), np.int64)


def check_problem(p, rows=None, plan_flags=0, tol=None, label=""):
    """Runs fwd+bwd on the GPU and compares all four outputs with the oracle."""
    import torch
    tol = tol or TOL[p.dtype]
    dp = bd.DeviceProblem(p, plan_flags)
    dp.step()
    torch.cuda.synchronize()
    assert dp.guards_intact(), (p.name, "a write outside y, dx, dA, dB, h_save or the workspace")
    o = make_oracle(p)
    if rows is None:
        y, dx = dp.host(dp.y), dp.host(dp.dx)
    else:
        idx = torch.from_numpy(rows).to(dp.dev)
        y, dx = dp.host(dp.y.index_select(0, idx)), dp.host(dp.dx.index_select(0, idx))
    errs = {"y": relerr(y, o.y(rows)), "dx": relerr(dx, o.dx(rows))}
    if p.R_tot:
        dA, dB = o.grads()
        errs["dA"] = relerr(dp.host(dp.dA), dA)
        errs["dB"] = relerr(dp.host(dp.dB), dB)
    print("%s %s errs=%s" % (label, p.name, {k: "%.2e" % v for k, v in errs.items()}), flush=True)
    for k, v in errs.items():
        assert v <= tol, (p.name, k, v, tol)
    return dp, errs


def check_index_probe(p):
    import torch
    dp_plan = bd.Plan.for_problem(p)
    out_task = torch.full((max(p.T, 1),), -7, dtype=torch.int32, device="cuda:0")
    out_cnt = torch.full((max(p.n_tasks, 1),), -7, dtype=torch.int64, device="cuda:0")
    bd.lobra_mlora_plan_token_task_map(dp_plan, out_task, out_cnt)
    torch.cuda.synchronize()
    ref = oracle.token_task(p.T, p.seg_off, p.seg_task, p.n_tasks)
    assert np.array_equal(out_task.cpu().numpy()[: p.T], ref)
    if p.n_tasks:
        assert np.array_equal(out_cnt.cpu().numpy(), np.bincount(ref[ref >= 0], minlength=p.n_tasks))
    dp_plan.close()


# ---------------------------------------------------------------------------------------------
def test_config1_fp32_full():
    p = wl.make_config(1)
    check_index_probe(p)
    check_problem(p)


SHRUNK = {2: (264, 328), 3: (192, 344), 4: (136, 200), 5: (328, 264)}


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
@pytest.mark.parametrize("order", ["shuffled", "sorted"])
def test_token_structure_of_each_workload_on_a_narrow_layer(cfg, order):
    """Real token counts and segment tables, layer shrunk so the oracle covers every element."""
    d_in, d_out = SHRUNK[cfg]
    p = wl.make_config(cfg, order, d_in=d_in, d_out=d_out)
    check_index_probe(p)
    check_problem(p, label=order)


# layer widths that are multiples of 64 take the direct-to-LDS GEMM pipeline (the widths above take
# the register-staged one); N = 448 / 576 leaves a ragged last column tile, T a ragged last row tile
SHRUNK_64 = {2: (320, 448), 3: (192, 576), 4: (128, 320), 5: (448, 320)}


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_token_structure_on_a_narrow_layer_whole_k_tiles(cfg):
    d_in, d_out = SHRUNK_64[cfg]
    p = wl.make_config(cfg, "shuffled", d_in=d_in, d_out=d_out)
    check_problem(p, label="k64")


@pytest.mark.parametrize("rank", [24, 32, 96])
def test_long_batch_at_medium_and_large_rank_takes_the_lds_staged_kernels(rank):
    """Workload 5's tokens at a uniform rank of 24 / 32 / 96: runs of four token blocks in the projection
    (two or eight rank blocks staged in LDS) and the 256-column tiles of the gradient reduction (rank 96:
    two passes of 64 ranks)."""
    p = wl.make_config(5, "shuffled", d_in=200, d_out=264, fill=False)
    p.ranks = np.full_like(p.ranks, rank)
    p.fill()
    plan = bd.Plan.for_problem(p, bd.PLAN_HOST_ONLY)
    assert int(np.diff(plan.query(bd.Q_BLOCK_RUNS)).max()) == 4
    plan.close()
    check_problem(p, label="rank %d" % rank)


@pytest.mark.parametrize("dims", [(8, 8), (16, 24), (64, 64), (72, 8), (8, 1032), (1024, 64), (2048, 256),
                                  (128, 192), (192, 320), (320, 128)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_extreme_layer_widths(dims, dtype):
    """Smallest legal widths, one K tile, K tails of 8, a single column chunk, long K."""
    d_in, d_out = dims
    lens = [3, 40, 0, 259, 1, 64, 130]
    p = wl.make_custom("widths", dtype, d_in, d_out, [1, 16, 128, 7],
                       np.concatenate([[0], np.cumsum(lens)]), [0, 1, 2, 2, -1, 3, 1], 7,
                       s=[2.0, 1.0, 0.25, -3.0], std_x=0.5, std_w=0.1, std_a=0.1, std_b=0.1)
    check_problem(p, label="%s %dx%d" % (dtype, d_in, d_out))


@pytest.mark.parametrize("T,d_in,d_out", [
    (256, 128, 256),      # one output tile, two K tiles: the stream's prologue is the whole product
    (257, 256, 384),      # one row over a tile: the second tile row is moved up by 255 rows; columns 256 .. 383 likewise
    (300, 384, 264),      # last column tile moved left by 248 columns
    (1000, 1024, 776),    # 4 x 4 tiles, both edges ragged, 16 K tiles forward and 12 (+ 8 columns: other kernel) backward
    (5000, 512, 1280),    # 20 x 5 = 100 tiles forward, 20 x 2 backward: fewer tiles than compute units
    (9000, 256, 2304),    # 36 x 9 = 324 tiles forward: more than one per compute unit, not a multiple of 8 per XCD
    (70000, 128, 256),    # 274 tile rows of one column: five tiles for some workgroups, ragged last rounds
])
def test_persistent_gemm_tile_edges_and_round_remainders(T, d_in, d_out):
    """Shapes around the persistent GEMM's assumptions (K a multiple of 128, at least one whole tile): tile rows and
    columns that are moved inwards, tile counts below, at and above the number of compute units, rounds that do not
    fill.  Segments are placed so that tile boundaries fall inside segments of every kind."""
    rng = np.random.default_rng(T + d_in)
    lens = []
    while sum(lens) < T:
        lens.append(int(rng.choice([1, 31, 100, 255, 257, 600])))
    lens[-1] -= sum(lens) - T
    seg_task = rng.integers(-1, 3, len(lens))
    p = wl.make_custom("edges-%dx%dx%d" % (T, d_in, d_out), "bf16", d_in, d_out, [16, 8, 40],
                       np.concatenate([[0], np.cumsum(lens)]), seg_task, 17, s=[2.0, -1.0, 0.5],
                       std_x=1.0, std_w=0.05, std_a=0.05, std_b=0.05)
    rows = None if T <= 9000 else sample_rows(p, 600, seed=1)
    check_problem(p, rows=rows, label="edges")


@pytest.mark.parametrize("n_proj", [1, 2])
def test_persistent_gemm_up_projection_at_every_kind_of_rank(n_proj):
    """The GEMM's fused up projection takes the operands of a tile's first segment from a copy made ahead of the
    epilogue when the rank window is at most 32, and loads them itself otherwise and for every further segment:
    ranks below, at and above 8, 16 and 32 (windows that end inside an 8-rank group rely on the masking), tiles
    crossed by one and by many segments, the last tile row moved up."""
    rng = np.random.default_rng(4400 + n_proj)
    ranks = [1, 3, 12, 17, 31, 32, 33, 8] if n_proj == 1 else [8, 16, 24, 32, 40]
    lens = []
    while sum(lens) < 3000:
        lens.append(int(rng.choice([1, 31, 100, 255, 257, 600])))
    lens[-1] -= sum(lens) - 3000
    seg_task = rng.integers(-1, len(ranks), len(lens))
    kw = dict(std_x=1.0, std_w=0.05, std_a=0.05, std_b=0.05)
    base = wl.make_custom("uprank-%d" % n_proj, "bf16", 256, 384, ranks, np.concatenate([[0], np.cumsum(lens)]), seg_task,
                          23, s=rng.uniform(-2, 2, len(ranks)).astype(np.float32), fill=(n_proj == 1), **kw)
    p = base if n_proj == 1 else wl.fuse_projections(base, n_proj, **kw)
    check_problem(p, label="up projection ranks %s x %d" % (ranks, n_proj))


def test_config3_reversed_rank_pairing():
    p = wl.make_config(3, "shuffled", d_in=192, d_out=344, reverse_ranks=True)
    check_problem(p)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_adapter_term_alone_w_zero(dtype):
    """W = 0 leaves only the adapter path under the tolerance; B_t scaled by (t+1) separates tasks."""
    p = wl.make_config(2, "shuffled", d_in=512, d_out=384)
    if dtype == "f32":
        for k in ("x", "W", "A", "B", "dy"):
            setattr(p, k, wl.bf16_bits_to_f32(getattr(p, k)))
        p.dtype = "f32"
    p.W = np.zeros_like(p.W)
    ro = p.rank_off
    for t in range(p.n_tasks):
        blk = wl.bf16_bits_to_f32(p.B[ro[t]:ro[t + 1]]) if dtype == "bf16" else p.B[ro[t]:ro[t + 1]]
        blk = blk * np.float32(t + 1)
        p.B[ro[t]:ro[t + 1]] = wl.f32_to_bf16_bits(blk) if dtype == "bf16" else blk
    check_problem(p, label="W=0 " + dtype)


def adversarial_tables():
    rng = np.random.default_rng(42)
    out = {}
    # boundaries at every residue of the tile sizes, one-token and empty segments, no-adapter spans
    lens = [1, 0, 31, 1, 33, 255, 2, 257, 0, 16, 16, 16, 16, 300, 1, 1, 1, 511, 17]
    out["residues"] = (np.concatenate([[0], np.cumsum(lens)]), rng.integers(-1, 4, len(lens)))
    out["alternate16"] = (np.arange(0, 16 * 41, 16), np.arange(40) % 4)
    out["single"] = (np.asarray([0, 777]), np.asarray([2]))
    out["task_without_tokens"] = (np.asarray([0, 100, 300, 301]), np.asarray([0, 3, 0]))
    out["no_adapter_only"] = (np.asarray([0, 130]), np.asarray([-1]))
    out["one_token_each"] = (np.arange(0, 70), np.arange(69) % 3)
    return out


@pytest.mark.parametrize("name", sorted(adversarial_tables()))
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_adversarial_segment_tables(name, dtype):
    seg_off, seg_task = adversarial_tables()[name]
    p = wl.make_custom(name, dtype, 136, 264, [8, 16, 5, 64], seg_off, seg_task, 99,
                       s=[2.0, 0.5, -1.0, 3.0])
    check_index_probe(p)
    dp, _ = check_problem(p, label=dtype)
    if name == "task_without_tokens":
        ro = p.rank_off
        for t in (1, 2):
            assert not dp.dA[ro[t]:ro[t + 1]].any().item() and not dp.dB[ro[t]:ro[t + 1]].any().item()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_flags_saved_h_determinism_and_canaries(dtype):
    import torch
    p = wl.make_config(2, "shuffled", d_in=264, d_out=328)
    if dtype == "f32":
        for k in ("x", "W", "A", "B", "dy"):
            setattr(p, k, wl.bf16_bits_to_f32(getattr(p, k)))
        p.dtype = "f32"
    dp = bd.DeviceProblem(p)
    # outputs live inside larger buffers whose margins must stay untouched
    pad = 1024

    def padded(t):
        big = torch.full((t.numel() + 2 * pad,), 7.0, dtype=t.dtype, device=t.device)
        return big, big[pad:pad + t.numel()].view(t.shape)
    bigs = {}
    for name in ("y", "dx", "dA", "dB"):
        bigs[name], view = padded(getattr(dp, name))
        setattr(dp, name, view)
    dp.step()
    torch.cuda.synchronize()
    first = {n: getattr(dp, n).clone() for n in ("y", "dx", "dA", "dB")}
    for name, big in bigs.items():
        assert (big[:pad] == 7.0).all().item() and (big[-pad:] == 7.0).all().item(), name
    # same call again: bit-identical (fixed reduction order)
    dp.step()
    torch.cuda.synchronize()
    for n, v in first.items():
        assert torch.equal(getattr(dp, n), v), n
    # recomputing h in bwd instead of using the saved copy gives the same bits
    dp.fwd(save_h=False)
    dp.bwd(use_saved_h=False)
    torch.cuda.synchronize()
    for n, v in first.items():
        assert torch.equal(getattr(dp, n), v), n
    # accumulate: dA, dB doubled; NO_DX leaves dx alone
    dp.dx.fill_(3.0)
    dp.bwd(flags=bd.FLAG_ACCUMULATE_GRADS | bd.FLAG_NO_DX)
    torch.cuda.synchronize()
    assert torch.equal(dp.dA, 2 * first["dA"]) and torch.equal(dp.dB, 2 * first["dB"])
    assert (dp.dx == 3.0).all().item()


def test_empty_batch_and_argument_errors():
    import torch
    p = wl.make_custom("empty", "bf16", 64, 64, [8], [0], [], 5)
    dp = bd.DeviceProblem(p)
    dp.dA.fill_(1.0)
    dp.step()
    torch.cuda.synchronize()
    assert not dp.dA.any().item()                 # no tokens: gradients are zero
    p = wl.make_config(1)
    dp = bd.DeviceProblem(p)
    st = bd.lobra_mlora_plan_fwd(dp.plan, None, dp.W, dp.A, dp.B, dp.s, dp.y, check=False)
    assert st == -1
    st = bd.lobra_mlora_plan_fwd(dp.plan, dp.x, dp.W, dp.A, dp.B, dp.s, dp.y, None, None, check=False)
    assert st == -7                               # needs scratch when h_save is not given
    st = bd.lobra_mlora_plan_bwd(dp.plan, dp.x, dp.W, dp.A, dp.B, dp.s, dp.dy, None, dp.dx, dp.dA, dp.dB,
                            0, dp.ws[:64], check=False)
    assert st == -7
    off = dp.x.view(-1)[1:1 + dp.x.numel() - 4]
    st = bd.lib().lobra_mlora_plan_fwd(dp.plan.handle, off.data_ptr(), dp.W.data_ptr(), dp.A.data_ptr(),
                                  dp.B.data_ptr(), dp.s.data_ptr(), dp.y.data_ptr(), None,
                                  dp.ws.data_ptr(), dp.ws.numel(), None)
    assert st == -8


def test_mfma_kernels_against_plain_kernels_every_element_full_size():
    """Workload 2 at full size: the MFMA path against the plain fp32-FMA kernels on the same bf16
    storage, all elements (the oracle covers sampled rows of this size in the test below)."""
    import torch
    p = wl.make_config(2, "shuffled")
    a = bd.DeviceProblem(p)
    a.step()
    b = bd.DeviceProblem(p, bd.PLAN_PLAIN_KERNELS)
    b.step()
    torch.cuda.synchronize()
    for name in ("y", "dx", "dA", "dB"):
        x, y = getattr(a, name).float(), getattr(b, name).float()
        err = ((x - y).abs().max() / y.abs().max()).item()
        print("mfma vs plain %s: %.2e" % (name, err), flush=True)
        assert err <= 1e-2, (name, err)


# ---------------------------------------------------------------------------------------------
# full-size workloads in the launch configuration bench.py times: sampled rows of y and dx that
# the oracle computes one by one, dA and dB in full
# ---------------------------------------------------------------------------------------------
FULL_ROWS = {2: 1024, 3: 768, 4: 96, 5: 256}


def test_full_size_workload2_with_unit_variance_activations():
    """Sensitivity row: x ~ N(0, 1) instead of N(0, 0.02) (the workload text fixes x only for workload 1)."""
    p = wl.make_config(2, "sorted", std_x=1.0)
    check_problem(p, rows=sample_rows(p, 512, seed=3), label="x~N(0,1)")


@pytest.mark.parametrize("cfg", [2, 3, 5, 4])
def test_full_size_workload_sampled_rows(cfg):
    p = wl.make_config(cfg, "shuffled")
    rows = sample_rows(p, FULL_ROWS[cfg])
    # the last rows sit beyond 2^32 bytes in y/dy at workload 4
    dp, errs = check_problem(p, rows=rows, label="full rows=%d" % len(rows))
    import torch
    if cfg in (2, 5):
        # the launch configuration bench.py times is a replay of a HIP graph of one step: at full size
        # every replay must reproduce, bit for bit, what the eager step just checked against the oracle
        want = [t.clone() for t in (dp.y, dp.dx, dp.dA, dp.dB)]
        g, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                dp.step()
        torch.cuda.synchronize()
        for rep in range(2):
            for t in (dp.y, dp.dx, dp.dA, dp.dB):
                t.fill_(5.0)
            g.replay()
            torch.cuda.synchronize()
            for a, b, name in zip(want, (dp.y, dp.dx, dp.dA, dp.dB), ("y", "dx", "dA", "dB")):
                assert torch.equal(a, b), (cfg, rep, name)
        del g, want
    del dp
    torch.cuda.empty_cache()


# ---------------------------------------------------------------------------------------------
# randomised problems: widths, ranks, tables and scales drawn from a seeded generator
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(12))
def test_random_problems(seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = "bf16" if seed % 3 else "f32"
    mult = 8 if dtype == "bf16" else 1
    d_in = int(rng.integers(1, 80)) * mult
    d_out = int(rng.integers(1, 80)) * mult
    n_tasks = int(rng.integers(1, 7))
    ranks = rng.choice([1, 2, 4, 8, 15, 16, 17, 32, 48, 64, 100, 128], n_tasks)
    S = int(rng.integers(1, 30))
    lens = rng.choice([0, 1, 2, 7, 16, 31, 32, 33, 63, 64, 65, 200, 256, 300, 700], S)
    seg_task = rng.integers(-1, n_tasks, S)
    seg_off = np.concatenate([[0], np.cumsum(lens)])
    s = rng.uniform(-2, 2, n_tasks).astype(np.float32)
    p = wl.make_custom("random%d" % seed, dtype, d_in, d_out, ranks, seg_off, seg_task, 500 + seed, s=s,
                       std_x=1.0, std_w=0.05, std_a=0.05, std_b=0.05)
    check_index_probe(p)
    check_problem(p, label="%s %dx%d n=%d T=%d" % (dtype, d_in, d_out, n_tasks, p.T))


def test_padded_bucket_layout_as_no_adapter_spans():
    """The paper's default layout pads every sequence of a chunk to a bucket boundary (section 2.1).
    Pad tokens are segments of task -1: they take the base product only and stay out of dA, dB."""
    import torch
    lens, tasks, bucket = [100, 250, 17, 256, 190], [0, 1, 1, 0, 2], 256
    # the [b, s_j] chunk with its valid lengths, turned into a segment table by the library's own helper
    seg_off, seg_task, T = bd.lobra_padded_segments(lens, tasks, 3, None, bucket)
    assert T == len(lens) * bucket and seg_off.tolist() == [0, 100, 256, 506, 512, 529, 768, 1024, 1024, 1214, 1280]
    padded = wl.make_custom("padded", "bf16", 320, 192, [16, 8, 32], seg_off, seg_task, 11)
    dp, _ = check_problem(padded, label="padded")
    # the packed batch of the same sequences gives the same adapter gradients
    keep = np.concatenate([np.arange(seg_off[k], seg_off[k + 1]) for k in range(len(seg_task)) if seg_task[k] >= 0])
    packed = wl.make_custom("packed", "bf16", 320, 192, [16, 8, 32], np.concatenate([[0], np.cumsum(lens)]), tasks, 11)
    packed.x, packed.dy = padded.x[keep], padded.dy[keep]
    packed.W, packed.A, packed.B = padded.W, padded.A, padded.B
    dq = bd.DeviceProblem(packed)
    dq.step()
    torch.cuda.synchronize()
    idx = torch.from_numpy(keep).to(dp.dev)
    assert torch.equal(dp.y.index_select(0, idx), dq.y) and torch.equal(dp.dx.index_select(0, idx), dq.dx)
    for a, b in ((dp.dA, dq.dA), (dp.dB, dq.dB)):
        assert ((a - b).abs().max() / b.abs().max()).item() < 1e-5      # same terms, other summation order


@pytest.mark.parametrize("kernels", ["register-staged-gemm", "persistent-gemm", "sliced-projection-fused-db"])
def test_fwd_bwd_under_hip_graph_capture(kernels):
    """fwd and bwd allocate nothing and never synchronise, so a step can be captured in a HIP graph.
    Every replay (with fresh inputs written into the same buffers and eager work in between) must
    reproduce the eager result bit for bit.  Once per family of kernels a step can consist of: the GEMM for
    widths that are not whole K tiles, the persistent GEMM (with the up projection's operands copied ahead), and
    the K-sliced projection with dB fused into the pass over dy."""
    import torch
    if kernels == "register-staged-gemm":
        p = wl.make_config(2, "shuffled", d_in=320, d_out=448)
    elif kernels == "persistent-gemm":
        p = wl.make_config(2, "shuffled", d_in=512, d_out=768)
    else:
        p = wl.make_config(4, "shuffled", d_in=1024, d_out=1024)
        q = bd.Plan.for_problem(p, bd.PLAN_HOST_ONLY).query(bd.Q_SLICED)
        assert q[0] > 0 and q[1] > 0 and q[2] == 1, q      # the plan does take the sliced kernels here
    dp = bd.DeviceProblem(p)
    dp.step()                                     # warm-up outside capture (first-call attribute set-up)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            dp.step()
    torch.cuda.synchronize()
    rng = torch.Generator(device="cuda").manual_seed(3)
    for rep in range(3):
        dp.x.copy_((torch.randn(dp.x.shape, device="cuda", generator=rng) * 0.02).to(dp.x.dtype))
        dp.dy.copy_(torch.randn(dp.dy.shape, device="cuda", generator=rng).to(dp.dy.dtype))
        for t in (dp.y, dp.dx, dp.dA, dp.dB):
            t.fill_(7.0)
        g.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (dp.y, dp.dx, dp.dA, dp.dB)]
        for t in (dp.y, dp.dx, dp.dA, dp.dB):
            t.fill_(-3.0)
        dp.step()                                 # eager, same inputs
        torch.cuda.synchronize()
        for a, b, name in zip(got, (dp.y, dp.dx, dp.dA, dp.dB), ("y", "dx", "dA", "dB")):
            assert torch.equal(a, b), (rep, name)


@pytest.mark.parametrize("which", ["cfg1-f32", "cfg2-bf16-narrow", "adversarial-bf16"])
def test_one_shot_descriptor_forms_against_the_oracle(which):
    """lobra_mlora_workspace_bytes / lobra_mlora_fwd / lobra_mlora_bwd / lobra_token_task_map on the descriptor
    itself: no plan object, the tables travel in the caller's workspace.  Compared with the oracle element by
    element; the workspace sits between sentinel margins that must survive."""
    import torch
    if which == "cfg1-f32":
        p = wl.make_config(1)
    elif which == "cfg2-bf16-narrow":
        p = wl.make_config(2, "shuffled", d_in=384, d_out=256)       # the persistent GEMM and the MFMA rank-r kernels
    else:
        seg_off, seg_task = adversarial_tables()["residues"]          # empty and one-token segments, no-adapter spans
        p = wl.make_custom("one-shot-residues", "bf16", 136, 72, [8, 16, 5, 64], seg_off, seg_task, 21)
    dp = bd.DeviceProblem(p)                      # only for the uploaded tensors and output buffers
    d, keep = bd.make_desc(p.dtype, p.T, p.d_in, p.d_out, p.rank_off, p.seg_off, p.seg_task)
    fwd_b, bwd_b = bd.lobra_mlora_workspace_bytes(d)
    margin = 4096
    buf = torch.full((max(fwd_b, bwd_b) + 2 * margin,), 0x5A, dtype=torch.uint8, device="cuda")
    ws_f, ws_b = buf[margin:margin + fwd_b], buf[margin:margin + bwd_b]
    for t in (dp.y, dp.dx):
        t.fill_(7.0)
    # forward without h_save, backward recomputing the projections
    bd.lobra_mlora_fwd(d, dp.x, dp.W, dp.A, dp.B, dp.s, dp.y, None, ws_f)
    bd.lobra_mlora_bwd(d, dp.x, dp.W, dp.A, dp.B, dp.s, dp.dy, None, dp.dx, dp.dA, dp.dB, 0, ws_b)
    torch.cuda.synchronize()
    assert bool((buf[:margin] == 0x5A).all()) and bool((buf[margin + max(fwd_b, bwd_b):] == 0x5A).all())
    o = make_oracle(p)
    dA, dB = o.grads()
    tol = TOL[p.dtype]
    errs = {"y": relerr(dp.host(dp.y), o.y()), "dx": relerr(dp.host(dp.dx), o.dx()),
            "dA": relerr(dp.host(dp.dA), dA), "dB": relerr(dp.host(dp.dB), dB)}
    print("one-shot", p.name, {k: "%.2e" % v for k, v in errs.items()}, flush=True)
    assert all(v <= tol for v in errs.values()), errs
    # with h_save handed from fwd to bwd: the same results as the plan forms, bit for bit
    y1, dx1, dA1, dB1 = (t.clone() for t in (dp.y, dp.dx, dp.dA, dp.dB))
    bd.lobra_mlora_fwd(d, dp.x, dp.W, dp.A, dp.B, dp.s, dp.y, dp.h_save, ws_f)
    bd.lobra_mlora_bwd(d, dp.x, dp.W, dp.A, dp.B, dp.s, dp.dy, dp.h_save, dp.dx, dp.dA, dp.dB, 0, ws_b)
    torch.cuda.synchronize()
    y2, dx2, dA2, dB2 = (t.clone() for t in (dp.y, dp.dx, dp.dA, dp.dB))
    dp.step()
    torch.cuda.synchronize()
    for a, b, c, name in ((y1, y2, dp.y, "y"), (dx1, dx2, dp.dx, "dx"), (dA1, dA2, dp.dA, "dA"), (dB1, dB2, dp.dB, "dB")):
        assert torch.equal(b, c), name
        assert torch.equal(a, c), name            # recomputed projections are the same numbers
    # index probe on the descriptor (its tables go into the library's static device array)
    out_task = torch.full((p.T,), -7, dtype=torch.int32, device="cuda")
    out_cnt = torch.full((p.n_tasks,), -7, dtype=torch.int64, device="cuda")
    bd.lobra_token_task_map(d, out_task, out_cnt)
    torch.cuda.synchronize()
    ref = oracle.token_task(p.T, p.seg_off, p.seg_task, p.n_tasks)
    assert np.array_equal(out_task.cpu().numpy(), ref)
    assert np.array_equal(out_cnt.cpu().numpy(), np.bincount(ref[ref >= 0], minlength=p.n_tasks))


def test_plan_in_caller_memory_and_under_graph_capture():
    """lobra_mlora_plan_init: the plan's device image lives in a buffer of the caller's (no hipMalloc, no blocking
    copy); its calls give the results of a lobra_mlora_plan_create plan bit for bit, also as replays of a HIP graph."""
    import torch
    p = wl.make_config(3, "shuffled", d_in=256, d_out=384)
    ref = bd.DeviceProblem(p)
    ref.step()
    torch.cuda.synchronize()
    d, keep = bd.make_desc(p.dtype, p.T, p.d_in, p.d_out, p.rank_off, p.seg_off, p.seg_task)
    n = bd.plan_device_bytes(d)
    margin = 1024
    mem = torch.full((n + 2 * margin,), 0xA5, dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        plan = bd.Plan(p.dtype, p.T, p.d_in, p.d_out, p.rank_off, p.seg_off, p.seg_task, device_mem=mem[margin:margin + n],
                       stream=side)
        assert (plan.h_save_bytes, plan.fwd_ws_bytes, plan.bwd_ws_bytes) == (ref.plan.h_save_bytes, ref.plan.fwd_ws_bytes,
                                                                              ref.plan.bwd_ws_bytes)
        dp = bd.DeviceProblem.__new__(bd.DeviceProblem)
        dp.__dict__.update(ref.__dict__)
        dp.plan = plan
        dp.y, dp.dx, dp.dA, dp.dB = (torch.full_like(t, 3.0) for t in (ref.y, ref.dx, ref.dA, ref.dB))
        dp.step()                                 # on the stream of the upload, hence behind it
    torch.cuda.synchronize()
    assert bool((mem[:margin] == 0xA5).all()) and bool((mem[margin + n:] == 0xA5).all())
    for a, b, name in ((dp.y, ref.y, "y"), (dp.dx, ref.dx, "dx"), (dp.dA, ref.dA, "dA"), (dp.dB, ref.dB, "dB")):
        assert torch.equal(a, b), name
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            dp.step()
    for rep in range(2):
        for t in (dp.y, dp.dx, dp.dA, dp.dB):
            t.fill_(-1.0)
        g.replay()
        torch.cuda.synchronize()
        for a, b, name in ((dp.y, ref.y, "y"), (dp.dx, ref.dx, "dx"), (dp.dA, ref.dA, "dA"), (dp.dB, ref.dB, "dB")):
            assert torch.equal(a, b), (rep, name)
    plan.close()


def test_shared_input_projection_fusion_through_the_same_entry_point():
    """q/k/v (or gate/up) LoRA-linears read the same x: one call with W concatenated along d_out, A_t
    stacked along the rank and B_t block-diagonal computes all three layers at once."""
    import torch
    d_in, d = 320, 128
    base = wl.make_config(2, "shuffled", d_in=d_in, d_out=d)
    parts = []
    for j in range(3):                                   # three layers on the same x and segment table
        q = wl.make_custom("proj%d" % j, "bf16", d_in, d, base.ranks, base.seg_off, base.seg_task, 40 + j, s=base.s)
        q.x = base.x
        parts.append(q)
    n, r = base.n_tasks, int(base.ranks[0])
    fused = wl.make_custom("fused", "bf16", d_in, 3 * d, base.ranks * 3, base.seg_off, base.seg_task, 50, s=base.s)
    fused.x = base.x
    fused.W = np.concatenate([q.W for q in parts], axis=1)
    fused.dy = np.concatenate([q.dy for q in parts], axis=1)
    fused.A = np.concatenate([np.concatenate([q.A[t * r:(t + 1) * r] for q in parts]) for t in range(n)])
    fused.B = np.zeros((3 * r * n, 3 * d), np.uint16)
    for t in range(n):
        for j, q in enumerate(parts):
            fused.B[(3 * t + j) * r:(3 * t + j + 1) * r, j * d:(j + 1) * d] = q.B[t * r:(t + 1) * r]
    df = bd.DeviceProblem(fused)
    df.step()
    dps = [bd.DeviceProblem(q) for q in parts]
    for dq in dps:
        dq.step()
    torch.cuda.synchronize()
    y = torch.cat([dq.y for dq in dps], dim=1).float()
    assert ((df.y.float() - y).abs().max() / y.abs().max()).item() < 1e-2     # bf16 outputs, other summation order
    dx = sum(dq.dx.float() for dq in dps)
    assert ((df.dx.float() - dx).abs().max() / dx.abs().max()).item() < 2e-2
    for t in range(n):
        for j, dq in enumerate(dps):
            rows = slice((3 * t + j) * r, (3 * t + j + 1) * r)
            a, b = df.dA[rows], dq.dA[t * r:(t + 1) * r]
            assert ((a - b).abs().max() / b.abs().max()).item() < 1e-2
            a, b = df.dB[rows, j * d:(j + 1) * d], dq.dB[t * r:(t + 1) * r]
            assert ((a - b).abs().max() / b.abs().max()).item() < 1e-2
    check_problem(fused, label="fused qkv")            # and the fused call itself against the oracle


# ---------------------------------------------------------------------------------------------
# fused shared-input projections (desc.n_proj > 1): stacked down factors, compact up factors
# ---------------------------------------------------------------------------------------------
def _fused_base(d_in, dg, ranks, dtype="bf16"):
    """Workload 2's token structure on a narrow layer with the given per-projection ranks."""
    base = wl.make_config(2, "shuffled", d_in=d_in, d_out=dg, fill=False)
    base.dtype = dtype
    base.ranks = np.asarray(ranks, np.int32)
    base.s = np.linspace(0.5, 2.0, len(ranks)).astype(np.float32)
    base.seg_off, base.seg_task = wl.segments_from_sequences(
        [(int(base.seg_off[k + 1] - base.seg_off[k]), int(base.seg_task[k]) % len(ranks)) for k in range(base.S)])
    return base


@pytest.mark.parametrize("n_proj,d_in,dg,ranks", [
    (3, 320, 256, [16, 16, 16, 16]),      # q/k/v at the benchmark's rank; whole K tiles
    (2, 256, 256, [16, 32, 8]),           # the persistent GEMM in both directions, one launch over both projections
    (2, 264, 192, [8, 16, 32, 64]),       # gate/up, heterogeneous ranks, widths off the tile grid
    (3, 128, 64, [8, 24, 40]),            # windows that are not multiples of 16
    (4, 192, 128, [32]),                  # one task, stacked rank 128
])
def test_fused_shared_input_projections(n_proj, d_in, dg, ranks):
    import torch
    base = _fused_base(d_in, dg, ranks)
    f = wl.fuse_projections(base, n_proj)
    dp, _ = check_problem(f, label="fused x%d" % n_proj)
    want = [t.clone() for t in (dp.y, dp.dx, dp.dA, dp.dB)]
    # recomputed H, dx skipped, gradients accumulated: same numbers
    dp.dA.fill_(1.0)
    dp.dB.fill_(-2.0)
    dp.dx.fill_(9.0)
    dp.bwd(use_saved_h=False, flags=bd.FLAG_ACCUMULATE_GRADS | bd.FLAG_NO_DX)
    torch.cuda.synchronize()
    assert bool((dp.dx.float() == 9.0).all())
    assert torch.allclose(dp.dA - 1.0, want[2], rtol=0, atol=1e-5 * float(want[2].abs().max()) + 1e-6)
    assert torch.allclose(dp.dB + 2.0, want[3], rtol=0, atol=1e-5 * float(want[3].abs().max()) + 1e-6)
    # against n_proj separate calls on the slices: y and the gradients are the same arithmetic
    ro = f.rank_off
    for j in range(n_proj):
        rows = np.concatenate([np.arange(ro[t] + j * r, ro[t] + (j + 1) * r) for t, r in enumerate(base.ranks)])
        q = wl.make_custom("part%d" % j, "bf16", d_in, dg, base.ranks, base.seg_off, base.seg_task, 1, s=base.s, fill=False)
        q.x, q.W, q.dy = f.x, np.ascontiguousarray(f.W[:, j * dg:(j + 1) * dg]), np.ascontiguousarray(f.dy[:, j * dg:(j + 1) * dg])
        q.A, q.B = np.ascontiguousarray(f.A[rows]), np.ascontiguousarray(f.B[rows])
        dq = bd.DeviceProblem(q)
        dq.step()
        torch.cuda.synchronize()
        idx = torch.from_numpy(rows).to(dp.dev)
        assert torch.equal(want[0][:, j * dg:(j + 1) * dg], dq.y), j
        # (the reductions may run in another kernel instantiation, i.e. another fixed summation order)
        for got, ref in ((want[3].index_select(0, idx), dq.dB), (want[2].index_select(0, idx), dq.dA)):
            assert float((got - ref).abs().max()) <= 1e-5 * float(ref.abs().max()), j


@pytest.mark.parametrize("dtype,flags", [("f32", 0), ("bf16", bd.PLAN_PLAIN_KERNELS)])
def test_fused_shared_input_projections_on_the_plain_kernels(dtype, flags):
    f = wl.fuse_projections(_fused_base(136, 72, [8, 16, 24], dtype), 3)
    dp, _ = check_problem(f, plan_flags=flags, label="fused x3 plain %s" % dtype)
    import torch
    want = [t.clone() for t in (dp.dA, dp.dB)]
    dp.bwd(use_saved_h=False)                     # recomputed H
    torch.cuda.synchronize()
    assert torch.equal(dp.dA, want[0]) and torch.equal(dp.dB, want[1])



@pytest.mark.parametrize("name", sorted(adversarial_tables()))
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fused_projections_adversarial_segment_tables(name, dtype):
    """The adversarial tables above under a fused two-layer call (per-projection ranks 8, 16, 24, 64)."""
    seg_off, seg_task = adversarial_tables()[name]
    base = wl.make_custom(name, dtype, 136, 128, [8, 16, 24, 64], seg_off, seg_task, 99,
                          s=[2.0, 0.5, -1.0, 3.0], fill=False)
    f = wl.fuse_projections(base, 2)
    dp, _ = check_problem(f, label="fused x2 %s" % dtype)
    if name == "task_without_tokens":
        ro = f.rank_off
        for t in (1, 2):
            assert not dp.dA[ro[t]:ro[t + 1]].any().item() and not dp.dB[ro[t]:ro[t + 1]].any().item()


def test_fused_projections_on_a_long_batch_with_large_stacked_ranks():
    """Two fused layers on workload 5's tokens, rank 32 each (stacked 64): the forward projection takes the
    LDS-staged kernel on runs of four blocks, dA the LDS-staged reduction over the stacked ranks, and dB the
    same kernel with every 256-column tile in its projection's rank window."""
    base = wl.make_config(5, "shuffled", d_in=136, d_out=256, fill=False)
    base.ranks = np.full_like(base.ranks, 32)
    f = wl.fuse_projections(base, 2)
    plan = bd.Plan.for_problem(f, bd.PLAN_HOST_ONLY)
    assert int(np.diff(plan.query(bd.Q_BLOCK_RUNS)).max()) == 4
    plan.close()
    check_problem(f, label="fused x2 long")


@pytest.mark.parametrize("seed", range(6))
def test_random_long_batches(seed):
    """Long packed batches (tens of thousands of tokens) of random shape: ranks up to 128, one to three
    fused projections, sampled rows of y and dx, dA and dB in full."""
    rng = np.random.default_rng(77000 + seed)
    P = int(rng.choice([1, 1, 2, 3]))
    d_in = int(rng.integers(1, 60)) * 8
    dg = int(rng.integers(1, 50)) * 8
    n_tasks = int(rng.integers(1, 6))
    ranks = rng.choice([8, 16, 24, 32, 40], n_tasks) if P > 1 else rng.choice([1, 3, 8, 16, 17, 24, 32, 48, 64, 96, 128], n_tasks)
    S = int(rng.integers(20, 60))
    lens = rng.choice([1, 33, 200, 700, 1500, 3000, 5000], S)
    seg_task = rng.integers(-1, n_tasks, S)
    seg_off = np.concatenate([[0], np.cumsum(lens)])
    s = rng.uniform(-2, 2, n_tasks).astype(np.float32)
    kw = dict(std_x=1.0, std_w=0.05, std_a=0.05, std_b=0.05)
    base = wl.make_custom("long%d" % seed, "bf16", d_in, dg, ranks, seg_off, seg_task, 900 + seed, s=s,
                          fill=(P == 1), **kw)
    p = base if P == 1 else wl.fuse_projections(base, P, **kw)
    check_problem(p, rows=sample_rows(p, 400, seed=seed), label="T=%d P=%d ranks=%s" % (p.T, P, list(map(int, p.ranks))))


# ---------------------------------------------------------------------------------------------
# the K-sliced projection of long batches at ranks up to 16, with and without dB fused into the pass
# over dy: adversarial tables at sizes where the plan chooses it
# ---------------------------------------------------------------------------------------------
def _sliced_case(name, seed):
    rng = np.random.default_rng(5100 + seed)
    if name == "mixed-small-ranks":
        # five tasks of ranks up to 16 in segments of every kind of length, with spans that carry no adapter
        n_tasks, ranks, d_in, d_out = 5, [16, 8, 4, 16, 12], 1024, 2048
        lens = rng.choice([1, 2, 31, 32, 33, 65, 700, 1500, 3000, 5000], 70)
        seg_task = rng.integers(-1, n_tasks, 70)
    elif name == "forty-tasks-some-empty":
        # many tasks, a third of them without a token: workgroups meet several (task, slice) runs each
        n_tasks, d_in, d_out = 40, 1536, 1024
        ranks = rng.choice([8, 16], n_tasks)
        live = rng.permutation(n_tasks)[:27]
        lens = rng.choice([40, 200, 900, 2500], 110)
        seg_task = rng.choice(live, 110)
    elif name == "one-task-one-segment":
        n_tasks, ranks, d_in, d_out = 1, [16], 2048, 1024
        lens, seg_task = np.asarray([50001]), np.asarray([0])
    else:   # "tiny-tasks": more rows of dB sums than the fused pass is worth: sliced projection, dB by the reduction kernels
        n_tasks, d_in, d_out = 750, 1024, 1024
        ranks = np.full(n_tasks, 16)
        lens = np.full(3000, 33)
        seg_task = np.arange(3000) % n_tasks
    seg_off = np.concatenate([[0], np.cumsum(lens)])
    s = rng.uniform(0.5, 2, n_tasks).astype(np.float32)
    return wl.make_custom(name, "bf16", d_in, d_out, ranks, seg_off, seg_task, 5100 + seed, s=s,
                          std_x=1.0, std_w=0.05, std_a=0.05, std_b=0.05)


@pytest.mark.parametrize("name,fused", [("mixed-small-ranks", True), ("forty-tasks-some-empty", True),
                                        ("one-task-one-segment", True), ("tiny-tasks", False)])
def test_sliced_projection_with_and_without_fused_db(name, fused):
    import torch
    p = _sliced_case(name, 0)
    plan = bd.Plan.for_problem(p, bd.PLAN_HOST_ONLY)
    nsl_in, nsl_out, is_fused = plan.query(bd.Q_SLICED)[:3].tolist()
    plan.close()
    assert nsl_in == p.d_in // 512 and nsl_out == p.d_out // 512 and bool(is_fused) == fused
    dp, _ = check_problem(p, rows=sample_rows(p, 400), label="sliced")
    # the same results on the next call (nothing of a call survives in the partial sums), with accumulation, and
    # with the down-projected activations recomputed by bwd
    first = {k: getattr(dp, k).clone() for k in ("y", "dx", "dA", "dB")}
    dp.step()
    torch.cuda.synchronize()
    for k, v in first.items():
        assert torch.equal(getattr(dp, k), v), k
    dp.bwd(flags=bd.FLAG_ACCUMULATE_GRADS)
    dp.bwd(use_saved_h=False, flags=bd.FLAG_ACCUMULATE_GRADS)
    torch.cuda.synchronize()
    for k in ("dA", "dB"):
        got, want = getattr(dp, k), 3 * first[k]
        assert ((got - want).abs().max() <= 1e-5 * want.abs().max()).item(), k
    assert dp.guards_intact()
    # the products read the projection that THIS call wrote: with all scales set to zero the adapter term is
    # exactly zero, so y and dx must equal the base-only products bit for bit - a projection left over from
    # the calls above (in the workspace, or in a cache) would show
    base = dp.base_only()                        # (shares y and dx with dp)
    base.step()
    torch.cuda.synchronize()
    y0, dx0 = dp.y.clone(), dp.dx.clone()
    dp.y.zero_()
    dp.dx.zero_()
    dp.s.zero_()
    dp.step()
    torch.cuda.synchronize()
    assert torch.equal(dp.y, y0) and torch.equal(dp.dx, dx0)
    assert float(dp.dA.abs().max()) == 0.0 and float(dp.dB.abs().max()) == 0.0


@pytest.mark.parametrize("seed", range(6))
def test_random_long_batches_at_ranks_up_to_16(seed):
    """Random long batches that the plan hands to the sliced projection in one or both directions (widths from
    512 to 4096, one to 33 tasks of ranks 1 to 16, segments from 1 token to 9000, spans without an adapter):
    sampled rows of y and dx, dA and dB in full, and bit-identical results over repeated steps."""
    import torch
    rng = np.random.default_rng(99000 + seed)
    n_tasks = int(rng.choice([1, 2, 5, 9, 33]))
    ranks = rng.choice([1, 4, 8, 12, 16], n_tasks)
    ranks[rng.integers(0, n_tasks)] = rng.choice([9, 16])
    d_in, d_out = [(512, 1024), (1024, 512), (1536, 2048), (4096, 1024), (2048, 2560)][seed % 5]
    S = int(rng.integers(max(2, n_tasks), 120))
    lens = rng.choice([1, 3, 16, 31, 32, 33, 64, 100, 500, 1500, 4000, 9000], S)
    if lens.sum() < 100000:
        lens = lens * max(1, int(110000 / max(1, lens.sum())))
    seg_task = rng.integers(-1, n_tasks, S)
    seg_off = np.concatenate([[0], np.cumsum(lens)])
    s = rng.uniform(-2, 2, n_tasks).astype(np.float32)
    p = wl.make_custom("long16-%d" % seed, "bf16", d_in, d_out, ranks, seg_off, seg_task, 99000 + seed, s=s,
                       std_x=1.0, std_w=0.05, std_a=0.05, std_b=0.05)
    plan = bd.Plan.for_problem(p, bd.PLAN_HOST_ONLY)
    q = plan.query(bd.Q_SLICED).tolist()
    plan.close()
    assert q[0] > 0 or q[1] > 0
    dp, _ = check_problem(p, rows=sample_rows(p, 300, seed=seed), label="T=%d slices=%s" % (p.T, q[:4]))
    first = {k: getattr(dp, k).clone() for k in ("y", "dx", "dA", "dB")}
    for _ in range(3):
        dp.step()
    torch.cuda.synchronize()
    for k, v in first.items():
        assert torch.equal(getattr(dp, k), v), k
    assert dp.guards_intact()
