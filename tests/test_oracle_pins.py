"""Pins of the fp64 oracle to things other than itself (CPU only).

The paper prints no worked number for the LoRA layer, so the oracle is pinned to
what the definition (section 2.1; fused batch of section 1 / Figure 1) and the
mathematics fix: a hand-computed integer case, the base-only reduction, the
merged weight W + s A^T B through a library matmul, fused batch == per-task runs,
adjoint identities, central finite differences, fp64 autograd of the per-task
formulation, structural invariances, and exact bf16 widening.  The last test
plants mistakes in copies of the oracle's C source and requires a pin to fail.
"""
import ctypes
import json
import os
import subprocess
import tempfile

import numpy as np
import pytest

import oracle
from oracle import oracle as orc_mod
from paper_2509_01193_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def small_problem(seed=7, d_in=24, d_out=20, ranks=(3, 5, 2), dtype="f32", with_gap=True):
    """Interleaved tasks, an empty segment, one no-adapter span, distinct scales."""
    seg_task = [0, 1, 2, 1, -1, 0, 2, 2] if with_gap else [0, 1, 2, 1, 0, 2, 1]
    lens = [5, 7, 1, 0, 4, 9, 3, 2][: len(seg_task)]
    seg_off = np.concatenate([[0], np.cumsum(lens)])
    p = wl.make_custom("small", dtype, d_in, d_out, ranks, seg_off, seg_task, seed,
                       s=[2.0, -0.5, 1.25], std_x=1.0, std_w=1.0, std_a=1.0, std_b=1.0)
    return p


def run(p, rows=None):
    o = oracle.Oracle(p.x, p.W, p.A, p.B, p.s, p.dy, p.rank_off, p.seg_off, p.seg_task)
    dA, dB = o.grads()
    return o.y(rows), o.dx(rows), dA, dB


def f64(p):
    conv = (lambda a: wl.bf16_bits_to_f32(a).astype(np.float64)) if p.dtype == "bf16" \
        else (lambda a: a.astype(np.float64))
    return conv(p.x), conv(p.W), conv(p.A), conv(p.B), conv(p.dy)


def relerr(a, b):
    den = np.abs(b).max()
    return np.abs(a - b).max() / (den if den > 0 else 1.0)


# ---------------------------------------------------------------------------
# the pins, as functions so that the mutation test can re-run them
# ---------------------------------------------------------------------------
def pin_golden_integer_case():
    g = json.load(open(os.path.join(GOLD, "tiny_integer_case.json")))
    a = lambda k: np.asarray(g[k], np.float32)
    o = oracle.Oracle(a("x"), a("W"), a("A"), a("B"), g["s"], a("dy"),
                      np.concatenate([[0], np.cumsum(g["ranks"])]), g["seg_off"], g["seg_task"])
    dA, dB = o.grads()
    assert np.array_equal(o.y(), np.asarray(g["y"], np.float64))
    assert np.array_equal(o.dx(), np.asarray(g["dx"], np.float64))
    assert np.array_equal(dA, np.asarray(g["dA"], np.float64))
    assert np.array_equal(dB, np.asarray(g["dB"], np.float64))


def pin_b_zero_is_base_only():
    p = small_problem()
    p.B = np.zeros_like(p.B)
    y, dx, dA, dB = run(p)
    q = small_problem()
    q.seg_task = np.full_like(q.seg_task, -1)
    yb, dxb, dAb, dBb = run(q)
    assert np.array_equal(y, yb)              # bitwise: adding s*0 changes nothing
    assert np.array_equal(dx, dxb)
    assert not dA.any() and not dAb.any() and not dBb.any()
    x, W, A, B, dy = f64(p)
    assert relerr(y, x @ W) < 1e-14 and relerr(dx, dy @ W.T) < 1e-14
    # dB does not vanish with B: it is s * h^T dy
    tok = oracle.token_task(p.T, p.seg_off, p.seg_task, p.n_tasks)
    for t in range(p.n_tasks):
        r0, r1 = p.rank_off[t], p.rank_off[t + 1]
        m = tok == t
        ref = float(p.s[t]) * (x[m] @ A[r0:r1].T).T @ dy[m]
        assert relerr(dB[r0:r1], ref) < 1e-13


def pin_single_task_merged_weight():
    p = wl.make_custom("one", "f32", 24, 20, [4], [0, 13], [0], 3, s=[1.75],
                       std_x=1.0, std_w=1.0, std_a=1.0, std_b=1.0)
    y, dx, dA, dB = run(p)
    x, W, A, B, dy = f64(p)
    M = W + 1.75 * A.T @ B                     # merged weight, section 2.1 (delta W = down * up)
    assert relerr(y, x @ M) < 1e-13
    assert relerr(dx, dy @ M.T) < 1e-13
    assert relerr(dA, 1.75 * (dy @ B.T).T @ x) < 1e-13
    assert relerr(dB, 1.75 * (x @ A.T).T @ dy) < 1e-13


def pin_fused_equals_per_task():
    p = small_problem()
    y, dx, dA, dB = run(p)
    tok = oracle.token_task(p.T, p.seg_off, p.seg_task, p.n_tasks)
    for t in range(p.n_tasks):
        m = np.nonzero(tok == t)[0]
        r0, r1 = p.rank_off[t], p.rank_off[t + 1]
        o = oracle.Oracle(p.x[m], p.W, p.A[r0:r1], p.B[r0:r1], p.s[t:t + 1], p.dy[m],
                          [0, r1 - r0], [0, len(m)], [0])
        dAt, dBt = o.grads()
        assert np.array_equal(y[m], o.y()) and np.array_equal(dx[m], o.dx())
        assert np.array_equal(dA[r0:r1], dAt) and np.array_equal(dB[r0:r1], dBt)
    m = np.nonzero(tok < 0)[0]
    x, W, A, B, dy = f64(p)
    assert relerr(y[m], x[m] @ W) < 1e-14


def pin_adjoint_identities():
    p = small_problem(seed=11)
    y, dx, dA, dB = run(p)
    x, W, A, B, dy = f64(p)
    rng = np.random.default_rng(5)
    ex = rng.standard_normal(p.x.shape).astype(np.float32)
    eA = rng.standard_normal(p.A.shape).astype(np.float32)
    eB = rng.standard_normal(p.B.shape).astype(np.float32)

    def fwd(xx, AA, BB, WW):
        o = oracle.Oracle(xx, WW, AA, BB, p.s, p.dy, p.rank_off, p.seg_off, p.seg_task)
        return o.y()
    zW = np.zeros_like(p.W)
    # y is linear in x; the adapter term is bilinear in (A, B)
    assert abs((dy * fwd(ex, p.A, p.B, p.W)).sum() - (dx * ex).sum()) < 1e-10 * np.abs(dy).sum()
    lhsA = (dy * fwd(p.x, eA, p.B, zW)).sum()
    lhsB = (dy * fwd(p.x, p.A, eB, zW)).sum()
    assert abs(lhsA - (dA * eA).sum()) < 1e-11 * max(1.0, abs(lhsA))
    assert abs(lhsB - (dB * eB).sum()) < 1e-11 * max(1.0, abs(lhsB))


def pin_finite_differences():
    p = small_problem(seed=13, d_in=6, d_out=5, ranks=(2, 1, 3))
    y, dx, dA, dB = run(p)
    dy = p.dy.astype(np.float64)

    def L(xx, AA, BB):
        o = oracle.Oracle(xx, p.W, AA, BB, p.s, p.dy, p.rank_off, p.seg_off, p.seg_task)
        return float((dy * o.y()).sum())
    eps = np.float32(0.25)     # exactly representable steps; L is (bi)linear so the quotient is exact
    for name, base, grad in (("x", p.x, dx), ("A", p.A, dA), ("B", p.B, dB)):
        worst = 0.0
        for idx in np.ndindex(base.shape):
            hi, lo = base.copy(), base.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args = {"x": (hi, p.A, p.B), "A": (p.x, hi, p.B), "B": (p.x, p.A, hi)}[name]
            args_lo = {"x": (lo, p.A, p.B), "A": (p.x, lo, p.B), "B": (p.x, p.A, lo)}[name]
            step = float(hi[idx]) - float(lo[idx])
            fd = (L(*args) - L(*args_lo)) / step
            worst = max(worst, abs(fd - grad[idx]))
        assert worst < 1e-8 * max(1.0, np.abs(grad).max()), (name, worst)


def pin_autograd_per_task():
    torch = pytest.importorskip("torch")
    p = small_problem(seed=17)
    y, dx, dA, dB = run(p)
    x, W, A, B, dy = [torch.tensor(a, dtype=torch.float64) for a in f64(p)]
    x.requires_grad_(True)
    A.requires_grad_(True)
    B.requires_grad_(True)
    out = []
    for k in range(p.S):                      # one independent LoRA layer per segment
        lo, hi, t = int(p.seg_off[k]), int(p.seg_off[k + 1]), int(p.seg_task[k])
        yk = x[lo:hi] @ W
        if t >= 0:
            r0, r1 = int(p.rank_off[t]), int(p.rank_off[t + 1])
            yk = yk + float(p.s[t]) * (x[lo:hi] @ A[r0:r1].T) @ B[r0:r1]
        out.append(yk)
    yt = torch.cat(out)
    (yt * dy).sum().backward()
    assert relerr(y, yt.detach().numpy()) < 1e-13
    assert relerr(dx, x.grad.numpy()) < 1e-13
    assert relerr(dA, A.grad.numpy()) < 1e-13
    assert relerr(dB, B.grad.numpy()) < 1e-13


def pin_structural_invariances():
    p = small_problem(seed=19)
    y, dx, dA, dB = run(p)
    # (a) permuting the segments permutes the rows of y and dx and leaves the gradients
    S = p.S
    perm = np.random.default_rng(3).permutation(S)
    lens = np.diff(p.seg_off)
    idx = np.concatenate([np.arange(p.seg_off[k], p.seg_off[k + 1]) for k in perm]).astype(np.int64)
    q = small_problem(seed=19)
    q.x, q.dy = p.x[idx], p.dy[idx]
    q.seg_task = p.seg_task[perm]
    q.seg_off = np.concatenate([[0], np.cumsum(lens[perm])]).astype(np.int32)
    y2, dx2, dA2, dB2 = run(q)
    assert np.array_equal(y2, y[idx]) and np.array_equal(dx2, dx[idx])
    assert relerr(dA2, dA) < 1e-12 and relerr(dB2, dB) < 1e-12
    # (b) splitting a segment in two changes nothing
    q = small_problem(seed=19)
    q.seg_off = np.insert(p.seg_off, 2, p.seg_off[1] + 3).astype(np.int32)
    q.seg_task = np.insert(p.seg_task, 1, p.seg_task[1]).astype(np.int32)
    for a, b in zip(run(q), (y, dx, dA, dB)):
        assert np.array_equal(a, b)
    # (c) padding a task with zero rank rows changes nothing
    q = small_problem(seed=19)
    r1 = int(p.rank_off[1])
    q.ranks = p.ranks.copy()
    q.ranks[0] += 2
    q.A = np.insert(p.A, [r1, r1], 0.0, axis=0)
    q.B = np.insert(p.B, [r1, r1], 0.0, axis=0)
    y3, dx3, dA3, dB3 = run(q)
    keep = np.r_[0:r1, r1 + 2:q.R_tot]
    assert np.array_equal(y3, y) and np.array_equal(dx3, dx)
    assert np.array_equal(dA3[keep], dA) and np.array_equal(dB3[keep], dB)
    # (d) the adapter term is linear in s_t
    q = small_problem(seed=19)
    q.s = (p.s * 3).astype(np.float32)
    y4 = run(q)[0]
    z = small_problem(seed=19)
    z.s = np.zeros_like(p.s)
    y0 = run(z)[0]
    assert relerr(y4 - y0, 3 * (y - y0)) < 1e-13


def pin_bf16_widening_and_row_subset():
    p = small_problem(seed=23, dtype="bf16")
    y, dx, dA, dB = run(p)
    q = small_problem(seed=23, dtype="bf16")
    for k in ("x", "W", "A", "B", "dy"):
        setattr(q, k, wl.bf16_bits_to_f32(getattr(p, k)))
    q.dtype = "f32"
    for a, b in zip(run(q), (y, dx, dA, dB)):
        assert np.array_equal(a, b)
    rows = np.asarray([p.T - 1, 0, 12, 12, 5], np.int64)
    ys, dxs, _, _ = run(p, rows)
    assert np.array_equal(ys, y[rows]) and np.array_equal(dxs, dx[rows])
    x, W, A, B, dy = f64(p)
    assert relerr(y[p.seg_off[4]:p.seg_off[5]], (x @ W)[p.seg_off[4]:p.seg_off[5]]) < 1e-14


def pin_token_task_map():
    rng = np.random.default_rng(1)
    for _ in range(20):
        S = int(rng.integers(1, 12))
        lens = rng.integers(0, 9, S)
        seg_off = np.concatenate([[0], np.cumsum(lens)])
        seg_task = rng.integers(-1, 4, S)
        ref = []
        for k in range(S):
            ref += [int(seg_task[k])] * int(lens[k])
        got = oracle.token_task(int(seg_off[-1]), seg_off, seg_task, 4)
        assert got.tolist() == ref
    with pytest.raises(ValueError):
        oracle.token_task(5, [0, 3, 2, 5], [0, 0, 0], 1)      # decreasing offsets
    with pytest.raises(ValueError):
        oracle.token_task(5, [0, 5], [2], 2)                  # task id out of range
    with pytest.raises(ValueError):
        oracle.token_task(6, [0, 5], [0], 1)                  # table does not cover T


def pin_projected_activations():
    """The optional outputs h_i = A_t x_i and g_i = B_t dy_i (section 2.1: the down factor applied to the token)
    against numpy's matmul per segment; rows without adapter and ranks beyond r_t are zero; a row subset gives
    the rows of the full result."""
    for dtype in ("f32", "bf16"):
        p = small_problem(dtype=dtype, d_in=24, d_out=16)
        x, W, A, B, dy = f64(p)
        task_of = oracle.token_task(p.T, p.seg_off, p.seg_task, p.n_tasks)
        y, h = oracle.forward(p.x, p.W, p.A, p.B, p.s, p.rank_off, task_of, want_h=True)
        dx, g = oracle.backward_dx(p.W, p.A, p.B, p.s, p.dy, p.rank_off, task_of, want_g=True)
        r_max = int(np.max(p.ranks))
        href, gref = np.zeros((p.T, r_max)), np.zeros((p.T, r_max))
        for k in range(p.S):
            t = int(p.seg_task[k])
            if t < 0:
                continue
            m = slice(int(p.seg_off[k]), int(p.seg_off[k + 1]))
            r0, r1 = int(p.rank_off[t]), int(p.rank_off[t + 1])
            href[m, : r1 - r0] = x[m] @ A[r0:r1].T
            gref[m, : r1 - r0] = dy[m] @ B[r0:r1].T
        assert h.shape == href.shape and relerr(h, href) < 1e-13 and relerr(g, gref) < 1e-13
        assert not h[task_of < 0].any() and not g[task_of < 0].any()
        for t in range(p.n_tasks):
            assert not h[task_of == t, int(p.ranks[t]):].any() and not g[task_of == t, int(p.ranks[t]):].any()
        # y and dx are what the calls return without the optional output
        assert np.array_equal(y, oracle.forward(p.x, p.W, p.A, p.B, p.s, p.rank_off, task_of))
        assert np.array_equal(dx, oracle.backward_dx(p.W, p.A, p.B, p.s, p.dy, p.rank_off, task_of))
        rows = np.asarray([p.T - 1, 0, 6, 6, 13], np.int64)
        assert np.array_equal(oracle.forward(p.x, p.W, p.A, p.B, p.s, p.rank_off, task_of, rows, want_h=True)[1], h[rows])
        assert np.array_equal(oracle.backward_dx(p.W, p.A, p.B, p.s, p.dy, p.rank_off, task_of, rows, want_g=True)[1], g[rows])


PINS = [pin_golden_integer_case, pin_projected_activations, pin_b_zero_is_base_only, pin_single_task_merged_weight,
        pin_fused_equals_per_task, pin_adjoint_identities, pin_finite_differences,
        pin_autograd_per_task, pin_structural_invariances, pin_bf16_widening_and_row_subset,
        pin_token_task_map]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin()


def test_config1_against_library_matmul():
    """Workload 1 in full against numpy fp64 matmul taken segment by segment."""
    p = wl.make_config(1)
    y, dx, dA, dB = run(p)
    x, W, A, B, dy = f64(p)
    yr, dxr = x @ W, dy @ W.T
    dAr, dBr = np.zeros_like(dA), np.zeros_like(dB)
    for k in range(p.S):
        lo, hi, t = p.seg_off[k], p.seg_off[k + 1], p.seg_task[k]
        r0, r1 = p.rank_off[t], p.rank_off[t + 1]
        h, g = x[lo:hi] @ A[r0:r1].T, dy[lo:hi] @ B[r0:r1].T
        yr[lo:hi] += 2.0 * h @ B[r0:r1]
        dxr[lo:hi] += 2.0 * g @ A[r0:r1]
        dAr[r0:r1] += 2.0 * g.T @ x[lo:hi]
        dBr[r0:r1] += 2.0 * h.T @ dy[lo:hi]
    for a, b in ((y, yr), (dx, dxr), (dA, dAr), (dB, dBr)):
        assert relerr(a, b) < 1e-13


# ---------------------------------------------------------------------------
# planted mistakes: each mutant of the C source must be caught by some pin
# ---------------------------------------------------------------------------
MUTANTS = [
    ("fwd scale dropped", "y[j] += st * lo;", "y[j] += lo;"),
    ("fwd W transposed", "load_elem(W, dtype, (size_t)k * d_out + j);\n        }\n        if (h_out)",
     "load_elem(W, dtype, ((size_t)j * d_in + k) % ((size_t)d_in * d_out));\n        }\n        if (h_out)"),
    ("dx adapter sign", "dx[k] += st * lo;", "dx[k] -= st * lo;"),
    ("dB scale dropped", "dBrow[j] *= st;", "dBrow[j] *= 1.0;"),
    ("dA uses h", "dArow[k] += gi *", "dArow[k] += hi *"),
    ("segment task reversed", "task_of[i] = seg_task[k];", "task_of[i] = seg_task[S - 1 - k];"),
    ("up projection ignores task offset",
     "lo += h[p] * load_elem(B, dtype, (size_t)(r0 + p) * d_out + j);",
     "lo += h[p] * load_elem(B, dtype, (size_t)(p) * d_out + j);"),
    ("gradient sums over every adapter token", "if (task_of[i] != t)", "if (task_of[i] < 0)"),
    ("bf16 widened wrongly", "[i] << 16;", "[i] << 15;"),
    ("h output scaled", "h_out[(size_t)q * r_max + p] = acc;", "h_out[(size_t)q * r_max + p] = 2.0 * acc;"),
    ("g output misplaced", "g_out[(size_t)q * r_max + p] = acc;", "g_out[(size_t)q * r_max + (r - 1 - p)] = acc;"),
    ("g uses A", "ag += load_elem(dy, dtype, (size_t)i * d_out + j) *\n                      load_elem(B, dtype, (size_t)(r0 + p) * d_out + j);",
     "ag += load_elem(dy, dtype, (size_t)i * d_out + j) *\n                      load_elem(A, dtype, ((size_t)(r0 + p) * d_in + j) % ((size_t)d_in));"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, old, new, monkeypatch):
    src = open(orc_mod._SRC).read()
    assert src.count(old) >= 1, "mutation site not found: " + name
    with tempfile.TemporaryDirectory() as d:
        c, so = os.path.join(d, "m.c"), os.path.join(d, "m.so")
        open(c, "w").write(src.replace(old, new, 1))
        subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", so, c,
                        orc_mod._SRC_ADAM, "-lm"], check=True)
        monkeypatch.setattr(orc_mod, "_handle", orc_mod._bind(ctypes.CDLL(so)))
        caught = []
        for pin in PINS:
            try:
                pin()
            except (AssertionError, ValueError):
                caught.append(pin.__name__)
        assert caught, "no pin noticed the planted mistake: " + name


def test_fused_projections_are_the_block_diagonal_dense_layer():
    """P layers that share x, as the oracle composes them, equal ONE layer of the pinned oracle whose up
    factors are block-diagonal over the concatenated outputs (and P = 1 is the layer itself)."""
    from paper_2509_01193_amd import workloads as wl
    base = wl.make_custom("b", "bf16", 24, 16, [8, 16], [0, 5, 9, 30, 41], [0, 1, -1, 0], 5)
    for P in (1, 2, 3):
        f = wl.fuse_projections(base, P)
        fo = oracle.FusedProjections(P, f.x, f.W, f.A, f.B, f.s, f.dy, f.rank_off, f.seg_off, f.seg_task)
        dg, ro = base.d_out, f.rank_off
        Bd = np.zeros((f.R_tot, P * dg), np.uint16)
        for t in range(f.n_tasks):
            r = int(f.ranks[t]) // P
            for j in range(P):
                rows = slice(ro[t] + j * r, ro[t] + (j + 1) * r)
                Bd[rows, j * dg:(j + 1) * dg] = f.B[rows]
        do = oracle.Oracle(f.x, f.W, f.A, Bd, f.s, f.dy, f.rank_off, f.seg_off, f.seg_task)
        assert np.array_equal(fo.y(), do.y())
        assert np.allclose(fo.dx(), do.dx(), rtol=1e-13, atol=0)
        (a1, b1), (a2, b2) = fo.grads(), do.grads()
        assert np.allclose(a1, a2, rtol=1e-13, atol=0)
        for t in range(f.n_tasks):
            r = int(f.ranks[t]) // P
            for j in range(P):
                rows = slice(ro[t] + j * r, ro[t] + (j + 1) * r)
                assert np.allclose(b1[rows], b2[rows, j * dg:(j + 1) * dg], rtol=1e-13, atol=0)
                off = np.ones(P * dg, bool)
                off[j * dg:(j + 1) * dg] = False
                # what the dense layer puts outside the diagonal blocks is the gradient of entries that are
                # structurally zero: it is not part of the fused layer
                assert b2[rows][:, off].shape[1] == (P - 1) * dg
