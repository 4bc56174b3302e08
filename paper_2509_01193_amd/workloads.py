"""Seeded synthetic workloads for the multi-adapter LoRA linear layer.

This module serves both the GPU path and the CPU oracle and therefore holds
none of the method's arithmetic: it only draws sequence lengths, builds the
task-segment table of a packed batch and fills the tensors with seeded normal
values (rounded once to bf16, round-to-nearest-even, for the bf16 workloads).

The five workloads stand in for the paper's joint fine-tuning batches (section
5.1 and the dataset statistics table of appendix B: heavily right-skewed
sequence lengths, tasks of very different sizes); the datasets themselves are
not used.  Lengths follow the recipe stated with each generator below.
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 20250901
_CHUNK = 1 << 23


# ----------------------------------------------------------------------------
# bf16 helpers (storage format only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(v: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(v, dtype=np.float32).view(np.uint32)
    rnd = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(seed, tag, shape, std, dtype):
    """N(0, std) tensor, generated in fixed chunks so the result does not depend on thread count."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16 if dtype == "bf16" else np.float32)
    nchunk = max(1, -(-n // _CHUNK))
    kids = np.random.SeedSequence([int(seed), int(tag)]).spawn(nchunk)

    def fill(c):
        lo, hi = c * _CHUNK, min(n, (c + 1) * _CHUNK)
        rng = np.random.Generator(np.random.PCG64(kids[c]))
        v = rng.standard_normal(hi - lo, dtype=np.float32)
        v *= np.float32(std)
        out[lo:hi] = f32_to_bf16_bits(v) if dtype == "bf16" else v

    workers = min(8, os.cpu_count() or 1, nchunk)
    if workers > 1:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(fill, range(nchunk)))
    else:
        for c in range(nchunk):
            fill(c)
    return out.reshape(shape)


# ----------------------------------------------------------------------------
# problem container
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class Problem:
    name: str
    dtype: str                 # "f32" or "bf16" (storage of x, W, A, B, dy, y, dx)
    T: int
    d_in: int
    d_out: int
    ranks: np.ndarray          # [n_tasks] int32
    s: np.ndarray              # [n_tasks] float32
    seg_off: np.ndarray        # [S+1] int32
    seg_task: np.ndarray       # [S] int32, -1 = no adapter
    seqs: list                 # [(length, task)] in packed order, before merging
    seed: int
    n_proj: int = 1            # > 1: that many layers reading the same x, fused (ranks stacked, B compact)
    x: np.ndarray = None       # [T, d_in]      float32, or uint16 bf16 bits
    W: np.ndarray = None       # [d_in, d_out]
    A: np.ndarray = None       # [R_tot, d_in]  (down projections, stacked by task)
    B: np.ndarray = None       # [R_tot, d_out] (up projections, stacked by task)
    dy: np.ndarray = None      # [T, d_out]

    @property
    def n_tasks(self):
        return int(self.ranks.shape[0])

    @property
    def rank_off(self):
        return np.concatenate([[0], np.cumsum(self.ranks)]).astype(np.int32)

    @property
    def R_tot(self):
        return int(self.ranks.sum())

    @property
    def S(self):
        return int(self.seg_task.shape[0])

    def task_tokens(self):
        cnt = np.zeros(self.n_tasks, dtype=np.int64)
        for k in range(self.S):
            if self.seg_task[k] >= 0:
                cnt[self.seg_task[k]] += self.seg_off[k + 1] - self.seg_off[k]
        return cnt

    def useful_flops(self):
        """fwd+bwd flops the method itself needs: base product twice plus six rank-r products."""
        cnt = self.task_tokens()
        base = 4.0 * self.T * self.d_in * self.d_out
        lora = 6.0 * float((cnt * self.ranks).sum()) * (self.d_in + self.d_out // self.n_proj)
        return base + lora

    def fill(self, std_x=0.02, std_w=0.02, std_a=0.02, std_b=0.02, std_dy=1.0):
        sd, dt = self.seed, self.dtype
        self.x = _normal(sd, 1, (self.T, self.d_in), std_x, dt)
        self.W = _normal(sd, 2, (self.d_in, self.d_out), std_w, dt)
        self.A = _normal(sd, 3, (self.R_tot, self.d_in), std_a, dt)
        self.B = _normal(sd, 4, (self.R_tot, self.d_out // self.n_proj), std_b, dt)
        self.dy = _normal(sd, 5, (self.T, self.d_out), std_dy, dt)
        return self


def segments_from_sequences(seqs):
    """Merge neighbouring sequences of one task into a segment; returns (seg_off, seg_task)."""
    off, task = [0], []
    for length, t in seqs:
        if length <= 0:
            continue
        if task and task[-1] == t:
            off[-1] += length
        else:
            task.append(t)
            off.append(off[-1] + length)
    return np.asarray(off, np.int32), np.asarray(task, np.int32)


def _order(seqs, order, rng):
    seqs = list(seqs)
    if order == "shuffled":
        perm = rng.permutation(len(seqs))
        return [seqs[i] for i in perm]
    if order == "sorted":
        return sorted(seqs, key=lambda q: q[1])
    if order == "as_drawn":
        return seqs
    raise ValueError("order must be shuffled, sorted or as_drawn")


def _fill_task(rng, total, draw, lo):
    """Draw lengths until they sum to `total`; the last one is cut to fit and a stub
    shorter than `lo` is merged into the previous sequence."""
    out, left = [], int(total)
    while left > 0:
        L = min(int(draw(rng)), left)
        if L < lo and out:
            out[-1] += L
        else:
            out.append(L)
        left -= L
    return out


def _lognormal(mu, sigma, lo, hi):
    def draw(rng):
        return int(np.clip(np.rint(rng.lognormal(mu, sigma)), lo, hi))
    return draw


def _largest_remainder(weights, total):
    w = np.asarray(weights, np.float64)
    q = w / w.sum() * total
    base = np.floor(q).astype(np.int64)
    rest = int(total - base.sum())
    for i in np.argsort(-(q - base), kind="stable")[:rest]:
        base[i] += 1
    return base


# ----------------------------------------------------------------------------
# the five workloads
# ----------------------------------------------------------------------------
def _seqs_cfg1(rng):
    # 8 sequences, length uniform in [16, 128], task ids round-robin over 2 tasks
    return [(int(rng.integers(16, 129)), i % 2) for i in range(8)], np.full(2, 8)


def _seqs_cfg2(rng, T=16384, n=4, r=16):
    # every task holds T/n tokens in lognormal(5.5, 1.0) sequences clipped to [32, 4096]
    seqs = []
    for t in range(n):
        for L in _fill_task(rng, T // n, _lognormal(5.5, 1.0, 32, 4096), 32):
            seqs.append((L, t))
    return seqs, np.full(n, r)


def _seqs_cfg3(rng, T=32768, ranks=(8, 8, 16, 16, 32, 32, 64, 64)):
    # task token shares follow Zipf(1.2) over the task index; lognormal(6, 1.2) in [16, 8192]
    n = len(ranks)
    shares = _largest_remainder([(k + 1) ** -1.2 for k in range(n)], T)
    seqs = []
    for t in range(n):
        for L in _fill_task(rng, shares[t], _lognormal(6.0, 1.2, 16, 8192), 16):
            seqs.append((L, t))
    return seqs, np.asarray(ranks)


def _seqs_cfg4(rng, T=65536, n=16, r=16):
    # 90 % lognormal(5.5, 0.8), 10 % uniform in [4096, 16384]; each sequence goes to the
    # task that holds the fewest tokens so far (exactly equal shares cannot hold a
    # 16384-token sequence)
    body = _lognormal(5.5, 0.8, 16, 16384)

    def draw(g):
        return int(g.integers(4096, 16385)) if g.random() < 0.1 else body(g)
    lens = _fill_task(rng, T, draw, 16)
    load = np.zeros(n, np.int64)
    seqs = []
    for L in lens:
        t = int(np.argmin(load))
        load[t] += L
        seqs.append((L, t))
    return seqs, np.full(n, r)


def _seqs_cfg5(rng, T=49152, n=32, r=64):
    # 4 heavy tasks hold 80 % of the tokens (one of them a single 16384-token sequence),
    # 28 light tasks the rest; 8 light tasks are one 16-token sequence each
    heavy = [16384, 10240, 7168, 5530]
    seqs = [(heavy[0], 0)]
    for t in (1, 2, 3):
        for L in _fill_task(rng, heavy[t], _lognormal(7.5, 1.0, 64, 16384), 64):
            seqs.append((L, t))
    rest = T - sum(heavy)
    tiny = list(range(n - 8, n))
    for t in tiny:
        seqs.append((16, t))
    rest -= 16 * len(tiny)
    light = list(range(4, n - 8))
    shares = _largest_remainder(np.ones(len(light)), rest)
    for t, sh in zip(light, shares):
        for L in _fill_task(rng, sh, _lognormal(5.0, 1.0, 16, 4096), 16):
            seqs.append((L, t))
    return seqs, np.full(n, r)


_CFG = {
    1: dict(dtype="f32", d_in=256, d_out=256, seqs=_seqs_cfg1, name="cfg1-tiny-f32"),
    2: dict(dtype="bf16", d_in=4096, d_out=4096, seqs=_seqs_cfg2, name="cfg2-llama7b-qproj"),
    3: dict(dtype="bf16", d_in=4096, d_out=11008, seqs=_seqs_cfg3, name="cfg3-llama7b-mlp-up"),
    4: dict(dtype="bf16", d_in=8192, d_out=28672, seqs=_seqs_cfg4, name="cfg4-llama70b-mlp"),
    5: dict(dtype="bf16", d_in=8192, d_out=8192, seqs=_seqs_cfg5, name="cfg5-skew-stress"),
}


def make_config(cfg: int, order: str = "shuffled", d_in: int = None, d_out: int = None,
                fill: bool = True, reverse_ranks: bool = False, scale: float = 2.0,
                **fill_kw) -> Problem:
    """Workload `cfg` (1..5).  `d_in`/`d_out` override the layer width (the parity tests
    shrink the layer so the oracle finishes in seconds; the token structure stays)."""
    c = _CFG[cfg]
    seed = BASE_SEED + cfg
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0])))
    seqs, ranks = c["seqs"](rng)
    ranks = np.asarray(ranks, np.int32)
    if reverse_ranks:
        ranks = ranks[::-1].copy()
    seqs = _order(seqs, "as_drawn" if cfg == 1 else order, rng)
    seg_off, seg_task = segments_from_sequences(seqs)
    p = Problem(name=c["name"] + ("" if cfg == 1 else "-" + order), dtype=c["dtype"],
                T=int(seg_off[-1]), d_in=d_in or c["d_in"], d_out=d_out or c["d_out"],
                ranks=ranks, s=np.full(len(ranks), scale, np.float32),
                seg_off=seg_off, seg_task=seg_task, seqs=seqs, seed=seed)
    return p.fill(**fill_kw) if fill else p


def fuse_projections(p: Problem, n_proj: int, fill: bool = True, **fill_kw) -> Problem:
    """`n_proj` layers of p's shape that read the same x (q/k/v, gate/up), as one fused problem:
    W [d_in, n_proj d_out], every task's ranks stacked n_proj times (rows j r_t .. of a task belong
    to projection j), B compact [R_tot, d_out], y/dy [T, n_proj d_out].  Token structure as in p."""
    q = Problem(name=p.name + "-x%d" % n_proj, dtype=p.dtype, T=p.T, d_in=p.d_in, d_out=n_proj * p.d_out,
                ranks=(n_proj * p.ranks).astype(np.int32), s=p.s.copy(), seg_off=p.seg_off.copy(),
                seg_task=p.seg_task.copy(), seqs=list(p.seqs), seed=p.seed + 7919 * n_proj, n_proj=n_proj)
    return q.fill(**fill_kw) if fill else q


def pad_to_buckets(p: Problem, bounds, fill: bool = True, **fill_kw) -> Problem:
    """The padded layout of the same sequences (paper section 2.1, "Processing Variable-length
    Data"): every sequence is followed by pad tokens up to the smallest boundary in `bounds` that
    holds it.  Pad tokens are segments of task -1 (base product only).  `bounds` comes from the
    caller (e.g. the dynamic bucketing entry point); this function only lays tokens out."""
    bounds = sorted(int(b) for b in bounds)
    seg_off, seg_task = [0], []
    for length, t in p.seqs:
        if length <= 0:
            continue
        b = next((u for u in bounds if u >= length), None)
        if b is None:
            raise ValueError("sequence of %d tokens exceeds the largest boundary" % length)
        seg_off.append(seg_off[-1] + length)
        seg_task.append(t)
        if b > length:
            seg_off.append(seg_off[-1] + b - length)
            seg_task.append(-1)
    q = Problem(name=p.name + "-padded", dtype=p.dtype, T=int(seg_off[-1]), d_in=p.d_in, d_out=p.d_out,
                ranks=p.ranks.copy(), s=p.s.copy(), seg_off=np.asarray(seg_off, np.int32),
                seg_task=np.asarray(seg_task, np.int32), seqs=list(p.seqs), seed=p.seed)
    return q.fill(**fill_kw) if fill else q


def make_custom(name, dtype, d_in, d_out, ranks, seg_off, seg_task, seed, s=None,
                fill=True, **fill_kw) -> Problem:
    """A problem from an explicit segment table (edge-case and adversarial tables)."""
    ranks = np.asarray(ranks, np.int32)
    seg_off = np.asarray(seg_off, np.int32)
    seg_task = np.asarray(seg_task, np.int32)
    s = np.full(len(ranks), 2.0, np.float32) if s is None else np.asarray(s, np.float32)
    p = Problem(name=name, dtype=dtype, T=int(seg_off[-1]) if len(seg_off) else 0,
                d_in=d_in, d_out=d_out, ranks=ranks, s=s, seg_off=seg_off,
                seg_task=seg_task, seqs=[], seed=seed)
    return p.fill(**fill_kw) if fill else p
