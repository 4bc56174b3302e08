"""Dynamic bucketing (paper section 4.3): oracle pins and the host implementation against the oracle. CPU only."""
import numpy as np
import pytest

from oracle import bucketing as ob
from paper_2509_01193_amd import binding as bd


def batches():
    rng = np.random.default_rng(5)
    for trial in range(40):
        U = int(rng.integers(1, 8))
        u = sorted(rng.choice(np.arange(1, 40), U, replace=False).tolist())
        n = int(rng.integers(0, 12))
        lens = rng.integers(1, u[-1] + 1, n).tolist()
        R = int(rng.integers(1, U + 2))
        yield lens, u, R


def test_oracle_dp_equals_brute_force_definition():
    for lens, u, R in batches():
        total, bounds = ob.dp_min_padding(lens, u, R)
        bf = ob.brute_force(lens, u, R)
        assert total == bf, (lens, u, R)
        if lens:
            assert len(bounds) <= R and ob.padding_for(lens, bounds) == total


def test_oracle_special_cases():
    u = [256, 512, 768, 1024]
    lens = [100, 300, 300, 700, 1000]
    # as many buckets as boundaries: only the padding inside each interval remains
    assert ob.dp_min_padding(lens, u, 4)[0] == sum(b - s for s, b in zip(lens, [256, 512, 512, 768, 1024]))
    # one bucket: everything is padded to the boundary that covers the longest sequence
    assert ob.dp_min_padding(lens, u, 1) == (sum(1024 - s for s in lens), [1024])
    # worked by hand: two buckets -> {512, 1024}: 412 + 212 + 212 + 324 + 24
    assert ob.dp_min_padding(lens, u, 2) == (1184, [512, 1024])
    with pytest.raises(ValueError):
        ob.dp_min_padding([2000], u, 2)


def test_host_implementation_equals_oracle():
    for lens, u, R in batches():
        total, _ = ob.dp_min_padding(lens, u, R)
        bounds, pad = bd.lobra_dynamic_buckets(lens, u, R)
        assert pad == (total if lens else 0)
        assert len(bounds) <= R and bounds == sorted(bounds) and set(bounds) <= set(u)
        if lens:
            assert ob.padding_for(lens, bounds) == total


def test_host_implementation_paper_scale_and_errors():
    # boundaries every 256 tokens up to 16384, R = 16 (the paper's defaults), a long-tailed batch
    rng = np.random.default_rng(0)
    u = list(range(256, 16385, 256))
    lens = np.clip(np.rint(rng.lognormal(6.0, 1.2, 4096)), 1, 16384).astype(int).tolist()
    b16, p16 = bd.lobra_dynamic_buckets(lens, u, 16)
    b8, p8 = bd.lobra_dynamic_buckets(lens, u, 8)
    b64, p64 = bd.lobra_dynamic_buckets(lens, u, 64)
    assert len(b16) == 16 and p64 <= p16 <= p8
    assert p16 == ob.padding_for(lens, b16) and p8 == ob.padding_for(lens, b8)
    assert p64 == sum(-(-s // 256) * 256 - s for s in lens)          # every occupied interval its own bucket
    assert b16[-1] == -(-max(lens) // 256) * 256
    assert bd.lib().lobra_dynamic_buckets(None, 0, None, 1, 1, None, None, None) == -1
    with pytest.raises(bd.LobraError):
        bd.lobra_dynamic_buckets([5], [4, 4], 1)
    with pytest.raises(bd.LobraError):
        bd.lobra_dynamic_buckets([9], [4, 8], 1)
    assert bd.lobra_dynamic_buckets([], [4, 8], 2) == ([], 0)


def test_padded_layout_of_a_workload_follows_the_chosen_boundaries():
    """Bucket boundaries -> padded batch: every sequence keeps its tokens and task and is followed
    by exactly the pad span (task -1) that brings it to its boundary; the pad total is the programme's."""
    from paper_2509_01193_amd import workloads as wl
    for cfg in (2, 3, 5):
        p = wl.make_config(cfg, "shuffled", fill=False)
        lens = [L for L, _ in p.seqs]
        cand = list(range(256, -(-max(lens) // 256) * 256 + 1, 256))
        bounds, pad = bd.lobra_dynamic_buckets(lens, cand, 8)
        q = wl.pad_to_buckets(p, bounds, fill=False)
        assert q.T == p.T + pad == p.T + ob.padding_for(lens, bounds)
        k = 0
        for L, t in p.seqs:
            assert q.seg_task[k] == t and q.seg_off[k + 1] - q.seg_off[k] == L
            k += 1
            b = min(u for u in bounds if u >= L)
            if b > L:
                assert q.seg_task[k] == -1 and q.seg_off[k + 1] - q.seg_off[k] == b - L
                k += 1
        assert k == q.S
        assert (q.task_tokens() == p.task_tokens()).all()
    with pytest.raises(ValueError):
        wl.pad_to_buckets(p, [16])


# ---- the padded chunk as a segment table (lobra_padded_segments) ---------------------------------------------
def test_padded_segments_oracle_pin_against_the_row_by_row_definition():
    """The oracle's table, expanded token by token with the layer oracle's own token -> task map, must be the
    definition: row r of sequence i belongs to task[i] when r < valid_len[i], to nobody otherwise."""
    import oracle
    rng = np.random.default_rng(9)
    for trial in range(30):
        n = int(rng.integers(0, 9))
        pl = rng.integers(0, 20, n)
        vl = np.asarray([int(rng.integers(0, p + 1)) for p in pl], np.int64)
        tk = rng.integers(-1, 4, n)
        seg_off, seg_task = ob.padded_segments(pl, vl, tk)
        want = np.concatenate([np.concatenate([np.full(v, t), np.full(p - v, -1)]) for p, v, t in zip(pl, vl, tk)]
                              + [np.zeros(0, np.int64)]).astype(np.int32)
        got = oracle.token_task(int(pl.sum()), np.asarray(seg_off, np.int32), np.asarray(seg_task, np.int32), 4)
        assert np.array_equal(got, want), (pl, vl, tk)
    # the worked case: [b, s_j] = [3, 8] with valid lengths 5, 8, 0
    assert ob.padded_segments([8, 8, 8], [5, 8, 0], [1, 0, 2]) == ([0, 5, 8, 16, 16, 16, 24], [1, -1, 0, -1, 2, -1])


def test_padded_segments_entry_point_against_the_oracle_bit_for_bit():
    rng = np.random.default_rng(10)
    for trial in range(60):
        n = int(rng.integers(0, 40))
        uniform = trial % 2 == 0
        pl = np.full(n, int(rng.integers(0, 600))) if uniform else rng.integers(0, 600, n)
        vl = np.asarray([int(rng.integers(0, p + 1)) for p in pl], np.int64)
        tk = rng.integers(-1, 5, n)
        so, stk, T = bd.lobra_padded_segments(vl, tk, 5, None if uniform else pl, int(pl[0]) if (uniform and n) else 0)
        ro, rt = ob.padded_segments(pl, vl, tk)
        assert so.tolist() == ro and stk.tolist() == rt and T == int(pl.sum())
        # what it writes is a table the layer accepts
        d, keep = bd.make_desc("bf16", T, 64, 64, np.arange(6) * 8, so, stk)
        assert bd.validate(d) == 0


@pytest.mark.parametrize("kw,code", [
    (dict(valid_len=[3, 9], task=[0, 1], padded_len=[4, 8]), -4),         # longer than its padded length
    (dict(valid_len=[3, -1], task=[0, 1], padded_len=[4, 8]), -4),
    (dict(valid_len=[3, 5], task=[0, 1], padded_len=[4, -8]), -4),
    (dict(valid_len=[3, 5], task=[0, 2], padded_len=[4, 8]), -5),         # n_tasks = 2
    (dict(valid_len=[3, 5], task=[-2, 1], padded_len=[4, 8]), -5),
    (dict(valid_len=[3, 5], task=[0, 1], uniform_len=-1), -2),
    (dict(valid_len=[1] * 3, task=[0] * 3, uniform_len=(1 << 30)), -2),   # 2^31 token rows and more
    (dict(valid_len=[3, 5], task=[0, 1], padded_len=[4, 8]), 0),
])
def test_padded_segments_argument_errors_write_nothing(kw, code):
    st, so, stk, T = bd.lobra_padded_segments(kw["valid_len"], kw["task"], 2, kw.get("padded_len"), kw.get("uniform_len", 0),
                                              check=False)
    assert st == code
    if code != 0:
        assert (so == -9).all() and (stk == -9).all() and T == -9

