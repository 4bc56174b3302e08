"""Oracle of the dynamic bucketing step that precedes the layer on the caller's side (test infrastructure).

Paper section 4.3, "Dynamic Bucketing": U pre-defined boundaries u_1 < ... < u_U split the length range
into U intervals; a batch is bucket-sorted by length; R of the boundaries are chosen so that padding
every sequence to the closest chosen boundary at or above its length costs the fewest pad tokens.

`dp_min_padding` follows the paper's dynamic programme in its order and notation (State_{i,j}, the
minimum over i', the explicit inner sum over i''); nothing is pre-summed.  As the paper's footnote on
the programme's cost says, empty intervals are ignored: the programme runs over the intervals that
hold at least one sequence (read literally over all U intervals, State_{U,R} would pad the whole
batch up to u_U even when no sequence is that long).  `brute_force` is the
definition itself: try every choice of at most R boundaries and pad.  Pure Python, small cases only.
"""
from itertools import combinations

INF = float("inf")


def interval_counts(lengths, u):
    """|I_i| for i = 1..U (returned 0-based): sequences with u_{i-1} < s <= u_i, u_0 = 0."""
    cnt = [0] * len(u)
    for s in lengths:
        if s < 1 or s > u[-1]:
            raise ValueError("sequence length outside (0, u_U]")
        i = 0
        while u[i] < s:
            i += 1
        cnt[i] += 1
    return cnt


def dp_min_padding(lengths, u, R):
    """State_{U,R} plus the padding inside the intervals: the total number of pad tokens (paper, footnote
    to the State equations), and the chosen boundaries (ascending)."""
    cnt_all = interval_counts(lengths, u)
    u = [b for b, c in zip(u, cnt_all) if c > 0]          # ignore empty intervals
    cnt = [c for c in cnt_all if c > 0]
    U = len(u)
    if U == 0:
        return 0, []
    # State[i][j]: least extra padding when the first i intervals form j buckets
    State = [[INF] * (R + 1) for _ in range(U + 1)]
    arg = [[-1] * (R + 1) for _ in range(U + 1)]
    for j in range(R + 1):
        State[0][j] = 0
    for i in range(U):               # computes State_{i+1, j+1}
        for j in range(R):
            best, best_ip = INF, -1
            for ip in range(i + 1):  # i' in [0, i]
                extra = 0
                for ipp in range(ip + 1, i + 1):           # i'' = i'+1 .. i  (1-based intervals)
                    extra += cnt[ipp - 1] * (u[i] - u[ipp - 1])   # u_{i+1} - u_{i''}
                cand = State[ip][j] + extra
                if cand < best:
                    best, best_ip = cand, ip
            State[i + 1][j + 1] = best
            arg[i + 1][j + 1] = best_ip
    inside = sum(u[i] - s for s in lengths for i in [next(k for k in range(U) if u[k] >= s)])
    # back-track the boundaries: bucket ending at interval i (1-based) uses boundary u_i
    bounds, i, j = [], U, R
    while i > 0 and j > 0:
        bounds.append(u[i - 1])
        i, j = arg[i][j], j - 1
    total = State[U][R] + inside
    return total, sorted(bounds)


def padding_for(lengths, chosen):
    """Pad tokens when every sequence goes to the smallest chosen boundary at or above its length."""
    tot = 0
    for s in lengths:
        fit = [b for b in chosen if b >= s]
        if not fit:
            return INF
        tot += min(fit) - s
    return tot


def brute_force(lengths, u, R):
    best = INF
    for k in range(1, R + 1):
        for chosen in combinations(u, k):
            best = min(best, padding_for(lengths, chosen))
    return best


def padded_segments(padded_len, valid_len, task):
    """Segment table of a padded chunk (paper section 2.1, "Processing Variable-length Data": sequences padded to a
    common length): sequence i occupies padded_len[i] token rows, the first valid_len[i] of them belong to
    task[i], the rest are pad tokens (task -1).  Written out row by row: the task of every token row, then the
    maximal description as (offsets, tasks) with two segments per sequence."""
    seg_off, seg_task = [0], []
    for pl, vl, t in zip(padded_len, valid_len, task):
        seg_off += [seg_off[-1] + int(vl), seg_off[-1] + int(pl)]
        seg_task += [int(t), -1]
    return seg_off, seg_task

