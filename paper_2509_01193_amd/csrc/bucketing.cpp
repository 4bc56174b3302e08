// Host-side dynamic bucketing (paper section 4.3): choose at most R of U candidate boundaries so that
// padding each sequence of a batch up to its bucket boundary costs the fewest tokens.
//
// The paper's programme is  State_{i+1,j+1} = min_{i' <= i} State_{i',j} + cost(i'+1 .. i+1)  where
// cost(a .. b) pads the sequences of the intervals a .. b up to u_b.  With C_i = number of sequences in
// the first i intervals and S_i = sum of |I_k| u_k over them, cost(a .. b) = u_b (C_b - C_{a-1}) -
// (S_b - S_{a-1}), so one transition is O(1).  Only intervals that hold sequences can end a bucket.
#include <algorithm>
#include <cstdint>
#include <limits>
#include <new>
#include <vector>

#include "lobra_mlora.h"

extern "C" lobra_status lobra_dynamic_buckets(const int32_t* seq_len, int64_t n_seq, const int32_t* bounds,
                                              int32_t U, int32_t R, int32_t* out_bounds, int32_t* out_n,
                                              int64_t* out_padding)
{
    if (!bounds || !out_bounds || !out_n || (n_seq > 0 && !seq_len)) return LOBRA_ERR_NULL;
    if (U < 1 || R < 1 || n_seq < 0 || bounds[0] < 1) return LOBRA_ERR_SHAPE;
    for (int32_t i = 1; i < U; ++i)
        if (bounds[i] <= bounds[i - 1]) return LOBRA_ERR_SHAPE;
    try {
        // bucket sort by interval; inside-interval padding is a constant of the batch
        std::vector<int64_t> cnt(size_t(U), 0);
        int64_t inside = 0;
        for (int64_t k = 0; k < n_seq; ++k) {
            const int32_t s = seq_len[k];
            if (s < 1 || s > bounds[U - 1]) return LOBRA_ERR_SHAPE;
            const int32_t i = int32_t(std::lower_bound(bounds, bounds + U, s) - bounds);
            ++cnt[size_t(i)];
            inside += bounds[i] - s;
        }
        // keep the intervals that hold sequences: e_0 < e_1 < ... (indices into bounds)
        std::vector<int32_t> e;
        for (int32_t i = 0; i < U; ++i)
            if (cnt[size_t(i)] > 0) e.push_back(i);
        const int32_t V = int32_t(e.size());
        for (int32_t j = 0; j < R; ++j) out_bounds[j] = 0;
        *out_n = 0;
        if (out_padding) *out_padding = 0;
        if (V == 0) return LOBRA_OK;
        std::vector<int64_t> C(size_t(V) + 1, 0), S(size_t(V) + 1, 0);
        for (int32_t i = 0; i < V; ++i) {
            C[size_t(i) + 1] = C[size_t(i)] + cnt[size_t(e[size_t(i)])];
            S[size_t(i) + 1] = S[size_t(i)] + cnt[size_t(e[size_t(i)])] * int64_t(bounds[e[size_t(i)]]);
        }
        const int32_t Rm = std::min(R, V);           // more buckets than occupied intervals gain nothing
        const int64_t INF = std::numeric_limits<int64_t>::max() / 4;
        // st[j][i]: least extra padding when the first i occupied intervals form j buckets (j >= 1)
        std::vector<std::vector<int64_t>> st(size_t(Rm) + 1, std::vector<int64_t>(size_t(V) + 1, INF));
        std::vector<std::vector<int32_t>> from(size_t(Rm) + 1, std::vector<int32_t>(size_t(V) + 1, -1));
        st[0][0] = 0;
        for (int32_t j = 1; j <= Rm; ++j) {
            st[size_t(j)][0] = 0;
            for (int32_t i = 1; i <= V; ++i) {
                const int64_t ub = bounds[e[size_t(i) - 1]];
                int64_t best = INF;
                int32_t arg = -1;
                for (int32_t ip = 0; ip < i; ++ip) {
                    const int64_t prev = (ip == 0) ? 0 : st[size_t(j) - 1][size_t(ip)];
                    if (prev >= INF) continue;
                    const int64_t cost = ub * (C[size_t(i)] - C[size_t(ip)]) - (S[size_t(i)] - S[size_t(ip)]);
                    if (prev + cost < best) {
                        best = prev + cost;
                        arg = ip;
                    }
                }
                st[size_t(j)][size_t(i)] = best;
                from[size_t(j)][size_t(i)] = arg;
            }
        }
        // the best count of buckets is Rm (more buckets never cost more); walk back
        std::vector<int32_t> chosen;
        for (int32_t i = V, j = Rm; i > 0 && j > 0; --j) {
            chosen.push_back(bounds[e[size_t(i) - 1]]);
            i = from[size_t(j)][size_t(i)];
        }
        std::sort(chosen.begin(), chosen.end());
        *out_n = int32_t(chosen.size());
        for (size_t q = 0; q < chosen.size(); ++q) out_bounds[q] = chosen[q];
        if (out_padding) *out_padding = st[size_t(Rm)][size_t(V)] + inside;
    } catch (const std::bad_alloc&) {
        return LOBRA_ERR_NOMEM;
    }
    return LOBRA_OK;
}

// The padded layout of a chunk (paper section 2.1, "Processing Variable-length Data": sequences of a chunk are
// padded to a common length) as a segment table of the packed operator: sequence i takes padded_len[i]
// consecutive token rows, the first valid_len[i] of them belong to task[i], the rest are pad tokens (task -1:
// base product only, no part in dA and dB).  Pure index arithmetic on the host.
extern "C" lobra_status lobra_padded_segments(int64_t n_seq, const int32_t* padded_len, int32_t uniform_len,
                                              const int32_t* valid_len, const int32_t* task, int32_t n_tasks,
                                              int32_t* seg_off, int32_t* seg_task, int64_t* T_out)
{
    if (n_seq < 0 || n_tasks < 0) return LOBRA_ERR_SHAPE;
    if (!seg_off || (n_seq > 0 && (!valid_len || !task || !seg_task))) return LOBRA_ERR_NULL;
    if (!padded_len && uniform_len < 0) return LOBRA_ERR_SHAPE;
    if (2 * n_seq > 0x7fffffff) return LOBRA_ERR_SHAPE;          // the table has 2 n_seq segments
    int64_t pos = 0;
    for (int64_t i = 0; i < n_seq; ++i) {                        // all checks first: on error nothing is written
        const int64_t pl = padded_len ? padded_len[i] : uniform_len;
        if (pl < 0 || valid_len[i] < 0 || valid_len[i] > pl) return LOBRA_ERR_SEGMENTS;
        if (task[i] < -1 || task[i] >= n_tasks) return LOBRA_ERR_TASK_ID;
        pos += pl;
        if (pos >= (int64_t(1) << 31)) return LOBRA_ERR_SHAPE;
    }
    pos = 0;
    seg_off[0] = 0;
    for (int64_t i = 0; i < n_seq; ++i) {
        const int64_t pl = padded_len ? padded_len[i] : uniform_len;
        seg_off[2 * i + 1] = int32_t(pos + valid_len[i]);
        seg_task[2 * i] = task[i];
        seg_off[2 * i + 2] = int32_t(pos + pl);
        seg_task[2 * i + 1] = -1;
        pos += pl;
    }
    if (T_out) *T_out = pos;
    return LOBRA_OK;
}
