// Validation of the problem descriptor and construction of the host-side work lists.
// The lists turn the packed batch's segment table (paper section 1: a fused batch holds the
// sequences of several tasks, each tagged with its task) into what the kernels iterate over.
#include "plan.h"

#include <algorithm>
#include <cstring>
#include <new>

namespace lobra {

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

lobra_status validate(const lobra_mlora_desc* d)
{
    if (!d) return LOBRA_ERR_NULL;
    if (d->dtype != LOBRA_F32 && d->dtype != LOBRA_BF16) return LOBRA_ERR_DTYPE;
    if (d->T < 0 || d->T >= (int64_t(1) << 31)) return LOBRA_ERR_SHAPE;
    if (d->d_in < 1 || d->d_out < 1 || d->n_tasks < 0 || d->S < 0) return LOBRA_ERR_SHAPE;
    // what the kernels' launch grids and 32-bit offsets inside a tile can address (checked here so that
    // no call fails after its first launch): widths, and the number of 256 x 256 output tiles
    if (d->d_in > LOBRA_MAX_WIDTH || d->d_out > LOBRA_MAX_WIDTH) return LOBRA_ERR_SHAPE;
    {
        const int64_t tiles_m = (d->T + 255) / 256, tiles_n = (int64_t(d->d_in > d->d_out ? d->d_in : d->d_out) + 255) / 256;
        if (tiles_m * tiles_n > 0x7fffffff) return LOBRA_ERR_SHAPE;
    }
    if (d->dtype == LOBRA_F32 && d->T > kPlainMaxTokens) return LOBRA_ERR_SHAPE;
    if (d->S == 0 && d->T != 0) return LOBRA_ERR_SEGMENTS;
    if (d->dtype == LOBRA_BF16 && (d->d_in % 8 != 0 || d->d_out % 8 != 0)) return LOBRA_ERR_ALIGN;
    if (d->n_proj < 0 || d->n_proj > 16) return LOBRA_ERR_SHAPE;
    const int32_t P = d->n_proj > 1 ? d->n_proj : 1;
    if (P > 1 && d->d_out % (8 * P) != 0) return LOBRA_ERR_ALIGN;
    if (d->n_tasks > 0) {
        if (!d->rank_off) return LOBRA_ERR_NULL;
        if (d->rank_off[0] != 0) return LOBRA_ERR_RANK;
        for (int32_t t = 0; t < d->n_tasks; ++t) {
            const int64_t r = int64_t(d->rank_off[t + 1]) - d->rank_off[t];
            if (r < 1 || r > LOBRA_MAX_RANK) return LOBRA_ERR_RANK;
            if (P > 1 && r % (8 * P) != 0) return LOBRA_ERR_RANK;
        }
    }
    if (d->S > 0) {
        if (!d->seg_off || !d->seg_task) return LOBRA_ERR_NULL;
        if (d->seg_off[0] != 0) return LOBRA_ERR_SEGMENTS;
        for (int32_t k = 0; k < d->S; ++k)
            if (d->seg_off[k + 1] < d->seg_off[k]) return LOBRA_ERR_SEGMENTS;
        if (int64_t(d->seg_off[d->S]) != d->T) return LOBRA_ERR_SEGMENTS;
        for (int32_t k = 0; k < d->S; ++k)
            if (d->seg_task[k] < -1 || d->seg_task[k] >= d->n_tasks) return LOBRA_ERR_TASK_ID;
    }
    return LOBRA_OK;
}

lobra_status build_host_plan(const lobra_mlora_desc* d, uint32_t flags, Plan* p)
{
    try {
        p->desc = *d;
        p->flags = flags;
        p->mfma = kMfmaKernels && d->dtype == LOBRA_BF16 && !(flags & LOBRA_PLAN_PLAIN_KERNELS);
        if (!p->mfma && d->T > kPlainMaxTokens) return LOBRA_ERR_SHAPE;   // the plain kernels' grid
        p->n_proj = d->n_proj > 1 ? d->n_proj : 1;
        p->dg = d->d_out / p->n_proj;

        const int32_t n = d->n_tasks;
        p->rank_off.assign(size_t(n) + 1, 0);
        for (int32_t t = 0; t <= n && n > 0; ++t) p->rank_off[t] = d->rank_off[t];
        p->R_tot = p->rank_off[n];
        p->r_max = 0;
        for (int32_t t = 0; t < n; ++t)
            p->r_max = std::max(p->r_max, p->rank_off[t + 1] - p->rank_off[t]);
        p->r_pad = (p->r_max + 15) / 16 * 16;
        p->seg_off_in.assign(d->seg_off ? d->seg_off : nullptr,
                             d->seg_off ? d->seg_off + d->S + 1 : nullptr);
        p->seg_task_in.assign(d->seg_task ? d->seg_task : nullptr,
                              d->seg_task ? d->seg_task + d->S : nullptr);
        p->desc.rank_off = p->rank_off.data();
        p->desc.seg_off = p->seg_off_in.data();
        p->desc.seg_task = p->seg_task_in.data();

        // 1. compacted table: no empty segments, no two neighbours with the same task
        p->cseg_off.assign(1, 0);
        p->cseg_task.clear();
        for (int32_t k = 0; k < d->S; ++k) {
            const int32_t len = d->seg_off[k + 1] - d->seg_off[k];
            if (len == 0) continue;
            if (!p->cseg_task.empty() && p->cseg_task.back() == d->seg_task[k]) {
                p->cseg_off.back() += len;
            } else {
                p->cseg_task.push_back(d->seg_task[k]);
                p->cseg_off.push_back(p->cseg_off.back() + len);
            }
        }
        const int32_t nseg = int32_t(p->cseg_task.size());
        const int32_t T = int32_t(d->T);

        // 2. first segment of every 32-row block
        const int32_t nrb = (T + kRowBlock - 1) / kRowBlock;
        p->rowblk_seg.assign(size_t(nrb), 0);
        for (int32_t b = 0, k = 0; b < nrb; ++b) {
            while (p->cseg_off[k + 1] <= b * kRowBlock) ++k;
            p->rowblk_seg[b] = k;
        }

        // 2b. what the first rows of every GEMM tile row belong to
        {
            const int32_t ntr = (T + kGemmTileRows - 1) / kGemmTileRows;
            p->gemm_tile_tab.assign(size_t(ntr) * kGemmTileRec, 0);
            for (int32_t i = 0, k = 0; i < ntr; ++i) {
                const int32_t row0 = std::max(0, std::min(i * kGemmTileRows, T - kGemmTileRows));
                while (p->cseg_off[k + 1] <= row0) ++k;      // row0 does not decrease with i
                const int32_t t = p->cseg_task[k];
                int32_t* rec = &p->gemm_tile_tab[size_t(i) * kGemmTileRec];
                rec[0] = k;
                rec[1] = p->cseg_off[k];
                rec[2] = p->cseg_off[k + 1];
                rec[3] = t;
                rec[4] = t >= 0 ? p->rank_off[t] : 0;
                rec[5] = t >= 0 ? p->rank_off[t + 1] - p->rank_off[t] : 0;
            }
        }

        // 3. token blocks, grouped by task (counting sort keeps token order inside a task)
        p->task_tb_off.assign(size_t(n) + 1, 0);
        for (int32_t k = 0; k < nseg; ++k) {
            const int32_t t = p->cseg_task[k];
            if (t < 0) continue;
            const int32_t len = p->cseg_off[k + 1] - p->cseg_off[k];
            p->task_tb_off[t + 1] += (len + kTokenBlock - 1) / kTokenBlock;
        }
        for (int32_t t = 0; t < n; ++t) p->task_tb_off[t + 1] += p->task_tb_off[t];
        p->tb.assign(size_t(p->task_tb_off[n]), TokenBlock{0, 0, 0, 0});
        {
            std::vector<int32_t> cur(p->task_tb_off.begin(), p->task_tb_off.end() - (n >= 0 ? 1 : 0));
            for (int32_t k = 0; k < nseg; ++k) {
                const int32_t t = p->cseg_task[k];
                if (t < 0) continue;
                for (int32_t r0 = p->cseg_off[k]; r0 < p->cseg_off[k + 1]; r0 += kTokenBlock) {
                    const int32_t nr = std::min(kTokenBlock, p->cseg_off[k + 1] - r0);
                    p->tb[size_t(cur[t]++)] = TokenBlock{r0, nr, t, p->rank_off[t]};
                }
            }
        }

        // 3b. runs of token blocks that one workgroup of the rank-r projection handles.  From rank 24 or
        //     so the adapter rows are most of what a single token block's workgroup reads (r_t rows
        //     per 32 token rows), so long batches are projected in runs of four blocks that share the
        //     rows staged in LDS; otherwise every block is its own run.
        {
            int64_t wsum = 0;                      // token-block-weighted sum of ranks
            const int64_t ntb_all = p->task_tb_off[n];
            for (int32_t t = 0; t < n; ++t)
                wsum += int64_t(p->task_tb_off[t + 1] - p->task_tb_off[t]) * (p->rank_off[t + 1] - p->rank_off[t]);
            const int32_t g = (p->mfma && ntb_all >= 1024 && wsum >= 24 * ntb_all) ? 4 : 1;
            p->shrink_group = g;
            p->sb_off.assign(1, 0);
            for (int32_t t = 0; t < n; ++t)
                for (int32_t b = p->task_tb_off[t]; b < p->task_tb_off[t + 1]; b += g)
                    p->sb_off.push_back(std::min(b + g, p->task_tb_off[t + 1]));
            // 3c. launch order of the projection's workgroups by descending rank.  A workgroup's cost grows with
            //     its task's rank (the adapter rows it reads next to its 32 token rows), and the lists above are
            //     in task order, so with mixed ranks whichever task comes last would make up the launch's tail.
            //     (Inside a rank the stored, task-grouped order stays: ordering the blocks by their position in
            //     the batch as well measured 2 us slower on the shuffled workload 2, although the kernels deal
            //     their work items to the XCDs in contiguous ranges.)
            auto by_rank = [&](size_t count, auto task_of, std::vector<int32_t>& order) {
                order.resize(count);
                for (size_t i = 0; i < count; ++i) order[i] = int32_t(i);
                auto rank_of = [&](int32_t i) { const int32_t t = task_of(i); return p->rank_off[t + 1] - p->rank_off[t]; };
                std::stable_sort(order.begin(), order.end(),
                                 [&](int32_t a, int32_t b) { return rank_of(a) > rank_of(b); });
                bool identity = true;
                for (size_t i = 0; i < count && identity; ++i) identity = order[i] == int32_t(i);
                if (identity) order.clear();
            };
            by_rank(p->tb.size(), [&](int32_t i) { return p->tb[size_t(i)].task; }, p->tb_order);
            by_rank(p->sb_off.size() - 1, [&](int32_t i) { return p->tb[size_t(p->sb_off[size_t(i)])].task; }, p->sb_order);
        }

        // 3d. the K-sliced projection (long batches, ranks up to 16) and whether dB rides with its pass over dy
        p->sliced_in = p->sliced_out = SlicedShape{};
        if (p->mfma && !p->tb.empty()) {
            p->sliced_in = sliced_shrink_shape(int64_t(p->tb.size()), p->r_pad, d->d_in);
            if (p->n_proj == 1) p->sliced_out = sliced_shrink_shape(int64_t(p->tb.size()), p->r_pad, d->d_out);
        }
        // dB fused into the sliced projection of dy: the runs of (task, slice) that every workgroup meets, by
        // the same split of the items as the kernel's (shrink_sliced_kernel)
        p->fused_db = false;
        p->fb_wg_run_off.clear();
        p->fb_run_row.clear();
        p->fb_cnt.clear();
        p->fb_task_row0.clear();
        p->fb_rows = 0;
        if (p->sliced_out.nsl > 0) {
            const int32_t nsl = p->sliced_out.nsl, per_xcd = kSlicedGrid / 8, ntb32 = int32_t(p->tb.size());
            std::vector<int32_t> run_task, run_k;
            p->fb_cnt.assign(size_t(n) * nsl, 0);
            p->fb_wg_run_off.assign(1, 0);
            for (int32_t wg = 0; wg < kSlicedGrid; ++wg) {
                const int32_t xcd = wg & 7, idx = wg >> 3;
                const int32_t bx0 = int32_t((int64_t(ntb32) * xcd) >> 3), bx1 = int32_t((int64_t(ntb32) * (xcd + 1)) >> 3);
                const int32_t nbx = bx1 - bx0;
                const int64_t nit = int64_t(nbx) * nsl;
                int64_t e = nit * idx / per_xcd;
                const int64_t e1 = nit * (idx + 1) / per_xcd;
                while (e < e1) {
                    const int32_t sl = int32_t(e / nbx), bo = int32_t(e - int64_t(sl) * nbx);
                    const int32_t t = p->tb[size_t(bx0 + bo)].task;
                    // the run ends with the workgroup's range, the slice, or the task's blocks inside the piece
                    const int64_t task_end = int64_t(sl) * nbx + std::min<int64_t>(nbx, p->task_tb_off[t + 1] - bx0);
                    const int64_t next = std::min(e1, task_end);
                    run_task.push_back(t);
                    run_k.push_back(p->fb_cnt[size_t(t) * nsl + sl]++);
                    e = next;
                }
                p->fb_wg_run_off.push_back(int32_t(run_task.size()));
            }
            p->fb_task_row0.assign(size_t(n), 0);
            int64_t rows = 0;
            for (int32_t t = 0; t < n; ++t) {
                int32_t most = 0;
                for (int32_t sl = 0; sl < nsl; ++sl) most = std::max(most, p->fb_cnt[size_t(t) * nsl + sl]);
                p->fb_task_row0[t] = int32_t(rows);
                rows += int64_t(most) * 16;
            }
            // worth it while the partial sums stay a small part of the pass over dy (4 bytes x rows per column,
            // written and read once, against 2 bytes x T)
            if (rows > 0 && rows <= int64_t(T) / 8 && rows < 0x7fffffff / 2) {
                p->fused_db = true;
                p->fb_rows = int32_t(rows);
                p->fb_run_row.resize(run_task.size());
                for (size_t i = 0; i < run_task.size(); ++i)
                    p->fb_run_row[i] = p->fb_task_row0[run_task[i]] + 16 * run_k[i];
            } else {
                p->fb_wg_run_off.clear();
                p->fb_cnt.clear();
                p->fb_task_row0.clear();
            }
        }
        // 4. reduction chunks: runs of token blocks of one task.  The chunk length is chosen so
        //    that (chunks x 128-column tiles) gives roughly a thousand workgroups, within
        //    [4, 64] token blocks ([1, 64] on the plain path); fewer, longer chunks mean less partial-sum traffic.
        const int64_t coltiles = (std::min(d->d_in, d->d_out) + 127) / 128;
        int64_t cb = (int64_t(T) * coltiles / 1024 + kTokenBlock - 1) / kTokenBlock;
        // Where dB rides with the projection of dy, stage 1 is one short launch for dA alone and what counts is
        // its balance: three workgroups per compute unit (at workload 2: 24 chunks of 21 or 22 blocks, 27.9 us,
        // against 36 of 16 or 3 blocks, 30.8 us; and a quarter fewer partial sums for stage 2)
        if (p->fused_db) cb = (int64_t(p->tb.size()) * ((d->d_in + 127) / 128) + 767) / 768;
        // (the MFMA kernel gives each of its four waves a token block of the chunk at a time; the plain
        //  kernel walks a chunk's tokens one after the other, so small batches want short chunks there)
        cb = std::max<int64_t>(p->mfma ? 4 : 1, std::min<int64_t>(64, cb));
        p->chunk_blocks = int32_t(cb);
        p->chunks.clear();
        p->task_chunk_off.assign(size_t(n) + 1, 0);
        p->part_rows = 0;
        for (int32_t t = 0; t < n; ++t) {
            const int32_t r = p->rank_off[t + 1] - p->rank_off[t];
            const int32_t nb = p->task_tb_off[t + 1] - p->task_tb_off[t];
            // (a task's blocks are split evenly among its chunks: no short chunk at the end of a task; workload 3:
            //  stage 1 177 -> 169 us)
            const int32_t nck = (nb + p->chunk_blocks - 1) / p->chunk_blocks;
            const int32_t len = nck > 0 ? (nb + nck - 1) / nck : p->chunk_blocks;
            for (int32_t b = p->task_tb_off[t]; b < p->task_tb_off[t + 1]; b += len) {
                const int32_t e = std::min(b + len, p->task_tb_off[t + 1]);
                p->chunks.push_back(GradChunk{b, e, t, p->part_rows});
                p->part_rows += r;
            }
            p->task_chunk_off[t + 1] = int32_t(p->chunks.size());
        }

        // (the reduction kernels put chunks x column tiles of at least 64 columns on grid.x)
        if (int64_t(p->chunks.size()) * ((int64_t(d->d_in) + 63) / 64 + (int64_t(d->d_out) + 63) / 64) > 0x7fffffff)
            return LOBRA_ERR_SHAPE;

        // 5. buffer sizes
        BufferLayout& L = p->p_layout;
        const size_t ntb = p->tb.size();
        if (ntb == 0) {
            L = BufferLayout{};
        } else if (p->mfma) {
            L.p_tok = 0;
            L.p_blk = align_up(size_t(T) * p->r_pad * 2, 256);
            L.total = L.p_blk + align_up(ntb * size_t(p->r_pad) * kTokenBlock * 2, 256);
        } else {
            L.p_tok = 0;
            L.p_blk = 0;
            L.total = align_up(size_t(T) * p->r_max * 4, 256);
        }
        const size_t spart_in = align_up(size_t(p->sliced_in.nsl) * size_t(T) * 64, 256);
        const size_t spart_out = align_up(size_t(p->sliced_out.nsl) * size_t(T) * 64, 256);
        p->h_save_bytes = L.total;
        p->fwd_off_p = spart_in;
        p->fwd_ws_bytes = spart_in + L.total;
        p->bwd_off_g = 0;
        p->bwd_off_h = L.total;
        p->bwd_off_part_b = 2 * L.total;
        // (with dB fused into the projection of dy, its partial sums are the fused kernel's)
        p->bwd_off_part_a = p->bwd_off_part_b +
                            align_up(size_t(p->fused_db ? p->fb_rows : p->part_rows) * size_t(d->d_out) * 4, 256);
        p->bwd_off_spart = p->bwd_off_part_a + align_up(size_t(p->part_rows) * size_t(d->d_in) * 4, 256);
        p->bwd_ws_bytes = p->bwd_off_spart + std::max(spart_in, spart_out);
    } catch (const std::bad_alloc&) {
        return LOBRA_ERR_NOMEM;
    }
    return LOBRA_OK;
}

SlicedShape sliced_shrink_shape(int64_t ntb, int32_t r_pad, int32_t D)
{
    SlicedShape none;
    // whole slices only (the kernel's copies carry no bound); at least a dozen items per compute unit
    if (r_pad != 16 || ntb <= 0 || D <= 0 || D % 512 != 0) return none;
    const int64_t nsl = D / 512;
    const int64_t items = ntb * nsl;
    if (items < 3072 || items >= 0x7fffffff) return none;
    return SlicedShape{1, int32_t(nsl)};
}

std::vector<int32_t> pack_blob(Plan* p)
{
    std::vector<int32_t> blob;
    auto put = [&](const int32_t* src, size_t n) {
        while (blob.size() % 4) blob.push_back(0);   // 16-byte alignment of every list
        const size_t off = blob.size();
        blob.insert(blob.end(), src, src + n);
        if (n == 0) blob.push_back(0);               // keep every list pointer valid
        return off;
    };
    p->o_cseg_off = put(p->cseg_off.data(), p->cseg_off.size());
    p->o_cseg_task = put(p->cseg_task.data(), p->cseg_task.size());
    p->o_rowblk = put(p->rowblk_seg.data(), p->rowblk_seg.size());
    p->o_tb = put(reinterpret_cast<const int32_t*>(p->tb.data()), p->tb.size() * 4);
    p->o_chunks = put(reinterpret_cast<const int32_t*>(p->chunks.data()), p->chunks.size() * 4);
    p->o_task_chunk = put(p->task_chunk_off.data(), p->task_chunk_off.size());
    p->o_rank_off = put(p->rank_off.data(), p->rank_off.size());
    p->o_task_tb = put(p->task_tb_off.data(), p->task_tb_off.size());
    p->o_sb = put(p->sb_off.data(), p->sb_off.size());
    p->o_tb_order = put(p->tb_order.data(), p->tb_order.size());
    p->o_sb_order = put(p->sb_order.data(), p->sb_order.size());
    p->o_fb_wg = put(p->fb_wg_run_off.data(), p->fb_wg_run_off.size());
    p->o_fb_run = put(p->fb_run_row.data(), p->fb_run_row.size());
    p->o_fb_cnt = put(p->fb_cnt.data(), p->fb_cnt.size());
    p->o_fb_row0 = put(p->fb_task_row0.data(), p->fb_task_row0.size());
    p->o_tile_tab = put(p->gemm_tile_tab.data(), p->gemm_tile_tab.size());
    while (blob.size() % 4) blob.push_back(0);
    return blob;
}

}  // namespace lobra
