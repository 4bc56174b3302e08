// extern "C" entry points declared in include/lobra_mlora.h: argument checks, plan life cycle,
// and the sequence of kernel launches of one forward / backward call.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <new>

#include "kernels.h"
#include "lobra_mlora.h"
#include "plan.h"

using namespace lobra;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

PlanDev device_view(const Plan& p)
{
    const int32_t* b = static_cast<const int32_t*>(p.dev_blob);
    PlanDev d;
    d.cseg_off = b + p.o_cseg_off;
    d.cseg_task = b + p.o_cseg_task;
    d.rowblk_seg = b + p.o_rowblk;
    d.tb = reinterpret_cast<const TokenBlock*>(b + p.o_tb);
    d.chunks = reinterpret_cast<const GradChunk*>(b + p.o_chunks);
    d.task_chunk_off = b + p.o_task_chunk;
    d.rank_off = b + p.o_rank_off;
    d.task_tb_off = b + p.o_task_tb;
    d.sb_off = b + p.o_sb;
    d.tb_order = p.tb_order.empty() ? nullptr : b + p.o_tb_order;
    d.sb_order = p.sb_order.empty() ? nullptr : b + p.o_sb_order;
    d.fb_wg_run_off = p.fused_db ? b + p.o_fb_wg : nullptr;
    d.fb_run_row = p.fused_db ? b + p.o_fb_run : nullptr;
    d.fb_cnt = p.fused_db ? b + p.o_fb_cnt : nullptr;
    d.fb_task_row0 = p.fused_db ? b + p.o_fb_row0 : nullptr;
    d.gemm_tile_tab = b + p.o_tile_tab;
    d.T = int32_t(p.desc.T);
    d.d_in = p.desc.d_in;
    d.d_out = p.desc.d_out;
    d.n_tasks = p.desc.n_tasks;
    d.nseg = int32_t(p.cseg_task.size());
    d.ntb = int32_t(p.tb.size());
    d.nchunks = int32_t(p.chunks.size());
    d.r_max = p.r_max;
    d.r_pad = p.r_pad;
    d.R_tot = p.R_tot;
    d.nsb = int32_t(p.sb_off.size()) - 1;
    d.shrink_group = p.shrink_group;
    d.n_proj = p.n_proj;
    d.dg = p.dg;
    return d;
}

// A plan can run only on the device it was uploaded to.
lobra_status runnable(const lobra_mlora_plan* plan)
{
    if (!plan) return LOBRA_ERR_PLAN;
    if (!plan->dev_blob) return LOBRA_ERR_PLAN;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return LOBRA_ERR_HIP;
    if (dev != plan->device) return LOBRA_ERR_PLAN;
    return LOBRA_OK;
}

#define LOBRA_HIP(expr)                                   \
    do {                                                  \
        if ((expr) != hipSuccess) return LOBRA_ERR_HIP;   \
    } while (0)

// One kernel launch, bracketed by the plan's trace events when a trace is attached.
#define LOBRA_LAUNCH(plan_ref, stream, kernel_id, expr)                                          \
    do {                                                                                         \
        const Plan& tp_ = (plan_ref);                                                            \
        const int32_t ti_ = tp_.trace_events ? tp_.trace_next++ : -1;                            \
        const bool tr_ = ti_ >= 0 && ti_ < tp_.trace_pairs;                                      \
        if (tp_.trace_count) *tp_.trace_count = tp_.trace_next;                                  \
        if (tr_) {                                                                               \
            if (tp_.trace_ids) tp_.trace_ids[ti_] = (kernel_id);                                 \
            LOBRA_HIP(hipEventRecord(static_cast<hipEvent_t>(tp_.trace_events[2 * ti_]), stream)); \
        }                                                                                        \
        LOBRA_HIP(expr);                                                                         \
        if (tr_)                                                                                 \
            LOBRA_HIP(hipEventRecord(static_cast<hipEvent_t>(tp_.trace_events[2 * ti_ + 1]), stream)); \
    } while (0)

// Argument checks of a forward call on plan p (everything except the plan itself): host only.
lobra_status fwd_check(const Plan& p, const void* x, const void* W, const void* A, const void* B, const float* s,
                       const void* y, const void* h_save, const void* ws, size_t ws_bytes, bool sliced = true)
{
    const bool adapters = !p.tb.empty();
    if (!x || !W || !y) return LOBRA_ERR_NULL;
    if (adapters && (!A || !B || !s)) return LOBRA_ERR_NULL;
    if (!aligned16(x) || !aligned16(W) || !aligned16(y) || !aligned16(A) || !aligned16(B) ||
        !aligned16(h_save) || !aligned16(ws))
        return LOBRA_ERR_ALIGN;
    // the workspace holds the sliced projection's partial sums (if the plan uses it) and, without h_save, the
    // projected activations behind them
    const size_t need = (sliced ? p.fwd_off_p : 0) + (h_save ? 0 : p.p_layout.total);
    if (adapters && need > 0 && (!ws || ws_bytes < need)) return LOBRA_ERR_WORKSPACE;
    return LOBRA_OK;
}

// The same for a backward call.
lobra_status bwd_check(const Plan& p, const void* x, const void* W, const void* A, const void* B, const float* s,
                       const void* dy, const void* h_saved, const void* dx, const float* dA, const float* dB,
                       uint32_t flags, const void* ws, size_t ws_bytes)
{
    const bool adapters = !p.tb.empty();
    const bool want_dx = !(flags & LOBRA_FLAG_NO_DX);
    if (p.R_tot > 0 && (!dA || !dB)) return LOBRA_ERR_NULL;
    if (p.desc.T > 0) {
        if (!W || !dy) return LOBRA_ERR_NULL;
        if (want_dx && !dx) return LOBRA_ERR_NULL;
        if (adapters && (!x || !A || !B || !s)) return LOBRA_ERR_NULL;
    }
    if (!aligned16(x) || !aligned16(W) || !aligned16(A) || !aligned16(B) || !aligned16(dy) ||
        !aligned16(h_saved) || !aligned16(dx) || !aligned16(dA) || !aligned16(dB) || !aligned16(ws))
        return LOBRA_ERR_ALIGN;
    if (p.bwd_ws_bytes > 0 && adapters && (!ws || ws_bytes < p.bwd_ws_bytes)) return LOBRA_ERR_WORKSPACE;
    return LOBRA_OK;
}

// Scratch of lobra_mlora_fwd_static_ws: device memory that is part of the library's code object, so that
// a call needs no allocation by anybody.  Every GPU the library runs on holds its own copy at its own
// address; the name below is only a handle for hipGetSymbolAddress, never a pointer to pass to a kernel.
static __device__ __align__(256) unsigned char scratch[LOBRA_STATIC_WS_BYTES];

// Address of `scratch` on the current device (looked up once per plan, at plan creation).
lobra_status static_scratch_address(void** out)
{
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LOBRA_ERR_HIP;
    *out = p;
    return LOBRA_OK;
}

}  // namespace

extern "C" {

lobra_status lobra_mlora_validate(const lobra_mlora_desc* desc) { return validate(desc); }

// Host side of a plan and its packed device image (kept in the plan: an asynchronous upload reads it later).
static lobra_status make_host_plan(const lobra_mlora_desc* desc, uint32_t plan_flags, lobra_mlora_plan** out)
{
    lobra_status st = validate(desc);
    if (st != LOBRA_OK) return st;
    lobra_mlora_plan* p = new (std::nothrow) lobra_mlora_plan();
    if (!p) return LOBRA_ERR_NOMEM;
    st = build_host_plan(desc, plan_flags, p);
    if (st == LOBRA_OK && !(plan_flags & LOBRA_PLAN_HOST_ONLY)) {
        try {
            p->host_blob = pack_blob(p);
            p->blob_bytes = p->host_blob.size() * sizeof(int32_t);
        } catch (const std::bad_alloc&) {
            st = LOBRA_ERR_NOMEM;
        }
    }
    if (st != LOBRA_OK) {
        delete p;
        return st;
    }
    *out = p;
    return LOBRA_OK;
}

lobra_status lobra_mlora_plan_create(const lobra_mlora_desc* desc, uint32_t plan_flags,
                                     lobra_mlora_plan** out)
{
    if (!out) return LOBRA_ERR_NULL;
    lobra_mlora_plan* p = nullptr;
    lobra_status st = make_host_plan(desc, plan_flags, &p);
    if (st != LOBRA_OK) return st;
    if (!(plan_flags & LOBRA_PLAN_HOST_ONLY)) {
        if (hipGetDevice(&p->device) != hipSuccess || static_scratch_address(&p->static_ws) != LOBRA_OK) {
            delete p;
            return LOBRA_ERR_HIP;
        }
        if (hipMalloc(&p->dev_blob, p->blob_bytes) != hipSuccess) {
            delete p;
            return LOBRA_ERR_NOMEM;
        }
        p->owns_blob = true;
        if (hipMemcpy(p->dev_blob, p->host_blob.data(), p->blob_bytes, hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipFree(p->dev_blob);
            delete p;
            return LOBRA_ERR_HIP;
        }
    }
    *out = p;
    return LOBRA_OK;
}

lobra_status lobra_mlora_plan_device_bytes(const lobra_mlora_desc* desc, uint32_t plan_flags, size_t* bytes)
{
    if (!bytes) return LOBRA_ERR_NULL;
    lobra_mlora_plan* p = nullptr;
    lobra_status st = make_host_plan(desc, plan_flags & ~uint32_t(LOBRA_PLAN_HOST_ONLY), &p);
    if (st != LOBRA_OK) return st;
    *bytes = p->blob_bytes;
    delete p;
    return LOBRA_OK;
}

lobra_status lobra_mlora_plan_init(const lobra_mlora_desc* desc, uint32_t plan_flags, void* device_mem,
                                   size_t device_bytes, void* hip_stream, lobra_mlora_plan** out)
{
    if (!out) return LOBRA_ERR_NULL;
    if (plan_flags & LOBRA_PLAN_HOST_ONLY) return LOBRA_ERR_PLAN;
    lobra_mlora_plan* p = nullptr;
    lobra_status st = make_host_plan(desc, plan_flags, &p);
    if (st != LOBRA_OK) return st;
    if (!device_mem || device_bytes < p->blob_bytes) st = LOBRA_ERR_WORKSPACE;
    else if (!aligned16(device_mem)) st = LOBRA_ERR_ALIGN;
    else if (hipGetDevice(&p->device) != hipSuccess || static_scratch_address(&p->static_ws) != LOBRA_OK) st = LOBRA_ERR_HIP;
    // the source of the copy is the plan's own host image, which lives as long as the plan
    else if (hipMemcpyAsync(device_mem, p->host_blob.data(), p->blob_bytes, hipMemcpyHostToDevice,
                            static_cast<hipStream_t>(hip_stream)) != hipSuccess) st = LOBRA_ERR_HIP;
    if (st != LOBRA_OK) {
        delete p;
        return st;
    }
    p->dev_blob = device_mem;
    p->owns_blob = false;
    *out = p;
    return LOBRA_OK;
}

lobra_status lobra_mlora_plan_destroy(lobra_mlora_plan* plan)
{
    if (!plan) return LOBRA_OK;
    lobra_status st = LOBRA_OK;
    if (plan->dev_blob && plan->owns_blob && hipFree(plan->dev_blob) != hipSuccess) st = LOBRA_ERR_HIP;
    delete plan;
    return st;
}

lobra_status lobra_mlora_plan_sizes(const lobra_mlora_plan* plan, size_t* h_save_bytes,
                                    size_t* fwd_ws_bytes, size_t* bwd_ws_bytes)
{
    if (!plan) return LOBRA_ERR_PLAN;
    if (h_save_bytes) *h_save_bytes = plan->h_save_bytes;
    if (fwd_ws_bytes) *fwd_ws_bytes = plan->fwd_ws_bytes;
    if (bwd_ws_bytes) *bwd_ws_bytes = plan->bwd_ws_bytes;
    return LOBRA_OK;
}

lobra_status lobra_mlora_plan_query(const lobra_mlora_plan* plan, int32_t what, int32_t* out,
                                    size_t capacity, size_t* count)
{
    if (!plan) return LOBRA_ERR_PLAN;
    if (!count) return LOBRA_ERR_NULL;
    std::vector<int32_t> tmp;
    const int32_t* src = nullptr;
    size_t n = 0;
    switch (what) {
    case LOBRA_Q_SEGMENTS:
        for (size_t k = 0; k < plan->cseg_task.size(); ++k) {
            tmp.push_back(plan->cseg_off[k]);
            tmp.push_back(plan->cseg_off[k + 1]);
            tmp.push_back(plan->cseg_task[k]);
        }
        src = tmp.data();
        n = tmp.size();
        break;
    case LOBRA_Q_ROWBLOCK_SEG:
        src = plan->rowblk_seg.data();
        n = plan->rowblk_seg.size();
        break;
    case LOBRA_Q_TOKEN_BLOCKS:
        src = reinterpret_cast<const int32_t*>(plan->tb.data());
        n = plan->tb.size() * 4;
        break;
    case LOBRA_Q_GRAD_CHUNKS:
        src = reinterpret_cast<const int32_t*>(plan->chunks.data());
        n = plan->chunks.size() * 4;
        break;
    case LOBRA_Q_TASK_CHUNKS:
        src = plan->task_chunk_off.data();
        n = plan->task_chunk_off.size();
        break;
    case LOBRA_Q_BLOCK_RUNS:
        src = plan->sb_off.data();
        n = plan->sb_off.size();
        break;
    case LOBRA_Q_BLOCK_ORDER:
        src = plan->tb_order.data();
        n = plan->tb_order.size();
        break;
    case LOBRA_Q_RUN_ORDER:
        src = plan->sb_order.data();
        n = plan->sb_order.size();
        break;
    case LOBRA_Q_SLICED:
        tmp = {plan->sliced_in.nsl, plan->sliced_out.nsl, plan->fused_db ? 1 : 0, plan->fb_rows, kSlicedGrid};
        src = tmp.data();
        n = tmp.size();
        break;
    case LOBRA_Q_FUSED_WG_RUNS:
        src = plan->fb_wg_run_off.data();
        n = plan->fb_wg_run_off.size();
        break;
    case LOBRA_Q_FUSED_RUN_ROW:
        src = plan->fb_run_row.data();
        n = plan->fb_run_row.size();
        break;
    case LOBRA_Q_FUSED_COUNT:
        src = plan->fb_cnt.data();
        n = plan->fb_cnt.size();
        break;
    case LOBRA_Q_FUSED_TASK_ROW:
        src = plan->fb_task_row0.data();
        n = plan->fb_task_row0.size();
        break;
    case LOBRA_Q_GEMM_TILE_ROWS:
        src = plan->gemm_tile_tab.data();
        n = plan->gemm_tile_tab.size();
        break;
    default:
        return LOBRA_ERR_SHAPE;
    }
    *count = n;
    if (out && n) std::memcpy(out, src, sizeof(int32_t) * (n < capacity ? n : capacity));
    return LOBRA_OK;
}

namespace {
// The forward pass.  sliced = false: without the K-sliced projection even where the plan would take it (its
// partial sums are most of the forward workspace): the projected activations then start at ws itself.
lobra_status plan_fwd(const lobra_mlora_plan* plan, const void* x, const void* W, const void* A, const void* B,
                      const float* s, void* y, void* h_save, void* ws, size_t ws_bytes, void* hip_stream, bool sliced)
{
    lobra_status rs = runnable(plan);
    if (rs != LOBRA_OK) return rs;
    const Plan& p = *plan;
    if (p.desc.T == 0) return LOBRA_OK;
    rs = fwd_check(p, x, W, A, B, s, y, h_save, ws, ws_bytes, sliced);
    if (rs != LOBRA_OK) return rs;
    const bool adapters = !p.tb.empty();
    void* hbuf = h_save ? h_save : static_cast<char*>(ws) + (sliced ? p.fwd_off_p : 0);
    const SlicedShape sliced_in = sliced ? p.sliced_in : SlicedShape{};
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const PlanDev pd = device_view(p);
    const int dt = p.desc.dtype;
    if (!p.mfma) {
        if (adapters)
            LOBRA_LAUNCH(p, st, LOBRA_K_SHRINK,
                         plain_shrink(pd, dt, x, A, s, static_cast<float*>(hbuf), pd.d_in, st));
        const size_t esz = dt == LOBRA_F32 ? 4 : 2;
        for (int32_t j = 0; j < p.n_proj; ++j) {        // one product per projection (one in all when n_proj = 1)
            const size_t col = size_t(j) * pd.dg * esz;   // bytes into a row of W / y
            LOBRA_LAUNCH(p, st, LOBRA_K_GEMM,
                         plain_gemm(pd, dt, false, x, static_cast<const char*>(W) + col,
                                    static_cast<const float*>(hbuf), B, static_cast<char*>(y) + col, pd.d_in,
                                    pd.dg, pd.d_out, st, pd.d_out, p.n_proj, j));
        }
        return LOBRA_OK;
    }
    // bf16 MFMA path
    char* hb = static_cast<char*>(hbuf);
    if (adapters)   // all projections' down factors are stacked in A: one pass over x
        LOBRA_LAUNCH(p, st, LOBRA_K_SHRINK,
                     shrink_mfma(pd, x, A, s, hb + p.p_layout.p_tok, hb + p.p_layout.p_blk, pd.d_in, pd.d_in, 1, 0, st,
                                 sliced_in, static_cast<float*>(ws)));
    if (p.n_proj == 1) {
        LOBRA_LAUNCH(p, st, LOBRA_K_GEMM,
                     gemm_mfma(pd, false, x, W, adapters ? hb + p.p_layout.p_tok : nullptr, B, y, pd.d_in,
                               pd.d_out, pd.d_out, st));
        return LOBRA_OK;
    }
    // fused shared-input projections: every column tile of y takes the rank window of H and the rows of
    // the compact B that belong to its projection - in one launch when no tile straddles two projections,
    // else in one launch per projection (its column block of W and y)
    if (pd.dg % 256 == 0) {
        LOBRA_LAUNCH(p, st, LOBRA_K_GEMM,
                     gemm_mfma(pd, false, x, W, adapters ? hb + p.p_layout.p_tok : nullptr, B, y, pd.d_in,
                               pd.d_out, pd.d_out, st, pd.d_out, p.n_proj, -1));
        return LOBRA_OK;
    }
    for (int32_t j = 0; j < p.n_proj; ++j) {
        const size_t col = size_t(j) * pd.dg * 2;                   // bytes into a row of W / y
        LOBRA_LAUNCH(p, st, LOBRA_K_GEMM,
                     gemm_mfma(pd, false, x, static_cast<const char*>(W) + col,
                               adapters ? hb + p.p_layout.p_tok : nullptr, B, static_cast<char*>(y) + col, pd.d_in,
                               pd.dg, pd.d_out, st, pd.d_out, p.n_proj, j));
    }
    return LOBRA_OK;
}
}  // namespace

lobra_status lobra_mlora_plan_fwd(const lobra_mlora_plan* plan, const void* x, const void* W,
                             const void* A, const void* B, const float* s, void* y,
                             void* h_save, void* ws, size_t ws_bytes, void* hip_stream)
{
    return plan_fwd(plan, x, W, A, B, s, y, h_save, ws, ws_bytes, hip_stream, true);
}

lobra_status lobra_mlora_fwd_static_ws(const lobra_mlora_plan* plan, const void* x, const void* W,
                                       const void* A, const void* B, const float* s, void* y,
                                       void* hip_stream)
{
    lobra_status rs = runnable(plan);
    if (rs != LOBRA_OK) return rs;
    // a batch whose K-sliced projection needs more than the array for its partial sums goes without it: the
    // one-block-per-workgroup projection needs the projected activations only
    const bool sliced = plan->fwd_ws_bytes <= size_t(LOBRA_STATIC_WS_BYTES);
    if (!sliced && plan->p_layout.total > size_t(LOBRA_STATIC_WS_BYTES)) return LOBRA_ERR_WORKSPACE;
    // the kernels get the array's device address, looked up when the plan was created on this device
    return plan_fwd(plan, x, W, A, B, s, y, nullptr, plan->static_ws, size_t(LOBRA_STATIC_WS_BYTES), hip_stream, sliced);
}

lobra_status lobra_mlora_plan_bwd(const lobra_mlora_plan* plan, const void* x, const void* W,
                             const void* A, const void* B, const float* s, const void* dy,
                             const void* h_saved, void* dx, float* dA, float* dB,
                             uint32_t flags, void* ws, size_t ws_bytes, void* hip_stream)
{
    lobra_status rs = runnable(plan);
    if (rs != LOBRA_OK) return rs;
    const Plan& p = *plan;
    rs = bwd_check(p, x, W, A, B, s, dy, h_saved, dx, dA, dB, flags, ws, ws_bytes);
    if (rs != LOBRA_OK) return rs;
    const bool adapters = !p.tb.empty();
    const bool want_dx = !(flags & LOBRA_FLAG_NO_DX);
    const bool accumulate = (flags & LOBRA_FLAG_ACCUMULATE_GRADS) != 0;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const PlanDev pd = device_view(p);
    const int dt = p.desc.dtype;
    char* wsb = static_cast<char*>(ws);
    float* part_b = adapters ? reinterpret_cast<float*>(wsb + p.bwd_off_part_b) : nullptr;
    float* part_a = adapters ? reinterpret_cast<float*>(wsb + p.bwd_off_part_a) : nullptr;
    if (!p.mfma) {
        float* G = adapters ? reinterpret_cast<float*>(wsb + p.bwd_off_g) : nullptr;
        const float* H = static_cast<const float*>(h_saved);
        if (adapters) {
            if (!H) {
                float* Hr = reinterpret_cast<float*>(wsb + p.bwd_off_h);
                LOBRA_LAUNCH(p, st, LOBRA_K_SHRINK, plain_shrink(pd, dt, x, A, s, Hr, pd.d_in, st));
                H = Hr;
            }
            const size_t esz = dt == LOBRA_F32 ? 4 : 2;
            for (int32_t j = 0; j < p.n_proj; ++j)
                LOBRA_LAUNCH(p, st, LOBRA_K_SHRINK,
                             plain_shrink(pd, dt, static_cast<const char*>(dy) + size_t(j) * pd.dg * esz, B, s, G,
                                          pd.dg, st, pd.d_out, p.n_proj, j));
        }
        if (want_dx && p.desc.T > 0)
            LOBRA_LAUNCH(p, st, LOBRA_K_GEMM,
                         plain_gemm(pd, dt, true, dy, W, G, A, dx, pd.d_out, pd.d_in, pd.d_out, st));
        if (p.R_tot > 0) {
            if (adapters) {
                const size_t esz = dt == LOBRA_F32 ? 4 : 2;
                if (p.n_proj == 1) {       // dB and dA in one launch
                    LOBRA_LAUNCH(p, st, LOBRA_K_GRAD_STAGE1,
                                 plain_grad_stage1(pd, dt, false, H, dy, part_b, pd.d_out, st, 0, 1, 0, G, x, part_a, pd.d_in));
                } else {
                    for (int32_t j = 0; j < p.n_proj; ++j)
                        LOBRA_LAUNCH(p, st, LOBRA_K_GRAD_STAGE1,
                                     plain_grad_stage1(pd, dt, false, H, static_cast<const char*>(dy) + size_t(j) * pd.dg * esz,
                                                       part_b, pd.dg, st, pd.d_out, p.n_proj, j));
                    LOBRA_LAUNCH(p, st, LOBRA_K_GRAD_STAGE1,
                                 plain_grad_stage1(pd, dt, false, G, x, part_a, pd.d_in, st));
                }
            }
            const GradJob jb{H, dy, part_b, dB, pd.dg}, ja{G, x, part_a, dA, pd.d_in};
            LOBRA_LAUNCH(p, st, LOBRA_K_GRAD_STAGE2, reduce_partials(pd, jb, ja, accumulate, st));
        }
        return LOBRA_OK;
    }
    // bf16 MFMA path
    char* G = adapters ? wsb + p.bwd_off_g : nullptr;
    float* spart = adapters ? reinterpret_cast<float*>(wsb + p.bwd_off_spart) : nullptr;
    // dB in the same pass over dy as G = s dy B^T (then stage 1 below is dA alone)
    const bool fused_db = adapters && p.fused_db && p.R_tot > 0;
    const char* H = static_cast<const char*>(h_saved);
    if (adapters) {
        if (!H) {
            char* Hr = wsb + p.bwd_off_h;
            LOBRA_LAUNCH(p, st, LOBRA_K_SHRINK,
                         shrink_mfma(pd, x, A, s, Hr + p.p_layout.p_tok, Hr + p.p_layout.p_blk, pd.d_in, pd.d_in, 1, 0, st,
                                     p.sliced_in, spart));
            H = Hr;
        }
        // G = s dy B^T; with fused projections one launch per projection: its column block of dy
        // against its rows of the compact B, written into its rank window of G
        for (int32_t j = 0; j < p.n_proj; ++j)
            LOBRA_LAUNCH(p, st, LOBRA_K_SHRINK,
                         shrink_mfma(pd, static_cast<const char*>(dy) + size_t(j) * pd.dg * 2, B, s,
                                     G + p.p_layout.p_tok, G + p.p_layout.p_blk, pd.dg, pd.d_out, p.n_proj, j, st,
                                     p.sliced_out, spart, fused_db ? H + p.p_layout.p_blk : nullptr, part_b));
    }
    if (want_dx && p.desc.T > 0)
        LOBRA_LAUNCH(p, st, LOBRA_K_GEMM,
                     gemm_mfma(pd, true, dy, W, adapters ? G + p.p_layout.p_tok : nullptr, A, dx, pd.d_out,
                               pd.d_in, pd.d_out, st));
    if (p.R_tot > 0) {
        // dB (from s h and dy) and dA (from s g and x) share one launch per stage
        GradJob jb{adapters ? H + p.p_layout.p_blk : nullptr, dy, part_b, dB, pd.dg};
        const GradJob ja{adapters ? G + p.p_layout.p_blk : nullptr, x, part_a, dA, pd.d_in};
        if (fused_db) {
            const GradJob none{nullptr, nullptr, nullptr, nullptr, 0};
            LOBRA_LAUNCH(p, st, LOBRA_K_GRAD_STAGE1, grad_mfma(pd, ja, none, st));
            jb.fcnt = pd.fb_cnt;
            jb.frow0 = pd.fb_task_row0;
            jb.fnsl = p.sliced_out.nsl;
        } else if (p.n_proj == 1) {
            if (adapters) LOBRA_LAUNCH(p, st, LOBRA_K_GRAD_STAGE1, grad_mfma(pd, jb, ja, st));
        } else if (adapters) {
            // dA over all stacked ranks in one pass over x; dB per projection (its column block of dy,
            // its rank window of H, its rows of the compact dB)
            const GradJob none{nullptr, nullptr, nullptr, nullptr, 0};
            LOBRA_LAUNCH(p, st, LOBRA_K_GRAD_STAGE1, grad_mfma(pd, ja, none, st));
            if (pd.dg % 128 == 0) {     // no column tile straddles two projections: one pass over all of dy
                GradJob jall = jb;
                jall.D = pd.d_out;
                jall.ldp = pd.dg;
                jall.nproj = p.n_proj;
                jall.proj = -1;
                LOBRA_LAUNCH(p, st, LOBRA_K_GRAD_STAGE1, grad_mfma(pd, jall, none, st));
            } else
            for (int32_t j = 0; j < p.n_proj; ++j) {
                GradJob jj = jb;
                jj.Z = static_cast<const char*>(dy) + size_t(j) * pd.dg * 2;
                jj.ldz = pd.d_out;
                jj.nproj = p.n_proj;
                jj.proj = j;
                LOBRA_LAUNCH(p, st, LOBRA_K_GRAD_STAGE1, grad_mfma(pd, jj, none, st));
            }
        }
        LOBRA_LAUNCH(p, st, LOBRA_K_GRAD_STAGE2, reduce_partials(pd, jb, ja, accumulate, st));
    }
    return LOBRA_OK;
}

lobra_status lobra_mlora_plan_token_task_map(const lobra_mlora_plan* plan, int32_t* out_task,
                                  int64_t* out_count, void* hip_stream)
{
    lobra_status rs = runnable(plan);
    if (rs != LOBRA_OK) return rs;
    const PlanDev pd = device_view(*plan);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    LOBRA_LAUNCH(*plan, st, LOBRA_K_TOKEN_TASK, token_task_map(pd, out_task, out_count, st));
    return LOBRA_OK;
}

// ---- descriptor-taking one-shot forms: the plan of the call is built on the host, its device image is placed
//      at the start of the caller's workspace by an asynchronous copy on the caller's stream, and the
//      plan-taking entry point does the rest with what remains of the workspace.
namespace {

inline size_t align256(size_t v) { return (v + 255) / 256 * 256; }

// Frees a one-shot plan (and with it the host image its upload reads) once the stream has passed the upload.
void free_oneshot_plan(void* p) { delete static_cast<lobra_mlora_plan*>(p); }

lobra_status release_after(hipStream_t st, lobra_mlora_plan* p)
{
    if (hipLaunchHostFunc(st, free_oneshot_plan, p) == hipSuccess) return LOBRA_OK;
    // no host callback on this stream: wait for the upload instead (slow path, never taken on a plain stream)
    const hipError_t e = hipStreamSynchronize(st);
    delete p;
    return e == hipSuccess ? LOBRA_OK : LOBRA_ERR_HIP;
}

// Places the device image of one-shot plan `p` at dev (device memory of at least align256(p->blob_bytes) bytes).
lobra_status upload_oneshot(lobra_mlora_plan* p, void* dev, hipStream_t st)
{
    if (hipGetDevice(&p->device) != hipSuccess) return LOBRA_ERR_HIP;
    if (hipMemcpyAsync(dev, p->host_blob.data(), p->blob_bytes, hipMemcpyHostToDevice, st) != hipSuccess)
        return LOBRA_ERR_HIP;
    p->dev_blob = dev;
    p->owns_blob = false;
    return LOBRA_OK;
}

}  // namespace

lobra_status lobra_mlora_workspace_bytes(const lobra_mlora_desc* desc, size_t* fwd_bytes, size_t* bwd_bytes)
{
    lobra_mlora_plan* p = nullptr;
    lobra_status st = make_host_plan(desc, 0, &p);
    if (st != LOBRA_OK) return st;
    const size_t img = align256(p->blob_bytes);
    if (fwd_bytes) *fwd_bytes = img + p->fwd_ws_bytes;
    if (bwd_bytes) *bwd_bytes = img + p->bwd_ws_bytes;
    delete p;
    return LOBRA_OK;
}

lobra_status lobra_mlora_fwd(const lobra_mlora_desc* desc, const void* x, const void* W, const void* A,
                             const void* B, const float* s, void* y, void* h_save, void* ws, size_t ws_bytes,
                             void* hip_stream)
{
    lobra_mlora_plan* p = nullptr;
    lobra_status st = make_host_plan(desc, 0, &p);
    if (st != LOBRA_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const size_t img = align256(p->blob_bytes);
    char* rest = static_cast<char*>(ws) + img;
    if (p->desc.T == 0) st = LOBRA_OK;
    else if (!ws || ws_bytes < img + p->fwd_off_p + (h_save ? 0 : p->p_layout.total)) st = LOBRA_ERR_WORKSPACE;
    else if (!aligned16(ws)) st = LOBRA_ERR_ALIGN;
    else if ((st = fwd_check(*p, x, W, A, B, s, y, h_save, rest, ws_bytes - img)) == LOBRA_OK &&
             (st = upload_oneshot(p, ws, stream)) == LOBRA_OK) {
        st = lobra_mlora_plan_fwd(p, x, W, A, B, s, y, h_save, rest, ws_bytes - img, hip_stream);
        const lobra_status rel = release_after(stream, p);
        return st != LOBRA_OK ? st : rel;
    }
    delete p;
    return st;
}

lobra_status lobra_mlora_bwd(const lobra_mlora_desc* desc, const void* x, const void* W, const void* A,
                             const void* B, const float* s, const void* dy, const void* h_saved, void* dx,
                             float* dA, float* dB, uint32_t flags, void* ws, size_t ws_bytes, void* hip_stream)
{
    lobra_mlora_plan* p = nullptr;
    lobra_status st = make_host_plan(desc, 0, &p);
    if (st != LOBRA_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const size_t img = align256(p->blob_bytes);
    char* rest = static_cast<char*>(ws) + img;
    if (!ws || ws_bytes < img + p->bwd_ws_bytes) st = LOBRA_ERR_WORKSPACE;
    else if (!aligned16(ws)) st = LOBRA_ERR_ALIGN;
    else if ((st = bwd_check(*p, x, W, A, B, s, dy, h_saved, dx, dA, dB, flags, rest, ws_bytes - img)) == LOBRA_OK &&
             (st = upload_oneshot(p, ws, stream)) == LOBRA_OK) {
        st = lobra_mlora_plan_bwd(p, x, W, A, B, s, dy, h_saved, dx, dA, dB, flags, rest, ws_bytes - img, hip_stream);
        const lobra_status rel = release_after(stream, p);
        return st != LOBRA_OK ? st : rel;
    }
    delete p;
    return st;
}

lobra_status lobra_token_task_map(const lobra_mlora_desc* desc, int32_t* out_task, int64_t* out_count,
                                  void* hip_stream)
{
    lobra_mlora_plan* p = nullptr;
    lobra_status st = make_host_plan(desc, 0, &p);
    if (st != LOBRA_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    void* dev = nullptr;
    // the call has no workspace argument: the tables go into the library's static device array
    if (p->blob_bytes > size_t(LOBRA_STATIC_WS_BYTES)) st = LOBRA_ERR_WORKSPACE;
    else if ((st = static_scratch_address(&dev)) == LOBRA_OK && (st = upload_oneshot(p, dev, stream)) == LOBRA_OK) {
        st = lobra_mlora_plan_token_task_map(p, out_task, out_count, hip_stream);
        const lobra_status rel = release_after(stream, p);
        return st != LOBRA_OK ? st : rel;
    }
    delete p;
    return st;
}

lobra_status lobra_mlora_adam_step(const lobra_mlora_plan* plan, const lobra_adam_config* cfg,
                                   const float* lr, const int32_t* step, const float* grad_scale,
                                   const float* dA, const float* dB, float* master_A,
                                   float* master_B, float* m_A, float* v_A, float* m_B, float* v_B,
                                   void* A, void* B, void* hip_stream)
{
    lobra_status rs = runnable(plan);
    if (rs != LOBRA_OK) return rs;
    const Plan& p = *plan;
    if (p.R_tot == 0) return LOBRA_OK;
    if (!cfg || !lr || !step || !dA || !dB || !master_A || !master_B || !m_A || !v_A || !m_B || !v_B)
        return LOBRA_ERR_NULL;
    if (!(cfg->beta1 >= 0.f && cfg->beta1 < 1.f && cfg->beta2 >= 0.f && cfg->beta2 < 1.f && cfg->eps >= 0.f))
        return LOBRA_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const PlanDev pd = device_view(p);
    const AdamTensor ta{dA, master_A, m_A, v_A, A, pd.d_in}, tb{dB, master_B, m_B, v_B, B, pd.dg};
    LOBRA_LAUNCH(p, st, LOBRA_K_ADAM,
                 adam_step(pd, p.desc.dtype, cfg->beta1, cfg->beta2, cfg->eps, cfg->weight_decay, lr, step,
                           grad_scale, ta, tb, st));
    return LOBRA_OK;
}

lobra_status lobra_mlora_plan_set_trace(lobra_mlora_plan* plan, void* const* events, int32_t n_pairs,
                                        int32_t* kernel_ids, int32_t* n_launched)
{
    if (!plan) return LOBRA_ERR_PLAN;
    if (n_pairs < 0) return LOBRA_ERR_SHAPE;
    const bool on = events && n_pairs > 0;
    plan->trace_events = on ? events : nullptr;
    plan->trace_pairs = on ? n_pairs : 0;
    plan->trace_ids = on ? kernel_ids : nullptr;
    plan->trace_count = on ? n_launched : nullptr;
    plan->trace_next = 0;
    if (on && n_launched) *n_launched = 0;
    return LOBRA_OK;
}

const char* lobra_status_string(lobra_status st)
{
    switch (st) {
    case LOBRA_OK: return "ok";
    case LOBRA_ERR_NULL: return "a required pointer is NULL";
    case LOBRA_ERR_SHAPE: return "shape out of range";
    case LOBRA_ERR_DTYPE: return "unsupported dtype";
    case LOBRA_ERR_SEGMENTS: return "malformed segment offsets";
    case LOBRA_ERR_TASK_ID: return "segment task id out of range";
    case LOBRA_ERR_RANK: return "adapter rank out of range";
    case LOBRA_ERR_WORKSPACE: return "workspace missing or too small";
    case LOBRA_ERR_ALIGN: return "pointer or row length not 16-byte aligned";
    case LOBRA_ERR_HIP: return "HIP runtime error";
    case LOBRA_ERR_PLAN: return "plan missing, host-only, or built for another device";
    case LOBRA_ERR_NOMEM: return "out of memory";
    }
    return "unknown status";
}

int lobra_version(void) { return 100; }

}  // extern "C"
