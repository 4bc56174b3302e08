// Host side of a batch plan: validation of the descriptor and the work lists that the
// kernels walk.  Pure C++ (no HIP), so that it can be built and tested without a GPU.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "lobra_mlora.h"

namespace lobra {

constexpr int kTokenBlock = 32;   // tokens per token block (one MFMA K step of the reductions)
constexpr int kRowBlock = 32;     // granularity of the row -> segment lookup table
constexpr int kGemmTileRows = 256;    // token rows of a base-GEMM output tile
constexpr int kGemmTileRec = 8;       // ints per record of Plan::gemm_tile_tab
constexpr bool kMfmaKernels = true;   // bf16 storage runs on the MFMA kernels
constexpr int64_t kPlainMaxTokens = 65535 * 64;   // the plain kernels put 64-token tiles on grid.y

struct TokenBlock { int32_t row0, nrows, task, rank_row0; };
struct GradChunk  { int32_t tb_begin, tb_end, task, part_row0; };

// The rank-r projection of a long batch of ranks up to 16 cuts K into slices of 512 columns and lets one
// workgroup per compute unit walk (token block, slice) items (shrink_sliced_kernel).  nsl = slices; nsl = 0: the
// one-block-per-workgroup kernels are used.  (m = slabs of 128 columns per wave and item: always 1.)
struct SlicedShape { int32_t m = 0, nsl = 0; };
constexpr int kSlicedGrid = 256;      // its workgroups: 8 XCDs x 32 compute units
// The shape for ntb token blocks projected from width D, or none: widths that are not a multiple of the slice,
// other ranks, too few items to keep every compute unit busy.
SlicedShape sliced_shrink_shape(int64_t ntb, int32_t r_pad, int32_t D);

// Byte offsets of the sub-buffers inside h_save and the workspaces.
struct BufferLayout {
    size_t p_tok = 0;     // token-major projected activations  [T][pstride]
    size_t p_blk = 0;     // block-transposed copy              [n_tb][rpad][32]  (MFMA path)
    size_t total = 0;
};

struct Plan {
    lobra_mlora_desc desc{};            // table pointers point into the vectors below
    uint32_t flags = 0;
    bool mfma = false;                  // bf16 storage and MFMA kernels
    int32_t r_max = 0, r_pad = 0, R_tot = 0;
    int32_t n_proj = 1;                 // shared-input projections fused into the call
    int32_t dg = 0;                     // d_out / n_proj: width of B and dB
    std::vector<int32_t> rank_off;      // [n_tasks+1]
    std::vector<int32_t> seg_off_in, seg_task_in;   // the caller's table, as given
    std::vector<int32_t> cseg_off, cseg_task;       // compacted table
    std::vector<int32_t> rowblk_seg;    // [ceil(T/32)]
    // One record of kGemmTileRec ints per tile row of the base GEMM (tile row i starts at token
    // min(i kGemmTileRows, T - kGemmTileRows), never below 0): the compacted segment that holds that token, its
    // first and last + 1 token, its task (-1: none), and that task's first rank row and stacked rank
    // (0, 0 without a task); the rest is padding.  One 32-byte read tells a GEMM workgroup what the fused
    // up projection of a tile starts with.
    std::vector<int32_t> gemm_tile_tab; // [ceil(T/kGemmTileRows)][kGemmTileRec]
    std::vector<TokenBlock> tb;         // grouped by task, token order inside a task
    std::vector<int32_t> task_tb_off;   // [n_tasks+1]
    std::vector<int32_t> sb_off;        // [nsb+1] runs of <= shrink_group token blocks of one task
    int32_t shrink_group = 1;           // token blocks that one shrink workgroup handles (1 or 4)
    // launch order of the shrink workgroups when ranks differ: token blocks / runs by descending rank
    // (stable), so that the most expensive ones do not form the tail of the launch.  Empty: as stored.
    std::vector<int32_t> tb_order, sb_order;
    std::vector<GradChunk> chunks;      // grouped by task
    std::vector<int32_t> task_chunk_off;// [n_tasks+1]
    int32_t part_rows = 0;              // rows of the partial-sum buffer = sum over chunks of r_t
    int32_t chunk_blocks = 0;           // token blocks per reduction chunk

    BufferLayout p_layout;              // layout of h_save (and of the G buffer in bwd)
    size_t h_save_bytes = 0, fwd_ws_bytes = 0, bwd_ws_bytes = 0;
    size_t bwd_off_g = 0, bwd_off_h = 0, bwd_off_part_b = 0, bwd_off_part_a = 0;
    // K-sliced projection: its shape for the projection from d_in (x, A) and from d_out (dy, B), and where its
    // fp32 partial projections [nsl][T][16] go: at the start of the forward workspace (the projected
    // activations follow at fwd_off_p unless the caller gives h_save), at bwd_off_spart in the backward one
    SlicedShape sliced_in, sliced_out;
    size_t fwd_off_p = 0, bwd_off_spart = 0;
    // dB fused into the sliced projection of dy (one pass over dy for s_t B_t dy_i and for dB): a workgroup
    // keeps the dB sums of the (task, slice) it is working on and writes them out - 16 rank rows x 512
    // columns - whenever task or slice changes.  These tables say where: the runs of workgroup g are
    // fb_wg_run_off[g] .. fb_wg_run_off[g + 1] - 1 in the order it meets them, run i goes to the rows
    // fb_run_row[i] .. + 15 of the partial array [fb_rows][d_out]; the k-th run of (task t, slice s) over all
    // workgroups sits at row fb_task_row0[t] + 16 k, and there are fb_cnt[t * nsl + s] of them (stage 2 adds
    // them in that order).
    bool fused_db = false;
    std::vector<int32_t> fb_wg_run_off, fb_run_row, fb_cnt, fb_task_row0;
    int32_t fb_rows = 0;

    // optional launch trace (see lobra_mlora_plan_set_trace)
    mutable void* const* trace_events = nullptr;
    mutable int32_t trace_pairs = 0;
    mutable int32_t* trace_ids = nullptr;
    mutable int32_t* trace_count = nullptr;
    mutable int32_t trace_next = 0;

    // device copy (absent for host-only plans)
    int device = -1;
    void* dev_blob = nullptr;
    bool owns_blob = false;             // dev_blob came from hipMalloc (plan_create), not from the caller (plan_init)
    std::vector<int32_t> host_blob;     // what dev_blob holds
    size_t blob_bytes = 0;
    void* static_ws = nullptr;          // this device's copy of the library's static scratch array
    // offsets (in int32 units) of the lists inside the blob
    size_t o_cseg_off = 0, o_cseg_task = 0, o_rowblk = 0, o_tb = 0, o_chunks = 0,
           o_task_chunk = 0, o_rank_off = 0, o_task_tb = 0, o_sb = 0, o_tb_order = 0, o_sb_order = 0,
           o_fb_wg = 0, o_fb_run = 0, o_fb_cnt = 0, o_fb_row0 = 0, o_tile_tab = 0;
};

lobra_status validate(const lobra_mlora_desc* d);
// Fills every host field of `p` (not the device copy).  `d` has been validated.
lobra_status build_host_plan(const lobra_mlora_desc* d, uint32_t flags, Plan* p);
// Packs the lists into one int32 blob; sets the o_* offsets.
std::vector<int32_t> pack_blob(Plan* p);

}  // namespace lobra

struct lobra_mlora_plan : lobra::Plan {};
