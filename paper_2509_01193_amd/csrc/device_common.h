// Shared by the HIP translation units: the device view of a plan and small helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

#include "plan.h"

namespace lobra {

// Device pointers into the plan blob, passed to kernels by value.
struct PlanDev {
    const int32_t* cseg_off;       // [nseg+1]
    const int32_t* cseg_task;      // [nseg]
    const int32_t* rowblk_seg;     // [ceil(T/32)]
    const TokenBlock* tb;          // [ntb]
    const GradChunk* chunks;       // [nchunks]
    const int32_t* task_chunk_off; // [n_tasks+1]
    const int32_t* rank_off;       // [n_tasks+1]
    const int32_t* task_tb_off;    // [n_tasks+1]
    const int32_t* sb_off;         // [nsb+1]
    const int32_t* tb_order;       // [ntb] launch order of the token blocks, or NULL = as stored
    const int32_t* sb_order;       // [nsb] launch order of the runs, or NULL = as stored
    // dB fused into the sliced projection of dy (NULL when the plan does not use it, see Plan::fused_db)
    const int32_t* fb_wg_run_off;  // [kSlicedGrid + 1]
    const int32_t* fb_run_row;     // [runs] first row of the run's partial sums
    const int32_t* fb_cnt;         // [n_tasks * slices] runs of (task, slice)
    const int32_t* fb_task_row0;   // [n_tasks] row of the first run of (task, any slice)
    const int32_t* gemm_tile_tab;  // [ceil(T/kGemmTileRows)][kGemmTileRec] (see Plan::gemm_tile_tab)
    int32_t T, d_in, d_out, n_tasks, nseg, ntb, nchunks, r_max, r_pad, R_tot, nsb, shrink_group, n_proj, dg;
};

// Index of the compacted segment that holds `row` (0 <= row < T): start from the table entry
// of the row's 32-row block and walk forward.
__device__ __forceinline__ int32_t segment_of_row(const PlanDev& pd, int32_t row)
{
    int32_t k = pd.rowblk_seg[row / kRowBlock];
    while (pd.cseg_off[k + 1] <= row) ++k;
    return k;
}

// Workgroup id -> work item, n items on a grid of n workgroups.  Consecutive workgroup ids run on different
// XCDs (8 of them, each with its own L2), so the identity map deals consecutive items - consecutive 32-row
// blocks of an activation tensor, 256 KiB apart - round-robin over the XCDs, and each XCD then reads addresses
// that all share bits 18-20 and, because its workgroups sweep their rows in step, nearly the same column
// bits: too little variety for the channel hashes, and a streaming kernel runs at 3.9 TB/s.  Giving every
// XCD a contiguous range of the items instead (6.2 TB/s for the same reads) is what this returns.
__device__ __forceinline__ int32_t xcd_contiguous(int32_t wg, int32_t n)
{
    const int32_t xcd = wg & 7, idx = wg >> 3;
    const int32_t per = n >> 3, rem = n & 7;
    return xcd * per + (xcd < rem ? xcd : rem) + idx;
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b)
{
    return __uint_as_float(uint32_t(b) << 16);
}

// Round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return uint16_t(u >> 16);
}

template <typename E> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p, size_t i) { return p[i]; }
    static __device__ __forceinline__ void store(float* p, size_t i, float v) { p[i] = v; }
};
template <> struct Elem<uint16_t> {
    static __device__ __forceinline__ float load(const uint16_t* p, size_t i) { return bf16_bits_to_float(p[i]); }
    static __device__ __forceinline__ void store(uint16_t* p, size_t i, float v) { p[i] = float_to_bf16_bits(v); }
};

}  // namespace lobra
