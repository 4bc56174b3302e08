// Launchers of the HIP kernels.  Each returns the hipError_t of its launches; none synchronises.
#pragma once
#include <hip/hip_runtime.h>

#include "device_common.h"

namespace lobra {

// One gradient reduction dM = sum_i P_i^T Z_i: stage 1 writes `part`, stage 2 writes `out` [R_tot, D].
struct GradJob {
    const void* P;   // projected activations (layout depends on the kernel family)
    const void* Z;   // [T, D]
    float* part;     // [sum over chunks of r_t, D]
    float* out;      // [R_tot, D]
    int32_t D;
    int32_t ldz = 0;    // row pitch of Z in elements (0: D)
    int32_t nproj = 1;  // > 1 (fused projections): only the rank window `proj` of every task;
    int32_t proj = 0;   //   proj < 0: D spans all projections (nproj * dg columns, dg a multiple of 128)
                        //   and a column tile takes the projection its columns lie in
    int32_t ldp = 0;    // row pitch of part (0: D); dg when proj < 0
    // stage 2 only: part holds the sums of the fused projection-and-dB pass instead of chunk sums: the k-th run
    // of (task t, 512-column slice c) at rows frow0[t] + 16 k .. + 15, fcnt[t * fnsl + c] of them
    const int32_t* fcnt = nullptr;
    const int32_t* frow0 = nullptr;
    int32_t fnsl = 0;
};

// ---- plain fp32-FMA kernels (fp32 path; bf16 storage as a cross-check) ---------------------
// P[row, :r_t] = s_t * Z[row, :] M_t^T for every token of an adapter segment (fp32, stride r_max).
// (ldz: row pitch of Z, 0 = D.  nproj > 1: projection `proj` of a fused shared-input call - only the
//  rank window [proj r, (proj+1) r) of every task; the same three arguments below mean the same.)
hipError_t plain_shrink(const PlanDev& pd, int dtype, const void* Z, const void* M, const float* s,
                        float* P, int32_t D, hipStream_t st, int32_t ldz = 0, int32_t nproj = 1,
                        int32_t proj = 0);
// C[T, N] = Z[T, K] * op(W) + P[:, :r_t] * M_t ;  transW = false: op(W)[k][n] = W[k*ldw + n]
// (forward), true: op(W)[k][n] = W[n*ldw + k] (backward).
hipError_t plain_gemm(const PlanDev& pd, int dtype, bool transW, const void* Z, const void* W,
                      const float* P, const void* M, void* C, int32_t K, int32_t N, int32_t ldw,
                      hipStream_t st, int32_t ldc = 0, int32_t nproj = 1, int32_t proj = 0);
// Stage 1 of dM_t = sum over the tokens of task t of P[i, :]^T Z[i, :]: one partial sum per
// reduction chunk, written to part[chunk.part_row0 + rho, :].
// P is fp32 [T][r_max], or (p_bf16) bf16 [T][r_pad].
hipError_t plain_grad_stage1(const PlanDev& pd, int dtype, bool p_bf16, const void* P, const void* Z,
                             float* part, int32_t D, hipStream_t st, int32_t ldz = 0, int32_t nproj = 1,
                             int32_t proj = 0, const void* P2 = nullptr, const void* Z2 = nullptr,
                             float* part2 = nullptr, int32_t D2 = 0);
// Stage 2 (also used by the MFMA path): out[R, :] (+)= sum of the partial sums of task(R), in
// chunk order, so that the result does not depend on scheduling.
// One launch for up to two gradients (jb.out == nullptr: only ja).
hipError_t reduce_partials(const PlanDev& pd, const GradJob& ja, const GradJob& jb, bool accumulate,
                           hipStream_t st);
// ---- bf16 MFMA kernels ------------------------------------------------------------------------
// C[T, N] = Z[T, K] * op(W) + P * M_t with P bf16 [T][r_pad] (already scaled by s_t, zero beyond r_t).
// ldc: row pitch of C (0: N).  nproj > 1: projection `proj` of a fused shared-input call - of every
// task's ranks only the window [proj r, (proj+1) r) takes part (rows of M, columns of P); proj < 0: one
// launch over all projections (N = nproj * pd.dg, pd.dg a multiple of 256), M compact [R_tot][pd.dg].
hipError_t gemm_mfma(const PlanDev& pd, bool transW, const void* Z, const void* W, const void* P,
                     const void* M, void* C, int32_t K, int32_t N, int32_t ldw, hipStream_t st,
                     int32_t ldc = 0, int32_t nproj = 1, int32_t proj = 0);
// The persistent direct-to-LDS kernel behind gemm_mfma for K % 64 == 0 (gemm_persistent.hip); gm = tile rows
// per sweep of the tile order.  Shapes the two kernels' 32-bit tile offsets cannot address are rejected by
// gemm_mfma_shape_ok, which plan creation consults so that no call fails after its first launch.
hipError_t gemm_persistent(const PlanDev& pd, bool transW, const void* Z, const void* W, const void* P,
                           const void* M, void* C, int32_t K, int32_t N, int32_t ldw, int32_t ldc, int32_t nproj,
                           int32_t proj, int32_t tiles_m, int32_t tiles_n, int32_t gm, hipStream_t st);
bool gemm_mfma_shape_ok(int64_t T, int32_t K, int32_t N, int32_t ldw);
// P = s_t Z M_t^T in bf16, written token-major [T][r_pad] and block-transposed [ntb][r_pad][32].
// (ldz: row pitch of Z; nproj > 1: projection `proj` of a fused call - rank window, see the kernel)
// sliced.nsl > 0 (chosen by the plan, see sliced_shrink_shape) and part != nullptr: the K-sliced kernel with its
// fp32 partial projections in part [nsl][T][16], followed by the finish kernel.  Hblk, partb (and a plan with
// fused_db): the same pass also accumulates sum_i Hblk_i^T Z_i (dB when Z = dy and Hblk = the block-transposed
// s_t h) into partb [fb_rows][D], to be added up by reduce_partials (GradJob::fcnt).

hipError_t shrink_mfma(const PlanDev& pd, const void* Z, const void* M, const float* s,
                       void* P_tok, void* P_blk, int32_t D, int32_t ldz, int32_t nproj, int32_t proj,
                       hipStream_t st, const SlicedShape& sliced = SlicedShape{}, float* part = nullptr,
                       const void* Hblk = nullptr, float* partb = nullptr);

// Stage 1 of dM_t = sum_i P_i^T Z_i from the block-transposed P; partial sums per reduction chunk.
// (P = block-transposed bf16 copy; one launch for up to two gradients, jb.P == nullptr: only ja.)
hipError_t grad_mfma(const PlanDev& pd, const GradJob& ja, const GradJob& jb, hipStream_t st);

// Fused Adam over the stacked adapters A [R_tot, d_in] and B [R_tot, d_out] (one launch).
struct AdamTensor {
    const float* grad;
    float* master;
    float* m;
    float* v;
    void* param;     // plan dtype, may be nullptr
    int32_t D;
};
hipError_t adam_step(const PlanDev& pd, int dtype, float beta1, float beta2, float eps, float wd,
                     const float* lr, const int32_t* step, const float* grad_scale,
                     const AdamTensor& ta, const AdamTensor& tb, hipStream_t st);

hipError_t token_task_map(const PlanDev& pd, int32_t* out_task, int64_t* out_count, hipStream_t st);

}  // namespace lobra
