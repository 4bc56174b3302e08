// bf16 MFMA GEMMs for gfx950 with the LoRA up projection fused into their epilogue:
//     C[T, N] = Z[T, K] * op(W) + P[T, r] * M_t[r, N]
// forward : Z = x,  op(W) = W   (W stored [K][N], N fastest),  P = s_t A_t x_i,  M = B  -> y
// backward: Z = dy, op(W) = W^T (W stored [N][K], K fastest),  P = s_t B_t dy_i, M = A  -> dx
// (paper section 2.1: X W + X (down)(up); section 1: one shared base product for the fused batch,
// a per-task adapter product on top of it).
//
// This file: the launcher that picks the kernel, and the register-staged kernel for K that is not a
// multiple of 128 (any multiple of 8) and for batches or layers smaller than one tile: one workgroup per
// 256 x 256 tile, eight waves of 64 x 128, global -> VGPR -> LDS with a zero-filled K tail, two LDS stages,
// the compiler schedules it.  K that is a multiple of 128 (every layer of the paper's model shapes) takes
// the persistent direct-to-LDS kernel of gemm_persistent.hip.
//
// Tiling: 256 x 256 x 64 per workgroup, blocks of v_mfma_f32_16x16x32_bf16 with fp32 accumulators.  The MFMA
// "A" operand is fed from W and the "B" operand from Z, so a lane ends up with four consecutive output columns
// of one row, which packs into 8-byte LDS writes in the epilogue.
//
// LDS layouts
//   Z tile, and the W tile when K is fastest (backward): [256 rows][64 k], 16-byte chunk c of a row
//       stored at c ^ ((row >> 1) & 7): the 16 rows of one ds_read_b128 pass hit 16 bank groups.
//   W tile when N is fastest (forward): [64 k][256 n + 32]; the MFMA operand (8 consecutive k of one column)
//       is gathered with two ds_read_b64_tr_b16.
//   adapter slice in the epilogue: [k][256 n], chunk c of k-row k stored at c ^ kn_swz(k).
//   C staging in the epilogue: per wave [rows][cols + 8] bf16, written back with non-temporal stores.
//
// Tuning macros (defaults are what the measurements chose): LOBRA_GEMM_GM tile-rows per sweep of the
// XCD-aware tile order, LOBRA_GEMM_NT_STORE.
#include <atomic>

#include "gemm_common.h"
#include "kernels.h"

#ifndef LOBRA_GEMM_GM
#define LOBRA_GEMM_GM 0      // 0: chosen from K by the launcher
#endif
#ifndef LOBRA_GEMM_NT_STORE
#define LOBRA_GEMM_NT_STORE 1
#endif

namespace lobra {

using namespace gemm;

namespace {

constexpr int ZT_BYTES = BM * BK * 2;               // 32 KiB
constexpr int WKN_PITCH = BN + 32;                  // elements
constexpr int WT_KN_BYTES = BK * WKN_PITCH * 2;     // 36 KiB
constexpr int WT_NK_BYTES = BN * BK * 2;            // 32 KiB

template <bool W_KN, int WN> constexpr int lds_bytes()
{
    const int loop = 2 * ZT_BYTES + 2 * (W_KN ? WT_KN_BYTES : WT_NK_BYTES);
    const int cs = BM * (BN + 8 * WN) * 2;          // all waves' C staging
    return loop > cs ? loop : cs;
}

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ swz_row(row); }

__device__ __forceinline__ u32x4 ldg16(const unsigned char* base, uint32_t off)
{
    return *reinterpret_cast<const u32x4*>(base + off);
}

}  // namespace

template <bool W_KN, int WM, int WN>
__global__ __launch_bounds__(64 * WM * WN)
void gemm_mfma_kernel(PlanDev pd, const uint16_t* __restrict__ Z, const uint16_t* __restrict__ W,
                      const uint16_t* __restrict__ P, const uint16_t* __restrict__ M,
                      uint16_t* __restrict__ C, int32_t K, int32_t N, int32_t ldw, int32_t ldc,
                      int32_t nproj, int32_t proj, int32_t tiles_m, int32_t tiles_n, int32_t GM)
{
    // ldc: row pitch of C.  nproj > 1: this launch is projection `proj` of a fused shared-input
    // call: of every task's rank rows (in M) and rank columns (in P) only the window
    // [proj r, (proj + 1) r) takes part, r = the task's stacked rank / nproj.  proj < 0: the launch
    // covers all projections (N = nproj * pd.dg, pd.dg a multiple of the tile width) and a tile takes
    // the projection its columns lie in; M is then the compact [R_tot][pd.dg] array.
    constexpr int NT = 64 * WM * WN;                // threads
    constexpr int TM = BM / WM, TN = BN / WN;       // wave tile
    constexpr int MB = TM / 16, NB = TN / 16;       // 16 x 16 blocks per wave
    constexpr int ZL = 2048 / NT;                   // 16-byte chunks per thread and tile
    constexpr int ZROWS = NT / 8;                   // rows covered by one pass of the [rows][64 k] loader
    constexpr int WKROWS = NT / 32;                 // k rows covered by one pass of the [64 k][256 n] loader
    constexpr int WT_BYTES = W_KN ? WT_KN_BYTES : WT_NK_BYTES;
    constexpr int CS_PITCH = TN + 8;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    // MFMA 16x16x32 lanes: j = row of the "B" operand (a token) and of the result, kg = group of 8 k
    // (operands) or of 4 result columns
    const int j = lane & 15, kg = lane >> 4;
    const int32_t T = pd.T;

    // ---- workgroup -> tile: consecutive ids go to different XCDs, so give each XCD a contiguous
    //      range of the tile order; inside it, GM tile-rows share one sweep over the tile-columns.
    int32_t tile_m, tile_n;
    {
        const int32_t ntiles = tiles_m * tiles_n;
        const int32_t wg = blockIdx.x;
        const int32_t xcd = wg & 7, idx = wg >> 3;
        const int32_t per = ntiles >> 3, rem = ntiles & 7;
        const int32_t id = xcd * per + (xcd < rem ? xcd : rem) + idx;   // XCD x holds per + (x < rem)
        const int32_t group = id / (GM * tiles_n);
        const int32_t first_m = group * GM;
        const int32_t gsz = min(tiles_m - first_m, GM);
        const int32_t in = id - group * GM * tiles_n;
        tile_m = first_m + in % gsz;
        tile_n = in / gsz;
    }
    const int32_t row0 = tile_m * BM, col0 = tile_n * BN;

    // The table entries of the first segment that crosses this tile are read now: after the main loop
    // (whose copies are opaque to the compiler) the chain of dependent loads would sit in front of the
    // epilogue.  Most tiles lie inside one segment.
    const int32_t sg_first = pd.rowblk_seg[row0 / kRowBlock];
    const int32_t sf_lo = pd.cseg_off[sg_first], sf_hi = pd.cseg_off[sg_first + 1];
    const int32_t sf_task = pd.cseg_task[sg_first];
    const int32_t pj = proj >= 0 ? proj : col0 / pd.dg;          // this tile's projection
    const int32_t mcol0 = proj >= 0 ? 0 : pj * pd.dg;            // first column of that projection
    const int32_t mpitch = proj >= 0 ? N : pd.dg;                // row pitch of M
    const int32_t sf_rw = sf_task >= 0 ? (pd.rank_off[sf_task + 1] - pd.rank_off[sf_task]) / nproj : 0;
    const int32_t sf_r0 = sf_task >= 0 ? pd.rank_off[sf_task] + pj * sf_rw : 0;
    const int32_t sf_r1 = sf_r0 + sf_rw;

    auto zs = [&](int buf) { return lds + buf * ZT_BYTES; };
    auto ws = [&](int buf) { return lds + 2 * ZT_BYTES + buf * WT_BYTES; };

    // acc[mb][nb][v]: token row mb 16 + j of the wave tile, column nb 16 + 4 kg + v
    f32x4 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int jj = 0; jj < NB; ++jj) acc[i][jj] = f32x4{0.f, 0.f, 0.f, 0.f};

    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    u32x4 zreg[ZL], wreg[ZL];

    // Per-thread byte offsets inside the tile's rows (loop invariant).  Rows of Z beyond T and columns
    // of W beyond N are clamped to the last valid one: they only feed output rows / columns that are
    // never stored.  The K tail (K % 64) is zero-filled by the guarded loader below.
    const int lc = tid & 7, lr = tid >> 3;          // [rows][64 k] loader: chunk, first row
    const int wnc = tid & 31, wkr = tid >> 5;       // [64 k][256 n] loader: n chunk, first k row
    uint32_t zoff[ZL], woff[ZL];
#pragma unroll
    for (int i = 0; i < ZL; ++i) {
        zoff[i] = (uint32_t(min(lr + ZROWS * i, T - 1 - row0)) * uint32_t(K) + 8u * lc) * 2u;
        if (W_KN)
            woff[i] = (uint32_t(wkr + WKROWS * i) * uint32_t(ldw) + uint32_t(min(8 * wnc, N - 8 - col0))) * 2u;
        else
            woff[i] = (uint32_t(min(lr + ZROWS * i, N - 1 - col0)) * uint32_t(ldw) + 8u * lc) * 2u;
    }
    const unsigned char* zbase = reinterpret_cast<const unsigned char*>(Z + size_t(row0) * K);
    const unsigned char* wbase = reinterpret_cast<const unsigned char*>(W_KN ? W + col0 : W + size_t(col0) * ldw);

    auto gload = [&](int32_t k0) {                  // full K tile, no guards
        const unsigned char* zb = zbase + size_t(k0) * 2;
        const unsigned char* wb = W_KN ? wbase + size_t(k0) * ldw * 2 : wbase + size_t(k0) * 2;
#pragma unroll
        for (int i = 0; i < ZL; ++i) zreg[i] = ldg16(zb, zoff[i]);
#pragma unroll
        for (int i = 0; i < ZL; ++i) wreg[i] = ldg16(wb, woff[i]);
    };
    auto gload_tail = [&](int32_t k0) {             // last, partial K tile: zero beyond K
        const unsigned char* zb = zbase + size_t(k0) * 2;
        const unsigned char* wb = W_KN ? wbase + size_t(k0) * ldw * 2 : wbase + size_t(k0) * 2;
#pragma unroll
        for (int i = 0; i < ZL; ++i) zreg[i] = (k0 + 8 * lc < K) ? ldg16(zb, zoff[i]) : zero4;
#pragma unroll
        for (int i = 0; i < ZL; ++i) {
            const bool in = W_KN ? (k0 + wkr + WKROWS * i < K) : (k0 + 8 * lc < K);
            wreg[i] = in ? ldg16(wb, woff[i]) : zero4;
        }
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < ZL; ++i) {
            const int row = lr + ZROWS * i;
            *reinterpret_cast<u32x4*>(zs(buf) + row * (BK * 2) + swz(row, lc) * 16) = zreg[i];
        }
#pragma unroll
        for (int i = 0; i < ZL; ++i) {
            if (W_KN) {
                *reinterpret_cast<u32x4*>(ws(buf) + (wkr + WKROWS * i) * (WKN_PITCH * 2) + wnc * 16) = wreg[i];
            } else {
                const int row = lr + ZROWS * i;
                *reinterpret_cast<u32x4*>(ws(buf) + row * (BK * 2) + swz(row, lc) * 16) = wreg[i];
            }
        }
    };
    // one K tile: 2 K steps of 32, each MB + NB operand fragments and MB * NB MFMAs
    auto compute = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 zf[MB], wf[NB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int row = wm * TM + mb * 16 + j;
                zf[mb] = *reinterpret_cast<const bf16x8*>(zs(buf) + row * (BK * 2) + swz(row, 4 * ks + kg) * 16);
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                if (W_KN) {
                    const int krow = 32 * ks + 8 * kg + (j >> 2);
                    const int n = wn * TN + nb * 16 + 4 * (j & 3);
                    wf[nb] = tr_pair(ws(buf) + krow * (WKN_PITCH * 2) + n * 2, WKN_PITCH * 2);
                } else {
                    const int row = wn * TN + nb * 16 + j;
                    wf[nb] = *reinterpret_cast<const bf16x8*>(ws(buf) + row * (BK * 2) + swz(row, 4 * ks + kg) * 16);
                }
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[nb], zf[mb], acc[mb][nb], 0, 0, 0);
        }
    };

    // ---- main loop ----------------------------------------------------------------------------
    const int32_t KT = (K + BK - 1) / BK;           // K tiles
    const int32_t KF = K / BK;                      // full K tiles
    if (KF > 0) gload(0); else gload_tail(0);
    lstore(0);
    __syncthreads();
    for (int32_t kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KF) gload((kt + 1) * BK);
        else if (kt + 1 < KT) gload_tail((kt + 1) * BK);
        compute(buf);
        if (kt + 1 < KT) lstore(buf ^ 1);
        __syncthreads();
    }

    // ---- fused up projection: for every adapter segment that crosses this tile, ceil(r_t / 32) extra
    //      K steps acc += M_t^T[:, cols] * P[rows, :]^T with the rows outside the segment masked to zero.
    //      The M_t slice [r_t][256 cols] is staged in LDS (free now) in the [k][n] layout of the forward W
    //      tile (rank rows up to the next multiple of 32 zero) and gathered with the transpose read; P comes
    //      straight from global memory, 16 bytes per lane.
    //      The segment loop and its barriers are uniform over the workgroup.
    {
        const int32_t row_end = min(row0 + BM, T);
        const int32_t wrow0 = row0 + wm * TM;       // the wave's rows are wrow0 .. wrow0 + TM - 1
        for (int32_t sg = sg_first; sg < pd.nseg; ++sg) {
            const bool cached = sg == sg_first;
            const int32_t seg_lo = cached ? sf_lo : pd.cseg_off[sg];
            if (seg_lo >= row_end) break;
            const int32_t t = cached ? sf_task : pd.cseg_task[sg];
            if (t < 0) continue;
            const int32_t seg_hi = cached ? sf_hi : pd.cseg_off[sg + 1];
            const int32_t lo = max(seg_lo, row0), hi = min(seg_hi, row_end);
            const int32_t r = cached ? sf_r1 - sf_r0 : (pd.rank_off[t + 1] - pd.rank_off[t]) / nproj;
            const int32_t r0 = cached ? sf_r0 : pd.rank_off[t] + pj * r;
            const int32_t rp = (r + 31) & ~31;
            const bool mine = hi > wrow0 && lo < wrow0 + TM;   // wave-uniform: the segment crosses this wave's rows
            // the P fragments of a rank step: lane (j, kg) holds the ranks kk + 8 kg .. + 7 of token row j of
            // each 16-row block; groups that start beyond r_t hold padding, or another projection's ranks,
            // and are not read.  The first step is fetched before the adapter slice is staged, so that its
            // latency overlaps the staging and its barriers
            u32x4 pv[MB];
            auto load_p = [&](int32_t kk) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const int32_t row = wrow0 + mb * 16 + j;
                    pv[mb] = (mine && kk + 8 * kg < r && row >= lo && row < hi)
                                 ? *reinterpret_cast<const u32x4*>(P + size_t(row) * pd.r_pad + pj * r + kk + 8 * kg) : zero4;
                }
            };
            load_p(0);
            // the adapter slice is rp * 32 chunks of 16 bytes; the first MCH * NT of them are fetched before
            // the barrier that frees the LDS and written after it
            constexpr int MCH = 4;
            u32x4 mreg[MCH];
            auto fetch_m = [&](int32_t base) {
#pragma unroll
                for (int q = 0; q < MCH; ++q) {
                    const int32_t ch = base + tid + q * NT, kr = ch >> 5, n = col0 + 8 * (ch & 31);
                    mreg[q] = (ch < rp * 32 && kr < r && n < N)
                                  ? *reinterpret_cast<const u32x4*>(M + size_t(r0 + kr) * mpitch + (n - mcol0)) : zero4;
                }
            };
            auto store_m = [&](int32_t base) {
#pragma unroll
                for (int q = 0; q < MCH; ++q) {
                    const int32_t ch = base + tid + q * NT, kr = ch >> 5, c = ch & 31;
                    if (ch < rp * 32) *reinterpret_cast<u32x4*>(lds + kr * 512 + ((c ^ kn_swz(kr)) << 4)) = mreg[q];
                }
            };
            fetch_m(0);
            __syncthreads();                        // everybody is done with what the LDS held before
            store_m(0);
            for (int32_t base = MCH * NT; base < rp * 32; base += MCH * NT) {
                fetch_m(base);
                store_m(base);
            }
            __syncthreads();
            if (!mine) continue;                    // wave-uniform; the barriers are above
            for (int32_t kk = 0; kk < rp; kk += 32) {
                if (kk > 0) load_p(kk);
                bf16x8 wf[NB];
                const int krow = kk + 8 * kg + (j >> 2);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int n = wn * TN + nb * 16 + 4 * (j & 3);
                    const int c = (n >> 3) ^ kn_swz(krow);
                    wf[nb] = tr_pair(lds + krow * 512 + c * 16 + (n & 7) * 2, 512);
                }
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const int32_t rb = wrow0 + mb * 16;
                    if (hi <= rb || lo >= rb + 16) continue;        // wave-uniform
                    const bf16x8 pf = as_bf16x8(pv[mb]);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[mb][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[nb], pf, acc[mb][nb], 0, 0, 0);
                }
            }
        }
        __syncthreads();                            // the C staging below reuses the same LDS
    }

    // ---- epilogue: fp32 -> bf16, stage the wave's block in LDS, store 16 bytes per lane
    {
        unsigned char* cs = lds + wave * (TM * CS_PITCH * 2);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                bf16x4 o;
#pragma unroll
                for (int q = 0; q < 4; ++q) o[q] = (__bf16)acc[mb][nb][q];
                const int m = mb * 16 + j, n = nb * 16 + 4 * kg;
                *reinterpret_cast<bf16x4*>(cs + (m * CS_PITCH + n) * 2) = o;
            }
        __syncthreads();
        constexpr int CPR = TN / 8;                  // 16-byte chunks per row of the wave tile
        constexpr int RPI = 64 / CPR;                // rows per store instruction
        const int cchunk = lane % CPR, rsub = lane / CPR;
        const int32_t col = col0 + wn * TN + cchunk * 8;
#pragma unroll 4
        for (int i = 0; i < TM / RPI; ++i) {
            const int m = i * RPI + rsub;
            const int32_t row = row0 + wm * TM + m;
            const u32x4 v = *reinterpret_cast<const u32x4*>(cs + (m * CS_PITCH + cchunk * 8) * 2);
            if (row < T && col < N) {
                if (LOBRA_GEMM_NT_STORE) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(C + size_t(row) * ldc + col));
                else *reinterpret_cast<u32x4*>(C + size_t(row) * ldc + col) = v;
            }
        }
    }
}

template <bool W_KN, int WM, int WN>
static hipError_t launch_gemm(const PlanDev& pd, const void* Z, const void* W, const void* P,
                              const void* M, void* C, int32_t K, int32_t N, int32_t ldw, int32_t ldc,
                              int32_t nproj, int32_t proj, int32_t tiles_m, int32_t tiles_n, int32_t gm,
                              hipStream_t st)
{
    constexpr int bytes = lds_bytes<W_KN, WN>();
    // the kernel needs more dynamic LDS than the default limit: raise it once per device
    static std::atomic<uint64_t> raised{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = uint64_t(1) << (dev & 63);
    if (!(raised.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_kernel<W_KN, WM, WN>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e != hipSuccess) return e;
        raised.fetch_or(bit, std::memory_order_release);
    }
    gemm_mfma_kernel<W_KN, WM, WN><<<dim3(uint32_t(tiles_m) * uint32_t(tiles_n)), 64 * WM * WN, bytes, st>>>(
        pd, (const uint16_t*)Z, (const uint16_t*)W, (const uint16_t*)P, (const uint16_t*)M, (uint16_t*)C,
        K, N, ldw, ldc, nproj, proj, tiles_m, tiles_n, gm);
    return hipGetLastError();
}

bool gemm_mfma_shape_ok(int64_t T, int32_t K, int32_t N, int32_t ldw)
{
    const int64_t tiles_m = (T + BM - 1) / BM, tiles_n = (int64_t(N) + BN - 1) / BN;
    if (tiles_m * tiles_n > 0x7fffffff) return false;
    // 32-bit byte offsets inside a tile: 256 rows of K (or ldw) elements, 64 rows of ldw elements
    if (int64_t(K) * 512 >= (int64_t(1) << 32) || int64_t(ldw) * 512 >= (int64_t(1) << 32)) return false;
    return N >= 8 && K >= 8;
}

hipError_t gemm_mfma(const PlanDev& pd, bool transW, const void* Z, const void* W, const void* P,
                     const void* M, void* C, int32_t K, int32_t N, int32_t ldw, hipStream_t st,
                     int32_t ldc, int32_t nproj, int32_t proj)
{
    if (pd.T == 0) return hipSuccess;
    if (ldc == 0) ldc = N;
    if (!gemm_mfma_shape_ok(pd.T, K, N, ldw)) return hipErrorInvalidValue;   // (plan creation has checked already)
    const int32_t tiles_m = (pd.T + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    // tile rows per sweep of the tile order: the workgroups that run on an XCD at one time share their
    // Z and W panels through its L2 only while they walk K nearly in step, and the row bands that the 8
    // XCDs sweep at one time (8 x rows x 256 x K x 2 bytes) should stay in the 256 MB infinity cache for
    // their re-reads; measured on the five workloads, long K wants shorter sweeps (K = 8192 .. 28672:
    // 4 rows up to 7 % faster than 8; K = 4096: 5 .. 8 alike)
    const int32_t gm = LOBRA_GEMM_GM > 0 ? LOBRA_GEMM_GM : (K > 4096 ? 4 : 6);
    // an even number of whole K tiles of 64 and at least one whole output tile: the persistent direct-to-LDS
    // kernel; other shapes: the register-staged kernel
    if (K % (2 * BK) == 0 && pd.T >= BM && N >= BN)
        return gemm_persistent(pd, transW, Z, W, P, M, C, K, N, ldw, ldc, nproj, proj, tiles_m, tiles_n, gm, st);
    if (!transW) return launch_gemm<true, 4, 2>(pd, Z, W, P, M, C, K, N, ldw, ldc, nproj, proj, tiles_m, tiles_n, gm, st);
    return launch_gemm<false, 4, 2>(pd, Z, W, P, M, C, K, N, ldw, ldc, nproj, proj, tiles_m, tiles_n, gm, st);
}

}  // namespace lobra
