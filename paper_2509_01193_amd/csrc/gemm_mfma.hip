// bf16 MFMA GEMM for gfx950 with the LoRA up projection fused into its epilogue:
//     C[T, N] = Z[T, K] * op(W) + P[T, r] * M_t[r, N]
// forward : Z = x,  op(W) = W   (W stored [K][N], N fastest),  P = s_t A_t x_i,  M = B  -> y
// backward: Z = dy, op(W) = W^T (W stored [N][K], K fastest),  P = s_t B_t dy_i, M = A  -> dx
// (paper section 2.1: X W + X (down)(up); section 1: one shared base product for the fused batch,
// a per-task adapter product on top of it).
//
// Tiling: 256 x 256 x 64 per workgroup of WM x WN waves (default 4 x 2 = 512 threads, two waves per
// SIMD), every wave owns (256/WM) x (256/WN) as blocks of v_mfma_f32_32x32x16_bf16 with fp32
// accumulators.  The MFMA "A" operand is fed from W and the "B" operand from Z, so a lane ends up
// with four consecutive output columns of one row, which packs into 8-byte LDS writes in the epilogue.
//
// Two loaders behind one kernel template:
//   DMA  (K a multiple of 64): K tiles go global -> LDS with global_load_lds_dwordx4, no registers
//        and no ds_write in between; two LDS stages; the copies of tile kt+1 are issued in the middle
//        of tile kt, after the barrier that freed their stage; every row segment is one 128-byte line.
//   register-staged (any K that is a multiple of 8): global -> VGPR -> LDS with a zero-filled K tail.
//
// LDS layouts (DMA path; the register-staged path pads the forward W tile instead of swizzling it)
//   Z tile, and the W tile when K is fastest (backward): [256 rows][64 k], 16-byte chunk c of a row
//       stored at c ^ ((row >> 1) & 7): the 16 rows of one ds_read_b128 pass hit 16 bank groups.
//   W tile when N is fastest (forward): [64 k][256 n], chunk c of k-row k stored at c ^ ((k & 3) << 2);
//       the MFMA operand (8 consecutive k of one column) is gathered with two ds_read_b64_tr_b16 and
//       the 4 k-rows of one such read sit in different bank quarters.
//   A wave-wide direct-to-LDS copy lands in lane order, so the swizzle is applied to the global
//       address each lane fetches from.
//   C staging in the epilogue: per wave [rows][cols + 8] bf16, written back with non-temporal stores.
//
// Tuning macros (defaults are what the measurements chose): LOBRA_GEMM_WM/WN wave grid, LOBRA_GEMM_DBK/
// DST K-tile width and stage count of the DMA path, LOBRA_GEMM_ISSUE_AT, LOBRA_GEMM_GM tile-rows per
// sweep of the XCD-aware tile order, LOBRA_GEMM_NT_STORE, LOBRA_GEMM_DMA.
#include <atomic>

#include "kernels.h"

#ifndef LOBRA_GEMM_DMA
#define LOBRA_GEMM_DMA 1
#endif
#ifndef LOBRA_GEMM_DBK
#define LOBRA_GEMM_DBK 64
#endif
#ifndef LOBRA_GEMM_DST
#define LOBRA_GEMM_DST 2
#endif
#ifndef LOBRA_GEMM_ISSUE_AT
#define LOBRA_GEMM_ISSUE_AT 0      // 1 or 2: K step of a tile after which the next tile's copies go out; 0: from K
#endif
#ifndef LOBRA_GEMM_GM
#define LOBRA_GEMM_GM 0      // 0: chosen from K by the launcher
#endif
#ifndef LOBRA_GEMM_NT_STORE
#define LOBRA_GEMM_NT_STORE 1
#endif
#ifndef LOBRA_GEMM_WM
#define LOBRA_GEMM_WM 4
#endif
#ifndef LOBRA_GEMM_WN
#define LOBRA_GEMM_WN 2
#endif

namespace lobra {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int ZT_BYTES = BM * BK * 2;               // 32 KiB
constexpr int WKN_PITCH = BN + 32;                  // elements
constexpr int WT_KN_BYTES = BK * WKN_PITCH * 2;     // 36 KiB
constexpr int WT_NK_BYTES = BN * BK * 2;            // 32 KiB

// direct-to-LDS variant: K tile of DBK, DST stages of (Z tile + W tile)
constexpr int DBK = LOBRA_GEMM_DBK, DST = LOBRA_GEMM_DST;
constexpr int DZT_BYTES = BM * DBK * 2, DSTAGE_BYTES = 2 * DZT_BYTES;
static_assert((DBK == 32 || DBK == 64) && DST >= 2 && DST <= 4 && DST * DSTAGE_BYTES <= 160 * 1024, "LDS budget");

template <bool W_KN, int WN, bool DMA> constexpr int lds_bytes()
{
    const int loop = DMA ? DST * DSTAGE_BYTES : 2 * ZT_BYTES + 2 * (W_KN ? WT_KN_BYTES : WT_NK_BYTES);
    const int cs = BM * (BN + 8 * WN) * 2;          // all waves' C staging
    return loop > cs ? loop : cs;
}

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v)
{
    union { u32x4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

__device__ __forceinline__ u32x4 ldg16(const unsigned char* base, uint32_t off)
{
    return *reinterpret_cast<const u32x4*>(base + off);
}

// One wave-wide global -> LDS copy of 64 x 16 bytes without passing through registers
// (global_load_lds_dwordx4): lane i fetches 16 bytes at gbase + voff and they land at LDS byte
// address lds_addr + 16 i.  lds_addr and gbase are wave-uniform.  The instruction counts on vmcnt;
// the compiler does not see it, so the caller places the matching s_waitcnt vmcnt itself.
__device__ __forceinline__ void dma16(uint32_t lds_addr, const unsigned char* gbase, uint32_t voff)
{
    const uint32_t la = __builtin_amdgcn_readfirstlane(lds_addr);
    const uint64_t gp = reinterpret_cast<uint64_t>(gbase);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(gp));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(uint32_t(gp >> 32));
    const uint64_t gu = (uint64_t(hi) << 32) | lo;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(la), "v"(voff), "s"(gu)
                 : "memory");     // m0 is a reserved register: the compiler re-loads it before each of its own uses
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

}  // namespace

template <bool W_KN, int WM, int WN, bool DMA, int IA>
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
    constexpr int MB = TM / 32, NB = TN / 32;       // 32 x 32 blocks per wave
    constexpr int ZL = 2048 / NT;                   // 16-byte chunks per thread and tile
    constexpr int ZROWS = NT / 8;                   // rows covered by one pass of the [rows][64 k] loader
    constexpr int WKROWS = NT / 32;                 // k rows covered by one pass of the [64 k][256 n] loader
    constexpr int WT_BYTES = W_KN ? WT_KN_BYTES : WT_NK_BYTES;
    constexpr int CS_PITCH = TN + 8;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, lh = lane >> 5;
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

    f32x16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    if constexpr (DMA) {
        // ---- direct-to-LDS pipeline: K tiles of DBK, DST LDS stages, loads issued DST-1 tiles ahead
        // Stage layout: Z [256 rows][DBK k] (DBK*2 bytes per row, 16-byte chunk c stored at c ^ f(row)),
        // then W either [256 n][DBK k] in the same layout (backward) or [DBK k][256 n] (forward, 512
        // bytes per k row, 16-byte chunk c stored at c ^ ((k & 3) << 2) so that the 4 k rows of one
        // transpose read sit in different bank quarters).  f spreads the 16 rows of one ds_read_b128
        // pass over all banks: (row >> 2) & 3 for 64-byte rows, (row >> 1) & 7 for 128-byte rows.
        // A wave-wide copy fills 1 KiB of LDS in lane order, so the swizzle is applied to the global
        // address each lane fetches from.
        constexpr int NW = WM * WN;
        constexpr int CPRW = DBK / 8;               // 16-byte chunks per row of the [rows][DBK] layout
        constexpr int RPB = 64 / CPRW;              // rows per 1 KiB block
        constexpr int NBZ = (DBK / 2) / NW;         // 1 KiB blocks per wave, for Z and for W each
        const uint32_t lds0 = uint32_t(uintptr_t((__attribute__((address_space(3))) unsigned char*)lds));
        auto fz = [](int row) { return DBK == 32 ? (row >> 2) & 3 : (row >> 1) & 7; };
        uint32_t zvo[NBZ], wvo[NBZ];
#pragma unroll
        for (int j = 0; j < NBZ; ++j) {
            const int blk = wave + NW * j;
            {
                const int row = RPB * blk + lane / CPRW;
                const int c = (lane % CPRW) ^ fz(row);
                zvo[j] = (uint32_t(min(row, T - 1 - row0)) * uint32_t(K) + 8u * c) * 2u;
                if (!W_KN) wvo[j] = (uint32_t(min(row, N - 1 - col0)) * uint32_t(ldw) + 8u * c) * 2u;
            }
            if (W_KN) {
                const int krow = 2 * blk + (lane >> 5);
                const int c = (lane & 31) ^ ((krow & 3) << 2);
                wvo[j] = (uint32_t(krow) * uint32_t(ldw) + uint32_t(min(8 * c, N - 8 - col0))) * 2u;
            }
        }
        const unsigned char* zbase = reinterpret_cast<const unsigned char*>(Z + size_t(row0) * K);
        const unsigned char* wbase = reinterpret_cast<const unsigned char*>(W_KN ? W + col0 : W + size_t(col0) * ldw);
        auto issue = [&](int32_t kt) {              // all of this wave's copies for K tile kt
            const uint32_t st = lds0 + uint32_t(kt % DST) * DSTAGE_BYTES;
            const unsigned char* zb = zbase + size_t(kt) * (DBK * 2);
            const unsigned char* wb = W_KN ? wbase + size_t(kt) * DBK * ldw * 2 : wbase + size_t(kt) * (DBK * 2);
#pragma unroll
            for (int j = 0; j < NBZ; ++j) dma16(st + (wave + NW * j) * 1024, zb, zvo[j]);
#pragma unroll
            for (int j = 0; j < NBZ; ++j) dma16(st + DZT_BYTES + (wave + NW * j) * 1024, wb, wvo[j]);
        };
        // operand fragments of K step ks of a stage
        auto load_frags = [&](int stage, int ks, bf16x8 (&zf)[MB], bf16x8 (&wf)[NB]) {
            const unsigned char* zs = lds + stage * DSTAGE_BYTES;
            const unsigned char* ws = zs + DZT_BYTES;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int row = wm * TM + mb * 32 + l32;
                zf[mb] = *reinterpret_cast<const bf16x8*>(zs + row * (DBK * 2) + ((2 * ks + lh) ^ fz(row)) * 16);
            }
            if (W_KN) {
                const int s = lane & 15, g = lane >> 4;
                const int krow = 16 * ks + 8 * (g >> 1) + (s >> 2);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int n = wn * TN + nb * 32 + 16 * (g & 1) + 4 * (s & 3);
                    const int c = (n >> 3) ^ ((krow & 3) << 2);
                    const unsigned char* p0 = ws + krow * 512 + c * 16 + (n & 7) * 2;
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (s16x4 __attribute__((address_space(3)))*)(p0));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (s16x4 __attribute__((address_space(3)))*)(p0 + 4 * 512));
                    union { s16x4 h[2]; bf16x8 b; } cv;
                    cv.h[0] = lo;
                    cv.h[1] = hi;
                    wf[nb] = cv.b;
                }
            } else {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int row = wn * TN + nb * 32 + l32;
                    wf[nb] = *reinterpret_cast<const bf16x8*>(ws + row * (DBK * 2) + ((2 * ks + lh) ^ fz(row)) * 16);
                }
            }
        };
        auto mma = [&](const bf16x8 (&zf)[MB], const bf16x8 (&wf)[NB]) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[nb], zf[mb], acc[mb][nb], 0, 0, 0);
        };
        // K steps ks0 .. ks1-1 of a stage (the compiler interleaves the LDS reads of a step with the MFMAs of the one before)
        auto compute = [&](int stage, int ks0, int ks1) {
#pragma unroll
            for (int ks = ks0; ks < ks1; ++ks) {
                bf16x8 zf[MB], wf[NB];
                load_frags(stage, ks, zf, wf);
                mma(zf, wf);
            }
        };
        constexpr int NPW = 2 * NBZ;                // copies per wave and K tile
        const int32_t KT = K / DBK;                 // the launcher guarantees K % DBK == 0
        for (int32_t s0 = 0; s0 < DST - 1; ++s0)
            if (s0 < KT) issue(s0);
        for (int32_t kt = 0; kt < KT; ++kt) {
            // this wave's copies of tile kt have landed once at most the copies of the (up to DST-2)
            // tiles issued after it are still outstanding; the barrier then covers the other waves'
            // copies and tells that everybody is done reading the stage that is refilled next
            if (DST >= 4 && kt + 2 < KT) wait_vmcnt<(DST >= 4 ? 2 : 0) * NPW>();
            else if (DST >= 3 && kt + 1 < KT) wait_vmcnt<(DST >= 3 ? 1 : 0) * NPW>();
            else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            // the copies of the tile that reuses the freed stage go out after one or two of this tile's
            // four K steps (right after the barrier they would compete with the tile's first LDS reads);
            // which of the two is faster depends on K, so the launcher chooses the instantiation
            compute(kt % DST, 0, IA);
            if (kt + DST - 1 < KT) issue(kt + DST - 1);
            compute(kt % DST, IA, DBK / 16);
        }
        wait_vmcnt<0>();
        __syncthreads();
    } else {
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
        // one K tile: 4 K steps of 16, each MB + NB operand fragments and MB * NB MFMAs
        auto compute = [&](int buf) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                bf16x8 zf[MB], wf[NB];
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const int row = wm * TM + mb * 32 + l32;
                    zf[mb] = *reinterpret_cast<const bf16x8*>(zs(buf) + row * (BK * 2) + swz(row, 2 * ks + lh) * 16);
                }
                if (W_KN) {
                    const int s = lane & 15, g = lane >> 4;
                    const int krow = 16 * ks + 8 * (g >> 1) + (s >> 2);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const int n = wn * TN + nb * 32 + 16 * (g & 1) + 4 * (s & 3);
                        const unsigned char* p0 = ws(buf) + krow * (WKN_PITCH * 2) + n * 2;
                        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (s16x4 __attribute__((address_space(3)))*)(p0));
                        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (s16x4 __attribute__((address_space(3)))*)(p0 + 4 * (WKN_PITCH * 2)));
                        union { s16x4 h[2]; bf16x8 b; } c;
                        c.h[0] = lo;
                        c.h[1] = hi;
                        wf[nb] = c.b;
                    }
                } else {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const int row = wn * TN + nb * 32 + l32;
                        wf[nb] = *reinterpret_cast<const bf16x8*>(ws(buf) + row * (BK * 2) + swz(row, 2 * ks + lh) * 16);
                    }
                }
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[nb], zf[mb], acc[mb][nb], 0, 0, 0);
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
    }

    // ---- fused up projection: for every adapter segment that crosses this tile, ceil(r_t / 16) extra
    //      K steps acc += M_t^T[:, cols] * P[rows, :]^T with the rows outside the segment masked to zero.
    //      The M_t slice [r_t][256 cols] is staged in LDS (free now) in the [k][n] layout of the forward W
    //      tile and gathered with the transpose read; P comes straight from global memory, 16 bytes per lane.
    //      The segment loop and its barriers are uniform over the workgroup.
    {
        constexpr int NT2 = 64 * WM * WN;
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
            const int32_t rp = (r + 15) & ~15;
            const bool mine = hi > wrow0 && lo < wrow0 + TM;   // wave-uniform: the segment crosses this wave's rows
            // P fragments of up to two rank steps are fetched before the adapter slice is staged, so
            // that their latency overlaps the staging and its barriers
            constexpr int KG = 2;
            u32x4 pv[KG][MB];
            auto load_p = [&](int32_t kk0) {
#pragma unroll
                for (int q = 0; q < KG; ++q)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        const int32_t row = wrow0 + mb * 32 + l32;
                        const int32_t kk = kk0 + 16 * q;
                        // (a lane's 8 ranks start at kk + 8 lh: groups that start beyond r_t hold padding,
                        //  or another projection's ranks, and are not read)
                        pv[q][mb] = (mine && kk + 8 * lh < r && row >= lo && row < hi)
                            ? *reinterpret_cast<const u32x4*>(P + size_t(row) * pd.r_pad + pj * r + kk + 8 * lh) : zero4;
                    }
            };
            load_p(0);
            // the adapter slice is rp * 32 chunks of 16 bytes; the first MCH * NT2 of them (ranks up to
            // 64 with 512 threads) are fetched before the barrier that frees the LDS and written after it
            constexpr int MCH = 4;
            u32x4 mreg[MCH];
            auto fetch_m = [&](int32_t base) {
#pragma unroll
                for (int q = 0; q < MCH; ++q) {
                    const int32_t ch = base + tid + q * NT2, kr = ch >> 5, n = col0 + 8 * (ch & 31);
                    mreg[q] = (ch < rp * 32 && kr < r && n < N)
                                  ? *reinterpret_cast<const u32x4*>(M + size_t(r0 + kr) * mpitch + (n - mcol0)) : zero4;
                }
            };
            auto store_m = [&](int32_t base) {
#pragma unroll
                for (int q = 0; q < MCH; ++q) {
                    const int32_t ch = base + tid + q * NT2, kr = ch >> 5, c = ch & 31;
                    if (ch < rp * 32) *reinterpret_cast<u32x4*>(lds + kr * 512 + ((c ^ ((kr & 3) << 2)) << 4)) = mreg[q];
                }
            };
            fetch_m(0);
            __syncthreads();                        // everybody is done with what the LDS held before
            store_m(0);
            for (int32_t base = MCH * NT2; base < rp * 32; base += MCH * NT2) {
                fetch_m(base);
                store_m(base);
            }
            __syncthreads();
            if (!mine) continue;                    // wave-uniform; the barriers are above
            const int s16 = lane & 15, g16 = lane >> 4;
            for (int32_t kk0 = 0; kk0 < rp; kk0 += 16 * KG) {
                if (kk0 > 0) load_p(kk0);
#pragma unroll
                for (int q = 0; q < KG; ++q) {
                    const int32_t kk = kk0 + 16 * q;
                    if (kk >= rp) break;            // wave-uniform
                    bf16x8 wf[NB];
                    const int krow = kk + 8 * (g16 >> 1) + (s16 >> 2);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const int n = wn * TN + nb * 32 + 16 * (g16 & 1) + 4 * (s16 & 3);
                        const int c = (n >> 3) ^ ((krow & 3) << 2);
                        const unsigned char* p0 = lds + krow * 512 + c * 16 + (n & 7) * 2;
                        const s16x4 vlo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (s16x4 __attribute__((address_space(3)))*)(p0));
                        const s16x4 vhi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (s16x4 __attribute__((address_space(3)))*)(p0 + 4 * 512));
                        union { s16x4 h[2]; bf16x8 b; } cv;
                        cv.h[0] = vlo;
                        cv.h[1] = vhi;
                        wf[nb] = cv.b;
                    }
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        const int32_t rb = wrow0 + mb * 32;
                        if (hi <= rb || lo >= rb + 32) continue;        // wave-uniform
                        const bf16x8 pf = as_bf16x8(pv[q][mb]);
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[nb], pf, acc[mb][nb], 0, 0, 0);
                    }
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
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 o;
#pragma unroll
                    for (int q = 0; q < 4; ++q) o[q] = (__bf16)acc[mb][nb][4 * g + q];
                    const int m = mb * 32 + l32, n = nb * 32 + 8 * g + 4 * lh;
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

template <bool W_KN, int WM, int WN, bool DMA, int IA>
static hipError_t launch_gemm(const PlanDev& pd, const void* Z, const void* W, const void* P,
                              const void* M, void* C, int32_t K, int32_t N, int32_t ldw, int32_t ldc,
                              int32_t nproj, int32_t proj, int32_t tiles_m, int32_t tiles_n, int32_t gm,
                              hipStream_t st)
{
    constexpr int bytes = lds_bytes<W_KN, WN, DMA>();
    // the kernel needs more dynamic LDS than the default limit: raise it once per device
    static std::atomic<uint64_t> raised{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = uint64_t(1) << (dev & 63);
    if (!(raised.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_kernel<W_KN, WM, WN, DMA, IA>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e != hipSuccess) return e;
        raised.fetch_or(bit, std::memory_order_release);
    }
    gemm_mfma_kernel<W_KN, WM, WN, DMA, IA><<<dim3(uint32_t(tiles_m) * uint32_t(tiles_n)), 64 * WM * WN, bytes, st>>>(
        pd, (const uint16_t*)Z, (const uint16_t*)W, (const uint16_t*)P, (const uint16_t*)M, (uint16_t*)C,
        K, N, ldw, ldc, nproj, proj, tiles_m, tiles_n, gm);
    return hipGetLastError();
}

hipError_t gemm_mfma(const PlanDev& pd, bool transW, const void* Z, const void* W, const void* P,
                     const void* M, void* C, int32_t K, int32_t N, int32_t ldw, hipStream_t st,
                     int32_t ldc, int32_t nproj, int32_t proj)
{
    if (pd.T == 0) return hipSuccess;
    if (ldc == 0) ldc = N;
    const int32_t tiles_m = (pd.T + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    if (int64_t(tiles_m) * tiles_n > 0x7fffffff) return hipErrorInvalidValue;
    // 32-bit byte offsets inside a tile: 256 rows of K (or ldw) elements, 64 rows of ldw elements
    if (int64_t(K) * 512 >= (int64_t(1) << 32) || int64_t(ldw) * 512 >= (int64_t(1) << 32))
        return hipErrorInvalidValue;
    if (N < 8 || K < 8) return hipErrorInvalidValue;
    // tile rows per sweep of the tile order: the workgroups that run on an XCD at one time share their
    // Z and W panels through its L2 only while they walk K nearly in step, and the row bands that the 8
    // XCDs sweep at one time (8 x rows x 256 x K x 2 bytes) should stay in the 256 MB infinity cache for
    // their re-reads; measured on the five workloads, long K wants shorter sweeps (K = 8192 .. 28672:
    // 4 rows up to 7 % faster than 8; K = 4096: 5 .. 8 alike)
    const int32_t gm = LOBRA_GEMM_GM > 0 ? LOBRA_GEMM_GM : (K > 4096 ? 4 : 6);
    // K step of a tile after which the next tile's copies are issued: long K gains 2-5 % from the earlier one
    const int32_t issue_at = LOBRA_GEMM_ISSUE_AT > 0 ? LOBRA_GEMM_ISSUE_AT : (K > 4096 ? 1 : 2);
    // the direct-to-LDS pipeline needs whole K tiles of 32; other K take the register-staged kernel
    const bool dma = LOBRA_GEMM_DMA && K % DBK == 0;
#define LOBRA_GEMM_GO(KN, DM, IA_) \
    return launch_gemm<KN, LOBRA_GEMM_WM, LOBRA_GEMM_WN, DM, IA_>(pd, Z, W, P, M, C, K, N, ldw, ldc, nproj, proj, tiles_m, tiles_n, gm, st)
    if (!transW) {
        if (!dma) LOBRA_GEMM_GO(true, false, 2);
        if (issue_at == 1) LOBRA_GEMM_GO(true, true, 1);
        LOBRA_GEMM_GO(true, true, 2);
    }
    if (!dma) LOBRA_GEMM_GO(false, false, 2);
    if (issue_at == 1) LOBRA_GEMM_GO(false, true, 1);
    LOBRA_GEMM_GO(false, true, 2);
#undef LOBRA_GEMM_GO
}

}  // namespace lobra
