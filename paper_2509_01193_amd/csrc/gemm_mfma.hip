// bf16 MFMA GEMM for gfx950 with the LoRA up projection fused into its epilogue:
//     C[T, N] = Z[T, K] * op(W) + P[T, r] * M_t[r, N]
// forward : Z = x,  op(W) = W   (W stored [K][N], N fastest),  P = s_t A_t x_i,  M = B  -> y
// backward: Z = dy, op(W) = W^T (W stored [N][K], K fastest),  P = s_t B_t dy_i, M = A  -> dx
// (paper section 2.1: X W + X (down)(up); section 1: one shared base product for the fused batch,
// a per-task adapter product on top of it).
//
// Tiling: 256 x 256 x 64 per workgroup, blocks of v_mfma_f32_16x16x32_bf16 with fp32 accumulators (on this
// chip a loop of nothing but these sustains 2.05 PFLOP/s, one of 32x32x16 blocks 1.79: the deeper K step
// moves each accumulator half as often per flop).  The MFMA "A" operand is fed from W and the "B" operand from
// Z, so a lane ends up with four consecutive output columns of one row, which packs into 8-byte LDS writes in
// the epilogue.
//
// Two main loops behind one kernel template:
//   DMA  (K a multiple of 64): four waves of 128 x 128 (one per SIMD, the 64 accumulators in the 256 AGPRs).
//        K tiles go global -> LDS with global_load_lds_dwordx4 (no registers, no ds_write) into two LDS
//        stages; every row segment a copy fetches is one 128-byte line.  With one wave per SIMD nothing
//        hides a wave's own latencies, so the loop is software-pipelined by hand and its order is pinned
//        (the MFMAs are volatile asm statements, sched_barrier between the slots): a K step of 32 is 16
//        sections of four MFMAs with one other piece of work behind each MFMA (an MFMA of this shape keeps
//        its pipe for 16 cycles, of which 12 are free for the wave to issue something else): the two
//        instructions of a copy, the address arithmetic, a fragment read.  The fragments of K step s + 1 are
//        read during step s (the token-side fragment of a row block straight back into its register once the
//        block is done, the other operand into a second register set); the barrier of a tile stands in front
//        of its last K step, whose fragments are already in registers, so MFMAs and not LDS latency follow
//        the barrier; the stage it frees is refilled by copies spread over the next one and a half K steps
//        (issued back to back they block their wave for as long as the texture unit takes to accept them).
//   register-staged (any K that is a multiple of 8): eight waves of 64 x 128, global -> VGPR -> LDS with
//        a zero-filled K tail; the compiler schedules it.
//
// LDS layouts (DMA path; the register-staged path pads the forward W tile instead of swizzling it)
//   Z tile, and the W tile when K is fastest (backward): [256 rows][64 k], 16-byte chunk c of a row
//       stored at c ^ ((row >> 1) & 7): the 16 rows of one ds_read_b128 pass hit 16 bank groups.
//   W tile when N is fastest (forward): [64 k][256 n], chunk c of k-row k stored at c ^ kn_swz(k);
//       the MFMA operand (8 consecutive k of one column) is gathered with two ds_read_b64_tr_b16 and
//       the k-rows that one such read touches sit in different bank groups.
//   A wave-wide direct-to-LDS copy lands in lane order, so the swizzle is applied to the global
//       address each lane fetches from.
//   C staging in the epilogue: per wave [rows][cols + 8] bf16, written back with non-temporal stores.
//
// Tuning macros (defaults are what the measurements chose): LOBRA_GEMM_GM tile-rows per sweep of the
// XCD-aware tile order, LOBRA_GEMM_NT_STORE, LOBRA_GEMM_DMA.
#include <atomic>

#include "kernels.h"

#ifndef LOBRA_GEMM_DMA
#define LOBRA_GEMM_DMA 1
#endif
#ifndef LOBRA_GEMM_GM
#define LOBRA_GEMM_GM 0      // 0: chosen from K by the launcher
#endif
#ifndef LOBRA_GEMM_NT_STORE
#define LOBRA_GEMM_NT_STORE 1
#endif

namespace lobra {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int ZT_BYTES = BM * BK * 2;               // 32 KiB
constexpr int WKN_PITCH = BN + 32;                  // elements
constexpr int WT_KN_BYTES = BK * WKN_PITCH * 2;     // 36 KiB
constexpr int WT_NK_BYTES = BN * BK * 2;            // 32 KiB

// direct-to-LDS loop: two stages of (Z tile + W tile)
constexpr int DBK = BK;
constexpr int DZT_BYTES = BM * DBK * 2, DSTAGE_BYTES = 2 * DZT_BYTES;
static_assert(2 * DSTAGE_BYTES <= 160 * 1024, "LDS budget");

template <bool W_KN, int WN, bool DMA> constexpr int lds_bytes()
{
    const int loop = DMA ? 2 * DSTAGE_BYTES : 2 * ZT_BYTES + 2 * (W_KN ? WT_KN_BYTES : WT_NK_BYTES);
    const int cs = BM * (BN + 8 * WN) * 2;          // all waves' C staging
    return loop > cs ? loop : cs;
}

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

// Swizzle of a [k][256 n] tile (512 bytes per k row): 16-byte chunk c of row k is stored at c ^ kn_swz(k).
// One transpose read of a 16-lane group takes 32 bytes from each of the k rows k0 .. k0 + 3, and the groups
// of a wave sit 8 rows apart: bits 0-1 of k pick the 64-byte quarter, bit 3 the 32-byte half of it.
__device__ __forceinline__ int kn_swz(int k) { return ((k & 3) << 2) | (((k >> 3) & 1) << 1); }

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

// acc += a * b with the accumulator pinned to the AGPRs and updated in place.  (With 64 accumulators of four
// registers the register allocator otherwise rotates them through VGPRs inside the main loop.)  The order of
// these statements is the order of the instructions.
__device__ __forceinline__ void mfma_acc(f32x4& acc, bf16x8 a, bf16x8 b)
{
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// The same copy in two instructions with room for another instruction between them (which also provides the
// wait state the M0 write needs): nothing that writes M0 may be scheduled between the two.
__device__ __forceinline__ void dma16_set_m0(uint32_t lds_addr)
{
    const uint32_t la = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %0" : : "s"(la) : "memory");
}
__device__ __forceinline__ void dma16_issue(const unsigned char* gbase, uint32_t voff)
{
    const uint64_t gp = reinterpret_cast<uint64_t>(gbase);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(gp));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(uint32_t(gp >> 32));
    const uint64_t gu = (uint64_t(hi) << 32) | lo;
    asm volatile("global_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(gu) : "memory");
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

}  // namespace

template <bool W_KN, int WM, int WN, bool DMA>
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

    // W operand (8 consecutive k of one column) out of a [k][n] tile with k rows `pitch` bytes apart:
    // two transpose reads of 4 k rows x 16 columns each.  `chunk_of(krow, c)` is the tile's swizzle.
    auto tr_pair = [&](const unsigned char* p0, int pitch) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 4 * pitch));
        union { s16x4 h[2]; bf16x8 b; } cv;
        cv.h[0] = lo;
        cv.h[1] = hi;
        return cv.b;
    };

    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    if constexpr (DMA) {
        // ---- direct-to-LDS pipeline, four waves of 128 x 128
        // Stage layout: Z [256 rows][64 k] (128 bytes per row, 16-byte chunk c stored at c ^ f(row)), then W
        // either [256 n][64 k] in the same layout (backward) or [64 k][256 n] (forward, 512 bytes per k row,
        // 16-byte chunk c stored at c ^ kn_swz(k) so that the k rows one transpose read touches sit in
        // different bank groups).  f(row) = (row >> 1) & 7 spreads the 16 rows of one ds_read_b128 pass
        // over all banks.  A wave-wide copy fills 1 KiB of LDS in lane order, so the swizzle is applied to
        // the global address each lane fetches from.
        constexpr int NW = WM * WN;
        constexpr int NBZ = (DBK / 2) / NW;         // 1 KiB blocks per wave, for Z and for W each
        constexpr int NU = MB + NB;                 // fragments per K step of 32 = sections per K step
        static_assert(NW == 4 && MB * NB == 4 * NU && 2 * NBZ == NU && DBK == 64,
                      "four waves of 128 x 128: four MFMAs and at most one copy per section");
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);
        const uint32_t lds0 = uint32_t(uintptr_t((__attribute__((address_space(3))) unsigned char*)lds));
        auto fz = [](int row) { return (row >> 1) & 7; };
        uint32_t zvo[NBZ], wvo[NBZ];                // per-lane source offsets of this wave's copies
#pragma unroll
        for (int c = 0; c < NBZ; ++c) {
            const int blk = wave + NW * c;
            {
                const int row = 8 * blk + lane / 8;
                const int ch = (lane % 8) ^ fz(row);
                zvo[c] = (uint32_t(min(row, T - 1 - row0)) * uint32_t(K) + 8u * ch) * 2u;
                if (!W_KN) wvo[c] = (uint32_t(min(row, N - 1 - col0)) * uint32_t(ldw) + 8u * ch) * 2u;
            }
            if (W_KN) {
                const int krow = 2 * blk + (lane >> 5);
                const int ch = (lane & 31) ^ kn_swz(krow);
                wvo[c] = (uint32_t(krow) * uint32_t(ldw) + uint32_t(min(8 * ch, N - 8 - col0))) * 2u;
            }
        }
        const unsigned char* zbase = reinterpret_cast<const unsigned char*>(Z + size_t(row0) * K);
        const unsigned char* wbase = reinterpret_cast<const unsigned char*>(W_KN ? W + col0 : W + size_t(col0) * ldw);
        const int32_t KT = K / DBK;                 // the launcher guarantees K % DBK == 0
        auto zsrc = [&](int32_t kt) { return zbase + size_t(kt) * (DBK * 2); };
        auto wsrc = [&](int32_t kt) { return W_KN ? wbase + size_t(kt) * DBK * ldw * 2 : wbase + size_t(kt) * (DBK * 2); };
        // copy c of a tile: c < NBZ is a Z block, the others are W blocks
        auto copy = [&](uint32_t stage_addr, const unsigned char* zb, const unsigned char* wb, int c) {
            if (c < NBZ) dma16(stage_addr + (wave_u + NW * c) * 1024, zb, zvo[c]);
            else dma16(stage_addr + DZT_BYTES + (wave_u + NW * (c - NBZ)) * 1024, wb, wvo[c - NBZ]);
        };
        // Operand fragments of K step ks (32 k) of a stage.  Block mb of a [rows][64 k] tile lies 16 rows =
        // 2048 bytes behind block 0 and (row >> 1) & 7 does not depend on mb, so one per-lane address per
        // step serves all blocks through the instruction's offset field.
        const int fzj = (j >> 1) & 7;
        auto zaddr = [&](int stage, int ks) {
            return lds + stage * DSTAGE_BYTES + (wm * TM + j) * (DBK * 2) + ((4 * ks + kg) ^ fzj) * 16;
        };
        auto waddr = [&](int stage, int ks) {       // backward layout only
            return lds + stage * DSTAGE_BYTES + DZT_BYTES + (wn * TN + j) * (DBK * 2) + ((4 * ks + kg) ^ fzj) * 16;
        };
        auto read_z = [&](const unsigned char* za, int mb, bf16x8 (&zf)[MB]) {
            zf[mb] = *reinterpret_cast<const bf16x8*>(za + mb * 16 * (DBK * 2));
        };
        auto read_w = [&](const unsigned char* wa, int stage, int ks, int nb, bf16x8 (&wf)[NB]) {
            if (W_KN) {
                const unsigned char* wst = lds + stage * DSTAGE_BYTES + DZT_BYTES;
                const int krow = 32 * ks + 8 * kg + (j >> 2);
                const int n = wn * TN + nb * 16 + 4 * (j & 3);
                const int ch = (n >> 3) ^ kn_swz(krow);
                wf[nb] = tr_pair(wst + krow * 512 + ch * 16 + (n & 7) * 2, 512);
            } else {
                wf[nb] = *reinterpret_cast<const bf16x8*>(wa + nb * 16 * (DBK * 2));
            }
        };
        // One K step of 32: the MB NB = 64 MFMAs in NU = 16 sections, each {2 MFMAs, copy, 2 MFMAs, fragment
        // read}: what is not an MFMA is issued while one runs.  Token-row block mb is done in sections 2 mb and
        // 2 mb + 1, after which its fragment zf[mb] is dead and is re-read at once for K step rks of stage
        // rstage (the step that follows); the other operand lives through the whole step, so its next
        // fragments go to a second register set (wn_), one in every even section.  Copies: the sections whose
        // bit is set in `mask` issue the next copy of the tile at (zb, wb) into the stage at cst, from copy c0 on.
        auto kstep = [&](int rstage, int rks, bf16x8 (&zf)[MB], bf16x8 (&wc)[NB], bf16x8 (&wn_)[NB],
                         int mask, int c0, uint32_t cst, const unsigned char* zb, const unsigned char* wb) {
            int c = c0;
            const unsigned char* za = zaddr(rstage, rks);
            const unsigned char* wa = waddr(rstage, rks);
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int mb = u / 2, nb0 = (NB / 2) * (u % 2);
                const bool cp = (mask >> u) & 1;
                // an MFMA of this shape keeps its pipe for 16 cycles, 12 of which are free to issue something
                // else: the copy goes out in two parts, each behind an MFMA
                mfma_acc(acc[mb][nb0], wc[nb0], zf[mb]);
                if (cp) dma16_set_m0(c < NBZ ? cst + (wave_u + NW * c) * 1024 : cst + DZT_BYTES + (wave_u + NW * (c - NBZ)) * 1024);
                __builtin_amdgcn_sched_barrier(0);
                mfma_acc(acc[mb][nb0 + 1], wc[nb0 + 1], zf[mb]);
                if (cp) {
                    if (c < NBZ) dma16_issue(zb, zvo[c]); else dma16_issue(wb, wvo[c - NBZ]);
                    ++c;
                }
                __builtin_amdgcn_sched_barrier(0);
                mfma_acc(acc[mb][nb0 + 2], wc[nb0 + 2], zf[mb]);
                __builtin_amdgcn_sched_barrier(0);
                mfma_acc(acc[mb][nb0 + 3], wc[nb0 + 3], zf[mb]);
                if (u % 2 == 0) read_w(wa, rstage, rks, u / 2, wn_);
                else read_z(za, mb, zf);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        static_assert(NB == 8 && MB == 8, "two sections of four MFMAs per token-row block");
        // the 2 NBZ = 16 copies of a tile go out in the K step behind the barrier that freed their stage, one
        // per section (measured against 14 + 2, 11 + 5, 10 + 6, 8 + 8 over this and the next step: the
        // earlier the better, by 1-4 %)
        constexpr int MD = 0xFFFF, MA = 0;
        constexpr int CD = __builtin_popcount(MD);
        static_assert(CD + __builtin_popcount(MA) == 2 * NBZ, "every copy once");

        bf16x8 zf[MB], wf[2][NB];
#pragma unroll
        for (int c = 0; c < 2 * NBZ; ++c) copy(lds0, zsrc(0), wsrc(0), c);
        if (KT > 1) {
#pragma unroll
            for (int c = 0; c < 2 * NBZ; ++c) copy(lds0 + DSTAGE_BYTES, zsrc(1), wsrc(1), c);
            wait_vmcnt<2 * NBZ>();
        } else {
            wait_vmcnt<0>();
        }
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int u = 0; u < MB; ++u) read_z(zaddr(0, 0), u, zf);
#pragma unroll
        for (int u = 0; u < NB; ++u) read_w(waddr(0, 0), 0, 0, u, wf[0]);
        for (int32_t kt = 0; kt < KT; ++kt) {
            const int stg = kt & 1;
            // Tile kt + 1 goes into the other stage (its first copies went out behind the previous barrier),
            // tile kt + 2 into this one once the barrier below has freed it.  Past the end a valid tile is
            // copied once more into a stage nobody reads any more, which keeps the loop free of branches.
            const int32_t k1 = min(kt + 1, KT - 1), k2 = min(kt + 2, KT - 1);
            const uint32_t st1 = lds0 + uint32_t(stg ^ 1) * DSTAGE_BYTES, st2 = lds0 + uint32_t(stg) * DSTAGE_BYTES;
            kstep(stg, 1, zf, wf[0], wf[1], MA, CD, st1, zsrc(k1), wsrc(k1));
            // every wave has read the last fragments of this stage and its copies of tile kt + 1 have landed
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            kstep(stg ^ 1, 0, zf, wf[1], wf[0], MD, 0, st2, zsrc(k2), wsrc(k2));
        }
        wait_vmcnt<0>();
        // the loop's MFMAs are asm statements, so the compiler does not know that the accumulators come out of
        // the matrix pipeline: keep its first read of them the documented number of wait states away
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
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

template <bool W_KN, int WM, int WN, bool DMA>
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
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_kernel<W_KN, WM, WN, DMA>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e != hipSuccess) return e;
        raised.fetch_or(bit, std::memory_order_release);
    }
    gemm_mfma_kernel<W_KN, WM, WN, DMA><<<dim3(uint32_t(tiles_m) * uint32_t(tiles_n)), 64 * WM * WN, bytes, st>>>(
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
    // the direct-to-LDS pipeline (four waves) needs whole K tiles of 64; other K take the register-staged
    // kernel (eight waves)
    const bool dma = LOBRA_GEMM_DMA && K % DBK == 0;
#define LOBRA_GEMM_GO(KN, WM_, WN_, DM) \
    return launch_gemm<KN, WM_, WN_, DM>(pd, Z, W, P, M, C, K, N, ldw, ldc, nproj, proj, tiles_m, tiles_n, gm, st)
    if (!transW) {
        if (dma) LOBRA_GEMM_GO(true, 2, 2, true);
        LOBRA_GEMM_GO(true, 4, 2, false);
    }
    if (dma) LOBRA_GEMM_GO(false, 2, 2, true);
    LOBRA_GEMM_GO(false, 4, 2, false);
#undef LOBRA_GEMM_GO
}

}  // namespace lobra
