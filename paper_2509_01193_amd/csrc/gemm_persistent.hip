// Persistent bf16 MFMA GEMM for gfx950 with the LoRA up projection fused into its epilogue (K a multiple of 64):
//     C[T, N] = Z[T, K] * op(W) + P[T, r] * M_t[r, N]
// forward : Z = x,  op(W) = W   (W stored [K][N], N fastest),  P = s_t A_t x_i,  M = B  -> y
// backward: Z = dy, op(W) = W^T (W stored [N][K], K fastest),  P = s_t B_t dy_i, M = A  -> dx
// (paper section 2.1: X W + X (down)(up); section 1: one shared base product for the fused batch,
// a per-task adapter product on top of it).
//
// One workgroup per compute unit walks a few 256 x 256 output tiles (LOBRA_GP_TPW of them; then the next round of
// workgroups is dispatched, which re-aligns the compute units of an XCD that share panels through its L2):
//   * the K tiles of ALL of a workgroup's output tiles form one stream through the two LDS stages: while the
//     last K tiles of an output tile are multiplied, the first K tiles of the next one are already being
//     copied, so no stage fill is exposed except the very first;
//   * the epilogue keeps its hands off the two stages: the adapter slice of the fused up projection is staged
//     in a third LDS region (for the tile's first segment it and the tile's rows of P are copied there while the
//     last K tile is multiplied, see prefetch_adapter), and the result is rounded, passed through the same region
//     (a 64 x 64 block per wave at a time) and stored in whole 128-byte lines; the stores drain under the next
//     tile's first MFMAs.
// One workgroup per output tile instead costs about 15 us per tile (workgroup start, two exposed stage fills,
// the epilogue and its store drain) next to 80 us of MFMAs at K = 4096; of that the stream hides what is not the
// stores and the epilogue's own instructions.
//
// Tile: 256 x 256 x 64, four waves of 128 x 128 (one per SIMD), blocks of v_mfma_f32_16x16x32_bf16 with the
// 64 accumulators of a wave in its 256 AGPRs, which the kernel names itself (gemm_common.h).  The MFMA "A"
// operand is fed from W and the "B" operand from Z, so a lane ends up with four output columns of one token row
// per block; block_col deals the columns of a wave tile to the blocks so that two blocks give a lane 8
// consecutive columns.
// K tiles go global -> LDS with global_load_lds_dwordx4 (no registers, no ds_write); every row segment a copy
// fetches is one 128-byte line.  With one wave per SIMD nothing hides a wave's own latencies, so the loop is
// software-pipelined by hand and its order is pinned (the MFMAs are volatile asm statements, sched_barrier
// between the slots); see kstep for the schedule of a K step.
//
// LDS: stage 0, stage 1 (64 KiB each: Z tile then W tile), adapter slice / result staging (32 KiB).
//   Z tile, and the W tile when K is fastest (backward): [256 rows][64 k], 16-byte chunk c of a row
//       stored at c ^ ((row >> 1) & 7): the 16 rows of one ds_read_b128 pass hit 16 bank groups.
//   W tile when N is fastest (forward), adapter slice: [k][256 n], chunk c of k-row k stored at c ^ kn_swz2(k);
//       the MFMA operand (8 consecutive k of one column) is gathered with two ds_read_b64_tr_b16.
//   A wave-wide direct-to-LDS copy lands in lane order, so the swizzle - and, backward, the dealing of the
//       columns to the MFMA blocks - is applied to the global address each lane fetches from.
#include <atomic>
#include <type_traits>

#include "gemm_common.h"
#include "kernels.h"

#ifndef LOBRA_GP_TPW
#define LOBRA_GP_TPW 4       // output tiles per workgroup
#endif
#ifndef LOBRA_GP_STORES_IN_FLIGHT
#define LOBRA_GP_STORES_IN_FLIGHT 32   // stores of an epilogue (MB x NB / 2 per wave); 0: wait for them at the next barrier
#endif
#ifndef LOBRA_GP_STORE
#define LOBRA_GP_STORE 1     // 1: non-temporal stores of whole lines through LDS (the product); 4: 64-byte pieces straight from the
                             // accumulators; 0 / 2: timing variants (hardly any stores / plain stores)
#endif

namespace lobra {

using namespace gemm;

namespace {

constexpr int WM = 2, WN = 2, NW = WM * WN;          // waves
constexpr int TM = BM / WM, TN = BN / WN;            // wave tile 128 x 128
constexpr int MB = TM / 16, NB = TN / 16;            // 16 x 16 blocks per wave
constexpr int ZT_BYTES = BM * BK * 2;                // one operand tile: 32 KiB
constexpr int STAGE_BYTES = 2 * ZT_BYTES;            // Z tile + W tile
constexpr int MROWS = 64;                            // rank rows of the adapter slice staged at a time
constexpr int MSLICE_OFF = 2 * STAGE_BYTES, MSLICE_BYTES = MROWS * BN * 2;
constexpr int LDS_BYTES = MSLICE_OFF + MSLICE_BYTES; // 160 KiB
constexpr int PRE_RANKS = 32;                        // rank windows up to this are copied ahead of the epilogue
constexpr int PRE_P_OFF = PRE_RANKS * BN * 2;        // where the P rows land in the adapter region
constexpr int PRE_COPIES = 8;                        // 1 KiB copies per wave: half for the M_t slice, half for P
static_assert(PRE_P_OFF + BM * PRE_RANKS * 2 <= MSLICE_BYTES && PRE_COPIES / 2 * NW * 1024 == PRE_P_OFF,
              "the copied-ahead operands fill the adapter region");
constexpr int NBZ = (BK / 2) / NW;                   // 1 KiB copy blocks per wave, for Z and for W each
constexpr int NU = MB + NB;                          // fragments per K step of 32 = sections per K step
static_assert(NW == 4 && MB == 8 && NB == 8 && MB * NB == 4 * NU && 2 * NBZ == NU && BK == 64,
              "four waves of 128 x 128: four MFMAs and at most one copy per section");
static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
static_assert(BM == kGemmTileRows, "the plan's tile-row table is made for this tile height");

// Column of the wave tile that MFMA block nb produces in its result row i (= row i of its "A" operand).
// Lane (j, kg) of a block holds result rows 4 kg .. 4 kg + 3, so with this dealing the blocks 2 p and
// 2 p + 1 together give it the 8 consecutive columns 32 p + 8 kg .. + 7 of token row j: the low four from block
// 2 p and the high four from block 2 p + 1 when kg is even, the other way round when kg is odd (the alternation
// is what lets the forward kernel's transpose reads use both halves of every 16-byte chunk, see kn_swz2).
__device__ __forceinline__ int block_col(int nb, int i)
{
    return 32 * (nb >> 1) + 8 * (i >> 2) + 4 * ((nb ^ (i >> 2)) & 1) + (i & 3);
}

constexpr int acc_reg(int mb, int nb) { return 4 * (NB * mb + nb); }   // first AGPR of accumulator (mb, nb)

}  // namespace

template <bool W_KN>
__global__ __launch_bounds__(64 * NW)
void gemm_persistent_kernel(PlanDev pd, const uint16_t* __restrict__ Z, const uint16_t* __restrict__ W,
                            const uint16_t* __restrict__ P, const uint16_t* __restrict__ M,
                            uint16_t* __restrict__ C, int32_t K, int32_t N, int32_t ldw, int32_t ldc,
                            int32_t nproj, int32_t proj, int32_t tiles_m, int32_t tiles_n, int32_t GM, int32_t cpx,
                            int32_t TPW, const int32_t* __restrict__ tile_tab, const int32_t* __restrict__ cseg_off,
                            const int32_t* __restrict__ cseg_task, const int32_t* __restrict__ rank_off)
{
    // tile_tab, cseg_off, cseg_task, rank_off: pd's tables of those names once more, as arguments of their own that
    // promise not to alias anything the kernel writes: their entries are the same for every lane, and with the
    // promise the compiler fetches them with scalar loads, which no vector memory operation in flight - copies,
    // stores - has to be waited for first.
    // cpx: workgroups an XCD runs at one time (one per compute unit); TPW: output tiles per workgroup.
    // ldc: row pitch of C.  nproj > 1: this launch is projection `proj` of a fused shared-input
    // call: of every task's rank rows (in M) and rank columns (in P) only the window
    // [proj r, (proj + 1) r) takes part, r = the task's stacked rank / nproj.  proj < 0: the launch
    // covers all projections (N = nproj * pd.dg, pd.dg a multiple of the tile width) and a tile takes
    // the projection its columns lie in; M is then the compact [R_tot][pd.dg] array.
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    // MFMA 16x16x32 lanes: j = row of the "B" operand (a token) and of the result, kg = group of 8 k
    // (operands) or of 4 result rows of the "A" operand (columns of C)
    const int j = lane & 15, kg = lane >> 4;
    const int32_t T = pd.T;
    const int32_t KT = K / BK;                       // the launcher guarantees K % (2 BK) == 0: an even number of K tiles

    // ---- this workgroup's output tiles.  Consecutive workgroup ids go to different XCDs (each with its own
    //      L2), so every XCD gets a contiguous range of the tile order; inside the order, GM tile-rows share one
    //      sweep over the tile-columns.  The cpx workgroups that an XCD runs at one time walk its range side by
    //      side - at any moment they work on cpx neighbouring tiles and share their panels through the L2 - but
    //      only for TPW tiles each: then the next cpx workgroups are dispatched.  (A workgroup that kept its
    //      place for the whole launch would drift: one that falls behind misses the panels its neighbours have
    //      fetched, which slows it further; at 112 tiles per compute unit that cost 5 % and 44 % more L2 misses.)
    const int32_t ntiles = tiles_m * tiles_n;
    const int32_t wg = blockIdx.x;
    const int32_t xcd = wg & 7, xidx = wg >> 3;
    const int32_t xper = ntiles >> 3, xrem = ntiles & 7;
    const int32_t xstart = xcd * xper + min(xcd, xrem), xcount = xper + (xcd < xrem ? 1 : 0);
    const int32_t xwgs = cpx;                        // stride between a workgroup's tiles
    const int32_t xfirst = (xidx / cpx) * (cpx * TPW) + xidx % cpx;      // its first tile within the XCD's range
    const int32_t my_tiles = xfirst < xcount ? min(TPW, (xcount - xfirst + cpx - 1) / cpx) : 0;
    if (my_tiles == 0) return;                       // uniform over the workgroup
    auto tile_origin = [&](int32_t n, int32_t& row0, int32_t& col0) {   // my n-th tile
        const int32_t id = xstart + xfirst + n * xwgs;
        const int32_t group = id / (GM * tiles_n);
        const int32_t first_m = group * GM;
        const int32_t gsz = min(tiles_m - first_m, GM);
        const int32_t in = id - group * GM * tiles_n;
        // The last tile row / column of a shape that is not a multiple of the tile is moved up / left until it
        // fits (the launcher guarantees T >= BM, N >= BN): it computes some elements of its neighbour once
        // more, bit for bit the same, and no tile needs clamped addresses or masked stores.
        row0 = min((first_m + in % gsz) * BM, T - BM);
        col0 = min((in / gsz) * BN, N - BN);
    };

    // Accumulator (mb, nb) of this wave is a[acc_reg(mb, nb) : + 3] (see gemm_common.h); its register v holds
    // token row mb 16 + j of the wave tile, column block_col(nb, 4 kg + v).  Nothing clears them: the first K
    // step of every output tile starts from zero.

    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = uint32_t(uintptr_t((__attribute__((address_space(3))) unsigned char*)lds));
    const uint32_t ldsw = lds0 + wave_u * 1024;      // where this wave's first copy block of stage 0 lands

    // ---- copy side: the stream of K tiles.  Copy block b (1 KiB) of an operand tile holds rows 8 b .. 8 b + 7
    //      of a [rows][64 k] tile or k rows 2 b, 2 b + 1 of a [64 k][256 n] tile; wave w moves blocks w, w + 4, ...
    //      The per-lane source offsets are the same for every tile.
    uint32_t zvo[NBZ], wvo[NBZ];
#pragma unroll
    for (int c = 0; c < NBZ; ++c) {
        const int blk = wave + NW * c;
        const int row = 8 * blk + lane / 8;
        const int ch = (lane % 8) ^ swz_row(row);
        zvo[c] = (uint32_t(row) * uint32_t(K) + 8u * ch) * 2u;
        if (W_KN) {
            const int krow = 2 * blk + (lane >> 5);
            const int chn = (lane & 31) ^ kn_swz2(krow);
            wvo[c] = (uint32_t(krow) * uint32_t(ldw) + 8u * chn) * 2u;
        } else {
            // LDS row `row` of the W tile feeds result row (row & 15) of block (row & 127) >> 4 of wave
            // row >> 7: it holds the column that block_col deals to it
            const int gcol = (row & ~127) + block_col((row & 127) >> 4, row & 15);
            wvo[c] = (uint32_t(gcol) * uint32_t(ldw) + 8u * ch) * 2u;
        }
    }
    const unsigned char *zcur, *wcur;                // K tile the next copies fetch
    const size_t wstep = W_KN ? size_t(BK) * ldw * 2 : size_t(BK) * 2;
    auto set_copy_tile = [&](int32_t n) {
        int32_t r0, c0;
        tile_origin(n, r0, c0);
        zcur = reinterpret_cast<const unsigned char*>(Z + size_t(r0) * K);
        wcur = reinterpret_cast<const unsigned char*>(W_KN ? W + c0 : W + size_t(c0) * ldw);
    };
    int32_t c_n = 0, c_kt = 0;                       // the copy cursor: my c_n-th tile, its K tile c_kt
    auto advance = [&]() __attribute__((always_inline)) {
        if (c_kt + 1 < KT) {
            ++c_kt;
            zcur += BK * 2;
            wcur += wstep;
        } else if (c_n + 1 < my_tiles) {
            ++c_n;
            c_kt = 0;
            set_copy_tile(c_n);
        }
        // else: past the end the last K tile is copied once more into a stage nobody reads any more,
        // which keeps the loop free of branches around the copies
    };
    // where copy c of a K tile lands: Z blocks, then W blocks.  stage_addr = the stage + 1024 x this wave's number
    auto copy_lds_addr = [&](uint32_t stage_addr, int c) {
        return c < NBZ ? stage_addr + NW * c * 1024 : stage_addr + ZT_BYTES + NW * (c - NBZ) * 1024;
    };

    // ---- compute side: operand fragments of K step ks (32 k) of a stage.  Block mb of a [rows][64 k] tile
    //      lies 16 rows = 2048 bytes behind block 0 and (row >> 1) & 7 does not depend on mb, so one per-lane
    //      address per step serves all blocks through the instruction's offset field.
    const int fzj = swz_row(j);
    auto zaddr = [&](int stage, int ks) {
        return lds + stage * STAGE_BYTES + (wm * TM + j) * (BK * 2) + ((4 * ks + kg) ^ fzj) * 16;
    };
    auto waddr = [&](int stage, int ks) {            // backward layout only
        return lds + stage * STAGE_BYTES + ZT_BYTES + (wn * TN + j) * (BK * 2) + ((4 * ks + kg) ^ fzj) * 16;
    };
    auto read_z = [&](const unsigned char* za, int mb, bf16x8 (&zf)[MB]) {
        zf[mb] = *reinterpret_cast<const bf16x8*>(za + mb * 16 * (BK * 2));
    };
    // "A" operand of block nb out of a [k][256 n] tile at `base`: k rows krow0 + 8 kg + (j >> 2) + {0, 4}, the
    // 4-column group (j & 3) of the block - with block_col's dealing that is columns 32 (nb / 2) + 8 (j & 3)
    // + 4 ((nb + j) % 2) .. + 3 of the wave tile
    auto read_kn = [&](const unsigned char* base, int krow0, int nb) __attribute__((always_inline)) {
        const int krow = krow0 + 8 * kg + (j >> 2);
        const int n = wn * TN + 32 * (nb >> 1) + 8 * (j & 3) + 4 * ((nb ^ j) & 1);
        const int ch = (n >> 3) ^ kn_swz2(krow);
        return tr_pair(base + krow * 512 + ch * 16 + (n & 7) * 2, 512);
    };
    auto read_w = [&](const unsigned char* wa, int stage, int ks, int nb, bf16x8 (&wf)[NB]) __attribute__((always_inline)) {
        if (W_KN) wf[nb] = read_kn(lds + stage * STAGE_BYTES + ZT_BYTES, 32 * ks, nb);
        else wf[nb] = *reinterpret_cast<const bf16x8*>(wa + nb * 16 * (BK * 2));
    };
    // One K step of 32: the MB NB = 64 MFMAs in NU = 16 sections of four.  A wave issues one instruction every
    // four cycles and an MFMA of this shape keeps its pipe for 16, so a section has room for 12 other
    // instructions before the matrix pipe runs dry; whatever is not an MFMA is placed behind one.
    // Token-row block mb is done in sections 2 mb and 2 mb + 1, after which its fragment zf[mb] is dead and is
    // re-read for K step rks of stage rstage (the step that follows); the other operand lives through the
    // whole step, so its next fragments go to a second register set (wn_).
    //   STEP_FIRST / STEP_PLAIN (K step 0 of a K tile; FIRST: of an output tile - its MFMAs start from zero):
    //       one fragment read per section; `hook` (the stream's bookkeeping, scalar) runs behind the first MFMA
    //       of section 1 instead of between two K steps, where nothing would cover it.
    //   STEP_COPY (K step 1 of a K tile): the K tile's barrier stands behind the first MFMA of section 1 - the
    //       last fragment read of the stage was issued a section and a half earlier, so the wait in front of
    //       the barrier finds it done (directly behind that read it cost the LDS latency once per K tile).
    //       Sections 2 .. 15 then read the first fragments of the next K tile from the other stage and issue
    //       the 16 copies of the K tile at (zcur, wcur) into the stage at cst, which the barrier has freed
    //       (issued back to back the copies block their wave for as long as the texture unit takes to accept
    //       them): one read and one copy per section, two of each in sections 2 and 3.
    enum { STEP_FIRST, STEP_PLAIN, STEP_COPY };
    auto kstep = [&](auto mode_c, int rstage, int rks, bf16x8 (&zf)[MB], bf16x8 (&wc)[NB], bf16x8 (&wn_)[NB], uint32_t cst,
                     auto&& hook) __attribute__((always_inline)) {
        constexpr int mode = decltype(mode_c)::value;
        // (opaque to the optimiser, so that the 16 landing addresses of a K tile are sums with a literal here
        //  instead of 16 loop-invariant registers that have to be spilled)
        asm volatile("" : "+s"(cst));
        agpr_fence();
        const unsigned char* za = zaddr(rstage, rks);
        const unsigned char* wa = waddr(rstage, rks);
        auto copy_src = [&](int c) { return c < NBZ ? zcur : wcur; };
        auto copy_off = [&](int c) { return c < NBZ ? zvo[c % NBZ] : wvo[c % NBZ]; };
        static_for<0, NU>([&](auto u_c) {
            constexpr int u = decltype(u_c)::value, mb = u / 2, nb0 = (NB / 2) * (u % 2);
            if constexpr (mode == STEP_COPY && u >= 2) {
                mfma2_dma16<acc_reg(mb, nb0), acc_reg(mb, nb0 + 1)>(wc[nb0], wc[nb0 + 1], zf[mb], copy_lds_addr(cst, u - 2),
                                                                   copy_src(u - 2), copy_off(u - 2));
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (u < 4) {
                    mfma2_dma16<acc_reg(mb, nb0 + 2), acc_reg(mb, nb0 + 3)>(wc[nb0 + 2], wc[nb0 + 3], zf[mb],
                                                                           copy_lds_addr(cst, 12 + u), copy_src(12 + u), copy_off(12 + u));
                } else {
                    mfma_acc<acc_reg(mb, nb0 + 2)>(wc[nb0 + 2], zf[mb]);
                    __builtin_amdgcn_sched_barrier(0);
                    mfma_acc<acc_reg(mb, nb0 + 3)>(wc[nb0 + 3], zf[mb]);
                }
            } else {
                static_for<0, 4>([&](auto q_c) {
                    constexpr int q = decltype(q_c)::value;
                    if constexpr (mode == STEP_FIRST) mfma_first<acc_reg(mb, nb0 + q)>(wc[nb0 + q], zf[mb]);
                    else mfma_acc<acc_reg(mb, nb0 + q)>(wc[nb0 + q], zf[mb]);
                    if constexpr (u == 1 && q == 0) hook();
                    if constexpr (q < 3) __builtin_amdgcn_sched_barrier(0);
                });
            }
            if constexpr (mode != STEP_COPY) {
                if constexpr (u % 2 == 0) read_w(wa, rstage, rks, u / 2, wn_);
                else read_z(za, mb, zf);
            } else if constexpr (u == 2) {
                read_w(wa, rstage, rks, 0, wn_);
                read_z(za, 0, zf);
            } else if constexpr (u == 3) {
                read_w(wa, rstage, rks, 1, wn_);
                read_z(za, 1, zf);
            } else if constexpr (u >= 4) {
                if constexpr (u % 2 == 0) read_w(wa, rstage, rks, u / 2, wn_);
                else read_z(za, mb, zf);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    using step_first = std::integral_constant<int, STEP_FIRST>;
    using step_plain = std::integral_constant<int, STEP_PLAIN>;
    using step_copy = std::integral_constant<int, STEP_COPY>;

    // ---- epilogue of the tile at (row0, col0): fused up projection, then fp32 -> bf16 and the stores.
    //      tab_*: the table entries of the first segment that crosses the tile, read when the tile's main loop
    //      began (a chain of dependent loads that would otherwise sit in front of the epilogue).
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    int32_t tab_sg = 0, tab_lo = 0, tab_hi = 0, tab_task = -1, tab_r0 = 0, tab_r1 = 0, tab_pcol = 0;
    bool tab_pre = false;                            // the first segment's operands are copied ahead (prefetch_adapter)
    auto rfl = [](int32_t v) { return __builtin_amdgcn_readfirstlane(v); };
    auto load_table = [&](int32_t row0, int32_t col0) {
        if (!P) return;
        // the record of this tile row (the last tile row may start above a multiple of the tile height)
        const int32_t* rec = tile_tab + size_t((row0 + BM - 1) / BM) * kGemmTileRec;
        tab_sg = rec[0];
        tab_lo = rec[1];
        tab_hi = rec[2];
        tab_task = rec[3];
        const int32_t pj = proj >= 0 ? proj : col0 / pd.dg;
        const int32_t rw = rec[5] / nproj;
        tab_r0 = rec[4] + pj * rw;
        tab_r1 = tab_r0 + rw;
        tab_pcol = pj * rw;
        tab_pre = tab_task >= 0 && rw > 0 && rw <= PRE_RANKS;
    };
    // ---- the up projection's operands for the first segment of the tile at (row0, col0), copied into the adapter
    //      region while the tile's last K tiles are multiplied, when that segment's rank window fits one rank step:
    //      k rows 0 .. 31 of the M_t slice in the [k][256 n] layout (16 KiB; rows from r_t on repeat row r_t - 1),
    //      then the tile's 256 rows of P, 64 bytes each (16 KiB; chunks from r_t on repeat chunk 0).  What lies
    //      beyond r_t is masked in registers, so only the addresses have to be valid.  Always PRE_COPIES copies
    //      per wave, whatever the rank.
    auto prefetch_adapter = [&](int32_t row0, int32_t col0) __attribute__((always_inline)) {
        if (!tab_pre) return;                        // uniform
        const int32_t r = tab_r1 - tab_r0;
        const int32_t mcol0 = proj >= 0 ? 0 : (col0 / pd.dg) * pd.dg;
        const int32_t mpitch = proj >= 0 ? N : pd.dg;
        const unsigned char* mbase = reinterpret_cast<const unsigned char*>(M + size_t(tab_r0) * mpitch + (col0 - mcol0));
        const unsigned char* pbase = reinterpret_cast<const unsigned char*>(P + size_t(row0) * pd.r_pad + tab_pcol);
        // (opaque to the optimiser: the per-lane offsets are worked out here, once per output tile, instead of
        //  living in eight loop-invariant registers through the main loop)
        int ln = lane;
        asm volatile("" : "+v"(ln));
#pragma unroll
        for (int c = 0; c < PRE_COPIES / 2; ++c) {
            const int blk = wave_u + NW * c;
            const int krow = 2 * blk + (ln >> 5);
            const int chn = (ln & 31) ^ kn_swz2(krow);
            dma16(lds0 + MSLICE_OFF + (wave_u + NW * c) * 1024, mbase,
                  (uint32_t(min(krow, r - 1)) * uint32_t(mpitch) + 8u * chn) * 2u);
        }
#pragma unroll
        for (int c = 0; c < PRE_COPIES / 2; ++c) {
            const int blk = wave_u + NW * c;
            const int row = 16 * blk + (ln >> 2), ch = ln & 3;
            dma16(lds0 + MSLICE_OFF + PRE_P_OFF + (wave_u + NW * c) * 1024, pbase,
                  (uint32_t(row) * uint32_t(pd.r_pad) + (8 * ch < r ? 8u * ch : 0u)) * 2u);
        }
    };
    auto epilogue = [&](int32_t row0, int32_t col0) __attribute__((always_inline)) {
        // the loop's MFMAs are asm statements, so the compiler does not know that the accumulators come out of
        // the matrix pipeline: keep the first read of them the documented number of wait states away
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        const int32_t row_end = min(row0 + BM, T);
        const int32_t wrow0 = row0 + wm * TM;        // the wave's rows are wrow0 .. wrow0 + TM - 1
        // ---- fused up projection: for every adapter segment that crosses this tile, ceil(r_t / 32) extra
        //      K steps acc += M_t^T[:, cols] * P[rows, :]^T with the rows outside the segment masked to zero.
        //      The M_t slice [r_t][256 cols] is staged in its own LDS region, MROWS rank rows at a time, in the
        //      [k][n] layout (rank rows up to the next multiple of 32 zero) and gathered with the transpose
        //      read; P comes straight from global memory, 16 bytes per lane.
        //      The segment loop and its barriers are uniform over the workgroup.
        if (P) {
            unsigned char* ml = lds + MSLICE_OFF;
            const int32_t pj = proj >= 0 ? proj : col0 / pd.dg;          // this tile's projection
            const int32_t mcol0 = proj >= 0 ? 0 : pj * pd.dg;            // first column of that projection
            const int32_t mpitch = proj >= 0 ? N : pd.dg;                // row pitch of M
            int32_t sg_first = tab_sg;
            if (tab_pre) {                           // uniform: the first segment's operands are in the region already
                sg_first = tab_sg + 1;
                const int32_t lo = max(tab_lo, row0), hi = min(tab_hi, row_end);
                if (hi > wrow0 && lo < wrow0 + TM) { // wave-uniform: the segment crosses this wave's rows
                    // lane (j, kg) holds ranks 8 kg .. 8 kg + 7 in both operands: those from r_t on are cleared
                    const int nv = min(max(tab_r1 - tab_r0 - 8 * kg, 0), 8);
                    u32x4 km;
#pragma unroll
                    for (int w = 0; w < 4; ++w) km[w] = (2 * w < nv ? 0xffffu : 0u) | (2 * w + 1 < nv ? 0xffff0000u : 0u);
                    const unsigned char* pl = ml + PRE_P_OFF + (wm * TM + j) * (PRE_RANKS * 2) + kg * 16;
                    u32x4 pv[MB];
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        const int32_t row = wrow0 + mb * 16 + j;
                        const u32x4 v = *reinterpret_cast<const u32x4*>(pl + mb * 16 * (PRE_RANKS * 2));
                        pv[mb] = (row >= lo && row < hi) ? (v & km) : zero4;
                    }
                    bf16x8 mf[NB];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        union { bf16x8 b; u32x4 u; } cv;
                        cv.b = read_kn(ml, 0, nb);
                        cv.u &= km;
                        mf[nb] = cv.b;
                    }
                    // The MFMAs are asm statements, which the compiler's hazard pass does not look into: an MFMA
                    // must not read a register in the two wait states after a vector ALU instruction has
                    // written it, and the masking above is such a write (operands that come straight from a
                    // load need nothing).  The statements below order the masking before the wait states and
                    // the MFMAs behind them.
                    asm volatile("s_nop 1" : "+v"(mf[0]), "+v"(mf[1]), "+v"(mf[2]), "+v"(mf[3]), "+v"(mf[4]), "+v"(mf[5]),
                                 "+v"(mf[6]), "+v"(mf[7]));
                    static_for<0, MB>([&](auto mb_c) {
                        constexpr int mb = decltype(mb_c)::value;
                        const int32_t rb = wrow0 + mb * 16;
                        if (hi <= rb || lo >= rb + 16) return;          // wave-uniform
                        bf16x8 pf = as_bf16x8(pv[mb]);
                        asm volatile("s_nop 1" : "+v"(pf));
                        static_for<0, NB>([&](auto nb_c) { mfma_acc<acc_reg(mb, decltype(nb_c)::value)>(mf[decltype(nb_c)::value], pf); });
                    });
                }
            }
            for (int32_t sg = sg_first; sg < pd.nseg; ++sg) {
                const bool cached = sg == tab_sg;
                const int32_t seg_lo = cached ? tab_lo : rfl(cseg_off[sg]);
                if (seg_lo >= row_end) break;
                const int32_t t = cached ? tab_task : rfl(cseg_task[sg]);
                if (t < 0) continue;
                const int32_t seg_hi = cached ? tab_hi : rfl(cseg_off[sg + 1]);
                const int32_t lo = max(seg_lo, row0), hi = min(seg_hi, row_end);
                const int32_t r = cached ? tab_r1 - tab_r0 : rfl(rank_off[t + 1] - rank_off[t]) / nproj;
                const int32_t r0 = cached ? tab_r0 : rfl(rank_off[t]) + pj * r;
                const int32_t rp = (r + 31) & ~31;
                const bool mine = hi > wrow0 && lo < wrow0 + TM;   // wave-uniform: the segment crosses this wave's rows
                // the P fragments of a rank step: lane (j, kg) holds the ranks kk + 8 kg .. + 7 of token row j of
                // each 16-row block; groups that start beyond r_t hold padding, or another projection's ranks,
                // and are not read
                u32x4 pv[MB];
                auto load_p = [&](int32_t kk) {
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        const int32_t row = wrow0 + mb * 16 + j;
                        pv[mb] = (mine && kk + 8 * kg < r && row >= lo && row < hi)
                                     ? *reinterpret_cast<const u32x4*>(P + size_t(row) * pd.r_pad + pj * r + kk + 8 * kg) : zero4;
                    }
                };
                for (int32_t k0 = 0; k0 < rp; k0 += MROWS) {           // rank rows k0 .. k0 + rows - 1 of the slice
                    const int32_t rows = min(rp - k0, MROWS);
                    load_p(k0);
                    // the slice is rows * 32 chunks of 16 bytes; the first MCH * 256 of them are fetched before
                    // the barrier that frees the region and written after it
                    constexpr int MCH = 2, NT = 64 * NW;
                    u32x4 mreg[MCH];
                    auto fetch_m = [&](int32_t base) {
#pragma unroll
                        for (int q = 0; q < MCH; ++q) {
                            const int32_t ch = base + tid + q * NT, kr = k0 + (ch >> 5), n = col0 + 8 * (ch & 31);
                            mreg[q] = (ch < rows * 32 && kr < r && n < N)
                                          ? *reinterpret_cast<const u32x4*>(M + size_t(r0 + kr) * mpitch + (n - mcol0)) : zero4;
                        }
                    };
                    auto store_m = [&](int32_t base) {
#pragma unroll
                        for (int q = 0; q < MCH; ++q) {
                            const int32_t ch = base + tid + q * NT, kr = ch >> 5, c = ch & 31;
                            if (ch < rows * 32) *reinterpret_cast<u32x4*>(ml + kr * 512 + ((c ^ kn_swz2(kr)) << 4)) = mreg[q];
                        }
                    };
                    fetch_m(0);
                    __syncthreads();                    // everybody is done with what the region held before
                    store_m(0);
                    for (int32_t base = MCH * NT; base < rows * 32; base += MCH * NT) {
                        fetch_m(base);
                        store_m(base);
                    }
                    __syncthreads();
                    if (!mine) continue;                // wave-uniform; the barriers are above
                    for (int32_t kk = 0; kk < rows; kk += 32) {
                        if (kk > 0) load_p(k0 + kk);
                        bf16x8 mf[NB];
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) mf[nb] = read_kn(ml, kk, nb);
                        static_for<0, MB>([&](auto mb_c) {
                            constexpr int mb = decltype(mb_c)::value;
                            const int32_t rb = wrow0 + mb * 16;
                            if (hi <= rb || lo >= rb + 16) return;          // wave-uniform
                            const bf16x8 pf = as_bf16x8(pv[mb]);
                            static_for<0, NB>([&](auto nb_c) { mfma_acc<acc_reg(mb, decltype(nb_c)::value)>(mf[decltype(nb_c)::value], pf); });
                        });
                    }
                }
            }
            asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        }
        // (block_col: a lane with odd kg holds its high four columns in block 2 p and its low four in block 2 p + 1)
        auto pair_order = [&](bf16x8 o) {
            union { bf16x8 b; uint64_t h[2]; } u, v;
            u.b = o;
            v.h[0] = (kg & 1) ? u.h[1] : u.h[0];
            v.h[1] = (kg & 1) ? u.h[0] : u.h[1];
            return v.b;
        };
        // ---- fp32 -> bf16 (one rounding, to nearest even) and the stores.  Blocks 2 p and 2 p + 1 hold this lane's
        //      columns 32 p + 8 kg .. + 7 of token row j.  Non-temporal, so that y / dx do not evict x / dy from the
        //      caches before the rank-r passes read them.
#if LOBRA_GP_STORE == 4
        //      Straight from the accumulators: 16 bytes per lane, 64 contiguous bytes per row and instruction.
        const int32_t orow = wrow0 + j, ocol = col0 + wn * TN + 8 * kg;
        uint16_t* cp = C + size_t(orow) * ldc + ocol;
        static_for<0, MB>([&](auto mb_c) {
            constexpr int mb = decltype(mb_c)::value;
            static_for<0, NB / 2>([&](auto p_c) {
                constexpr int p = decltype(p_c)::value;
                bf16x8 o;
                static_for<0, 8>([&](auto q_c) {     // accumulators (mb, 2 p) and (mb, 2 p + 1) are neighbours
                    constexpr int q = decltype(q_c)::value;
                    o[q] = (__bf16)acc_read<acc_reg(mb, 2 * p) + q>();
                });
                o = pair_order(o);
                __builtin_nontemporal_store(o, reinterpret_cast<bf16x8*>(cp + size_t(16 * mb) * ldc + 32 * p));
            });
        });
#else
        //      Through the wave's quarter of the adapter-slice region (8 KiB, free now), a 64 x 64 block at a time,
        //      so that every store instruction writes whole 128-byte lines (8 rows of them): written 64 bytes at a
        //      time the result costs 40 % more write requests between L2 and memory.  Rows of a block are 128 bytes
        //      apart in LDS, 16-byte chunk c of row r stored at c ^ ((r >> 1) & 7); a wave's LDS operations are
        //      carried out in order, so the reads of a block need no wait for its writes.
        if (P) __syncthreads();                      // other waves may still read the adapter slice
        unsigned char* cs = lds + MSLICE_OFF + wave * 8192;
        static_for<0, 4>([&](auto b_c) {
            constexpr int hm = decltype(b_c)::value / 2, hn = decltype(b_c)::value % 2;
            static_for<0, 4>([&](auto m_c) {
                constexpr int mb = 4 * hm + decltype(m_c)::value;
                static_for<0, 2>([&](auto p_c) {
                    constexpr int p = 2 * hn + decltype(p_c)::value;
                    bf16x8 o;
                    static_for<0, 8>([&](auto q_c) {     // accumulators (mb, 2 p) and (mb, 2 p + 1) are neighbours
                        constexpr int q = decltype(q_c)::value;
                        o[q] = (__bf16)acc_read<acc_reg(mb, 2 * p) + q>();
                    });
                    o = pair_order(o);
                    const int r = 16 * (mb % 4) + j, c = 4 * (p % 2) + kg;
                    *reinterpret_cast<bf16x8*>(cs + r * 128 + ((c ^ swz_row(r)) << 4)) = o;
                });
            });
            static_for<0, 8>([&](auto i_c) {
                const int r = 8 * decltype(i_c)::value + (lane >> 3), pos = lane & 7;
                const bf16x8 o = *reinterpret_cast<const bf16x8*>(cs + r * 128 + (pos << 4));
                uint16_t* dst = C + size_t(wrow0 + 64 * hm + r) * ldc + (col0 + wn * TN + 64 * hn + 8 * (pos ^ swz_row(r)));
#if LOBRA_GP_STORE == 0     // timing variant: only a token store, so that the result is not dead code
                if (decltype(b_c)::value == 0 && decltype(i_c)::value == 0) __builtin_nontemporal_store(o, reinterpret_cast<bf16x8*>(dst));
                else asm volatile("" : : "v"(o));
#elif LOBRA_GP_STORE == 2
                *reinterpret_cast<bf16x8*>(dst) = o;
#else
                __builtin_nontemporal_store(o, reinterpret_cast<bf16x8*>(dst));
#endif
            });
        });
#endif
        // (the accumulators are not cleared here: the first K step of the next tile starts from zero)
    };

    // ---- the stream: K tile g of it sits in stage g & 1 and is copied two K tiles ahead of its use.  The loop
    //      body handles two K tiles, so that the stages are compile-time constants.
    bf16x8 zf[MB], wf[2][NB];
    set_copy_tile(0);
#pragma unroll
    for (int c = 0; c < 2 * NBZ; ++c) dma16(copy_lds_addr(ldsw, c), c < NBZ ? zcur : wcur, c < NBZ ? zvo[c] : wvo[c - NBZ]);
    advance();
#pragma unroll
    for (int c = 0; c < 2 * NBZ; ++c)
        dma16(copy_lds_addr(ldsw + STAGE_BYTES, c), c < NBZ ? zcur : wcur, c < NBZ ? zvo[c] : wvo[c - NBZ]);
    int32_t t_n = 0, t_kt = 0, t_row0, t_col0;       // the compute cursor
    tile_origin(0, t_row0, t_col0);
    load_table(t_row0, t_col0);
    wait_vmcnt<0>();                                 // the first two K tiles have landed
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int u = 0; u < MB; ++u) read_z(zaddr(0, 0), u, zf);
#pragma unroll
    for (int u = 0; u < NB; ++u) read_w(waddr(0, 0), 0, 0, u, wf[0]);
    // every wave has read the last fragments of this stage, and the copies of the next K tile have landed
    auto tile_barrier = []() __attribute__((always_inline)) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
    };
    // The same in the first K tile of an output tile: the 32 stores of the previous tile's epilogue were
    // issued after the copies this barrier is about, and vector memory operations complete in the order they
    // were issued, so the barrier does not have to wait for the stores: they drain under the MFMAs that follow.
    // (The workgroup's very first tile has no stores behind its copies: the prologue waits for them itself.)
    auto tile_barrier_after_stores = []() __attribute__((always_inline)) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        wait_vmcnt<LOBRA_GP_STORES_IN_FLIGHT>();
        __builtin_amdgcn_s_barrier();
    };
    // One K tile in stage STG: K step 0 (fragments in registers) reads the fragments of K step 1 and moves the
    // copy cursor on to the K tile after next; K step 1, once the barrier in its second section is passed,
    // reads the first fragments of the next K tile from the other stage and copies the K tile after next
    // into this one.
    auto ktile = [&](auto stg_c, auto mode_c) __attribute__((always_inline)) {
        constexpr int STG = decltype(stg_c)::value;
        kstep(mode_c, STG, 1, zf, wf[0], wf[1], 0, advance);
        if constexpr (decltype(mode_c)::value == STEP_FIRST)
            kstep(step_copy{}, STG ^ 1, 0, zf, wf[1], wf[0], ldsw + uint32_t(STG) * STAGE_BYTES, tile_barrier_after_stores);
        else
            kstep(step_copy{}, STG ^ 1, 0, zf, wf[1], wf[0], ldsw + uint32_t(STG) * STAGE_BYTES, tile_barrier);
    };
    using stage0 = std::integral_constant<int, 0>;
    using stage1 = std::integral_constant<int, 1>;
    for (;;) {
        if (t_kt == 0) ktile(stage0{}, step_first{});
        else ktile(stage0{}, step_plain{});
        if (t_kt + 2 == KT) prefetch_adapter(t_row0, t_col0);   // waited for at the tile barrier that follows
        ktile(stage1{}, step_plain{});
        t_kt += 2;
        if (t_kt == KT) {                            // uniform: an output tile is complete
            epilogue(t_row0, t_col0);
            t_kt = 0;
            if (++t_n == my_tiles) break;
            tile_origin(t_n, t_row0, t_col0);
            load_table(t_row0, t_col0);
            // the first fragments of the next output tile once more: holding 64 registers of them through
            // the epilogue costs more (spills) than these sixteen reads
#pragma unroll
            for (int u = 0; u < MB; ++u) read_z(zaddr(0, 0), u, zf);
#pragma unroll
            for (int u = 0; u < NB; ++u) read_w(waddr(0, 0), 0, 0, u, wf[0]);
        }
    }
    // copies past the end are still in flight: they must have landed before the LDS is given back
    wait_vmcnt<0>();
}

namespace {
template <bool W_KN>
hipError_t launch_persistent(const PlanDev& pd, const void* Z, const void* W, const void* P, const void* M, void* C,
                             int32_t K, int32_t N, int32_t ldw, int32_t ldc, int32_t nproj, int32_t proj,
                             int32_t tiles_m, int32_t tiles_n, int32_t gm, hipStream_t st)
{
    // once per device: the kernel needs more dynamic LDS than the default limit; one workgroup per compute unit
    static std::atomic<int32_t> cus[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    int32_t ncu = cus[dev].load(std::memory_order_acquire);
    if (ncu == 0) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_persistent_kernel<W_KN>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        int n = 0;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        ncu = n > 0 ? n : 1;
        cus[dev].store(ncu, std::memory_order_release);
    }
    const int64_t ntiles = int64_t(tiles_m) * tiles_n;
    const int32_t cpx = ncu >= 8 ? ncu / 8 : 1;
    const int32_t tpw = LOBRA_GP_TPW;
    const int64_t xmax = (ntiles + 7) / 8;                                    // tiles of the fullest XCD
    const int64_t rounds = (xmax + int64_t(cpx) * tpw - 1) / (int64_t(cpx) * tpw);
    const int64_t wgs = ntiles <= 8 * int64_t(cpx) ? ntiles : 8 * rounds * cpx;   // few tiles: one workgroup each
    gemm_persistent_kernel<W_KN><<<dim3(uint32_t(wgs)), 64 * NW, LDS_BYTES, st>>>(
        pd, (const uint16_t*)Z, (const uint16_t*)W, (const uint16_t*)P, (const uint16_t*)M, (uint16_t*)C,
        K, N, ldw, ldc, nproj, proj, tiles_m, tiles_n, gm, cpx, tpw, pd.gemm_tile_tab, pd.cseg_off, pd.cseg_task, pd.rank_off);
    return hipGetLastError();
}
}  // namespace

hipError_t gemm_persistent(const PlanDev& pd, bool transW, const void* Z, const void* W, const void* P,
                           const void* M, void* C, int32_t K, int32_t N, int32_t ldw, int32_t ldc, int32_t nproj,
                           int32_t proj, int32_t tiles_m, int32_t tiles_n, int32_t gm, hipStream_t st)
{
    if (transW) return launch_persistent<false>(pd, Z, W, P, M, C, K, N, ldw, ldc, nproj, proj, tiles_m, tiles_n, gm, st);
    return launch_persistent<true>(pd, Z, W, P, M, C, K, N, ldw, ldc, nproj, proj, tiles_m, tiles_n, gm, st);
}

}  // namespace lobra
