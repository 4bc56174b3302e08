// HBM-bound rank-r kernels of the bf16 path (gfx950 MFMA, operands streamed straight from
// global memory into MFMA registers: the skinny operand needs no LDS tile at all).
//
//   shrink_mfma      P = s_t Z M_t^T   (Z = x, M = A gives s_t A_t x_i; Z = dy, M = B gives s_t B_t dy_i)
//   grad_mfma        stage 1 of dM_t = sum_i P_i^T Z_i over a reduction chunk (dB from P = s h,
//                    Z = dy; dA from P = s g, Z = x), partial sums per chunk
// (paper section 2.1: the two low-rank factors of X (down)(up) and their gradients; section 1:
// each task of the fused batch has its own pair.)
#include <atomic>

#include "gemm_common.h"
#include "kernels.h"

#ifndef LOBRA_GRAD_ORDER
#define LOBRA_GRAD_ORDER 2      // reduction kernels: 2 column tile fastest, 0 chunk fastest, 1 column tile fastest and XCD-contiguous
#endif
#ifndef LOBRA_SKINNY_XCD
#define LOBRA_SKINNY_XCD 1      // work items dealt to the XCDs in contiguous ranges (see xcd_contiguous)
#endif

namespace lobra {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {
// Load of data that is read once per launch and in whole cache lines (the gradient kernels' token
// rows): marked non-temporal (STREAM), it does not displace the rank-r operand that every workgroup
// re-reads.  Measured 7-11 % on the gradient kernels at ranks from 32 and on batches far larger than the
// 256 MB infinity cache; a batch that fits that cache is better left in it for the kernels that follow
// (the projection kernels, which read half lines per instruction, lose 15-20 % with the hint and never use it).
template <bool STREAM, typename V> __device__ __forceinline__ V stream_load(const V* p)
{
    if constexpr (STREAM) return __builtin_nontemporal_load(p);
    else return *p;
}
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v)
{
    union { u32x4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}
}  // namespace

// -------------------------------------------------------------------------------------------------
// shrink: one workgroup per token block (<= 32 tokens of one task), 4 waves split K.
// v_mfma_f32_16x16x32_bf16 with the MFMA "A" operand = 16 rank rows of M_t and the "B" operand =
// 16 token rows of Z, so a lane ends up with 4 consecutive ranks of one token.  K is walked in
// slabs of 128 = 4 MFMA steps of 32: in step q lane (row, kg) loads the 8 elements
// slab + 32 q + 8 kg .. + 7 of its row, so the four lanes of a row read one 64-byte sector per
// load instruction and a whole 256-byte run per slab.  Rank blocks beyond the task's rank are
// skipped.
// -------------------------------------------------------------------------------------------------
// NRB: rank blocks of 16 (r_t <= 16 NRB); NWV: waves; DEPTH: slabs in flight per wave
template <int NRB, int NWV, int DEPTH>
__global__ __launch_bounds__(64 * NWV) void shrink_mfma_kernel(PlanDev pd, const uint16_t* __restrict__ Z,
                                                          const uint16_t* __restrict__ M,
                                                          const float* __restrict__ s,
                                                          uint16_t* __restrict__ P_tok,
                                                          uint16_t* __restrict__ P_blk, int32_t D,
                                                          int32_t ldz, int32_t nproj, int32_t proj)
{
    // nproj > 1 (fused shared-input projections): this launch handles projection `proj` only - Z is
    // that projection's column block of dy (row pitch ldz), M its rows of the compact up factors,
    // and the task's rank rows it reads and writes are the window [proj r, (proj + 1) r).
    __shared__ float red[NWV][2][NRB][64][4];   // [wave][token half][rank block][lane][4]
    // (a launch order by rank is dealt round-robin: contiguous ranges of it would give one XCD all the expensive blocks)
    const int32_t bi = pd.tb_order ? pd.tb_order[blockIdx.x]
                                   : (LOBRA_SKINNY_XCD ? xcd_contiguous(blockIdx.x, gridDim.x) : int32_t(blockIdx.x));
    const TokenBlock b = pd.tb[bi];
    const int32_t r = (pd.rank_off[b.task + 1] - b.rank_row0) / nproj;
    const int32_t pofs = proj * r;               // first rank of the window inside the task's rows
    const int32_t rank_row0 = b.rank_row0 + pofs;
    const int32_t plim = proj == nproj - 1 ? pd.r_pad - pofs : r;   // ranks (and zero padding) stored by this launch
    const int32_t nrb_t = (r + 15) >> 4;        // rank blocks this task needs (uniform)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, kg = lane >> 4;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    f32x4 acc[2][NRB];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) acc[h][rb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // rows beyond the block repeat its last row (their results are never stored)
    const uint16_t* zrow[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
        zrow[h] = Z + size_t(b.row0 + min(16 * h + j, b.nrows - 1)) * ldz;
    const uint16_t* mrow[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) mrow[rb] = M + size_t(rank_row0 + min(16 * rb + j, r - 1)) * D;

    // operands of one slab: 4 steps x (2 token halves of Z, NRB rank blocks of M).
    // Rank rows beyond r_t and token rows beyond the block repeat a valid row: what they produce
    // is dropped at the store, so the loads of a whole slab need no per-lane condition.
    struct Slab { u32x4 zv[2][4], mv[NRB][4]; };
    auto load = [&](Slab& sl, int32_t slab) {
        const int32_t k = slab + 8 * kg;
        if (slab + 128 <= D) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
#pragma unroll
                for (int rb = 0; rb < NRB; ++rb)
                    if (NRB == 1 || rb < nrb_t)
                        sl.mv[rb][q] = *reinterpret_cast<const u32x4*>(mrow[rb] + k + 32 * q);
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    sl.zv[h][q] = *reinterpret_cast<const u32x4*>(zrow[h] + k + 32 * q);
            }
        } else {   // the last slab of a width that is not a multiple of 128: columns beyond D read as 0
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool kin = k + 32 * q < D;
#pragma unroll
                for (int rb = 0; rb < NRB; ++rb)
                    if (NRB == 1 || rb < nrb_t)
                        sl.mv[rb][q] = kin ? *reinterpret_cast<const u32x4*>(mrow[rb] + k + 32 * q) : zero4;
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    sl.zv[h][q] = kin ? *reinterpret_cast<const u32x4*>(zrow[h] + k + 32 * q) : zero4;
            }
        }
    };
    auto mac = [&](const Slab& sl) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int rb = 0; rb < NRB; ++rb)
                    if (NRB == 1 || rb < nrb_t)
                        acc[h][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            as_bf16x8(sl.mv[rb][q]), as_bf16x8(sl.zv[h][q]), acc[h][rb], 0, 0, 0);
    };
    const int32_t nsl = (D + 127) >> 7;
    // DEPTH slabs in flight per wave: the loads of slab i + DEPTH - 1 are issued before the MFMAs
    // of slab i (DEPTH = 1: load, then multiply).
    Slab buf[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH - 1; ++d)
        if (wave + NWV * d < nsl) load(buf[d], (wave + NWV * d) << 7);
    for (int32_t i = wave; i < nsl; i += NWV * DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int32_t nx = i + NWV * (d + DEPTH - 1);
            if (nx < nsl) load(buf[(d + DEPTH - 1) % DEPTH], nx << 7);
            if (i + NWV * d < nsl) mac(buf[d]);
        }
    }
    // cross-wave sum through LDS, then lane (token j, rank group kg) of wave 0/1 stores half h
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
            if (rb < nrb_t)
#pragma unroll
                for (int v = 0; v < 4; ++v) red[wave][h][rb][lane][v] = acc[h][rb][v];
    __syncthreads();
    if (wave < 2) {
        const int h = wave;
        const int32_t tok = 16 * h + j;
        const float st = s[b.task];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            bf16x4 o;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float sum = 0.f;
                if (rb < nrb_t)
#pragma unroll
                    for (int w = 0; w < NWV; ++w) sum += red[w][h][rb][lane][v];   // fixed order
                const int32_t p = 16 * rb + 4 * kg + v;
                o[v] = (__bf16)((p < r && tok < b.nrows) ? st * sum : 0.f);
            }
            const int32_t p0 = 16 * rb + 4 * kg;
            if (p0 < plim) {
                if (tok < b.nrows)
                    *reinterpret_cast<bf16x4*>(P_tok + size_t(b.row0 + tok) * pd.r_pad + pofs + p0) = o;
                // block-transposed copy [block][rank][32 tokens]; tokens beyond the block hold 0
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    union { __bf16 b; uint16_t u; } c;
                    c.b = o[v];
                    P_blk[(size_t(bi) * pd.r_pad + pofs + p0 + v) * kTokenBlock + tok] = c.u;
                }
            }
        }
    }
}

// -------------------------------------------------------------------------------------------------
// shrink for ranks from about 24 up (chosen by the plan for long batches): one workgroup per run of up to 4 token blocks of one task, wave w owns
// block w over the whole of K.  The rank rows of a slab (16 NRB x 128 columns) are staged in LDS once
// per workgroup and read by all four waves, so the adapter traffic is r_t rows per 128 token rows
// instead of per 32; a wave's sums are complete when its loop ends (no cross-wave reduction).
// LDS layout of a staged slab: [rank row][16 chunks of 16 bytes], chunk c of row R at c ^ (R & 15), so
// that the 16 rank rows of one ds_read_b128 pass hit 16 different bank groups; two slabs are staged
// alternately (one barrier per slab).
// -------------------------------------------------------------------------------------------------
template <int NRB, int DEPTH>
__global__ __launch_bounds__(256) void shrink_lds_kernel(PlanDev pd, const uint16_t* __restrict__ Z,
                                                      const uint16_t* __restrict__ M,
                                                      const float* __restrict__ s,
                                                      uint16_t* __restrict__ P_tok,
                                                      uint16_t* __restrict__ P_blk, int32_t D)
{
    constexpr int ROWS = 16 * NRB;                       // staged rank rows
    constexpr int CH = ROWS * 16;                        // 16-byte chunks per staged slab
    constexpr int MLD = (CH + 255) / 256;                // chunks per thread
    __shared__ __attribute__((aligned(16))) unsigned char ms[2][ROWS * 256];
    const int32_t run = pd.sb_order ? pd.sb_order[blockIdx.x]
                                    : (LOBRA_SKINNY_XCD ? xcd_contiguous(blockIdx.x, gridDim.x) : int32_t(blockIdx.x));
    const int32_t tb0 = pd.sb_off[run];
    const int32_t cnt = pd.sb_off[run + 1] - tb0;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool active = wave < cnt;                      // wave-uniform: this wave has a token block
    const TokenBlock b = pd.tb[tb0 + min(wave, cnt - 1)];
    const int32_t r = pd.rank_off[b.task + 1] - b.rank_row0;
    const int32_t nrb_t = (r + 15) >> 4;
    const int j = lane & 15, kg = lane >> 4;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    f32x4 acc[2][NRB];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) acc[h][rb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const uint16_t* zrow[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) zrow[h] = Z + size_t(b.row0 + min(16 * h + j, b.nrows - 1)) * D;

    // staging: thread tid moves chunks tid, tid + 256, ...: chunk id = (rank row, 16-byte column chunk)
    u32x4 mreg[MLD];
    auto fetch_m = [&](int32_t slab) {
#pragma unroll
        for (int u = 0; u < MLD; ++u) {
            const int ch = threadIdx.x + 256 * u, R = ch >> 4, c = ch & 15;
            const int32_t k = slab + 8 * c;
            mreg[u] = (ch < CH && R < 16 * nrb_t && k < D)
                          ? *reinterpret_cast<const u32x4*>(M + size_t(b.rank_row0 + min(R, r - 1)) * D + k) : zero4;
        }
    };
    auto stash_m = [&](int buf) {
#pragma unroll
        for (int u = 0; u < MLD; ++u) {
            const int ch = threadIdx.x + 256 * u, R = ch >> 4, c = ch & 15;
            if (ch < CH) *reinterpret_cast<u32x4*>(&ms[buf][R * 256 + ((c ^ (R & 15)) << 4)]) = mreg[u];
        }
    };
    struct ZSlab { u32x4 zv[2][4]; };
    auto load_z = [&](ZSlab& sl, int32_t slab) {
        const int32_t k = slab + 8 * kg;
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                sl.zv[h][q] = (slab + 128 <= D || k + 32 * q < D)
                                  ? *reinterpret_cast<const u32x4*>(zrow[h] + min(k + 32 * q, D - 8)) : zero4;
    };
    auto mac = [&](const ZSlab& sl, int buf) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb)
                if (rb < nrb_t) {
                    const int R = 16 * rb + j;
                    const u32x4 mv = *reinterpret_cast<const u32x4*>(&ms[buf][R * 256 + (((4 * q + kg) ^ (R & 15)) << 4)]);
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        acc[h][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(mv), as_bf16x8(sl.zv[h][q]),
                                                                         acc[h][rb], 0, 0, 0);
                }
    };
    const int32_t nsl = (D + 127) >> 7;
    ZSlab zb[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH - 1; ++d)
        if (d < nsl && active) load_z(zb[d], d << 7);
    fetch_m(0);
    for (int32_t i = 0; i < nsl; i += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            const int32_t sl = i + d;
            if (sl >= nsl) break;                            // uniform
            stash_m(sl & 1);
            __syncthreads();                                 // slab sl is staged; slab sl - 1 has been consumed
            if (sl + 1 < nsl) fetch_m((sl + 1) << 7);
            if (active) {
                if (sl + DEPTH - 1 < nsl) load_z(zb[(d + DEPTH - 1) % DEPTH], (sl + DEPTH - 1) << 7);
                mac(zb[d], sl & 1);
            }
        }
    }
    if (!active) return;
    const float st = s[b.task];
    const int32_t bi = tb0 + wave;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int32_t tok = 16 * h + j;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            bf16x4 o;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int32_t p = 16 * rb + 4 * kg + v;
                o[v] = (__bf16)((p < r && tok < b.nrows) ? st * acc[h][rb][v] : 0.f);
            }
            const int32_t p0 = 16 * rb + 4 * kg;
            if (p0 < pd.r_pad) {
                if (tok < b.nrows)
                    *reinterpret_cast<bf16x4*>(P_tok + size_t(b.row0 + tok) * pd.r_pad + p0) = o;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    union { __bf16 b; uint16_t u; } c;
                    c.b = o[v];
                    P_blk[(size_t(bi) * pd.r_pad + p0 + v) * kTokenBlock + tok] = c.u;
                }
            }
        }
    }
}

// -------------------------------------------------------------------------------------------------
// shrink for ranks up to 16 on long batches: K is cut into slices of 512 columns, a work item is (token
// block, slice), and one workgroup per compute unit walks a contiguous range of the items of its XCD's
// token blocks in slice-major order.  What the one-block-per-workgroup kernel above loses on such a batch,
// measured: (a) its workgroups all start, stream and finish in step, so the dependent loads at the start
// and the reduction and stores at the end of a block are exposed once per launch with nothing behind them;
// (b) a compute unit sustains about 20 GB/s of token rows however many workgroups it holds, so a launch of
// 513 blocks on 256 compute units takes as long as one of 768 (one unit gets three blocks instead of two);
// (c) the adapter rows are a third of what passes through the vector memory path.  Here a wave keeps the
// adapter columns of its part of the slice in registers for as long as task and slice stay the same (they are
// read once per dozen token blocks), the loads of the next three items are in flight while an item is
// multiplied, reduced and stored, and the items are dealt to the workgroups to within one item.
// The eight waves of a workgroup share an item: wave (h, w) takes token half h (16 tokens) and the 128 columns
// number w of the slice; the four waves of a half add their sums through LDS (fixed order) and wave (h, 0)
// writes the fp32 partial projection part[slice][token][16]; the finish kernel below adds the slices in
// order, scales, rounds and writes both bf16 layouts.
// The token rows go global -> LDS without passing through registers (global_load_lds_dwordx4, lane-linear:
// the lane that fetched 16 bytes reads them back as its MFMA operand), into a ring of R slots of 4 KiB per
// wave.  The compiler does not see these copies, so the kernel places their waits itself (s_waitcnt vmcnt
// with the number of younger copies): with ordinary loads under the loop's conditions the compiler's own
// waits drained every wave's prefetched loads at every item.  For the same reason the item barrier is a bare
// s_barrier (no fence), and the tables are restrict-qualified arguments of their own rather than members of
// the plan structure: only then are they read with scalar loads, which vmcnt does not count.
//
// WITH_DB (the backward pass over dy): the same pass also accumulates dB_t = sum_i (s_t h_i)^T dy_i (section 2.1:
// the gradient of the up factor), so that dy is read once for both.  The block-transposed s_t h of an item
// (P_blk: 16 ranks x 32 tokens, 1 KiB) comes in with one more copy of wave 0 and is read by all waves behind
// the item's barrier (one such copy per wave measured 4 us slower at workload 2); the dy
// operand - 4 tokens of one column per lane - is gathered out of the ring with transposing reads
// (ds_read_b64_tr_b16); eight v_mfma_f32_16x16x16_bf16 add the item to the wave's 16 ranks x 128 columns of sums,
// which stay in registers for as long as task and slice stay the same.  When they change (and at the end) the
// two token halves are added through LDS and written to the rows that the plan has assigned to this run of
// the workgroup (Plan::fb_*); stage 2 of the reductions adds the runs of a (task, slice) in the plan's order.
// -------------------------------------------------------------------------------------------------
constexpr int kSlicedRing = 4;                                     // ring slots per wave
constexpr int kSlicedRedOff = 8 * kSlicedRing * 4096;              // the two reduction buffers (also the dB exchange)
constexpr int kSlicedHOff = kSlicedRedOff + 2 * 8 * 64 * 16;       // WITH_DB: ring of the items' s_t h blocks, 1 KiB per slot
constexpr int kSlicedLds = kSlicedHOff, kSlicedLdsDb = kSlicedHOff + (kSlicedRing + 1) * 1024;

typedef short s16x4 __attribute__((ext_vector_type(4)));

template <bool WITH_DB>
__global__ __launch_bounds__(512) void shrink_sliced_kernel(const TokenBlock* __restrict__ tbs,
                                                           const int32_t* __restrict__ rank_off, int32_t ntb,
                                                           int32_t T, const uint16_t* __restrict__ Z,
                                                           const uint16_t* __restrict__ Mx,
                                                           float* __restrict__ part, int32_t D, int32_t ldz,
                                                           int32_t nsl, const uint16_t* __restrict__ Hblk,
                                                           float* __restrict__ partb,
                                                           const int32_t* __restrict__ wg_run_off,
                                                           const int32_t* __restrict__ run_row)
{
    constexpr int R = kSlicedRing;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x >> 6));
    const int h = wave >> 2, w = wave & 3;
    const int j = lane & 15, kg = lane >> 4;
    unsigned char* ring = lds + wave * (R * 4096);                 // this wave's ring
    const uint32_t ring_addr = uint32_t(uintptr_t((__attribute__((address_space(3))) unsigned char*)ring));
    float* red = reinterpret_cast<float*>(lds + kSlicedRedOff);    // [item parity][wave][lane][4]
    unsigned char* hring = lds + kSlicedHOff;                      // WITH_DB: [slot][16 ranks][32 tokens] bf16
    const uint32_t hring_addr = uint32_t(uintptr_t((__attribute__((address_space(3))) unsigned char*)hring));

    // consecutive workgroup ids run on different XCDs: XCD x takes the token blocks [bx0, bx1) - a
    // contiguous piece of the activation tensor when the batch is sorted - and its workgroups split the
    // items (slice, block) of that piece, slice-major, into contiguous ranges
    const int32_t per_xcd = int32_t(gridDim.x >> 3), xcd = int32_t(blockIdx.x & 7), idx = int32_t(blockIdx.x >> 3);
    const int32_t bx0 = int32_t((int64_t(ntb) * xcd) >> 3), bx1 = int32_t((int64_t(ntb) * (xcd + 1)) >> 3);
    const int32_t nbx = bx1 - bx0;
    const int64_t nit = int64_t(nbx) * nsl;
    const int32_t e0 = int32_t(nit * idx / per_xcd), e1 = int32_t(nit * (idx + 1) / per_xcd);
    const int32_t n = e1 - e0;                   // the same for all waves of the workgroup
    if (n <= 0) return;

    // slice, block offset inside the XCD's piece, ring slot, slot in the ring of s_t h blocks.  (That ring is
    // shared by the waves and has one slot more: wave 0 overwrites the slot of the item before the one its
    // fellow waves may still be reading.)
    struct Cursor { int32_t sl, bo, slot, hslot; };
    auto advance = [&](Cursor& c) {
        if (++c.bo == nbx) { c.bo = 0; ++c.sl; }
        if (++c.slot == R) c.slot = 0;
        if (++c.hslot == R + 1) c.hslot = 0;
    };
    // the four copies of an item: lane (j, kg) of copy q fetches the 8 columns 32 q + 8 kg .. + 7 of its row
    // out of this wave's 128 columns (one 64-byte piece per four lanes, a 256-byte run of the row in all);
    // rows beyond the block repeat its last row (what they produce is never stored)
    auto issue = [&](const Cursor& c) {
        const TokenBlock b = tbs[bx0 + c.bo];
        const unsigned char* base = reinterpret_cast<const unsigned char*>(Z) +
                                    (size_t(b.row0) * ldz + size_t(c.sl) * 512 + w * 128) * 2;
        const uint32_t voff = (uint32_t(min(16 * h + j, b.nrows - 1)) * uint32_t(ldz) + 8u * kg) * 2u;
#pragma unroll
        for (int q = 0; q < 4; ++q) gemm::dma16(ring_addr + c.slot * 4096 + q * 1024, base + q * 64, voff);
        if constexpr (WITH_DB) {
            // the item's block of s_t h (1 KiB, as stored) for the whole workgroup: one more copy of wave 0,
            // which the other waves read behind the item's barrier
            if (wave == 0)
                gemm::dma16(hring_addr + c.hslot * 1024,
                            reinterpret_cast<const unsigned char*>(Hblk) + size_t(bx0 + c.bo) * (16 * kTokenBlock * 2),
                            uint32_t(lane) * 16u);
        }
    };
    // vector memory operations complete in order: with the copies of y younger items behind it, an item has
    // landed when at most y times the copies per item are outstanding (wave (h, 0)'s stores also count: they
    // only make the wait stricter)
    auto wait_item = [&](auto younger) {
        constexpr int y = decltype(younger)::value;
        if (WITH_DB && wave == 0) gemm::wait_vmcnt<5 * y>();
        else gemm::wait_vmcnt<4 * y>();
    };

    // WITH_DB: this wave's dB sums, 8 column tiles of 16: lane (n, kg) holds ranks 4 kg .. 4 kg + 3 of column n
    f32x4 dbacc[WITH_DB ? 8 : 1];
    int32_t run_idx = -1;                        // runs of (task, slice) this workgroup has met so far, minus 1
    if constexpr (WITH_DB) {
#pragma unroll
        for (int tl = 0; tl < 8; ++tl) dbacc[tl] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // the run's sums go out: the halves are added through LDS (h = 0 plus h = 1, four column tiles at a time:
    // the exchange memory is the two reduction buffers), wave (0, w) stores its 128 columns
    auto flush_db = [&](int32_t sl) {
        if constexpr (WITH_DB) {
            const int32_t row0 = run_row[wg_run_off[blockIdx.x] + run_idx];
            float* ex = red + (w * 4 * 64) * 4;      // [tile of the round][lane][4]
            float* dst = partb + size_t(row0 + 4 * kg) * D + sl * 512 + w * 128 + j;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                // (first round: wave (h, 0) has read the last item's sums out of this memory; second: the
                //  first round's reads are done)
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                if (h == 1) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) *reinterpret_cast<f32x4*>(ex + (u * 64 + lane) * 4) = dbacc[4 * half + u];
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                if (h == 0) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int tl = 4 * half + u;
                        const f32x4 o = dbacc[tl] + *reinterpret_cast<const f32x4*>(ex + (u * 64 + lane) * 4);
#pragma unroll
                        for (int v = 0; v < 4; ++v) dst[size_t(v) * D + tl * 16] = o[v];
                    }
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();        // the memory is free for the next item's sums
            asm volatile("" ::: "memory");
#pragma unroll
            for (int tl = 0; tl < 8; ++tl) dbacc[tl] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    };

    u32x4 av[4];                                 // the adapter columns of this wave's part of the slice
    int32_t cur_task = -1, cur_sl = -1;
    auto consume = [&](const Cursor& c, int32_t it) {
        const TokenBlock b = tbs[bx0 + c.bo];
        if (b.task != cur_task || c.sl != cur_sl) {          // uniform; once per dozen items
            if (WITH_DB && run_idx >= 0) flush_db(cur_sl);
            ++run_idx;
            const int32_t r = rank_off[b.task + 1] - b.rank_row0;
            // rank rows beyond r_t repeat a valid row; the finish kernel drops what they produce
            const uint16_t* mrow = Mx + size_t(b.rank_row0 + min(j, r - 1)) * D + c.sl * 512 + w * 128 + 8 * kg;
#pragma unroll
            for (int q = 0; q < 4; ++q) av[q] = *reinterpret_cast<const u32x4*>(mrow + 32 * q);
            // the values are "used" here so that the compiler waits for them inside this branch: a wait behind
            // the branch would also wait, at every item, for the copies in flight
#pragma unroll
            for (int q = 0; q < 4; ++q) asm volatile("" : "+v"(av[q]));
            cur_task = b.task;
            cur_sl = c.sl;
        }
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const u32x4 zv = *reinterpret_cast<const u32x4*>(ring + c.slot * 4096 + q * 1024 + lane * 16);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(av[q]), as_bf16x8(zv), acc, 0, 0, 0);
        }
        // WITH_DB: the dy operands of the dB product are gathered here, in front of the barrier, whose wait then
        // covers their latency.  "B" operand of column tile tl: lane (n, kg) needs tokens 4 kg .. 4 kg + 3 of column
        // 16 tl + n.  A transposing read of a 16-lane group takes 8 bytes (4 columns) from each lane's address and
        // hands lane 4 g + e element e of what the lanes 4 kr + g, kr = 0 .. 3, supplied: so lane j supplies token
        // 4 kg + (j >> 2), columns 16 tl + 4 (j & 3) .. + 3.  In the ring, column c of token t lies in copy c / 32
        // at lane t + 16 ((c / 8) & 3), 2 (c & 7) bytes in.
        s16x4 bv[WITH_DB ? 8 : 1];
        if constexpr (WITH_DB) {
            const unsigned char* zb = ring + c.slot * 4096 + ((4 * kg + (j >> 2)) + 16 * ((j & 3) >> 1)) * 16 + (j & 1) * 8;
#pragma unroll
            for (int tl = 0; tl < 8; ++tl)
                bv[tl] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (s16x4 __attribute__((address_space(3)))*)(zb + (tl >> 1) * 1024 + (tl & 1) * 512));
        }
        float* rbuf = red + (it & 1) * (8 * 64 * 4);
        *reinterpret_cast<f32x4*>(rbuf + (wave * 64 + lane) * 4) = acc;
        // one barrier per item: the next write to this half of red follows the next item's barrier,
        // which wave (h, 0) reaches only after the reads below
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");           // the reads below stay behind the barrier
        if (w == 0) {
            const f32x4 s0 = *reinterpret_cast<const f32x4*>(rbuf + ((4 * h + 0) * 64 + lane) * 4);
            const f32x4 s1 = *reinterpret_cast<const f32x4*>(rbuf + ((4 * h + 1) * 64 + lane) * 4);
            const f32x4 s2 = *reinterpret_cast<const f32x4*>(rbuf + ((4 * h + 2) * 64 + lane) * 4);
            const f32x4 s3 = *reinterpret_cast<const f32x4*>(rbuf + ((4 * h + 3) * 64 + lane) * 4);
            const int32_t tok = 16 * h + j;
            if (tok < b.nrows)     // lane (j, kg): ranks 4 kg .. 4 kg + 3 of token j
                *reinterpret_cast<f32x4*>(part + (size_t(c.sl) * T + b.row0 + tok) * 16 + 4 * kg) = ((s0 + s1) + s2) + s3;
        }
        if constexpr (WITH_DB) {
            // (behind the barrier: wave 0 has seen the block of s_t h land before it came here)
            // "A" operand: s_t h transposed, lane (i, kg): rank i, tokens 16 h + 4 kg .. + 3 of the block
            union { uint64_t u; s16x4 v; } hv;
            hv.u = *reinterpret_cast<const uint64_t*>(hring + c.hslot * 1024 + (j * kTokenBlock + 16 * h + 4 * kg) * 2);
#pragma unroll
            for (int tl = 0; tl < 8; ++tl)
                dbacc[tl] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(hv.v, bv[tl], dbacc[tl], 0, 0, 0);
        }
    };

    Cursor pc, cc;                               // next item to fetch, next item to consume
    pc.sl = e0 / nbx;
    pc.bo = e0 - pc.sl * nbx;
    pc.slot = 0;
    pc.hslot = 0;
    cc = pc;
    if (n >= R - 1) {
        for (int d = 0; d < R - 1; ++d) {
            issue(pc);
            advance(pc);
        }
        int32_t it = 0;
        for (; it + R - 1 < n; ++it) {
            issue(pc);
            advance(pc);
            wait_item(std::integral_constant<int, R - 1>{});
            consume(cc, it);
            advance(cc);
        }
        gemm::static_for<0, R - 1>([&](auto t) {
            wait_item(std::integral_constant<int, R - 2 - decltype(t)::value>{});
            consume(cc, it);
            advance(cc);
            ++it;
        });
    } else {
        for (int32_t it = 0; it < n; ++it) {
            issue(pc);
            advance(pc);
            gemm::wait_vmcnt<0>();
            consume(cc, it);
            advance(cc);
        }
    }
    if (WITH_DB) flush_db(cur_sl);
}

// Second pass of the sliced projection: P = s_t * (sum of the slices' partial projections, in slice order),
// rounded to bf16 and written token-major and block-transposed.  Two token blocks per workgroup; thread
// (block, token, kg) owns the ranks 4 kg .. 4 kg + 3 of its token.
__global__ __launch_bounds__(256) void shrink_finish_kernel(PlanDev pd, const float* __restrict__ part,
                                                           const float* __restrict__ s,
                                                           uint16_t* __restrict__ P_tok,
                                                           uint16_t* __restrict__ P_blk, int32_t nsl)
{
    const int32_t bi = int32_t(blockIdx.x) * 2 + int32_t(threadIdx.x >> 7);
    if (bi >= pd.ntb) return;
    const int tok = (threadIdx.x >> 2) & 31, kg = threadIdx.x & 3;
    const TokenBlock b = pd.tb[bi];
    const int32_t r = pd.rank_off[b.task + 1] - b.rank_row0;
    const bool live = tok < b.nrows;
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    if (live) {
        const float* p = part + size_t(b.row0 + tok) * 16 + 4 * kg;
        const size_t pitch = size_t(pd.T) * 16;
        int32_t sl = 0;
        for (; sl + 8 <= nsl; sl += 8) {         // eight loads in flight (this kernel is all latency), added in slice order
            f32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f32x4*>(p + (sl + u) * pitch);
#pragma unroll
            for (int u = 0; u < 8; ++u) sum = sum + v[u];
        }
        for (; sl < nsl; ++sl) sum = sum + *reinterpret_cast<const f32x4*>(p + sl * pitch);
    }
    const float st = s[b.task];
    bf16x4 o;
#pragma unroll
    for (int v = 0; v < 4; ++v) o[v] = (__bf16)((live && 4 * kg + v < r) ? st * sum[v] : 0.f);
    if (live) *reinterpret_cast<bf16x4*>(P_tok + size_t(b.row0 + tok) * pd.r_pad + 4 * kg) = o;
    // block-transposed copy [block][rank][32 tokens]; tokens beyond the block hold 0
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        union { __bf16 b; uint16_t u; } c;
        c.b = o[v];
        P_blk[(size_t(bi) * pd.r_pad + 4 * kg + v) * kTokenBlock + tok] = c.u;
    }
}

namespace {
// once per device: the sliced kernel's rings need more dynamic LDS than the default limit
hipError_t sliced_setup()
{
    static std::atomic<int32_t> done[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (done[dev].load(std::memory_order_acquire) == 0) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&shrink_sliced_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kSlicedLds);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&shrink_sliced_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kSlicedLdsDb);
        if (e != hipSuccess) return e;
        done[dev].store(1, std::memory_order_release);
    }
    return hipSuccess;
}
}  // namespace

hipError_t shrink_mfma(const PlanDev& pd, const void* Z, const void* M, const float* s,
                       void* P_tok, void* P_blk, int32_t D, int32_t ldz, int32_t nproj, int32_t proj,
                       hipStream_t st, const SlicedShape& sliced, float* part, const void* Hblk, float* partb)
{
    if (pd.ntb == 0) return hipSuccess;
    if (sliced.nsl > 0 && part && nproj == 1) {
        hipError_t e = sliced_setup();
        if (e != hipSuccess) return e;
        // a fixed grid - one workgroup per compute unit of the chip this is written for - so that the split
        // of the items, and with it the order of every sum, does not depend on the device
        if (Hblk && partb && pd.fb_run_row)
            shrink_sliced_kernel<true><<<kSlicedGrid, 512, kSlicedLdsDb, st>>>(
                pd.tb, pd.rank_off, pd.ntb, pd.T, (const uint16_t*)Z, (const uint16_t*)M, part, D, ldz, sliced.nsl,
                (const uint16_t*)Hblk, partb, pd.fb_wg_run_off, pd.fb_run_row);
        else
            shrink_sliced_kernel<false><<<kSlicedGrid, 512, kSlicedLds, st>>>(
                pd.tb, pd.rank_off, pd.ntb, pd.T, (const uint16_t*)Z, (const uint16_t*)M, part, D, ldz, sliced.nsl,
                nullptr, nullptr, nullptr, nullptr);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        shrink_finish_kernel<<<(pd.ntb + 1) / 2, 256, 0, st>>>(pd, part, s, (uint16_t*)P_tok, (uint16_t*)P_blk, sliced.nsl);
        return hipGetLastError();
    }
    // rank blocks of the widest window (nproj = 1: of the widest task)
    const int nrb = (pd.r_max / nproj + 15) / 16;
    if (pd.shrink_group == 4 && nproj == 1 && ldz == D) {
        // ranks from about 24 up and a long batch: runs of four token blocks share the staged adapter rows
        if (nrb <= 2)
            shrink_lds_kernel<2, 2><<<pd.nsb, 256, 0, st>>>(pd, (const uint16_t*)Z, (const uint16_t*)M, s,
                                                            (uint16_t*)P_tok, (uint16_t*)P_blk, D);
        else if (nrb <= 4)
            shrink_lds_kernel<4, 2><<<pd.nsb, 256, 0, st>>>(pd, (const uint16_t*)Z, (const uint16_t*)M, s,
                                                            (uint16_t*)P_tok, (uint16_t*)P_blk, D);
        else
            shrink_lds_kernel<8, 2><<<pd.nsb, 256, 0, st>>>(pd, (const uint16_t*)Z, (const uint16_t*)M, s,
                                                            (uint16_t*)P_tok, (uint16_t*)P_blk, D);
        return hipGetLastError();
    }
#define LOBRA_SHRINK(NRB, DEPTH)                                                                       \
    shrink_mfma_kernel<NRB, 4, DEPTH><<<pd.ntb, 256, 0, st>>>(                                           \
        pd, (const uint16_t*)Z, (const uint16_t*)M, s, (uint16_t*)P_tok, (uint16_t*)P_blk, D, ldz, nproj, proj)
    if (nrb <= 1) LOBRA_SHRINK(1, 3);
    else if (nrb <= 2) LOBRA_SHRINK(2, 2);
    else if (nrb <= 4) LOBRA_SHRINK(4, 2);
    else LOBRA_SHRINK(8, 1);
#undef LOBRA_SHRINK
    return hipGetLastError();
}

// -------------------------------------------------------------------------------------------------
// grad stage 1: partial dM over one reduction chunk and 16 CW columns per workgroup of 4 waves
// (CW = 8: 128 columns; CW = 4: 64 columns, for large ranks, where the accumulators of a
// 128-column tile would leave room for one wave per SIMD only).
// Wave w takes the chunk's token blocks w, w+4, ...  For one block, lane (c, g) loads the 8 token
// rows 8g .. 8g+7 at the CW columns CW c .. CW c + CW-1 (so 16 lanes read 256 or 128 contiguous
// bytes of a row), transposes the 8 x CW patch in registers (v_perm_b32) into CW MFMA "B"
// operands - operand jj holds 8 tokens of column CW c + jj - and multiplies each with the "A"
// operand P_blk[rank][32 tokens].  MFMA jj therefore produces the columns {CW c + jj}, and a lane
// ends up with CW consecutive columns.  Rank blocks beyond the task's rank are skipped.
// The four waves' sums are combined through LDS in two steps (fixed order: ((w0+w2)+(w1+w3))).
// -------------------------------------------------------------------------------------------------
template <int NRB, int CW, bool STREAM>
__global__ __launch_bounds__(256) void grad_mfma_kernel(PlanDev pd, GradJob ja, GradJob jb, int32_t tiles_a, int32_t tiles_all)
{
    typedef uint32_t zvec __attribute__((ext_vector_type(CW / 2)));
    typedef float ovec __attribute__((ext_vector_type(4)));
    // The grid is one-dimensional in (chunk, column tile), column tile fastest, workgroup ids as dispatched
    // (round-robin over the XCDs): the workgroups in flight at one time then cover whole rows of a few chunks.
    // Measured against chunk fastest (the order of a two-dimensional grid) and against contiguous ranges per
    // XCD: 287 / 352 / 484 us at workload 5, 881 / 908 / 972 us at workload 4, 178 / 187 / 182 us at workload 3,
    // 50 / 51 / 50 us at workload 2 (58 for chunk fastest on a task-sorted batch).
#if LOBRA_GRAD_ORDER == 0        // chunk fastest, workgroup ids as dispatched
    const int32_t nch = int32_t(gridDim.x) / tiles_all;
    const int32_t tile_y = int32_t(blockIdx.x) / nch, chunk_x = int32_t(blockIdx.x) % nch;
#else
    const int32_t wi = LOBRA_GRAD_ORDER == 1 ? xcd_contiguous(blockIdx.x, gridDim.x) : int32_t(blockIdx.x);
    const int32_t tile_y = wi % tiles_all, chunk_x = wi / tiles_all;
#endif
    // one launch serves both gradients: column tiles [0, tiles_a) belong to job a, the rest to job b
    const bool first = tile_y < tiles_a;
    const uint16_t* __restrict__ P_blk = static_cast<const uint16_t*>(first ? ja.P : jb.P);
    const uint16_t* __restrict__ Z = static_cast<const uint16_t*>(first ? ja.Z : jb.Z);
    float* __restrict__ part = first ? ja.part : jb.part;
    const int32_t D = first ? ja.D : jb.D;
    const int32_t ldz = (first ? ja.ldz : jb.ldz) ? (first ? ja.ldz : jb.ldz) : D;   // row pitch of Z (elements)
    const int32_t nproj = first ? ja.nproj : jb.nproj;    // > 1: only the rank window of one projection
    const int32_t coltile = first ? tile_y : tile_y - tiles_a;
    const int32_t proj_in = first ? ja.proj : jb.proj;
    const int32_t proj = proj_in >= 0 ? proj_in : coltile * (16 * CW) / pd.dg;   // projection of this column tile
    const int32_t pcol0 = proj_in >= 0 ? 0 : proj * pd.dg;                      // its first column
    const int32_t ldp = (first ? ja.ldp : jb.ldp) ? (first ? ja.ldp : jb.ldp) : D;   // row pitch of part
    __shared__ float red[2][NRB][CW][64][4];
    const GradChunk ch = pd.chunks[chunk_x];
    const int32_t r = (pd.rank_off[ch.task + 1] - pd.rank_off[ch.task]) / nproj;
    const int32_t pofs = proj * r;                        // first rank of the window inside the task's rows
    const int32_t rb0 = blockIdx.y * NRB;                 // first rank block of this pass
    if (16 * rb0 >= r) return;                            // uniform: nothing to do for this task
    const int32_t nrb_t = min(NRB, (r - 16 * rb0 + 15) >> 4);   // rank blocks needed (uniform)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int32_t col = coltile * (16 * CW) + CW * c;
    const bool col_in = col < D;
    const bool tile_full = (coltile + 1) * (16 * CW) <= D;   // uniform: no lane of this tile is beyond D

    f32x4 acc[NRB][CW];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int jj = 0; jj < CW; ++jj) acc[rb][jj] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int32_t bi = ch.tb_begin + wave; bi < ch.tb_end; bi += 4) {
        const TokenBlock b = pd.tb[bi];
        zvec zin[8];
        // rows beyond the block repeat its last row; their P entries are zero
        if (tile_full) {
#pragma unroll
            for (int q = 0; q < 8; ++q)
                zin[q] = stream_load<STREAM>(reinterpret_cast<const zvec*>(Z + size_t(b.row0 + min(8 * g + q, b.nrows - 1)) * ldz + col));
        } else {
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int32_t row = b.row0 + min(8 * g + q, b.nrows - 1);
                zin[q] = col_in ? stream_load<STREAM>(reinterpret_cast<const zvec*>(Z + size_t(row) * ldz + col)) : zvec(0u);
            }
        }
        u32x4 pf[NRB];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
            if (rb < nrb_t)
                pf[rb] = *reinterpret_cast<const u32x4*>(
                    P_blk + (size_t(bi) * pd.r_pad + min(pofs + 16 * (rb0 + rb) + c, pd.r_pad - 1)) * kTokenBlock + 8 * g);
#pragma unroll
        for (int jj = 0; jj < CW; ++jj) {
            u32x4 f;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                f[e] = __builtin_amdgcn_perm(zin[2 * e + 1][jj >> 1], zin[2 * e][jj >> 1],
                                             (jj & 1) ? 0x07060302u : 0x05040100u);
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb)
                if (rb < nrb_t)
                    acc[rb][jj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(pf[rb]), as_bf16x8(f),
                                                                          acc[rb][jj], 0, 0, 0);
        }
    }
    // first waves 2, 3 hand their sums to waves 0, 1; then wave 1 hands its sum to wave 0
    if (wave >= 2)
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
            if (rb < nrb_t)
#pragma unroll
                for (int jj = 0; jj < CW; ++jj)
#pragma unroll
                    for (int v = 0; v < 4; ++v) red[wave - 2][rb][jj][lane][v] = acc[rb][jj][v];
    __syncthreads();
    if (wave < 2)
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
            if (rb < nrb_t)
#pragma unroll
                for (int jj = 0; jj < CW; ++jj)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[rb][jj][v] += red[wave][rb][jj][lane][v];
    __syncthreads();
    if (wave == 1)
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
            if (rb < nrb_t)
#pragma unroll
                for (int jj = 0; jj < CW; ++jj)
#pragma unroll
                    for (int v = 0; v < 4; ++v) red[0][rb][jj][lane][v] = acc[rb][jj][v];
    __syncthreads();
    if (wave == 0 && col_in) {
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int32_t p = 16 * (rb0 + rb) + 4 * g + v;
                if (p >= r) continue;
                float* dst = part + size_t(ch.part_row0 + pofs + p) * ldp + (col - pcol0);
#pragma unroll
                for (int j4 = 0; j4 < CW; j4 += 4) {
                    ovec o;
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) o[jj] = acc[rb][j4 + jj][v] + red[0][rb][j4 + jj][lane][v];
                    *reinterpret_cast<ovec*>(dst + j4) = o;
                }
            }
    }
}

// -------------------------------------------------------------------------------------------------
// grad stage 1 for ranks above 16 (NRB = 2: r_pad = 32, NRB = 4: r_pad >= 48, in passes of 64 ranks):
// partial dM over one reduction chunk and 256 columns per
// workgroup.  Wave w owns the 64 columns 64 w .. of the tile for ALL token blocks of the chunk (so its
// sums are final: no cross-wave reduction), and the P_blk tile of a token block ([16 NRB ranks][32
// tokens]) is staged in LDS once for the four waves instead of being fetched by each of them - with 64
// ranks it is as many bytes as the wave's own slice of Z.  Two LDS buffers alternate, one barrier per
// token block; the next block's Z rows and P tile are fetched before the current block is multiplied.
// Operand layouts as in grad_mfma_kernel with CW = 4.
// -------------------------------------------------------------------------------------------------
template <int NRB>
__global__ __launch_bounds__(256) void grad_lds_kernel(PlanDev pd, GradJob ja, GradJob jb, int32_t tiles_a, int32_t tiles_all)
{
    constexpr int CW = 4, TW = 4 * 16 * CW;     // rank blocks per pass, columns per lane, tile width
    typedef uint32_t zvec __attribute__((ext_vector_type(CW / 2)));
    typedef float ovec __attribute__((ext_vector_type(4)));
    __shared__ __attribute__((aligned(16))) unsigned char ps[2][16 * NRB * 64];
    // (work order as in grad_mfma_kernel)
#if LOBRA_GRAD_ORDER == 0        // chunk fastest, workgroup ids as dispatched
    const int32_t nch = int32_t(gridDim.x) / tiles_all;
    const int32_t tile_y = int32_t(blockIdx.x) / nch, chunk_x = int32_t(blockIdx.x) % nch;
#else
    const int32_t wi = LOBRA_GRAD_ORDER == 1 ? xcd_contiguous(blockIdx.x, gridDim.x) : int32_t(blockIdx.x);
    const int32_t tile_y = wi % tiles_all, chunk_x = wi / tiles_all;
#endif
    const bool first = tile_y < tiles_a;
    const uint16_t* __restrict__ P_blk = static_cast<const uint16_t*>(first ? ja.P : jb.P);
    const uint16_t* __restrict__ Z = static_cast<const uint16_t*>(first ? ja.Z : jb.Z);
    float* __restrict__ part = first ? ja.part : jb.part;
    const int32_t D = first ? ja.D : jb.D;
    const int32_t ldz = (first ? ja.ldz : jb.ldz) ? (first ? ja.ldz : jb.ldz) : D;
    const int32_t nproj = first ? ja.nproj : jb.nproj;
    const int32_t coltile = first ? tile_y : tile_y - tiles_a;
    const int32_t proj_in = first ? ja.proj : jb.proj;
    const int32_t proj = proj_in >= 0 ? proj_in : coltile * TW / pd.dg;   // pd.dg is a multiple of TW then
    const int32_t pcol0 = proj_in >= 0 ? 0 : proj * pd.dg;
    const int32_t ldp = (first ? ja.ldp : jb.ldp) ? (first ? ja.ldp : jb.ldp) : D;
    const GradChunk ch = pd.chunks[chunk_x];
    const int32_t r = (pd.rank_off[ch.task + 1] - pd.rank_off[ch.task]) / nproj;
    const int32_t pofs = proj * r;
    const int32_t rb0 = blockIdx.y * NRB;
    if (16 * rb0 >= r) return;                            // uniform
    const int32_t nrb_t = min(NRB, (r - 16 * rb0 + 15) >> 4);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int32_t col = coltile * TW + wave * (16 * CW) + CW * c;
    const bool col_in = col < D;

    f32x4 acc[NRB][CW];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int jj = 0; jj < CW; ++jj) acc[rb][jj] = f32x4{0.f, 0.f, 0.f, 0.f};

    // staging: thread tid moves 16 bytes: rank row tid / 4 of the pass, tokens 8 (tid % 4) ..
    const int prow = min(int(threadIdx.x >> 2), 16 * NRB - 1), pchunk = threadIdx.x & 3;
    const int32_t prank = min(pofs + 16 * rb0 + prow, pd.r_pad - 1);
    auto fetch_p = [&](int32_t bi) {
        return *reinterpret_cast<const u32x4*>(P_blk + (size_t(bi) * pd.r_pad + prank) * kTokenBlock + 8 * pchunk);
    };
    auto load_z = [&](zvec (&zin)[8], int32_t bi) {
        const TokenBlock b = pd.tb[bi];
#pragma unroll
        for (int q = 0; q < 8; ++q)   // rows beyond the block repeat its last row; their P entries are zero
            zin[q] = col_in ? stream_load<true>(reinterpret_cast<const zvec*>(Z + size_t(b.row0 + min(8 * g + q, b.nrows - 1)) * ldz + col))
                            : zvec(0u);
    };
    auto mac = [&](const zvec (&zin)[8], int buf) {
        u32x4 pf[NRB];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
            if (rb < nrb_t) pf[rb] = *reinterpret_cast<const u32x4*>(&ps[buf][(16 * rb + c) * 64 + 16 * g]);
#pragma unroll
        for (int jj = 0; jj < CW; ++jj) {
            u32x4 f;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                f[e] = __builtin_amdgcn_perm(zin[2 * e + 1][jj >> 1], zin[2 * e][jj >> 1],
                                             (jj & 1) ? 0x07060302u : 0x05040100u);
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb)
                if (rb < nrb_t)
                    acc[rb][jj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(pf[rb]), as_bf16x8(f),
                                                                          acc[rb][jj], 0, 0, 0);
        }
    };
    const int32_t n = ch.tb_end - ch.tb_begin;
    zvec za[8], zb[8];
    u32x4 preg = fetch_p(ch.tb_begin);
    load_z(za, ch.tb_begin);
    for (int32_t i = 0; i < n; i += 2) {
        // block i (Z rows in za), then block i + 1 (zb): the buffers alternate without register copies
        *reinterpret_cast<u32x4*>(&ps[0][prow * 64 + 16 * pchunk]) = preg;
        __syncthreads();                                 // tile i is staged; tile i - 1 has been consumed
        if (i + 1 < n) {
            preg = fetch_p(ch.tb_begin + i + 1);
            load_z(zb, ch.tb_begin + i + 1);
        }
        mac(za, 0);
        if (i + 1 >= n) break;                           // uniform
        *reinterpret_cast<u32x4*>(&ps[1][prow * 64 + 16 * pchunk]) = preg;
        __syncthreads();
        if (i + 2 < n) {
            preg = fetch_p(ch.tb_begin + i + 2);
            load_z(za, ch.tb_begin + i + 2);
        }
        mac(zb, 1);
    }
    if (!col_in) return;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int32_t p = 16 * (rb0 + rb) + 4 * g + v;
            if (p >= r) continue;
            ovec o;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) o[jj] = acc[rb][jj][v];
            *reinterpret_cast<ovec*>(part + size_t(ch.part_row0 + pofs + p) * ldp + (col - pcol0)) = o;
        }
}

hipError_t grad_mfma(const PlanDev& pd, const GradJob& ja, const GradJob& jb, hipStream_t st)
{
    if (pd.nchunks == 0) return hipSuccess;
    // rank blocks of the widest window (both jobs of a launch have the same nproj)
    const int nrb = ja.nproj > 1 ? (pd.r_max / ja.nproj + 15) / 16 : pd.r_pad / 16;
    const int NRB = nrb <= 1 ? 1 : (nrb <= 2 ? 2 : 4);
    // ranks above 16: the kernel that stages P_blk in LDS (its 256-column tiles must not straddle projections)
    if (NRB >= 2 &&
        (ja.proj >= 0 || pd.dg % 256 == 0) && (!jb.P || jb.proj >= 0 || pd.dg % 256 == 0)) {
        const int32_t ta = (ja.D + 255) / 256, tb = jb.P ? (jb.D + 255) / 256 : 0;
        const dim3 grid(uint32_t(pd.nchunks) * uint32_t(ta + tb), (nrb + 3) / 4);     // (plan creation bounds the product)
        if (NRB == 2) grad_lds_kernel<2><<<dim3(grid.x, 1), 256, 0, st>>>(pd, ja, jb, ta, ta + tb);
        else grad_lds_kernel<4><<<grid, 256, 0, st>>>(pd, ja, jb, ta, ta + tb);
        return hipGetLastError();
    }
    const int cw = NRB == 4 ? 4 : 8;
    const int32_t tw = 16 * cw;
    const int32_t tiles_a = (ja.D + tw - 1) / tw, tiles_b = jb.P ? (jb.D + tw - 1) / tw : 0;
    const dim3 grid(uint32_t(pd.nchunks) * uint32_t(tiles_a + tiles_b), (nrb + NRB - 1) / NRB);
    // token rows that cannot stay in the 256 MB infinity cache anyway are streamed past the caches
    const bool stream = int64_t(pd.T) * (int64_t(ja.D) + (jb.P ? jb.D : 0)) * 2 > (int64_t(512) << 20);
#define LOBRA_GRAD(NRB_, CW_)                                                                  \
    do {                                                                                       \
        if (stream) grad_mfma_kernel<NRB_, CW_, true><<<grid, 256, 0, st>>>(pd, ja, jb, tiles_a, tiles_a + tiles_b);  \
        else grad_mfma_kernel<NRB_, CW_, false><<<grid, 256, 0, st>>>(pd, ja, jb, tiles_a, tiles_a + tiles_b);        \
    } while (0)
    if (NRB == 1) LOBRA_GRAD(1, 8);
    else if (NRB == 2) LOBRA_GRAD(2, 8);
    else LOBRA_GRAD(4, 4);
#undef LOBRA_GRAD
    return hipGetLastError();
}

}  // namespace lobra
