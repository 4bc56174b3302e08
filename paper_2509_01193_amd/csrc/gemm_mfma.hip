// bf16 MFMA GEMM for gfx950 with the LoRA up projection fused into its epilogue:
//     C[T, N] = Z[T, K] * op(W) + P[T, r] * M_t[r, N]
// forward : Z = x,  op(W) = W   (W stored [K][N], N fastest),  P = s_t A_t x_i,  M = B  -> y
// backward: Z = dy, op(W) = W^T (W stored [N][K], K fastest),  P = s_t B_t dy_i, M = A  -> dx
// (paper section 2.1: X W + X (down)(up); section 1: one shared base product for the fused batch,
// a per-task adapter product on top of it).
//
// Tiling: 256 x 256 x 64 per workgroup of 4 waves (2 x 2), every wave owns 128 x 128 as 4 x 4
// v_mfma_f32_32x32x16_bf16 blocks (256 fp32 accumulators per lane), LDS double buffered,
// global -> register -> LDS prefetch of the next K tile while the current one is multiplied.
// The MFMA "A" operand is fed from W and the "B" operand from Z, so a lane ends up with four
// consecutive output columns of one row, which packs into 8-byte LDS writes in the epilogue.
//
// LDS layouts
//   Z tile, and the W tile when K is fastest: [256 rows][64 k], 16-byte chunks XOR-swizzled
//       with (row >> 1) & 7 so that the 16 rows of one ds_read_b128 pass hit 16 bank groups.
//   W tile when N is fastest (forward): [64 k][256 + 32 n]; the MFMA operand (8 consecutive k
//       of one column) is gathered with two ds_read_b64_tr_b16, the row pitch of 576 bytes puts
//       the 4 k-rows of one pass in different bank quarters.
//   C staging in the epilogue: per wave [128 rows][128 + 8 cols] bf16.
#include "kernels.h"

namespace lobra {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int ZT_BYTES = BM * BK * 2;               // 32 KiB
constexpr int WKN_PITCH = BN + 32;                  // elements
constexpr int WT_KN_BYTES = BK * WKN_PITCH * 2;     // 36 KiB
constexpr int WT_NK_BYTES = BN * BK * 2;            // 32 KiB
constexpr int CS_PITCH = 128 + 8;                   // elements, per-wave C staging
constexpr int CS_BYTES = 4 * 128 * CS_PITCH * 2;    // 136 KiB

template <bool W_KN> constexpr int lds_bytes()
{
    const int loop = 2 * ZT_BYTES + 2 * (W_KN ? WT_KN_BYTES : WT_NK_BYTES);
    return loop > CS_BYTES ? loop : CS_BYTES;
}

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v)
{
    union { u32x4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

}  // namespace

template <bool W_KN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_mfma_kernel(PlanDev pd, const uint16_t* __restrict__ Z, const uint16_t* __restrict__ W,
                      const uint16_t* __restrict__ P, const uint16_t* __restrict__ M,
                      uint16_t* __restrict__ C, int32_t K, int32_t N, int32_t ldw,
                      int32_t tiles_m, int32_t tiles_n)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int32_t T = pd.T;

    // ---- workgroup -> tile: consecutive ids go to different XCDs, so give each XCD a contiguous
    //      range of the tile order; inside it, 8 tile-rows share one sweep over the tile-columns.
    int32_t tile_m, tile_n;
    {
        const int32_t ntiles = tiles_m * tiles_n;
        const int32_t wg = blockIdx.x;
        const int32_t xcd = wg & 7, idx = wg >> 3;
        const int32_t per = ntiles >> 3, rem = ntiles & 7;
        const int32_t id = xcd * per + (xcd < rem ? xcd : rem) + idx;   // XCD x holds per + (x < rem)
        constexpr int GM = 8;
        const int32_t group = id / (GM * tiles_n);
        const int32_t first_m = group * GM;
        const int32_t gsz = min(tiles_m - first_m, GM);
        const int32_t in = id - group * GM * tiles_n;
        tile_m = first_m + in % gsz;
        tile_n = in / gsz;
    }
    const int32_t row0 = tile_m * BM, col0 = tile_n * BN;

    constexpr int WT_BYTES = W_KN ? WT_KN_BYTES : WT_NK_BYTES;
    auto zs = [&](int buf) { return lds + buf * ZT_BYTES; };
    auto ws = [&](int buf) { return lds + 2 * ZT_BYTES + buf * WT_BYTES; };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    u32x4 zreg[8], wreg[8];
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    auto gload = [&](int32_t k0) {
        {   // Z tile: thread -> chunk tid % 8 of rows tid / 8 + 32 i
            const int c = tid & 7, rb = tid >> 3;
            const int32_t k = k0 + 8 * c;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int32_t row = row0 + rb + 32 * i;
                zreg[i] = (row < T && k < K)
                              ? *reinterpret_cast<const u32x4*>(Z + size_t(row) * K + k) : zero4;
            }
        }
        if (W_KN) {   // W tile [64 k][256 n]: thread -> n chunk tid % 32 of k rows tid / 32 + 8 i
            const int nc = tid & 31, kb = tid >> 5;
            const int32_t n = col0 + 8 * nc;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int32_t k = k0 + kb + 8 * i;
                wreg[i] = (k < K && n < N)
                              ? *reinterpret_cast<const u32x4*>(W + size_t(k) * ldw + n) : zero4;
            }
        } else {      // W tile [256 n][64 k]
            const int c = tid & 7, rb = tid >> 3;
            const int32_t k = k0 + 8 * c;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int32_t n = col0 + rb + 32 * i;
                wreg[i] = (n < N && k < K)
                              ? *reinterpret_cast<const u32x4*>(W + size_t(n) * ldw + k) : zero4;
            }
        }
    };
    auto lstore = [&](int buf) {
        {
            const int c = tid & 7, rb = tid >> 3;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = rb + 32 * i;
                *reinterpret_cast<u32x4*>(zs(buf) + row * (BK * 2) + swz(row, c) * 16) = zreg[i];
            }
        }
        if (W_KN) {
            const int nc = tid & 31, kb = tid >> 5;
#pragma unroll
            for (int i = 0; i < 8; ++i)
                *reinterpret_cast<u32x4*>(ws(buf) + (kb + 8 * i) * (WKN_PITCH * 2) + nc * 16) = wreg[i];
        } else {
            const int c = tid & 7, rb = tid >> 3;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int row = rb + 32 * i;
                *reinterpret_cast<u32x4*>(ws(buf) + row * (BK * 2) + swz(row, c) * 16) = wreg[i];
            }
        }
    };
    // one K tile: 4 K steps of 16, each 4 + 4 operand fragments and 16 MFMAs
    auto compute = [&](int buf) {
        const int l32 = lane & 31, lh = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 zf[4], wf[4];
#pragma unroll
            for (int mb = 0; mb < 4; ++mb) {
                const int row = wm * 128 + mb * 32 + l32;
                zf[mb] = *reinterpret_cast<const bf16x8*>(zs(buf) + row * (BK * 2) + swz(row, 2 * ks + lh) * 16);
            }
            if (W_KN) {
                const int s = lane & 15, g = lane >> 4;
                const int krow = 16 * ks + 8 * (g >> 1) + (s >> 2);
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {
                    const int n = wn * 128 + nb * 32 + 16 * (g & 1) + 4 * (s & 3);
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
                for (int nb = 0; nb < 4; ++nb) {
                    const int row = wn * 128 + nb * 32 + l32;
                    wf[nb] = *reinterpret_cast<const bf16x8*>(ws(buf) + row * (BK * 2) + swz(row, 2 * ks + lh) * 16);
                }
            }
#pragma unroll
            for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                for (int nb = 0; nb < 4; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[nb], zf[mb], acc[mb][nb], 0, 0, 0);
        }
    };

    // ---- main loop ----------------------------------------------------------------------------
    const int32_t KT = (K + BK - 1) / BK;
    gload(0);
    lstore(0);
    __syncthreads();
    for (int32_t kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) gload((kt + 1) * BK);
        compute(buf);
        if (kt + 1 < KT) lstore(buf ^ 1);
        __syncthreads();
    }

    // ---- fused up projection: one extra K step of 16 ranks per (segment in this tile, rank block)
    {
        const int l32 = lane & 31, lh = lane >> 5;
        const int32_t row_end = min(row0 + BM, T);
        int32_t sg = pd.rowblk_seg[row0 / kRowBlock];
        for (; sg < pd.nseg && pd.cseg_off[sg] < row_end; ++sg) {
            const int32_t t = pd.cseg_task[sg];
            if (t < 0) continue;
            const int32_t lo = max(pd.cseg_off[sg], row0), hi = min(pd.cseg_off[sg + 1], row_end);
            const int32_t r0 = pd.rank_off[t], r = pd.rank_off[t + 1] - r0;
            // the wave's rows are row0 + wm*128 .. +127
            if (hi <= row0 + wm * 128 || lo >= row0 + wm * 128 + 128) continue;
            for (int32_t kk = 0; kk < r; kk += 16) {
                bf16x8 wf[4];
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {
                    const int32_t n = col0 + wn * 128 + nb * 32 + l32;
                    union { uint16_t h[8]; bf16x8 b; } c;
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        const int32_t p = kk + 8 * lh + q;
                        c.h[q] = (p < r && n < N) ? M[size_t(r0 + p) * N + n] : uint16_t(0);
                    }
                    wf[nb] = c.b;
                }
#pragma unroll
                for (int mb = 0; mb < 4; ++mb) {
                    const int32_t rb = row0 + wm * 128 + mb * 32;
                    if (hi <= rb || lo >= rb + 32) continue;        // wave-uniform
                    const int32_t row = rb + l32;
                    const u32x4 pv = (row >= lo && row < hi)
                        ? *reinterpret_cast<const u32x4*>(P + size_t(row) * pd.r_pad + kk + 8 * lh) : zero4;
                    const bf16x8 pf = as_bf16x8(pv);
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb)
                        acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[nb], pf, acc[mb][nb], 0, 0, 0);
                }
            }
        }
    }

    // ---- epilogue: fp32 -> bf16, stage the wave's 128 x 128 block in LDS, store 16 bytes per lane
    {
        unsigned char* cs = lds + wave * (128 * CS_PITCH * 2);
        const int l32 = lane & 31, lh = lane >> 5;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 o;
#pragma unroll
                    for (int q = 0; q < 4; ++q) o[q] = (__bf16)acc[mb][nb][4 * g + q];
                    const int m = mb * 32 + l32, n = nb * 32 + 8 * g + 4 * lh;
                    *reinterpret_cast<bf16x4*>(cs + (m * CS_PITCH + n) * 2) = o;
                }
        __syncthreads();
        const int cchunk = lane & 15, rsub = lane >> 4;
        const int32_t col = col0 + wn * 128 + cchunk * 8;
#pragma unroll 4
        for (int i = 0; i < 32; ++i) {
            const int m = i * 4 + rsub;
            const int32_t row = row0 + wm * 128 + m;
            const u32x4 v = *reinterpret_cast<const u32x4*>(cs + (m * CS_PITCH + cchunk * 8) * 2);
            if (row < T && col < N) *reinterpret_cast<u32x4*>(C + size_t(row) * N + col) = v;
        }
    }
}

hipError_t gemm_mfma(const PlanDev& pd, bool transW, const void* Z, const void* W, const void* P,
                     const void* M, void* C, int32_t K, int32_t N, int32_t ldw, hipStream_t st)
{
    if (pd.T == 0) return hipSuccess;
    const int32_t tiles_m = (pd.T + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int64_t ntiles = int64_t(tiles_m) * tiles_n;
    if (ntiles > 0x7fffffff) return hipErrorInvalidValue;
    static bool attr_set[2] = {false, false};
    hipError_t e;
    if (!transW) {
        constexpr int bytes = lds_bytes<true>();
        if (!attr_set[0]) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_kernel<true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
            if (e != hipSuccess) return e;
            attr_set[0] = true;
        }
        gemm_mfma_kernel<true><<<dim3(uint32_t(ntiles)), 256, bytes, st>>>(
            pd, (const uint16_t*)Z, (const uint16_t*)W, (const uint16_t*)P, (const uint16_t*)M,
            (uint16_t*)C, K, N, ldw, tiles_m, tiles_n);
    } else {
        constexpr int bytes = lds_bytes<false>();
        if (!attr_set[1]) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_kernel<false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
            if (e != hipSuccess) return e;
            attr_set[1] = true;
        }
        gemm_mfma_kernel<false><<<dim3(uint32_t(ntiles)), 256, bytes, st>>>(
            pd, (const uint16_t*)Z, (const uint16_t*)W, (const uint16_t*)P, (const uint16_t*)M,
            (uint16_t*)C, K, N, ldw, tiles_m, tiles_n);
    }
    return hipGetLastError();
}

}  // namespace lobra
