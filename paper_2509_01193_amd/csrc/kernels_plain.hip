// Plain fp32-FMA kernels: the fp32 path of the library, and (on bf16 storage) a slow
// cross-check of the MFMA kernels.  Straightforward tiling, no matrix cores.
//
// They implement the four products of the LoRA layer (paper section 2.1: X W + X (down)(up),
// applied per task to a fused batch, section 1) and their derivatives:
//   shrink      P = s_t Z M_t^T            (Z = x, M = A: s_t A_t x_i;  Z = dy, M = B: s_t B_t dy_i)
//   gemm        C = Z op(W) + P M_t        (y = x W + P B_t;  dx = dy W^T + P A_t)
//   gradreduce  dM_t = sum_i P_i^T Z_i     (dB_t from P = s h, Z = dy;  dA_t from P = s g, Z = x)
#include "kernels.h"

namespace lobra {

// -------------------------------------------------------------------------------------------
// shrink: one workgroup per token block; wave w takes the rows 8w .. 8w+7 and, eight ranks at a
// time, keeps an 8 x 8 block of sums in registers while its lanes stride over D four elements at
// a time (so a rank row fetched from the cache serves eight token rows); the 64 lanes' partial
// sums are combined with shuffles at the end.  Widths that are not a multiple of 4 take the
// same loop one element at a time.
// -------------------------------------------------------------------------------------------
namespace {
template <typename E> struct Vec4;
template <> struct Vec4<float> {
    static __device__ __forceinline__ void load(const float* p, size_t i, float (&v)[4])
    {
        typedef float f4 __attribute__((ext_vector_type(4)));
        const f4 t = *reinterpret_cast<const f4*>(p + i);
        v[0] = t[0], v[1] = t[1], v[2] = t[2], v[3] = t[3];
    }
};
template <> struct Vec4<uint16_t> {
    static __device__ __forceinline__ void load(const uint16_t* p, size_t i, float (&v)[4])
    {
        typedef uint32_t u2 __attribute__((ext_vector_type(2)));
        const u2 t = *reinterpret_cast<const u2*>(p + i);
        v[0] = __uint_as_float(t[0] << 16), v[1] = __uint_as_float(t[0] & 0xffff0000u);
        v[2] = __uint_as_float(t[1] << 16), v[3] = __uint_as_float(t[1] & 0xffff0000u);
    }
};
}  // namespace

template <typename E, int VW>   // VW: elements per lane and step (4, or 1 for odd widths)
__global__ __launch_bounds__(256) void plain_shrink_kernel(PlanDev pd, const E* __restrict__ Z,
                                                           const E* __restrict__ M,
                                                           const float* __restrict__ s,
                                                           float* __restrict__ P, int32_t D, int32_t ldz,
                                                           int32_t nproj, int32_t proj)
{
    // nproj > 1 (fused shared-input projections): projection `proj` only - Z is its column block of
    // dy (row pitch ldz), M its rows of the compact up factors, and of the task's ranks the window
    // [proj r, (proj + 1) r) is read and written
    const TokenBlock b = pd.tb[blockIdx.x];
    const int32_t r = (pd.rank_off[b.task + 1] - pd.rank_off[b.task]) / nproj;
    const int32_t pofs = proj * r;
    const int32_t plim = proj == nproj - 1 ? pd.r_max - pofs : r;   // ranks (and zero padding) stored here
    const float st = s[b.task];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int32_t rr0 = 8 * wave;
    if (rr0 >= b.nrows) return;
    size_t zoff[8];          // rows beyond the block repeat its last row; their sums are not stored
#pragma unroll
    for (int i = 0; i < 8; ++i) zoff[i] = size_t(b.row0 + min(rr0 + i, b.nrows - 1)) * ldz;
    for (int32_t p0 = 0; p0 < plim; p0 += 8) {
        float acc[8][8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[i][q] = 0.f;
        if (p0 < r) {
            size_t moff[8];  // ranks beyond r_t repeat the last rank row; their sums are not stored
#pragma unroll
            for (int q = 0; q < 8; ++q) moff[q] = size_t(b.rank_row0 + pofs + min(p0 + q, r - 1)) * D;
            for (int32_t k = VW * lane; k < D; k += VW * 64) {
                float z[8][VW], m[8][VW];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    if constexpr (VW == 4) Vec4<E>::load(Z, zoff[i] + k, z[i]);
                    else z[i][0] = Elem<E>::load(Z, zoff[i] + k);
                }
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    if constexpr (VW == 4) Vec4<E>::load(M, moff[q] + k, m[q]);
                    else m[q][0] = Elem<E>::load(M, moff[q] + k);
                }
#pragma unroll
                for (int e = 0; e < VW; ++e)
#pragma unroll
                    for (int i = 0; i < 8; ++i)
#pragma unroll
                        for (int q = 0; q < 8; ++q) acc[i][q] = fmaf(z[i][e], m[q][e], acc[i][q]);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    for (int off = 32; off > 0; off >>= 1) acc[i][q] += __shfl_xor(acc[i][q], off, 64);
        }
        // lane 8 i + q stores the sum of row i and rank p0 + q
        float v = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (lane == 8 * i + q) v = acc[i][q];
        const int i = lane >> 3, q = lane & 7;
        if (rr0 + i < b.nrows && p0 + q < plim)
            P[size_t(b.row0 + rr0 + i) * pd.r_max + pofs + p0 + q] = (p0 + q < r) ? st * v : 0.f;
    }
}

hipError_t plain_shrink(const PlanDev& pd, int dtype, const void* Z, const void* M, const float* s,
                        float* P, int32_t D, hipStream_t st, int32_t ldz, int32_t nproj, int32_t proj)
{
    if (pd.ntb == 0) return hipSuccess;
    if (ldz == 0) ldz = D;
    const bool vec = (D & 3) == 0 && (ldz & 3) == 0;   // rows then start on 16-byte (fp32) or 8-byte (bf16) boundaries
#define LOBRA_PLAIN_SHRINK(E, VW) \
    plain_shrink_kernel<E, VW><<<pd.ntb, 256, 0, st>>>(pd, (const E*)Z, (const E*)M, s, P, D, ldz, nproj, proj)
    if (dtype == LOBRA_F32) {
        if (vec) LOBRA_PLAIN_SHRINK(float, 4); else LOBRA_PLAIN_SHRINK(float, 1);
    } else {
        if (vec) LOBRA_PLAIN_SHRINK(uint16_t, 4); else LOBRA_PLAIN_SHRINK(uint16_t, 1);
    }
#undef LOBRA_PLAIN_SHRINK
    return hipGetLastError();
}

// -------------------------------------------------------------------------------------------
// gemm: 64 x 64 tile, K step 16, 4 x 4 outputs per thread, the adapter term as further K steps per segment
// -------------------------------------------------------------------------------------------
template <typename E, bool TRANSW>
__global__ __launch_bounds__(256) void plain_gemm_kernel(PlanDev pd, const E* __restrict__ Z,
                                                         const E* __restrict__ W,
                                                         const float* __restrict__ P,
                                                         const E* __restrict__ M, E* __restrict__ C,
                                                         int32_t K, int32_t N, int32_t ldw, int32_t ldc,
                                                         int32_t nproj, int32_t proj)
{
    // ldc: row pitch of C.  nproj > 1: projection `proj` of a fused shared-input call - of every task's
    // ranks only the window [proj r, (proj + 1) r) takes part (columns of P, rows of M; M pitch N)
    __shared__ float Zs[16][64 + 4];
    __shared__ float Ws[16][64 + 4];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int32_t row0 = blockIdx.y * 64, col0 = blockIdx.x * 64;
    const int32_t T = pd.T;
    float acc[4][4] = {};
    // each thread moves 4 elements of the Z tile and 4 of the W tile per K step; the elements of
    // step k0 + 16 are fetched into registers before the products of step k0 are formed
    float zr[4], wr[4];
    auto fetch = [&](int32_t k0) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = tid + 256 * u;
            {   // Z tile: 64 rows x 16 k, k fastest in memory
                const int kk = e & 15, m = e >> 4;
                const int32_t row = row0 + m, k = k0 + kk;
                zr[u] = (row < T && k < K) ? Elem<E>::load(Z, size_t(row) * K + k) : 0.f;
            }
            if (TRANSW) {   // op(W)[k][n] = W[n*ldw + k]: k fastest
                const int kk = e & 15, nn = e >> 4;
                const int32_t n = col0 + nn, k = k0 + kk;
                wr[u] = (n < N && k < K) ? Elem<E>::load(W, size_t(n) * ldw + k) : 0.f;
            } else {        // op(W)[k][n] = W[k*ldw + n]: n fastest
                const int nn = e & 63, kk = e >> 6;
                const int32_t n = col0 + nn, k = k0 + kk;
                wr[u] = (n < N && k < K) ? Elem<E>::load(W, size_t(k) * ldw + n) : 0.f;
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = tid + 256 * u;
            Zs[e & 15][e >> 4] = zr[u];
            if (TRANSW) Ws[e & 15][e >> 4] = wr[u];
            else Ws[e >> 6][e & 63] = wr[u];
        }
    };
    fetch(0);
    for (int32_t k0 = 0; k0 < K; k0 += 16) {
        stash();
        __syncthreads();
        if (k0 + 16 < K) fetch(k0 + 16);
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = Zs[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Ws[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    // adapter term: for every adapter segment that crosses the tile, the task's ranks are further K steps of
    // the same tile product, acc += P[rows, ranks] M_t[ranks, cols], with the rows outside the segment masked
    // (the loops are uniform over the workgroup)
    {
        const int32_t row_end = min(row0 + 64, T);
        for (int32_t sg = pd.rowblk_seg[row0 / kRowBlock]; sg < pd.nseg; ++sg) {
            const int32_t seg_lo = pd.cseg_off[sg];
            if (seg_lo >= row_end) break;
            const int32_t t = pd.cseg_task[sg];
            if (t < 0) continue;
            const int32_t lo = max(seg_lo, row0), hi = min(pd.cseg_off[sg + 1], row_end);
            const int32_t r = (pd.rank_off[t + 1] - pd.rank_off[t]) / nproj, pofs = proj * r;
            const int32_t r0 = pd.rank_off[t] + pofs;
            for (int32_t c0 = 0; c0 < r; c0 += 16) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int e = tid + 256 * u;
                    {
                        const int kk = e & 15, m = e >> 4;
                        const int32_t row = row0 + m;
                        Zs[kk][m] = (row >= lo && row < hi && c0 + kk < r) ? P[size_t(row) * pd.r_max + pofs + c0 + kk] : 0.f;
                    }
                    {
                        const int nn = e & 63, kk = e >> 6;
                        const int32_t n = col0 + nn;
                        Ws[kk][nn] = (c0 + kk < r && n < N) ? Elem<E>::load(M, size_t(r0 + c0 + kk) * N + n) : 0.f;
                    }
                }
                __syncthreads();
#pragma unroll
                for (int kk = 0; kk < 16; ++kk) {
                    float a[4], b[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) a[i] = Zs[kk][ty * 4 + i];
#pragma unroll
                    for (int j = 0; j < 4; ++j) b[j] = Ws[kk][tx * 4 + j];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
                }
                __syncthreads();
            }
        }
    }
    for (int i = 0; i < 4; ++i) {
        const int32_t row = row0 + ty * 4 + i;
        if (row >= T) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int32_t col = col0 + tx * 4 + j;
            if (col < N) Elem<E>::store(C, size_t(row) * ldc + col, acc[i][j]);
        }
    }
}

hipError_t plain_gemm(const PlanDev& pd, int dtype, bool transW, const void* Z, const void* W,
                      const float* P, const void* M, void* C, int32_t K, int32_t N, int32_t ldw,
                      hipStream_t st, int32_t ldc, int32_t nproj, int32_t proj)
{
    if (pd.T == 0) return hipSuccess;
    if (ldc == 0) ldc = N;
    const dim3 grid((N + 63) / 64, (pd.T + 63) / 64);
    if (grid.y > 65535u) return hipErrorInvalidValue;
#define LOBRA_LAUNCH(E, TR) \
    plain_gemm_kernel<E, TR><<<grid, 256, 0, st>>>(pd, (const E*)Z, (const E*)W, P, (const E*)M, (E*)C, K, N, ldw, ldc, nproj, proj)
    if (dtype == LOBRA_F32) {
        if (transW) LOBRA_LAUNCH(float, true); else LOBRA_LAUNCH(float, false);
    } else {
        if (transW) LOBRA_LAUNCH(uint16_t, true); else LOBRA_LAUNCH(uint16_t, false);
    }
#undef LOBRA_LAUNCH
    return hipGetLastError();
}

// -------------------------------------------------------------------------------------------
// gradreduce stage 1: one workgroup per (chunk, 256 columns), one thread per column
// -------------------------------------------------------------------------------------------
template <typename E, typename PE>
__global__ __launch_bounds__(256) void plain_gradreduce_kernel(PlanDev pd, const PE* __restrict__ P,
                                                               int32_t pstride, const E* __restrict__ Z,
                                                               float* __restrict__ part, int32_t D, int32_t ldz,
                                                               int32_t nproj, int32_t proj, int32_t tiles_a,
                                                               const PE* __restrict__ P2, const E* __restrict__ Z2,
                                                               float* __restrict__ part2, int32_t D2)
{
    // nproj > 1: projection `proj` of a fused call - Z is its column block (row pitch ldz), and of the
    // task's ranks only the window [proj r, (proj + 1) r) is reduced (columns of P, rows of part).
    // One launch can serve two gradients (nproj = 1): column tiles from tiles_a on belong to (P2, Z2, part2, D2).
    int32_t coltile = blockIdx.y;
    if (coltile >= tiles_a) {
        coltile -= tiles_a;
        P = P2;
        Z = Z2;
        part = part2;
        D = ldz = D2;
    }
    const GradChunk c = pd.chunks[blockIdx.x];
    const int32_t r = (pd.rank_off[c.task + 1] - pd.rank_off[c.task]) / nproj;
    const int32_t pofs = proj * r;
    const int32_t col = coltile * 256 + threadIdx.x;
    const bool live = col < D;
    for (int32_t p0 = 0; p0 < r; p0 += 16) {
        float acc[16] = {};
        for (int32_t bi = c.tb_begin; bi < c.tb_end; ++bi) {
            const TokenBlock b = pd.tb[bi];
            // four rows at a time, so that their loads are in flight together (rows in order:
            // the sum does not depend on the grouping)
            for (int32_t rr = 0; rr < b.nrows; rr += 4) {
                float z[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    z[u] = (live && rr + u < b.nrows) ? Elem<E>::load(Z, size_t(b.row0 + rr + u) * ldz + col) : 0.f;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (rr + u >= b.nrows) break;
                    const size_t row = size_t(b.row0 + rr + u);
#pragma unroll
                    for (int q = 0; q < 16; ++q)
                        if (p0 + q < r) acc[q] = fmaf(Elem<PE>::load(P, row * pstride + pofs + p0 + q), z[u], acc[q]);
                }
            }
        }
        if (live)
#pragma unroll
            for (int q = 0; q < 16; ++q)
                if (p0 + q < r) part[size_t(c.part_row0 + pofs + p0 + q) * D + col] = acc[q];
    }
}

// stage 2: out[R, col] (+)= sum over the chunks of task(R), in chunk order.  One workgroup per
// (rank row, 1024 columns), one float4 per thread, four chunk loads in flight.
__global__ __launch_bounds__(256) void reduce_partials_kernel(PlanDev pd, GradJob ja, GradJob jb,
                                                              int32_t tiles_a, int accumulate)
{
    const bool first = int32_t(blockIdx.y) < tiles_a;
    const float* __restrict__ part = first ? ja.part : jb.part;
    float* __restrict__ out = first ? ja.out : jb.out;
    const int32_t D = first ? ja.D : jb.D;
    const int32_t coltile = first ? int32_t(blockIdx.y) : int32_t(blockIdx.y) - tiles_a;
    const int32_t R = blockIdx.x;
    int32_t t = 0;
    while (pd.rank_off[t + 1] <= R) ++t;
    const int32_t p = R - pd.rank_off[t];
    const int32_t col = coltile * 1024 + threadIdx.x * 4;
    if (col >= D) return;
    // the partial sums of a task: one per reduction chunk, or (fcnt) one per run of the fused pass that covers
    // this thread's 512-column slice
    const int32_t* fcnt = first ? ja.fcnt : jb.fcnt;
    const int32_t c0 = fcnt ? 0 : pd.task_chunk_off[t];
    const int32_t c1 = fcnt ? fcnt[t * (first ? ja.fnsl : jb.fnsl) + (col >> 9)] : pd.task_chunk_off[t + 1];
    const int32_t frow = fcnt ? (first ? ja.frow0 : jb.frow0)[t] + p : 0;
    const int nv = min(4, D - col);                 // D need not be a multiple of 4 on the fp32 path
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    auto row_ptr = [&](int32_t c) {
        return part + size_t(fcnt ? frow + 16 * c : pd.chunks[c].part_row0 + p) * D + col;
    };
    if (nv == 4 && (D & 3) == 0) {
        typedef float f4 __attribute__((ext_vector_type(4)));
        int32_t c = c0;
        for (; c + 8 <= c1; c += 8) {            // eight loads in flight, added in order
            f4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f4*>(row_ptr(c + u));
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] += v[u][q];
        }
        for (; c + 4 <= c1; c += 4) {
            const f4 v0 = *reinterpret_cast<const f4*>(row_ptr(c));
            const f4 v1 = *reinterpret_cast<const f4*>(row_ptr(c + 1));
            const f4 v2 = *reinterpret_cast<const f4*>(row_ptr(c + 2));
            const f4 v3 = *reinterpret_cast<const f4*>(row_ptr(c + 3));
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = (((acc[q] + v0[q]) + v1[q]) + v2[q]) + v3[q];
        }
        for (; c < c1; ++c) {
            const f4 v = *reinterpret_cast<const f4*>(row_ptr(c));
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] += v[q];
        }
        float* o = out + size_t(R) * D + col;
        f4 res;
#pragma unroll
        for (int q = 0; q < 4; ++q) res[q] = accumulate ? o[q] + acc[q] : acc[q];
        *reinterpret_cast<f4*>(o) = res;
    } else {
        for (int32_t c = c0; c < c1; ++c)
            for (int q = 0; q < nv; ++q) acc[q] += row_ptr(c)[q];
        float* o = out + size_t(R) * D + col;
        for (int q = 0; q < nv; ++q) o[q] = accumulate ? o[q] + acc[q] : acc[q];
    }
}

hipError_t reduce_partials(const PlanDev& pd, const GradJob& ja, const GradJob& jb, bool accumulate,
                           hipStream_t st)
{
    if (pd.R_tot == 0) return hipSuccess;
    const int32_t tiles_a = (ja.D + 1023) / 1024, tiles_b = jb.out ? (jb.D + 1023) / 1024 : 0;
    const dim3 grid(pd.R_tot, tiles_a + tiles_b);
    if (grid.y > 65535u) return hipErrorInvalidValue;
    reduce_partials_kernel<<<grid, 256, 0, st>>>(pd, ja, jb, tiles_a, accumulate ? 1 : 0);
    return hipGetLastError();
}

hipError_t plain_grad_stage1(const PlanDev& pd, int dtype, bool p_bf16, const void* P, const void* Z,
                             float* part, int32_t D, hipStream_t st, int32_t ldz, int32_t nproj, int32_t proj,
                             const void* P2, const void* Z2, float* part2, int32_t D2)
{
    // (P2, Z2, part2, D2): a second gradient served by the same launch (nproj = 1 only), or P2 = NULL
    if (pd.nchunks == 0) return hipSuccess;
    if (ldz == 0) ldz = D;
    if (P2 && nproj != 1) return hipErrorInvalidValue;
    const int32_t tiles_a = (D + 255) / 256, tiles_b = P2 ? (D2 + 255) / 256 : 0;
    const dim3 grid(pd.nchunks, tiles_a + tiles_b);
    if (grid.y > 65535u) return hipErrorInvalidValue;
    if (dtype == LOBRA_F32)
        plain_gradreduce_kernel<float, float><<<grid, 256, 0, st>>>(pd, (const float*)P, pd.r_max, (const float*)Z, part, D, ldz, nproj, proj,
                                                                     tiles_a, (const float*)P2, (const float*)Z2, part2, D2);
    else if (!p_bf16)
        plain_gradreduce_kernel<uint16_t, float><<<grid, 256, 0, st>>>(pd, (const float*)P, pd.r_max, (const uint16_t*)Z, part, D, ldz, nproj, proj,
                                                                        tiles_a, (const float*)P2, (const uint16_t*)Z2, part2, D2);
    else
        plain_gradreduce_kernel<uint16_t, uint16_t><<<grid, 256, 0, st>>>(pd, (const uint16_t*)P, pd.r_pad, (const uint16_t*)Z, part, D, ldz, nproj, proj,
                                                                           tiles_a, (const uint16_t*)P2, (const uint16_t*)Z2, part2, D2);
    return hipGetLastError();
}

// -------------------------------------------------------------------------------------------
// fused multi-adapter Adam (Kingma & Ba, Algorithm 1; decoupled decay of Loshchilov & Hutter):
// one workgroup per (rank row, 1024 columns) of A, then of B; the row's task supplies lr, step
// count and gradient scale; bias corrections are taken in double once per workgroup
// -------------------------------------------------------------------------------------------
template <typename E>
__global__ __launch_bounds__(256) void adam_kernel(PlanDev pd, float beta1, float beta2, float eps, float wd,
                                                   const float* __restrict__ lr,
                                                   const int32_t* __restrict__ step,
                                                   const float* __restrict__ grad_scale, AdamTensor ta,
                                                   AdamTensor tb, int32_t tiles_a)
{
    const bool first = int32_t(blockIdx.y) < tiles_a;
    const AdamTensor& tn = first ? ta : tb;
    const int32_t coltile = first ? int32_t(blockIdx.y) : int32_t(blockIdx.y) - tiles_a;
    const int32_t R = blockIdx.x;
    int32_t t = 0;
    while (pd.rank_off[t + 1] <= R) ++t;
    const int32_t k = step[t];
    if (k <= 0) return;
    const float c1 = float(1.0 - pow(double(beta1), double(k)));
    const float c2 = float(1.0 - pow(double(beta2), double(k)));
    const float lrt = lr[t], sc = grad_scale ? grad_scale[t] : 1.f;
    E* param = static_cast<E*>(tn.param);
    for (int32_t col = coltile * 1024 + threadIdx.x; col < min(tn.D, (coltile + 1) * 1024); col += 256) {
        const size_t i = size_t(R) * tn.D + col;
        const float g = sc * tn.grad[i];
        const float m = beta1 * tn.m[i] + (1.f - beta1) * g;
        const float v = beta2 * tn.v[i] + (1.f - beta2) * g * g;
        const float th = tn.master[i];
        const float upd = (m / c1) / (sqrtf(v / c2) + eps) + wd * th;
        const float nt = th - lrt * upd;
        tn.m[i] = m;
        tn.v[i] = v;
        tn.master[i] = nt;
        if (param) Elem<E>::store(param, i, nt);
    }
}

hipError_t adam_step(const PlanDev& pd, int dtype, float beta1, float beta2, float eps, float wd,
                     const float* lr, const int32_t* step, const float* grad_scale,
                     const AdamTensor& ta, const AdamTensor& tb, hipStream_t st)
{
    if (pd.R_tot == 0) return hipSuccess;
    const int32_t tiles_a = (ta.D + 1023) / 1024, tiles_b = (tb.D + 1023) / 1024;
    const dim3 grid(pd.R_tot, tiles_a + tiles_b);
    if (grid.y > 65535u) return hipErrorInvalidValue;
    if (dtype == LOBRA_F32)
        adam_kernel<float><<<grid, 256, 0, st>>>(pd, beta1, beta2, eps, wd, lr, step, grad_scale, ta, tb, tiles_a);
    else
        adam_kernel<uint16_t><<<grid, 256, 0, st>>>(pd, beta1, beta2, eps, wd, lr, step, grad_scale, ta, tb, tiles_a);
    return hipGetLastError();
}

// -------------------------------------------------------------------------------------------
// index probe
// -------------------------------------------------------------------------------------------
__global__ void zero_counts_kernel(unsigned long long* cnt, int32_t n)
{
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) cnt[i] = 0ull;
}

__global__ __launch_bounds__(256) void token_task_kernel(PlanDev pd, int32_t* __restrict__ out_task,
                                                         unsigned long long* __restrict__ cnt)
{
    const int32_t row = blockIdx.x * 256 + threadIdx.x;
    if (row >= pd.T) return;
    const int32_t t = pd.cseg_task[segment_of_row(pd, row)];
    if (out_task) out_task[row] = t;
    if (cnt && t >= 0) atomicAdd(&cnt[t], 1ull);   // integer sum: order does not matter
}

hipError_t token_task_map(const PlanDev& pd, int32_t* out_task, int64_t* out_count, hipStream_t st)
{
    if (out_count && pd.n_tasks > 0) {
        zero_counts_kernel<<<(pd.n_tasks + 255) / 256, 256, 0, st>>>((unsigned long long*)out_count, pd.n_tasks);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (pd.T > 0) {
        token_task_kernel<<<(pd.T + 255) / 256, 256, 0, st>>>(pd, out_task, (unsigned long long*)out_count);
        return hipGetLastError();
    }
    return hipSuccess;
}

}  // namespace lobra
