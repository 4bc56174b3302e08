// Measured ceilings for bench.py (built into liblobra_ceilings.so, NOT into the product library): what this
// chip sustains on the two resources the layer's kernels are bound by, measured in the same process and under
// the same power and clock conditions as the benchmark itself.
//   lobra_ceiling_mfma      a loop of nothing but v_mfma_f32_16x16x32_bf16 in the GEMM's register shape (four
//                           waves per compute unit, 8 x 8 accumulators of 16 x 16 per wave, operands that change
//                           with every MFMA): the matrix cores' sustained rate under the power limit
//   lobra_ceiling_read      a streaming read of a buffer with 16-byte loads (whole 1 KiB runs per wave instruction)
//   lobra_ceiling_copy      the same with a 16-byte store of every element read
// Each entry point only enqueues its kernel on the given stream; the caller times it.
#include <hip/hip_runtime.h>
#include <cstdint>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define LOBRA_CEIL_API extern "C" __attribute__((visibility("default")))

namespace {

// in: at least 16 * 64 * 4 operands of 16 bytes (any finite bf16 values); out: one float per thread
__global__ __launch_bounds__(256) void mfma_only_kernel(const bf16x8* __restrict__ in, float* __restrict__ out, int iters)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bf16x8 zf[8], wf[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        zf[i] = in[(wave * 16 + i) * 64 + lane];
        wf[i] = in[(wave * 16 + 8 + i) * 64 + lane];
    }
    f32x4 acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j], zf[i], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int v = 0; v < 4; ++v) s += acc[i][j][v];
    out[size_t(blockIdx.x) * 256 + threadIdx.x] = s;
}

// n16 = number of 16-byte elements; every workgroup walks the buffer with the grid's stride
template <bool COPY>
__global__ __launch_bounds__(256) void stream_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16,
                                                     uint32_t* __restrict__ sink)
{
    const size_t stride = size_t(gridDim.x) * 256 * 4;
    u32x4 acc = {0u, 0u, 0u, 0u};
    size_t i = size_t(blockIdx.x) * 256 * 4 + threadIdx.x;
    for (; i + 3 * 256 < n16; i += stride) {
        u32x4 v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = __builtin_nontemporal_load(src + i + q * 256);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (COPY) __builtin_nontemporal_store(v[q], dst + i + q * 256);
            else acc ^= v[q];
        }
    }
    for (; i < n16; i += 256) {         // the last, partial group of this workgroup's walk
        const u32x4 v = src[i];
        if (COPY) dst[i] = v;
        else acc ^= v;
    }
    if (!COPY && (acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = 1u;   // keeps the loads alive
}

}  // namespace

// flops of one launch: workgroups * 4 waves * iters * 64 MFMAs * 2 * 16 * 16 * 32
LOBRA_CEIL_API int lobra_ceiling_mfma(const void* operands, float* out, int workgroups, int iters, void* stream)
{
    if (!operands || !out || workgroups < 1 || iters < 1) return -1;
    mfma_only_kernel<<<workgroups, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const bf16x8*>(operands), out, iters);
    return hipGetLastError() == hipSuccess ? 0 : -9;
}

LOBRA_CEIL_API int lobra_ceiling_read(const void* src, size_t bytes, uint32_t* sink, int workgroups, void* stream)
{
    if (!src || !sink || bytes % 16 || workgroups < 1) return -1;
    stream_kernel<false><<<workgroups, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const u32x4*>(src), nullptr, bytes / 16, sink);
    return hipGetLastError() == hipSuccess ? 0 : -9;
}

LOBRA_CEIL_API int lobra_ceiling_copy(const void* src, void* dst, size_t bytes, int workgroups, void* stream)
{
    if (!src || !dst || bytes % 16 || workgroups < 1) return -1;
    stream_kernel<true><<<workgroups, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), bytes / 16, nullptr);
    return hipGetLastError() == hipSuccess ? 0 : -9;
}
