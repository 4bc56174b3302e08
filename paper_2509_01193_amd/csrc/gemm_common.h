// Pieces shared by the bf16 MFMA kernels (the persistent direct-to-LDS GEMM, the K-sliced rank-r kernel and the
// register-staged kernel for K that is not a multiple of 64): vector types, the LDS swizzles, the
// direct global -> LDS copy and the in-place MFMA on AGPR accumulators.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>
#include <type_traits>

namespace lobra {
namespace gemm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 256, BN = 256, BK = 64;

// [rows][64 k] tile, 128 bytes per row: 16-byte chunk c of a row is stored at c ^ swz_row(row), so that
// the 16 rows of one ds_read_b128 pass hit 16 bank groups.
__device__ __forceinline__ int swz_row(int row) { return (row >> 1) & 7; }

// Swizzle of a [k][256 n] tile (512 bytes per k row): 16-byte chunk c of row k is stored at c ^ kn_swz(k).
// One transpose read of a 16-lane group takes 4 x 8 bytes from each of the k rows k0 .. k0 + 3, and the groups
// of a wave sit 8 rows apart: bits 0-1 of k pick the 64-byte quarter, bit 3 the 32-byte half of it.
__device__ __forceinline__ int kn_swz(int k) { return ((k & 3) << 2) | (((k >> 3) & 1) << 1); }

// The same for the persistent kernel's dealing of columns to MFMA blocks (block_col in gemm_persistent.hip): there
// the four 8-byte pieces a k row contributes to one transpose read lie in four different 16-byte chunks, in the low
// or the high half of each by the parity of lane group and block; bits 0-1 of k pick the 64-byte quarter as
// above, bit 3 the neighbouring chunk - whose piece lies in the other half - so that the k rows 8 apart, which the
// two lane groups of a 32-lane pass read, never meet in a bank.
__device__ __forceinline__ int kn_swz2(int k) { return ((k & 3) << 2) | ((k >> 3) & 1); }

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v)
{
    union { u32x4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

// MFMA "A" operand (8 consecutive k of one column) out of a [k][n] tile with k rows `pitch` bytes apart:
// two transpose reads of 4 k rows x 16 columns each.  p0 = this lane's 4-column group at its k row.
__device__ __forceinline__ bf16x8 tr_pair(const unsigned char* p0, int pitch)
{
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 4 * pitch));
    union { s16x4 h[2]; bf16x8 b; } cv;
    cv.h[0] = lo;
    cv.h[1] = hi;
    return cv.b;
}

// One wave-wide global -> LDS copy of 64 x 16 bytes without passing through registers
// (global_load_lds_dwordx4): lane i fetches 16 bytes at gbase + voff and they land at LDS byte
// address lds_addr + 16 i.  lds_addr and gbase are wave-uniform.  The LDS address travels in M0: the
// write of M0 and the copy that consumes it are ONE asm statement, so nothing can come between them.
// The instruction counts on vmcnt; the compiler does not see it, so the caller places the matching
// s_waitcnt vmcnt itself.
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
                 : "memory");
}

// ---- accumulators in explicitly named AGPRs --------------------------------------------------------------
// The persistent kernel keeps the 64 four-register accumulators of a wave in a[0:255] for its whole life,
// across output tiles, epilogues and a loop nest.  Handed to the register allocator as 64 values they get
// spilled at the loop header (all 256 AGPRs are taken, so every live-range split needs a spill), so the
// kernel names the registers itself: accumulator R lives in a[R : R + 3], the statements below are the only
// ones that touch AGPRs, and each one that writes them lists all of a0 .. a255 as clobbered, which keeps the
// compiler's own values out of them and makes the kernel allocate all 256.  (tests/test_kernel_isa.py checks on
// the generated code that nothing else touches an AGPR and that nothing is spilled.)
#define LOBRA_A10(p) "a" #p "0", "a" #p "1", "a" #p "2", "a" #p "3", "a" #p "4", "a" #p "5", "a" #p "6", "a" #p "7", "a" #p "8", "a" #p "9"
#define LOBRA_ALL_AGPRS                                                                                     \
    "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", LOBRA_A10(1), LOBRA_A10(2), LOBRA_A10(3),       \
    LOBRA_A10(4), LOBRA_A10(5), LOBRA_A10(6), LOBRA_A10(7), LOBRA_A10(8), LOBRA_A10(9), LOBRA_A10(10),          \
    LOBRA_A10(11), LOBRA_A10(12), LOBRA_A10(13), LOBRA_A10(14), LOBRA_A10(15), LOBRA_A10(16), LOBRA_A10(17),     \
    LOBRA_A10(18), LOBRA_A10(19), LOBRA_A10(20), LOBRA_A10(21), LOBRA_A10(22), LOBRA_A10(23), LOBRA_A10(24),     \
    "a250", "a251", "a252", "a253", "a254", "a255"

#ifndef LOBRA_MFMA_CLOBBER
#define LOBRA_MFMA_CLOBBER 0
#endif
#if LOBRA_MFMA_CLOBBER
#define LOBRA_MFMA_CLOB LOBRA_ALL_AGPRS
#define LOBRA_MFMA_CLOB_MEM "memory", LOBRA_ALL_AGPRS
#else
#define LOBRA_MFMA_CLOB
#define LOBRA_MFMA_CLOB_MEM "memory"
#endif
// Nothing of the compiler's may live in an AGPR across this point.
__device__ __forceinline__ void agpr_fence() { asm volatile("" : : : LOBRA_ALL_AGPRS); }

// a[R : R + 3] += a * b.  The order of these statements is the order of the instructions.
template <int R> __device__ __forceinline__ void mfma_acc(bf16x8 a, bf16x8 b)
{
    asm volatile("v_mfma_f32_16x16x32_bf16 a[%2:%3], %0, %1, a[%2:%3]"
                 :
                 : "v"(a), "v"(b), "n"(R), "n"(R + 3)
                 : LOBRA_MFMA_CLOB);
}

// a[R : R + 3] = a * b: the first MFMA of an output tile starts from zero instead of from what the previous
// tile left in the accumulator.
template <int R> __device__ __forceinline__ void mfma_first(bf16x8 a, bf16x8 b)
{
    asm volatile("v_mfma_f32_16x16x32_bf16 a[%2:%3], %0, %1, 0"
                 :
                 : "v"(a), "v"(b), "n"(R), "n"(R + 3)
                 : LOBRA_MFMA_CLOB);
}

// Two such MFMAs with a copy issued behind them, as one statement: an MFMA of this shape keeps its pipe for
// 16 cycles, 12 of which are free for the wave to issue something else, so the M0 write goes out behind the
// first and the copy behind the second (the MFMA between them is also the wait state the M0 write needs).
template <int R0, int R1>
__device__ __forceinline__ void mfma2_dma16(bf16x8 a0, bf16x8 a1, bf16x8 b, uint32_t lds_addr,
                                            const unsigned char* gbase, uint32_t voff)
{
    const uint32_t la = __builtin_amdgcn_readfirstlane(lds_addr);
    const uint64_t gp = reinterpret_cast<uint64_t>(gbase);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(uint32_t(gp));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(uint32_t(gp >> 32));
    const uint64_t gu = (uint64_t(hi) << 32) | lo;
    asm volatile("v_mfma_f32_16x16x32_bf16 a[%6:%7], %0, %2, a[%6:%7]\n\t"
                 "s_mov_b32 m0, %3\n\t"
                 "v_mfma_f32_16x16x32_bf16 a[%8:%9], %1, %2, a[%8:%9]\n\t"
                 "global_load_lds_dwordx4 %4, %5"
                 :
                 : "v"(a0), "v"(a1), "v"(b), "s"(la), "v"(voff), "s"(gu), "n"(R0), "n"(R0 + 3), "n"(R1), "n"(R1 + 3)
                 : LOBRA_MFMA_CLOB_MEM);
}

// One register of an accumulator, for the epilogue.  (Volatile: it stays behind the MFMAs before it.)
template <int R> __device__ __forceinline__ float acc_read()
{
    float v;
    asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(v) : "n"(R));
    return v;
}

// Compile-time loop: f(std::integral_constant<int, B>{}), ..., f(std::integral_constant<int, E - 1>{}).
template <int B, int E, typename F> __device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

}  // namespace gemm
}  // namespace lobra
