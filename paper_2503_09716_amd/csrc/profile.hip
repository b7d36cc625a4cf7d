// Measured ceiling of the matrix cores: a register-only loop of the MFMA instruction the grouped
// GEMMs use (v_mfma_f32_16x16x32_bf16), with no LDS and no memory traffic inside the loop.
// The chip is power-limited on dense bf16 work and what it sustains depends on the operand
// VALUES (zeros toggle no multiplier inputs), so the loop takes its operand fragments from
// caller-supplied buffers: the workload's own activations and weights give the rate a GEMM on
// that data could reach if feeding the matrix cores were free; NULL buffers give the rate on
// zeros.  Reported beside the published peak by bench.py.
#include "common.h"

namespace moe {
namespace {

// The instruction as the GEMM tile routine issues it: accumulator tied to an AGPR quad (left to
// the register allocator, part of the 256 accumulators travel through temporaries, several
// copies per MFMA, and the loop measures the copies).  Every accumulator is re-used only 64
// instructions later, so no hazard needs covering inside the loop.
__device__ __forceinline__ void mfma(f32x4& c, const bf16x8& a, const bf16x8& b) {
#if defined(__gfx950__)
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
#endif
}

constexpr int CEIL_FRAGS = 8;   // 8 x 8 accumulator blocks of 16 x 16: all 256 accumulator registers, as in the GEMM tile

__global__ __launch_bounds__(256, 1) void mfma_ceiling_kernel(const bf16x8* __restrict__ a_src, const bf16x8* __restrict__ b_src,
                                                              uint32_t n_frags, int iters, float* __restrict__ sink) {
    f32x4 acc[CEIL_FRAGS][CEIL_FRAGS];
#pragma unroll
    for (int j = 0; j < CEIL_FRAGS; ++j)
#pragma unroll
        for (int i = 0; i < CEIL_FRAGS; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[j][i][r] = 0.f;
    bf16x8 a[CEIL_FRAGS], b[CEIL_FRAGS];
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
#pragma unroll
    for (int j = 0; j < CEIL_FRAGS; ++j) {
        bf16x8 z;
#pragma unroll
        for (int q = 0; q < 8; ++q) z[q] = (__bf16)0.0f;
        // consecutive lanes read consecutive 16-byte pieces; every (block, fragment) pair reads another part of the buffer
        const uint32_t at = (uint32_t)(((uint64_t)t * CEIL_FRAGS + j) % n_frags);
        a[j] = a_src ? a_src[at] : z;
        b[j] = b_src ? b_src[at] : z;
    }
    // Instruction order of the GEMM's half sub-tile: the first operand alternates between two
    // fragments, the second changes with every second instruction.  What the chip sustains under
    // its power limit depends on this order too: on the Mixtral-shaped workload's data this one
    // measured 2.10 PFLOP/s, one first operand for eight instructions in a row 2.04, both
    // operands new with every instruction 1.98 (all 2.43 on zeros).
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int h = 0; h < CEIL_FRAGS; h += 2)
#pragma unroll
            for (int i = 0; i < CEIL_FRAGS; ++i)
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
                    mfma(acc[h + jj][i], a[h + jj], b[i]);
    }
    // the last instructions are still in the matrix pipe; the compiler does not track inline assembly
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < CEIL_FRAGS; ++j)
#pragma unroll
        for (int i = 0; i < CEIL_FRAGS; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) s += acc[j][i][r];
    sink[t] = s;   // keeps the loop alive
}

}  // namespace

// FLOPs of one launch: blocks x 4 waves x iters x 64 MFMAs x 2*16*16*32.
double mfma_ceiling_flops(int blocks, int iters) {
    return (double)blocks * 4.0 * (double)iters * (CEIL_FRAGS * CEIL_FRAGS) * 2.0 * 16 * 16 * 32;
}

hipError_t launch_mfma_ceiling(const void* a, const void* b, size_t bytes, int blocks, int iters, float* sink, hipStream_t st) {
    const uint32_t n_frags = (uint32_t)(bytes / 16);
    hipLaunchKernelGGL(mfma_ceiling_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const bf16x8*)a, (const bf16x8*)b,
                       n_frags ? n_frags : 1u, iters, sink);
    return hipGetLastError();
}

}  // namespace moe
