// Weighted combine back to token order, and the one-time weight transpose.
// (Sec. 2: the layer output is the weighted sum of the k experts' outputs, plus the shared
// expert every token passes through.)
//
// combine: one workgroup per token; every lane owns 8 consecutive hidden elements (16 B) and
// gathers the k expert rows of its token through inv_perm.  Sums are fp32 in the fixed order
// j = 0..k-1 then shared, every output element is written exactly once: no atomics, and the
// result is bit-identical from run to run.  HBM-bound: reads k+1 rows, writes 1 row per token.
#include "common.h"

namespace moe {
namespace {

// acc += w * (8 consecutive elements of a row, starting at element 8*c)
template <bool F32>
__device__ __forceinline__ void accum8(float (&acc)[8], const void* __restrict__ row, const int c, const float w) {
    if (F32) {
        const float4* p = reinterpret_cast<const float4*>(row) + 2 * c;
        const float4 a = p[0], b = p[1];
        const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = fmaf(w, v[i], acc[i]);
    } else {
        const uint4 v = reinterpret_cast<const uint4*>(row)[c];
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            acc[2 * q] = fmaf(w, __uint_as_float(u[q] << 16), acc[2 * q]);
            acc[2 * q + 1] = fmaf(w, __uint_as_float(u[q] & 0xffff0000u), acc[2 * q + 1]);
        }
    }
}

template <bool YF32, bool OF32>
__global__ __launch_bounds__(256) void combine_kernel(const char* __restrict__ y_perm, const int32_t* __restrict__ inv_perm,
                                                      const float* __restrict__ w, const char* __restrict__ y_shared,
                                                      int k, int H, char* __restrict__ out) {
    const int t = blockIdx.x;
    const size_t ybytes = (size_t)H * (YF32 ? 4 : 2);
    for (int c = threadIdx.x; c < H / 8; c += 256) {
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        for (int j = 0; j < k; ++j) {
            const int r = inv_perm[(size_t)t * k + j];
            const float wj = w[(size_t)t * k + j];
            accum8<YF32>(acc, y_perm + (size_t)r * ybytes, c, wj);
        }
        if (y_shared) accum8<YF32>(acc, y_shared + (size_t)t * ybytes, c, 1.0f);
        if (OF32) {
            float4* o = reinterpret_cast<float4*>(out + (size_t)t * H * 4) + 2 * c;
            o[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
            o[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
        } else {
            bf16x8 o;
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = (__bf16)acc[i];
            reinterpret_cast<bf16x8*>(out + (size_t)t * H * 2)[c] = o;
        }
    }
}

// out[c][r] = in[r][c] for a [rows, cols] bf16 matrix, 64x64 tiles through LDS.
__global__ __launch_bounds__(256) void transpose_kernel(const uint16_t* __restrict__ in, int rows, int cols,
                                                        uint16_t* __restrict__ out) {
    __shared__ uint16_t tile[64][66];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4) {
        const int r = r0 + i, c = c0 + tx;
        tile[i][tx] = (r < rows && c < cols) ? in[(size_t)r * cols + c] : (uint16_t)0;
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        const int c = c0 + i, r = r0 + tx;
        if (c < cols && r < rows) out[(size_t)c * rows + r] = tile[tx][i];
    }
}

}  // namespace

hipError_t launch_combine(const moe_shape& s, const void* y_perm, const int32_t* inv_perm, const float* w,
                          const void* y_shared, void* out, bool y_fp32, bool out_fp32, hipStream_t st) {
#define COMBINE(Y, O)                                                                                           \
    hipLaunchKernelGGL((combine_kernel<Y, O>), dim3(s.T), dim3(256), 0, st, (const char*)y_perm, inv_perm, w,   \
                       (const char*)y_shared, s.top_k, s.H, (char*)out)
    if (y_fp32 && out_fp32) COMBINE(true, true);
    else if (y_fp32) COMBINE(true, false);
    else if (out_fp32) COMBINE(false, true);
    else COMBINE(false, false);
#undef COMBINE
    return hipGetLastError();
}

hipError_t launch_transpose(const void* in, int rows, int cols, void* out, hipStream_t st) {
    const dim3 grid((cols + 63) / 64, (rows + 63) / 64);
    hipLaunchKernelGGL(transpose_kernel, grid, dim3(256), 0, st, (const uint16_t*)in, rows, cols, (uint16_t*)out);
    return hipGetLastError();
}

}  // namespace moe
