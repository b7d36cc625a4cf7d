// Weighted combine back to token order, and the one-time weight packing.
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

// YF32 / SF32: y_perm / y_shared hold fp32 (else bf16); OF32: out is fp32 (else bf16, RNE).
template <bool YF32, bool SF32, bool OF32>
__global__ __launch_bounds__(256) void combine_kernel(const char* __restrict__ y_perm, const int32_t* __restrict__ inv_perm,
                                                      const float* __restrict__ w, const char* __restrict__ y_shared,
                                                      int k, int H, char* __restrict__ out) {
    const int t = blockIdx.x;
    const size_t ybytes = (size_t)H * (YF32 ? 4 : 2);
    const size_t sbytes = (size_t)H * (SF32 ? 4 : 2);
    for (int c = threadIdx.x; c < H / 8; c += 256) {
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        for (int j = 0; j < k; ++j) {
            const int r = inv_perm[(size_t)t * k + j];
            const float wj = w[(size_t)t * k + j];
            accum8<YF32>(acc, y_perm + (size_t)r * ybytes, c, wj);
        }
        if (y_shared) accum8<SF32>(acc, y_shared + (size_t)t * sbytes, c, 1.0f);
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

// One-time weight packing.  in: logical [K, N] bf16 row-major (K = contraction dimension).
// out: the tiled layout the GEMM loads, i.e. the matrix W[n][k] = in[k][n] cut into blocks of
// 16 rows x 32 k (1 KiB), blocks ordered [N/16][K/32]; inside a block, row r (0..15) occupies
// bytes r*64..r*64+63 and its 16-byte piece c (k = 8c..8c+7) sits at slot c ^ ((4 - r/4) & 3).
// Rows keep their logical order.
// One workgroup transposes a 32 k x 32 n patch through LDS.
// N columns exist in `in`; blocks past them (the router pads its expert count to 32) are zero.
__global__ __launch_bounds__(256) void pack_weight_kernel(const uint16_t* __restrict__ in, int K, int N,
                                                          uint16_t* __restrict__ out) {
    __shared__ uint16_t patch[32][34];
    const int kt = blockIdx.x, b = blockIdx.y;      // k sub-tile, 32-row block of W
    const int tid = threadIdx.x;
    for (int i = tid; i < 32 * 32; i += 256) {
        const int kk = i >> 5, nn = i & 31;
        const int n = b * 32 + nn;
        patch[kk][nn] = n < N ? in[(size_t)(kt * 32 + kk) * N + n] : (uint16_t)0;
    }
    __syncthreads();
    if (tid < 128) {
        // 2 groups x 64 pieces; piece id inside the group = r*4 + slot
        const int grp = tid >> 6, pid = tid & 63;
        const int r = pid >> 2, slot = pid & 3;
        const int c = slot ^ block_swizzle(r);
        const int rho = grp * 16 + r;
        const int nloc = rho;
        uint16_t v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = patch[c * 8 + i][nloc];
        const size_t block = ((size_t)(b * 2 + grp) * (size_t)(K >> 5) + kt) * 512;  // in uint16 units
        uint4 q;
        q.x = v[0] | ((uint32_t)v[1] << 16);
        q.y = v[2] | ((uint32_t)v[3] << 16);
        q.z = v[4] | ((uint32_t)v[5] << 16);
        q.w = v[6] | ((uint32_t)v[7] << 16);
        *reinterpret_cast<uint4*>(out + block + pid * 8) = q;
    }
}

}  // namespace

hipError_t launch_combine(const moe_shape& s, const void* y_perm, const int32_t* inv_perm, const float* w,
                          const void* y_shared, void* out, bool y_fp32, bool shared_fp32, bool out_fp32, hipStream_t st) {
#define COMBINE(Y, S, O)                                                                                          \
    hipLaunchKernelGGL((combine_kernel<Y, S, O>), dim3(s.T), dim3(256), 0, st, (const char*)y_perm, inv_perm, w,  \
                       (const char*)y_shared, s.top_k, s.H, (char*)out)
#define COMBINE_O(Y, S)                 \
    do {                                \
        if (out_fp32) COMBINE(Y, S, true); \
        else COMBINE(Y, S, false);      \
    } while (0)
    if (y_fp32 && shared_fp32) COMBINE_O(true, true);
    else if (y_fp32) COMBINE_O(true, false);
    else if (shared_fp32) COMBINE_O(false, true);
    else COMBINE_O(false, false);
#undef COMBINE_O
#undef COMBINE
    return hipGetLastError();
}

hipError_t launch_pack_weight(const void* in, int rows, int cols, int cols_padded, void* out, hipStream_t st) {
    const dim3 grid(rows / 32, cols_padded / 32);   // rows = K, cols = N
    hipLaunchKernelGGL(pack_weight_kernel, grid, dim3(256), 0, st, (const uint16_t*)in, rows, cols, (uint16_t*)out);
    return hipGetLastError();
}

}  // namespace moe
