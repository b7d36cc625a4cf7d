// Router: fp32 gate logits, softmax over all experts, wavefront-level top-k.
// (Sec. 2 "MoE inference": the router assigns each token to its top-k experts.)
//
// bf16 x bf16 products are exact in fp32, so the GPU logits differ from a correctly rounded
// reference only through the order of the fp32 additions; both paths below keep the sums short
// enough that top-k agrees except at genuine near-ties.  Both multiply x with the PACKED gate
// matrix on the matrix cores:
//   E <= 16 : one kernel (HBM-bound: it streams x once): 16 tokens per workgroup, K cut over 8
//             waves, the selection in the same workgroup with a token's logits in 16 lanes.
//   E  > 16 : the logits go through the MFMA tile routine of the grouped GEMM (K cut into
//             independent chains); route_topk_kernel then sums the partials, adds the bias and
//             selects: 64 lanes hold a token's logits.
// Selection: max / sum are butterfly reductions and top-k is k rounds of an arg-max on the
// logits (ties resolved towards the lower expert id).
#include <type_traits>

#include "common.h"

namespace moe {
namespace {

// Butterfly step M of a wave-wide reduction: the value held by this lane's partner, the lane
// that differs from it in bit log2(M) and agrees in all higher bits.  Inside a row of 16 lanes
// the partner comes through the VALU's data-parallel-primitive path (quad permutes for M = 1, 2;
// half-row and row mirrors for M = 4, 8: lane i with 7-i, 15-i, which also flip the lower bits,
// and any partner with the same higher bits will do for a reduction); only M = 16, 32 go
// through the LDS crossbar, whose throughput per CU is what bounded the top-k kernels.
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
template <int M>
__device__ __forceinline__ int pair_i(int v) {
    if constexpr (M == 1) return dpp_move<0xB1>(v);        // quad_perm [1,0,3,2]
    else if constexpr (M == 2) return dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
    else if constexpr (M == 4) return dpp_move<0x141>(v);  // row_half_mirror
    else if constexpr (M == 8) return dpp_move<0x140>(v);  // row_mirror
    else return __shfl_xor(v, M, 64);
}
template <int M>
__device__ __forceinline__ float pair_f(float v) {
    return __int_as_float(pair_i<M>(__float_as_int(v)));
}

__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, pair_f<1>(v));
    v = fmaxf(v, pair_f<2>(v));
    v = fmaxf(v, pair_f<4>(v));
    v = fmaxf(v, pair_f<8>(v));
    v = fmaxf(v, pair_f<16>(v));
    v = fmaxf(v, pair_f<32>(v));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
    v += pair_f<1>(v);
    v += pair_f<2>(v);
    v += pair_f<4>(v);
    v += pair_f<8>(v);
    v += pair_f<16>(v);
    v += pair_f<32>(v);
    return v;
}

// Softmax over all experts + top-k for ONE token held by one wavefront: lane l holds the logits
// of experts l, l+64, ... in v[] (-inf past E).  Max and sum are butterfly reductions; top-k is
// k rounds of a wave-wide arg-max on the logits (ties -> lower expert id), so rounding in exp /
// division can never change the selection.
template <int NV>
__device__ __forceinline__ void route_finish(const float (&v)[NV], const int lane, const int t, const int E, const int k,
                                             const int renorm, const float scale, int32_t* __restrict__ idx_out,
                                             float* __restrict__ w_out, float* __restrict__ logits_out) {
    float p[NV];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int e = lane + 64 * i;
        m = fmaxf(m, v[i]);
        if (logits_out && e < E) logits_out[(size_t)t * E + e] = v[i];
    }
    m = wave_max(m);
    float z = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        p[i] = expf(v[i] - m);  // exp(-inf) = 0 for padded experts
        z += p[i];
    }
    z = wave_sum(z);
    const float rz = 1.0f / z;
    float my_w = 0.f;
    int my_e = 0;
    unsigned taken = 0;
    for (int j = 0; j < k; ++j) {
        // lane-local best among the not-yet-selected (ascending expert id, strict >)
        float bv = -INFINITY, bp = 0.f;
        int be = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int e = lane + 64 * i;
            const bool ok = e < E && !((taken >> i) & 1u);
            if (ok && (be == 0x7fffffff || v[i] > bv)) { bv = v[i]; be = e; bp = p[i]; }
        }
        // wave arg-max, ties -> lower expert id ((value, -id) is a total order, so the result does
        // not depend on how the lanes are paired)
        auto step = [&](auto m_tag) __attribute__((always_inline)) {
            constexpr int M = decltype(m_tag)::value;
            const float ov = pair_f<M>(bv);
            const int oe = pair_i<M>(be);
            const float op = pair_f<M>(bp);
            if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; bp = op; }
        };
        step(std::integral_constant<int, 1>{});
        step(std::integral_constant<int, 2>{});
        step(std::integral_constant<int, 4>{});
        step(std::integral_constant<int, 8>{});
        step(std::integral_constant<int, 16>{});
        step(std::integral_constant<int, 32>{});
        if (lane == j) { my_e = be; my_w = bp * rz; }
        // retire the winner
#pragma unroll
        for (int i = 0; i < NV; ++i)
            if (lane + 64 * i == be) taken |= 1u << i;
    }
    const float wsum = wave_sum(lane < k ? my_w : 0.f);
    if (lane < k) {
        float wv = my_w;
        if (renorm) wv = wv / wsum;
        idx_out[(size_t)t * k + lane] = my_e;
        w_out[(size_t)t * k + lane] = wv * scale;
    }
}

// Few experts (E <= 16) on the matrix cores.  One workgroup of 8 wavefronts takes 16 tokens; a
// wavefront multiplies every 8th K sub-tile of 32 (the eight waves read neighbouring 64-byte
// pieces of the same 16 rows of x at the same time) with v_mfma_f32_16x16x32_bf16: x is the row
// operand (lane l: token l%16, k = 8*(l/16)..+7, 16 bytes straight from the row), the packed
// gate matrix the column operand (lane l: expert l%16, the same k: one 1 KiB block per sub-tile,
// in lane order).  All loads of up to 16 sub-tiles are issued before the first multiply, so a
// wave has 32 KiB in flight.  The eight partial sums of a logit meet in LDS and are added in
// wave order; then wave r (r < 4) finishes tokens 4q + r, q = 0..3, all four at once: the 16
// logits of a token sit in one row of 16 lanes, so max / sum / arg-max are four butterfly steps
// inside a row, none through LDS.  No per-lane FMA loop and no cross-lane reduction of partial
// sums: the matrix instruction adds over K.

constexpr int ROUTE_MFMA_WAVES = 8;
constexpr int ROUTE_MFMA_AHEAD = 16;   // sub-tiles whose loads a wave issues before its first multiply

__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, pair_f<1>(v));
    v = fmaxf(v, pair_f<2>(v));
    v = fmaxf(v, pair_f<4>(v));
    v = fmaxf(v, pair_f<8>(v));
    return v;
}
__device__ __forceinline__ float row16_sum(float v) {
    v += pair_f<1>(v);
    v += pair_f<2>(v);
    v += pair_f<4>(v);
    v += pair_f<8>(v);
    return v;
}

// Softmax over all experts + top-k (k <= 16) for the token held by one ROW of 16 lanes: the lane
// with row index c holds the logits of experts c, c+16, ... in v[] (-inf past E); a wavefront
// finishes four tokens at once.  Max, sum and the k arg-max rounds (ties -> lower expert id, on
// the logits, so rounding in exp / division can never change the selection) are four butterfly
// steps inside the row, all on the VALU's DPP path.  Lane j of the row ends up with the j-th pick.
// WIDE: the lane holds experts 4c..4c+3, 64+4c..64+4c+3, ... instead (what 16-byte loads of a
// row of logits deliver); either way its experts ascend with i.
template <bool WIDE>
__device__ __forceinline__ int row16_expert(const int row, const int i) {
    return WIDE ? row * 4 + (i & 3) + 64 * (i >> 2) : row + 16 * i;
}
template <int NV, bool WIDE = false>
__device__ __forceinline__ void route_finish_row16(const float (&v)[NV], const int row, const int tok, const bool valid,
                                                   const int E, const int k, const int renorm, const float scale,
                                                   int32_t* __restrict__ idx_out, float* __restrict__ w_out,
                                                   float* __restrict__ logits_out) {
    float p[NV];
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int e = row16_expert<WIDE>(row, i);
        m = fmaxf(m, v[i]);
        if (logits_out && valid && e < E) logits_out[(size_t)tok * E + e] = v[i];
    }
    m = row16_max(m);
    float z = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        p[i] = expf(v[i] - m);   // exp(-inf) = 0 for padded experts
        z += p[i];
    }
    const float rz = 1.0f / row16_sum(z);
    float my_w = 0.f;
    int my_e = 0;
    unsigned taken = 0;
    for (int j = 0; j < k; ++j) {
        // lane-local best among the not-yet-selected (ascending expert id, strict >)
        float bv = -INFINITY, bp = 0.f;
        int be = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int e = row16_expert<WIDE>(row, i);
            const bool ok = e < E && !((taken >> i) & 1u);
            if (ok && (be == 0x7fffffff || v[i] > bv)) { bv = v[i]; be = e; bp = p[i]; }
        }
        auto step = [&](auto m_tag) __attribute__((always_inline)) {
            constexpr int M = decltype(m_tag)::value;
            const float ov = pair_f<M>(bv);
            const int oe = pair_i<M>(be);
            const float op = pair_f<M>(bp);
            // (value, -id) is a total order over the lanes that still hold a candidate
            if (oe != 0x7fffffff && (be == 0x7fffffff || ov > bv || (ov == bv && oe < be))) { bv = ov; be = oe; bp = op; }
        };
        step(std::integral_constant<int, 1>{});
        step(std::integral_constant<int, 2>{});
        step(std::integral_constant<int, 4>{});
        step(std::integral_constant<int, 8>{});
        if (row == j) { my_e = be; my_w = bp * rz; }
#pragma unroll
        for (int i = 0; i < NV; ++i)
            if (row16_expert<WIDE>(row, i) == be) taken |= 1u << i;
    }
    const float wsum = row16_sum(row < k ? my_w : 0.f);
    if (valid && row < k) {
        float wv = my_w;
        if (renorm) wv = wv / wsum;
        idx_out[(size_t)tok * k + row] = my_e;
        w_out[(size_t)tok * k + row] = wv * scale;
    }
}

__global__ __launch_bounds__(ROUTE_MFMA_WAVES * 64) void route_mfma_kernel(
    const char* __restrict__ x, const char* __restrict__ wg_packed, const float* __restrict__ bias, int T, int H, int E, int k,
    int renorm, float scale, int32_t* __restrict__ idx_out, float* __restrict__ w_out, float* __restrict__ logits_out) {
    __shared__ float part[ROUTE_MFMA_WAVES][4][64];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int row = lane & 15, g = lane >> 4;
    const int t0 = blockIdx.x * 16;
    const char* xa = x + (size_t)min(t0 + row, T - 1) * H * 2 + g * 16;
    const char* wb = wg_packed + row * 64 + ((g ^ block_swizzle(row)) << 4);
    const int KS = H >> 5;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int ks0 = wave; ks0 < KS; ks0 += ROUTE_MFMA_WAVES * ROUTE_MFMA_AHEAD) {
        bf16x8 a[ROUTE_MFMA_AHEAD], b[ROUTE_MFMA_AHEAD];
#pragma unroll
        for (int u = 0; u < ROUTE_MFMA_AHEAD; ++u) {
            const int ks = ks0 + u * ROUTE_MFMA_WAVES;
            if (ks < KS) {   // wave-uniform
                a[u] = *reinterpret_cast<const bf16x8*>(xa + (size_t)ks * 64);
                b[u] = *reinterpret_cast<const bf16x8*>(wb + (size_t)ks * 1024);
            } else {
#pragma unroll
                for (int q = 0; q < 8; ++q) { a[u][q] = (__bf16)0.0f; b[u][q] = (__bf16)0.0f; }
            }
        }
#pragma unroll
        for (int u = 0; u < ROUTE_MFMA_AHEAD; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u], b[u], acc, 0, 0, 0);
    }
    // acc[r]: token t0 + 4*g + r, expert `row` (partial over this wave's sub-tiles)
#pragma unroll
    for (int r = 0; r < 4; ++r) part[wave][r][lane] = acc[r];
    __syncthreads();
    if (wave >= 4) return;   // wave-uniform; no barrier follows
    const int r = wave;
    float v = 0.f;
#pragma unroll
    for (int w8 = 0; w8 < ROUTE_MFMA_WAVES; ++w8) v += part[w8][r][lane];
    const int tok = t0 + 4 * g + r;
    const float one[1] = {row < E ? v + (bias ? bias[row] : 0.f) : -INFINITY};
    route_finish_row16<1>(one, row, tok, tok < T, E, k, renorm, scale, idx_out, w_out, logits_out);
}

// E > 16: the logits come from the grouped-GEMM tile routine (x row-major against the packed
// gate matrix, K cut into `splits` independent accumulation chains to keep the fp32 rounding
// error of the long sums small).  This kernel adds the partial sums in a fixed order, adds the
// bias, and runs the wave-level softmax / top-k: one wavefront per token.
template <int NV>
__global__ __launch_bounds__(256) void route_topk_kernel(const float* __restrict__ partial, int splits, int T, int EP,
                                                         int E, int k, const float* __restrict__ bias, int renorm,
                                                         float scale, int32_t* __restrict__ idx_out,
                                                         float* __restrict__ w_out, float* __restrict__ logits_out) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;  // wave-uniform
    float v[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int e = lane + 64 * i;
        v[i] = -INFINITY;
        if (e < E) {
            float a = 0.f;
            for (int s = 0; s < splits; ++s) a += partial[((size_t)s * T + t) * EP + e];
            v[i] = a + (bias ? bias[e] : 0.f);
        }
    }
    route_finish<NV>(v, lane, t, E, k, renorm, scale, idx_out, w_out, logits_out);
}

// The same for k <= 16 with a token's logits in a row of 16 lanes: four tokens per wavefront, no
// step through the LDS crossbar.  Lane c of a row reads experts 4c..4c+3 of every 64 as one
// 16-byte load per partial matrix (NB = blocks of 64 experts).
template <int NB>
__global__ __launch_bounds__(256) void route_topk_row16_kernel(const float* __restrict__ partial, int splits, int T, int EP,
                                                               int E, int k, const float* __restrict__ bias, int renorm,
                                                               float scale, int32_t* __restrict__ idx_out,
                                                               float* __restrict__ w_out, float* __restrict__ logits_out) {
    const int lane = threadIdx.x & 63, row = lane & 15;
    const int tok = (blockIdx.x * 4 + (threadIdx.x >> 6)) * 4 + (lane >> 4);
    const int t = min(tok, T - 1);   // rows past the end redo the last token and write nothing
    float v[4 * NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int e0 = row * 4 + 64 * b;
        f32x4 a = {0.f, 0.f, 0.f, 0.f};
        if (e0 < EP)   // EP is a multiple of 32: the four values are all inside the row or all outside
            for (int s = 0; s < splits; ++s) a += *reinterpret_cast<const f32x4*>(partial + ((size_t)s * T + t) * EP + e0);
#pragma unroll
        for (int q = 0; q < 4; ++q) v[4 * b + q] = e0 + q < E ? a[q] + (bias ? bias[e0 + q] : 0.f) : -INFINITY;
    }
    route_finish_row16<4 * NB, true>(v, row, tok, tok < T, E, k, renorm, scale, idx_out, w_out, logits_out);
}

}  // namespace

hipError_t launch_route_topk(const moe_shape& s, const float* partial, int splits, int ep, const float* bias,
                             int32_t* idx, float* w, float* logits, hipStream_t st) {
    if (s.top_k <= 16) {
        const dim3 grid((s.T + 15) / 16), block(256);
#define TOPK16(NB_)                                                                                                 \
    hipLaunchKernelGGL(route_topk_row16_kernel<NB_>, grid, block, 0, st, partial, splits, s.T, ep, s.E, s.top_k, bias, \
                       s.renormalize, s.routed_scale, idx, w, logits)
        if (s.E <= 64) TOPK16(1);
        else if (s.E <= 128) TOPK16(2);
        else if (s.E <= 192) TOPK16(3);
        else TOPK16(4);
#undef TOPK16
        return hipGetLastError();
    }
    const dim3 grid((s.T + 3) / 4), block(256);
#define TOPK(NV_)                                                                                              \
    hipLaunchKernelGGL(route_topk_kernel<NV_>, grid, block, 0, st, partial, splits, s.T, ep, s.E, s.top_k, bias,  \
                       s.renormalize, s.routed_scale, idx, w, logits)
    if (s.E <= 64) TOPK(1);
    else if (s.E <= 128) TOPK(2);
    else if (s.E <= 192) TOPK(3);
    else TOPK(4);
#undef TOPK
    return hipGetLastError();
}

hipError_t launch_route_mfma(const moe_shape& s, const void* x, const void* wg_packed, const float* bias, int32_t* idx,
                             float* w, float* logits, hipStream_t st) {
    hipLaunchKernelGGL(route_mfma_kernel, dim3((s.T + 15) / 16), dim3(ROUTE_MFMA_WAVES * 64), 0, st, (const char*)x,
                       (const char*)wg_packed, bias, s.T, s.H, s.E, s.top_k, s.renormalize, s.routed_scale, idx, w, logits);
    return hipGetLastError();
}

}  // namespace moe
