// Router: fp32 gate logits, softmax over all experts, wavefront-level top-k.
// (Sec. 2 "MoE inference": the router assigns each token to its top-k experts.)
//
// bf16 x bf16 products are exact in fp32, so the GPU logits differ from a correctly rounded
// reference only through the order of the fp32 additions; both paths below keep the sums short
// enough that top-k agrees except at genuine near-ties.
//   E <= 16 : one streaming kernel (HBM-bound): fp32 FMAs per lane, reduction over lanes and waves.
//   E  > 16 : the logits are a dense contraction and go through the MFMA tile routine of the
//             grouped GEMM (x against the packed gate matrix, K cut into independent chains);
//             route_topk_kernel then sums the partials, adds the bias and selects.
// Selection: 64 lanes hold a token's logits, max / sum are butterfly reductions and top-k is k
// rounds of a wave-wide arg-max on the logits (ties resolved towards the lower expert id).
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

// Sum over the 64 lanes of N per-lane values (N = 64 or 128) in N - N/64 exchange steps instead
// of 6N: at the step with lane mask m every lane keeps one half of its values (upper half if its
// bit m is set) and adds the partner's copy of that half.  Afterwards lane l holds the complete
// sums of values l*(N/64) .. +N/64-1 in v[0..N/64).  fp32 addition is commutative, so every value
// is added up along the same tree of lanes whatever its index.
template <int N, int HALF = N / 2, int MASK = 32>
__device__ __forceinline__ void lane_reduce_scatter(float (&v)[N], const int lane) {
    const bool up = (lane & MASK) != 0;
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
        const float keep = up ? v[i + HALF] : v[i];
        const float send = up ? v[i] : v[i + HALF];
        v[i] = keep + pair_f<MASK>(send);
    }
    if constexpr (MASK > 1) lane_reduce_scatter<N, HALF / 2, MASK / 2>(v, lane);
}

// Few experts (E <= 16): HBM-bound.  One workgroup of 4 wavefronts takes TOK tokens; every wave
// works on all TOK tokens but only on a quarter of the hidden dimension (thread i owns
// h = 2048*it + 8*i .. +7), so a wave has TOK 16-byte loads in flight per step and reads a quarter
// of Wg (8*E contiguous bf16 per 8 hidden elements, cache resident).  The per-lane partial sums
// go through lane_reduce_scatter, the four waves' results through LDS (added in wave order), and
// each wave then finishes TOK/4 tokens.  The sum that makes a logit does not depend on TOK, on
// the token's slot in the workgroup or on T.
template <int EP, bool EXACT, int TOK>  // EP: padded expert count (8 or 16); EXACT: E == EP, rows of Wg are 16-byte vectors
__global__ __launch_bounds__(256) void route_small_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg,
                                                          const float* __restrict__ bias, int T, int H, int E, int k,
                                                          int renorm, float scale, int32_t* __restrict__ idx_out,
                                                          float* __restrict__ w_out, float* __restrict__ logits_out) {
    constexpr int NVAL = TOK * EP;   // 64 or 128
    constexpr int PER = NVAL / 64;
    static_assert(NVAL == 64 || NVAL == 128, "lane_reduce_scatter needs 64 or 128 values");
    __shared__ float part[4][NVAL];
    __shared__ float logit_s[NVAL];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t0 = blockIdx.x * TOK;
    float acc[NVAL];   // [token slot a][expert e] at a*EP + e
#pragma unroll
    for (int i = 0; i < NVAL; ++i) acc[i] = 0.f;
    for (int h0 = threadIdx.x * 8; h0 < H; h0 += 2048) {
        uint4 xv[TOK];
#pragma unroll
        for (int a = 0; a < TOK; ++a) {
            const int t = min(t0 + a, T - 1);
            xv[a] = *reinterpret_cast<const uint4*>(x + (size_t)t * H + h0);
        }
#pragma unroll
        for (int hh = 0; hh < 8; ++hh) {
            float xa[TOK];
#pragma unroll
            for (int a = 0; a < TOK; ++a) {
                const uint32_t u = (&xv[a].x)[hh >> 1];
                xa[a] = (hh & 1) ? __uint_as_float(u & 0xffff0000u) : __uint_as_float(u << 16);
            }
            const uint16_t* wr = wg + (size_t)(h0 + hh) * E;
            float wv[EP];
            if (EXACT) {
#pragma unroll
                for (int c = 0; c < EP / 8; ++c) {
                    const uint4 q = reinterpret_cast<const uint4*>(wr)[c];
                    const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        wv[c * 8 + 2 * i] = __uint_as_float(u[i] << 16);
                        wv[c * 8 + 2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < EP; ++e) wv[e] = e < E ? __uint_as_float((uint32_t)wr[e] << 16) : 0.f;
            }
#pragma unroll
            for (int e = 0; e < EP; ++e)
#pragma unroll
                for (int a = 0; a < TOK; ++a) acc[a * EP + e] = fmaf(xa[a], wv[e], acc[a * EP + e]);
        }
    }
    lane_reduce_scatter<NVAL>(acc, lane);
#pragma unroll
    for (int i = 0; i < PER; ++i) part[wave][lane * PER + i] = acc[i];
    __syncthreads();
    if (threadIdx.x < NVAL) {
        const int i = threadIdx.x;
        logit_s[i] = ((part[0][i] + part[1][i]) + part[2][i]) + part[3][i];
    }
    __syncthreads();
    for (int a = wave; a < TOK; a += 4) {
        const int t = t0 + a;
        if (t >= T) break;  // wave-uniform; no barrier follows
        float mine = -INFINITY;
        if (lane < E) mine = logit_s[a * EP + lane] + (bias ? bias[lane] : 0.f);
        const float v[1] = {mine};
        route_finish<1>(v, lane, t, E, k, renorm, scale, idx_out, w_out, logits_out);
    }
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

}  // namespace

hipError_t launch_route_topk(const moe_shape& s, const float* partial, int splits, int ep, const float* bias,
                             int32_t* idx, float* w, float* logits, hipStream_t st) {
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

hipError_t launch_route(const moe_shape& s, const void* x, const void* wg, const float* bias, int32_t* idx,
                        float* w, float* logits, hipStream_t st) {
    if (s.E <= 16) {
        // Tokens per workgroup: as many as the registers hold (16 with 8 experts, 8 with 16) when
        // that still gives every CU two workgroups, else half of that.
        const bool big = s.T >= 2 * 256 * (s.E <= 8 ? 16 : 8);
#define ROUTE_SMALL(EP_, EX_, TOK_)                                                                                 \
    hipLaunchKernelGGL((route_small_kernel<EP_, EX_, TOK_>), dim3((s.T + TOK_ - 1) / TOK_), dim3(256), 0, st,          \
                       (const uint16_t*)x, (const uint16_t*)wg, bias, s.T, s.H, s.E, s.top_k, s.renormalize,          \
                       s.routed_scale, idx, w, logits)
#define ROUTE_SMALL_T(EP_, EX_, TB_, TS_)      \
    do {                                       \
        if (big) ROUTE_SMALL(EP_, EX_, TB_);   \
        else ROUTE_SMALL(EP_, EX_, TS_);       \
    } while (0)
        if (s.E == 8) ROUTE_SMALL_T(8, true, 16, 8);
        else if (s.E < 8) ROUTE_SMALL_T(8, false, 16, 8);
        else if (s.E == 16) ROUTE_SMALL_T(16, true, 8, 4);
        else ROUTE_SMALL_T(16, false, 8, 4);
#undef ROUTE_SMALL_T
#undef ROUTE_SMALL
        return hipGetLastError();
    }
    return hipErrorInvalidValue;  // E > 16 goes through the GEMM path (launch_route_plan / launch_route_topk)
}

}  // namespace moe
