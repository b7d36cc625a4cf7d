// Router: fp32 gate GEMM + softmax over all experts + wavefront-level top-k.
// (Sec. 2 "MoE inference": the router assigns each token to its top-k experts.)
//
// One workgroup owns ROUTE_TOK tokens.  Phase 1 streams x and Wg through LDS in K-chunks and
// accumulates logits with fp32 FMAs (bf16 x bf16 products are exact in fp32; a chunk-local
// accumulator is folded into the running sum once per chunk to keep the rounding error of
// the long sum small, which is what makes top-k agree with a correctly rounded reference
// except at genuine near-ties).  Phase 2 parks the logits in LDS; each wavefront then takes
// one token at a time: 64 lanes hold the token's logits, max / sum are butterfly reductions
// and top-k is k rounds of a wave-wide arg-max (ties resolved towards the lower expert id).
#include "common.h"

namespace moe {
namespace {

constexpr int ROUTE_TOK = 32;  // tokens per workgroup
constexpr int ROUTE_KC = 64;   // K elements per LDS chunk
constexpr int ROUTE_LD = ROUTE_KC + 8;  // padded row length (bf16) -> 144 B rows, conflict-free 16 B reads

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
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
        // wave arg-max, ties -> lower expert id
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) {
            const float ov = __shfl_xor(bv, s, 64);
            const int oe = __shfl_xor(be, s, 64);
            const float op = __shfl_xor(bp, s, 64);
            if (ov > bv || (ov == bv && oe < be)) { bv = ov; be = oe; bp = op; }
        }
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

// TE = experts per thread in phase 1 (thread tid%32 owns experts tid%32 + 32*i, i < TE).
template <int TE>
__global__ __launch_bounds__(256) void route_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg,
                                                    const float* __restrict__ bias, int T, int H, int E, int k,
                                                    int renorm, float scale, int32_t* __restrict__ idx_out,
                                                    float* __restrict__ w_out, float* __restrict__ logits_out) {
    constexpr int EP = TE * 32;  // padded expert count
    __shared__ __attribute__((aligned(16))) uint16_t xs[ROUTE_TOK * ROUTE_LD];
    __shared__ __attribute__((aligned(16))) uint16_t ws[EP * ROUTE_LD];
    // the logits (ROUTE_TOK x EP fp32 = 128*EP bytes) reuse the Wg staging buffer (144*EP bytes)
    float* lg = reinterpret_cast<float*>(ws);
    static_assert(ROUTE_TOK * 4 <= ROUTE_LD * 2, "logit tile must fit in the Wg staging buffer");

    const int tid = threadIdx.x;
    const int t0 = blockIdx.x * ROUTE_TOK;
    const int tg = tid >> 5;  // token group: tokens tg*4 .. tg*4+3
    const int el = tid & 31;

    float acc[4][TE];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int i = 0; i < TE; ++i) acc[a][i] = 0.f;

    // zero the padded expert rows once (they are never written by the staging loop)
    for (int i = tid; i < EP * ROUTE_LD; i += 256) ws[i] = 0;

    for (int h0 = 0; h0 < H; h0 += ROUTE_KC) {
        __syncthreads();
        // stage x: ROUTE_TOK rows x 64 bf16 = 8 x 16 B per row; 256 threads, one 16 B piece each
        {
            const int r = tid >> 3, c = tid & 7;
            int t = t0 + r;
            if (t >= T) t = T - 1;
            const uint4 v = *reinterpret_cast<const uint4*>(x + (size_t)t * H + h0 + c * 8);
            *reinterpret_cast<uint4*>(xs + r * ROUTE_LD + c * 8) = v;
        }
        // stage Wg transposed: ws[e][hh] = wg[h0+hh][e]
        for (int i = tid; i < ROUTE_KC * E; i += 256) {
            const int hh = i / E, e = i - hh * E;
            ws[e * ROUTE_LD + hh] = wg[(size_t)(h0 + hh) * E + e];
        }
        __syncthreads();
        float part[4][TE];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int i = 0; i < TE; ++i) part[a][i] = 0.f;
#pragma unroll
        for (int k8 = 0; k8 < ROUTE_KC; k8 += 8) {
            uint4 xv[4], wv[TE];
#pragma unroll
            for (int a = 0; a < 4; ++a) xv[a] = *reinterpret_cast<const uint4*>(xs + (tg * 4 + a) * ROUTE_LD + k8);
#pragma unroll
            for (int i = 0; i < TE; ++i) wv[i] = *reinterpret_cast<const uint4*>(ws + (el + 32 * i) * ROUTE_LD + k8);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float xl[4], xh[4], wl[TE], wh[TE];
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const uint32_t u = (&xv[a].x)[q];
                    xl[a] = __uint_as_float(u << 16);
                    xh[a] = __uint_as_float(u & 0xffff0000u);
                }
#pragma unroll
                for (int i = 0; i < TE; ++i) {
                    const uint32_t u = (&wv[i].x)[q];
                    wl[i] = __uint_as_float(u << 16);
                    wh[i] = __uint_as_float(u & 0xffff0000u);
                }
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int i = 0; i < TE; ++i) {
                        part[a][i] = fmaf(xl[a], wl[i], part[a][i]);
                        part[a][i] = fmaf(xh[a], wh[i], part[a][i]);
                    }
            }
        }
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int i = 0; i < TE; ++i) acc[a][i] += part[a][i];
    }

    // park logits (+bias) in LDS; padded experts get -inf
    __syncthreads();  // every thread is done reading ws
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int i = 0; i < TE; ++i) {
            const int e = el + 32 * i;
            float v = -INFINITY;
            if (e < E) v = acc[a][i] + (bias ? bias[e] : 0.f);
            lg[(tg * 4 + a) * EP + e] = v;
        }
    __syncthreads();

    // phase 2: one wavefront per token
    constexpr int NV = (EP + 63) / 64;
    const int lane = tid & 63, wave = tid >> 6;
    for (int tt = wave; tt < ROUTE_TOK; tt += 4) {
        const int t = t0 + tt;
        if (t >= T) break;  // wave-uniform
        float v[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int e = lane + 64 * i;
            v[i] = (e < EP) ? lg[tt * EP + e] : -INFINITY;
        }
        route_finish<NV>(v, lane, t, E, k, renorm, scale, idx_out, w_out, logits_out);
    }
}

// Few experts (E <= 16): HBM-bound.  One wavefront takes SMALL_TOK tokens; lane l owns the hidden
// elements h = 512*it + 8*l .. +7, so a wave reads 1 KiB of each token row per step and the
// matching 8 rows of Wg (8*E contiguous bf16, cache resident).  Per-lane partial sums are
// combined by a butterfly, after which every lane holds every logit.
constexpr int SMALL_TOK = 4;

template <int EP, bool EXACT>  // EP: padded expert count (8 or 16); EXACT: E == EP, rows of Wg are 16-byte vectors
__global__ __launch_bounds__(256) void route_small_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg,
                                                          const float* __restrict__ bias, int T, int H, int E, int k,
                                                          int renorm, float scale, int32_t* __restrict__ idx_out,
                                                          float* __restrict__ w_out, float* __restrict__ logits_out) {
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int t0 = wave * SMALL_TOK;
    if (t0 >= T) return;
    float acc[SMALL_TOK][EP];
#pragma unroll
    for (int a = 0; a < SMALL_TOK; ++a)
#pragma unroll
        for (int e = 0; e < EP; ++e) acc[a][e] = 0.f;
    for (int h0 = lane * 8; h0 < H; h0 += 512) {
        uint4 xv[SMALL_TOK];
#pragma unroll
        for (int a = 0; a < SMALL_TOK; ++a) {
            const int t = min(t0 + a, T - 1);
            xv[a] = *reinterpret_cast<const uint4*>(x + (size_t)t * H + h0);
        }
#pragma unroll
        for (int hh = 0; hh < 8; ++hh) {
            float xa[SMALL_TOK];
#pragma unroll
            for (int a = 0; a < SMALL_TOK; ++a) {
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
                for (int a = 0; a < SMALL_TOK; ++a) acc[a][e] = fmaf(xa[a], wv[e], acc[a][e]);
        }
    }
#pragma unroll
    for (int a = 0; a < SMALL_TOK; ++a) {
        const int t = t0 + a;
        if (t >= T) break;  // wave-uniform
        float mine = -INFINITY;
#pragma unroll
        for (int e = 0; e < EP; ++e) {
            const float tot = wave_sum(acc[a][e]);
            if (lane == e && e < E) mine = tot + (bias ? bias[e] : 0.f);
        }
        const float v[1] = {mine};
        route_finish<1>(v, lane, t, E, k, renorm, scale, idx_out, w_out, logits_out);
    }
}

}  // namespace

hipError_t launch_route(const moe_shape& s, const void* x, const void* wg, const float* bias, int32_t* idx,
                        float* w, float* logits, hipStream_t st) {
    if (s.E <= 16) {
        const dim3 g((s.T + 4 * SMALL_TOK - 1) / (4 * SMALL_TOK)), b(256);
#define ROUTE_SMALL(EP_, EX_)                                                                                  \
    hipLaunchKernelGGL((route_small_kernel<EP_, EX_>), g, b, 0, st, (const uint16_t*)x, (const uint16_t*)wg, bias, \
                       s.T, s.H, s.E, s.top_k, s.renormalize, s.routed_scale, idx, w, logits)
        if (s.E == 8) ROUTE_SMALL(8, true);
        else if (s.E < 8) ROUTE_SMALL(8, false);
        else if (s.E == 16) ROUTE_SMALL(16, true);
        else ROUTE_SMALL(16, false);
#undef ROUTE_SMALL
        return hipGetLastError();
    }
    const dim3 grid((s.T + ROUTE_TOK - 1) / ROUTE_TOK), block(256);
    const int te = (s.E + 31) / 32;
#define ROUTE_CASE(N)                                                                                         \
    case N:                                                                                                   \
        hipLaunchKernelGGL(route_kernel<N>, grid, block, 0, st, (const uint16_t*)x, (const uint16_t*)wg, bias, \
                           s.T, s.H, s.E, s.top_k, s.renormalize, s.routed_scale, idx, w, logits);            \
        break;
    switch (te) {
        ROUTE_CASE(1) ROUTE_CASE(2) ROUTE_CASE(3) ROUTE_CASE(4) ROUTE_CASE(5) ROUTE_CASE(6) ROUTE_CASE(7) ROUTE_CASE(8)
        default: return hipErrorInvalidValue;
    }
#undef ROUTE_CASE
    return hipGetLastError();
}

}  // namespace moe
