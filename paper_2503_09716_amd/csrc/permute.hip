// Permutation of (token, rank) pairs into per-expert contiguous groups: histogram, prefix
// sums, stable placement, and the coalesced row gather.  (Sec. 2: each token is processed by
// its k selected experts; Sec. 4.3: the per-expert token counts are only known at run time.)
//
// Canonical order = ascending expert id, then ascending token id, so the result is unique
// and every run is bit-identical.  Tokens are cut into chunks of PERMUTE_CHUNK_TOKENS; one
// workgroup owns one chunk:
//   count : per-chunk per-expert histogram
//   scan  : per-expert exclusive prefix over chunks, then exclusive prefix over experts
//   place : a 64-bit lane mask per expert and wavefront (built with integer OR in LDS) gives
//           each (token, rank) pair its position among its expert's rows of the chunk
//           (popcount of the lower lanes and of the lower wavefronts' masks)
//   gather: x_perm[r,:] = x[perm[r]/k,:] in 16-byte pieces, one row per wavefront pass
// Launches: one for small batches (every workgroup counts everything itself), two for the
// usual sizes (count; scan + place), three when the table of histograms is too large for every
// workgroup to add up.
#include "common.h"

namespace moe {
namespace {

constexpr int MAX_E = 256;

__global__ __launch_bounds__(256) void permute_count_kernel(const int32_t* __restrict__ idx, int T, int k, int E,
                                                            int32_t* __restrict__ chunk_counts) {
    __shared__ int cnt[MAX_E];
    const int tid = threadIdx.x, chunk = blockIdx.x;
    for (int e = tid; e < E; e += 256) cnt[e] = 0;
    __syncthreads();
    const int t0 = chunk * PERMUTE_CHUNK_TOKENS;
    const int t1 = min(T, t0 + PERMUTE_CHUNK_TOKENS);
    const int n = (t1 - t0) * k;
    const int32_t* p = idx + (size_t)t0 * k;
    for (int i = tid; i < n; i += 256) {
        const int e = p[i];
        if ((unsigned)e < (unsigned)E) atomicAdd(&cnt[e], 1);  // integer LDS counters: order-independent
    }
    __syncthreads();
    for (int e = tid; e < E; e += 256) chunk_counts[(size_t)chunk * E + e] = cnt[e];
}

// chunk_counts[c][e] -> exclusive prefix over c (in place); offsets[e] = exclusive prefix over experts.
__global__ __launch_bounds__(256) void permute_scan_kernel(int32_t* __restrict__ chunk_counts, int nchunks, int E,
                                                           int32_t* __restrict__ offsets) {
    __shared__ int total[MAX_E];
    const int tid = threadIdx.x;
    for (int e = tid; e < E; e += 256) {
        int run = 0;
        for (int c0 = 0; c0 < nchunks; c0 += 16) {
            int v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = (c0 + u < nchunks) ? chunk_counts[(size_t)(c0 + u) * E + e] : 0;
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                if (c0 + u < nchunks) chunk_counts[(size_t)(c0 + u) * E + e] = run;
                run += v[u];
            }
        }
        total[e] = run;
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) {
            offsets[e] = run;
            run += total[e];
        }
        offsets[E] = run;
    }
}

// Placement: one wavefront per chunk, 64 tokens per step.  Every lane ORs its lane bit into a
// 64-bit LDS mask per selected expert (an order-independent integer operation); the rank of a
// token inside its expert's rows of this step is then the number of lower lanes in that mask,
// which is exactly the stable token order.  The per-expert cursors live in LDS and advance by
// the mask's population count after each step.  Work per step is O(k) per lane plus O(E/64)
// for the cursor update, independent of how many experts the step touches.
__global__ __launch_bounds__(64) void permute_place_kernel(const int32_t* __restrict__ idx, int T, int k, int E,
                                                           const int32_t* __restrict__ chunk_prefix,
                                                           const int32_t* __restrict__ offsets,
                                                           int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
                                                           int32_t* __restrict__ row_token) {
    __shared__ unsigned long long mask[MAX_E];
    __shared__ int cur[MAX_E];
    const int lane = threadIdx.x, chunk = blockIdx.x;
    for (int e = lane; e < E; e += 64) {
        cur[e] = offsets[e] + chunk_prefix[(size_t)chunk * E + e];
        mask[e] = 0ull;
    }
    __syncthreads();
    const unsigned long long bit = 1ull << lane, lt = bit - 1ull;
    const int t0 = chunk * PERMUTE_CHUNK_TOKENS;
    for (int s = 0; s < PERMUTE_CHUNK_TOKENS; s += 64) {
        if (t0 + s >= T) break;
        const int t = t0 + s + lane;
        const bool valid = t < T;
        const int32_t* mine = idx + (size_t)t * k;
        if (valid)
            for (int j = 0; j < k; ++j) {
                const int e = mine[j];
                if ((unsigned)e < (unsigned)E) atomicOr(&mask[e], bit);
            }
        __syncthreads();
        if (valid)
            for (int j = 0; j < k; ++j) {
                const int e = mine[j];
                if ((unsigned)e >= (unsigned)E) continue;
                const int slot = cur[e] + __popcll(mask[e] & lt);
                perm[slot] = t * k + j;
                inv_perm[(size_t)t * k + j] = slot;
                if (row_token) row_token[slot] = t;
            }
        __syncthreads();
        for (int e = lane; e < E; e += 64) {
            cur[e] += __popcll(mask[e]);
            mask[e] = 0ull;
        }
        __syncthreads();
    }
}

// Common tail of the two kernels below.  Thread e < E comes in with its expert's pair count over
// all chunks (total) and over the chunks before this workgroup's (before); mask[][] is zero.
// Exclusive prefix sum of the totals over the experts (-> expert_offsets, written by chunk 0, and
// this chunk's cursors), then the placement of the chunk: wavefront w takes tokens 64w .. 64w+63,
// the lane masks of all four wavefronts give a pair its rank.
__device__ __forceinline__ void scan_and_place_chunk(const int32_t* __restrict__ idx, const int T, const int k, const int E,
                                                     const int total, const int before,
                                                     unsigned long long (&mask)[4][MAX_E], int (&cur)[MAX_E],
                                                     int (&wave_sum)[4], int32_t* __restrict__ offsets,
                                                     int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
                                                     int32_t* __restrict__ row_token) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, chunk = blockIdx.x;
    int incl = total;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int t = __shfl_up(incl, d, 64);
        if (lane >= d) incl += t;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    int base = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w)
        if (w < wave) base += wave_sum[w];
    const int excl = base + incl - total;
    if (tid < E) {
        cur[tid] = excl + before;
        if (chunk == 0) offsets[tid] = excl;
    }
    if (chunk == 0 && tid == E - 1) offsets[E] = excl + total;
    // placement of this chunk: wave w owns tokens 64w .. 64w+63
    const int t = chunk * PERMUTE_CHUNK_TOKENS + tid;
    const bool valid = t < T;
    const int32_t* mine = idx + (size_t)t * k;
    const unsigned long long bit = 1ull << lane, lt = bit - 1ull;
    if (valid)
        for (int j = 0; j < k; ++j) {
            const int e = mine[j];
            if ((unsigned)e < (unsigned)E) atomicOr(&mask[wave][e], bit);
        }
    __syncthreads();
    if (valid)
        for (int j = 0; j < k; ++j) {
            const int e = mine[j];
            if ((unsigned)e >= (unsigned)E) continue;
            int slot = cur[e] + __popcll(mask[wave][e] & lt);
            for (int w = 0; w < wave; ++w) slot += __popcll(mask[w][e]);
            perm[slot] = t * k + j;
            inv_perm[(size_t)t * k + j] = slot;
            if (row_token) row_token[slot] = t;
        }
}

// All three steps in ONE launch, for small batches (T*k <= FUSED_MAX_PAIRS), where two extra
// launches cost more than the work (256 tokens top-2: 6 us against 13; from a few thousand pairs
// on, the three kernels win: every workgroup here reads the whole index array): every workgroup
// (one per chunk, 4 wavefronts) histograms ALL pairs into wave-private LDS counters, once counting everything (-> expert_offsets, the same in
// every workgroup) and once counting only the chunks before its own (-> its cursors), then
// places its chunk: wavefront w takes tokens 64w .. 64w+63 of the chunk, the lane masks of all
// four wavefronts give a pair its rank.  Same result as the three kernels above, bit for bit,
// without their two extra launches.
constexpr int FUSED_MAX_PAIRS = 1 << 12;
static_assert(PERMUTE_CHUNK_TOKENS == 256, "the fused kernel gives each of its 4 wavefronts 64 tokens of a chunk");

__global__ __launch_bounds__(256) void permute_index_fused_kernel(const int32_t* __restrict__ idx, int T, int k, int E,
                                                                  int32_t* __restrict__ offsets, int32_t* __restrict__ perm,
                                                                  int32_t* __restrict__ inv_perm, int32_t* __restrict__ row_token) {
    __shared__ int hist[4][2][MAX_E];              // [wave][0: all chunks, 1: chunks before mine][expert]
    __shared__ unsigned long long mask[4][MAX_E];  // [wave][expert]: lanes of that wave that picked the expert
    __shared__ int cur[MAX_E];
    __shared__ int wave_sum[4];
    const int tid = threadIdx.x, wave = tid >> 6, chunk = blockIdx.x;
    for (int i = tid; i < 4 * 2 * MAX_E; i += 256) (&hist[0][0][0])[i] = 0;
    for (int i = tid; i < 4 * MAX_E; i += 256) (&mask[0][0])[i] = 0ull;
    __syncthreads();
    const int n = T * k;
    const int mine_begin = chunk * PERMUTE_CHUNK_TOKENS * k;   // pairs of earlier chunks come before this index
    for (int i = tid; i < n; i += 256) {
        const int e = idx[i];
        if ((unsigned)e < (unsigned)E) {
            atomicAdd(&hist[wave][0][e], 1);                   // integer LDS counters: order-independent
            if (i < mine_begin) atomicAdd(&hist[wave][1][e], 1);
        }
    }
    __syncthreads();
    int total = 0, before = 0;
    if (tid < E) {
#pragma unroll
        for (int w = 0; w < 4; ++w) { total += hist[w][0][tid]; before += hist[w][1][tid]; }
    }
    scan_and_place_chunk(idx, T, k, E, total, before, mask, cur, wave_sum, offsets, perm, inv_perm, row_token);
}

// Scan + placement in one launch, from the per-chunk histograms of permute_count_kernel: every
// workgroup adds up the histograms of all chunks (-> expert_offsets) and of the chunks before its
// own (-> its cursors), then places its chunk like the kernel above.  Thread i sums expert
// i % EP2 over the chunks i / EP2, i / EP2 + 256 / EP2, ... (EP2 = E rounded up to a power of two),
// the partial sums meet in integer LDS counters.  nchunks * E integers are read by every
// workgroup, so the launcher takes this path only while that stays small.
constexpr int PLACE_SCAN_MAX_COUNTS = 1 << 14;

__global__ __launch_bounds__(256) void permute_place_scan_kernel(const int32_t* __restrict__ idx, int T, int k, int E, int ep2,
                                                                 const int32_t* __restrict__ chunk_counts, int nchunks,
                                                                 int32_t* __restrict__ offsets, int32_t* __restrict__ perm,
                                                                 int32_t* __restrict__ inv_perm, int32_t* __restrict__ row_token) {
    __shared__ int sum[2][MAX_E];                  // [0: all chunks, 1: chunks before mine][expert]
    __shared__ unsigned long long mask[4][MAX_E];
    __shared__ int cur[MAX_E];
    __shared__ int wave_sum[4];
    const int tid = threadIdx.x, chunk = blockIdx.x;
    for (int i = tid; i < 2 * MAX_E; i += 256) (&sum[0][0])[i] = 0;
    for (int i = tid; i < 4 * MAX_E; i += 256) (&mask[0][0])[i] = 0ull;
    __syncthreads();
    const int e = tid & (ep2 - 1), step = 256 / ep2;
    if (e < E) {
        int all = 0, before = 0;
        for (int c = tid / ep2; c < nchunks; c += step) {
            const int v = chunk_counts[(size_t)c * E + e];
            all += v;
            if (c < chunk) before += v;
        }
        atomicAdd(&sum[0][e], all);                // integer LDS counters: order-independent
        atomicAdd(&sum[1][e], before);
    }
    __syncthreads();
    const int total = tid < E ? sum[0][tid] : 0, before = tid < E ? sum[1][tid] : 0;
    scan_and_place_chunk(idx, T, k, E, total, before, mask, cur, wave_sum, offsets, perm, inv_perm, row_token);
}

// One wavefront copies one row per pass; 16 bytes per lane, consecutive lanes consecutive addresses.
__global__ __launch_bounds__(256) void permute_gather_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ perm,
                                                             int R, int k, int row16, uint4* __restrict__ x_perm) {
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int nwaves = gridDim.x * 4;
    for (int r = wave; r < R; r += nwaves) {
        const int t = perm[r] / k;
        const uint4* src = x + (size_t)t * row16;
        uint4* dst = x_perm + (size_t)r * row16;
        for (int c = lane; c < row16; c += 64) dst[c] = src[c];
    }
}

// Gather into the tiled layout: one wavefront fills one 1 KiB block (16 permuted rows x 32
// columns): lane l reads the 16-byte piece (l%4) ^ block_swizzle(l/4) of row 16g + l/4 and writes
// slot l of the block, so every store instruction covers 1 KiB of consecutive memory.
__global__ __launch_bounds__(256) void permute_gather_tiled_kernel(const char* __restrict__ x,
                                                                   const int32_t* __restrict__ row_token, int R, int H,
                                                                   char* __restrict__ xt) {
    const int lane = threadIdx.x & 63;
    const int KT = H >> 5;
    const int nblocks = ((R + 15) >> 4) * KT;
    const int nwaves = gridDim.x * 4;
    const int piece = (lane & 3) ^ block_swizzle(lane >> 2);
    for (int b = blockIdx.x * 4 + (threadIdx.x >> 6); b < nblocks; b += nwaves) {
        const int g = b / KT, kt = b - g * KT;
        int r = g * 16 + (lane >> 2);
        if (r > R - 1) r = R - 1;
        const int t = row_token[r];
        const uint4 v = *reinterpret_cast<const uint4*>(x + ((size_t)t * H + kt * 32 + piece * 8) * 2);
        *reinterpret_cast<uint4*>(xt + (size_t)b * 1024 + lane * 16) = v;
    }
}

}  // namespace

hipError_t launch_permute_gather_tiled(const moe_shape& s, const void* x, const int32_t* row_token, void* x_tiled,
                                       hipStream_t st) {
    const int R = s.T * s.top_k;
    const int nblocks = ((R + 15) / 16) * (s.H / 32);
    const int blocks = (nblocks + 3) / 4 < 16384 ? (nblocks + 3) / 4 : 16384;
    hipLaunchKernelGGL(permute_gather_tiled_kernel, dim3(blocks), dim3(256), 0, st, (const char*)x, row_token, R, s.H,
                       (char*)x_tiled);
    return hipGetLastError();
}

hipError_t launch_permute_index(const moe_shape& s, const int32_t* idx, int32_t* chunk_counts, int32_t* offsets,
                                int32_t* perm, int32_t* inv_perm, int32_t* row_token, hipStream_t st) {
    const int nchunks = permute_chunks(s);
    if ((int64_t)s.T * s.top_k <= FUSED_MAX_PAIRS) {
        hipLaunchKernelGGL(permute_index_fused_kernel, dim3(nchunks), dim3(256), 0, st, idx, s.T, s.top_k, s.E, offsets, perm,
                           inv_perm, row_token);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(permute_count_kernel, dim3(nchunks), dim3(256), 0, st, idx, s.T, s.top_k, s.E, chunk_counts);
    if ((int64_t)nchunks * s.E <= PLACE_SCAN_MAX_COUNTS) {
        int ep2 = 1;
        while (ep2 < s.E) ep2 <<= 1;
        hipLaunchKernelGGL(permute_place_scan_kernel, dim3(nchunks), dim3(256), 0, st, idx, s.T, s.top_k, s.E, ep2,
                           (const int32_t*)chunk_counts, nchunks, offsets, perm, inv_perm, row_token);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(256), 0, st, chunk_counts, nchunks, s.E, offsets);
    hipLaunchKernelGGL(permute_place_kernel, dim3(nchunks), dim3(64), 0, st, idx, s.T, s.top_k, s.E,
                       (const int32_t*)chunk_counts, (const int32_t*)offsets, perm, inv_perm, row_token);
    return hipGetLastError();
}

// expert_offsets of an empty batch: the scan over zero chunks writes E + 1 zeros
hipError_t launch_zero_offsets(int E, int32_t* offsets, hipStream_t st) {
    hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(256), 0, st, (int32_t*)nullptr, 0, E, offsets);
    return hipGetLastError();
}

hipError_t launch_permute_gather(const moe_shape& s, const void* x, const int32_t* perm, void* x_perm,
                                 hipStream_t st) {
    const int R = s.T * s.top_k;
    const int blocks = (R + 3) / 4 < 8192 ? (R + 3) / 4 : 8192;
    hipLaunchKernelGGL(permute_gather_kernel, dim3(blocks), dim3(256), 0, st, (const uint4*)x, perm, R, s.top_k,
                       s.H / 8, (uint4*)x_perm);
    return hipGetLastError();
}

}  // namespace moe
