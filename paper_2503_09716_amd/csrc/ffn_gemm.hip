// Grouped SwiGLU FFN as two grouped bf16 MFMA GEMMs with fp32 accumulation.
// (Sec. 2: each token is processed by its k selected experts; Sec. 4.2: experts see one large
// accumulated batch, so each expert's rows form a tall matrix and the GEMMs are compute bound.)
//
//   GEMM 1 (gated):  h[r, f]  = silu(X_e[r,:] . W1p_e[f,:]) * (X_e[r,:] . W3p_e[f,:])      -> bf16
//   GEMM 2        :  y[r, n]  = h[r,:] . W2p_e[n,:]                                        -> bf16
// Both operands are K-contiguous ("packed" weights), so one tile routine serves both.
//
// Tile routine (one workgroup = 4 wavefronts, one per SIMD, up to 512 registers each):
//   * macro tile: BM rows of X (256/128/64/32) x 256 rows of W (GEMM 1: 128 gate + 128 up rows,
//     so the SiLU-gate product is formed in registers), K step 64.
//   * global -> LDS with global_load_lds_dwordx4 (no VGPR round trip), two LDS stages
//     (2 x 64 KiB at BM = 256), one barrier per K step.
//   * LDS layout: 128-byte rows (64 bf16), the eight 16-byte pieces of a row XOR-swizzled by
//     (row ^ row/8) & 7 so that the 16-byte MFMA operand reads of 16 consecutive rows fall in
//     distinct banks.  The swizzle is applied by choosing which global piece each lane of the
//     direct-to-LDS load fetches, since the LDS side of that load is fixed (lane * 16 bytes).
//   * v_mfma_f32_32x32x16_bf16 with W as the row (A) operand and X as the column (B) operand:
//     a lane's 16 accumulator registers then belong to ONE output row.  W rows are placed in
//     LDS in the order that makes those 16 registers 16 CONSECUTIVE output columns, so the
//     epilogue writes 2 x 16-byte stores per 32x32 block straight from registers.
//   * ragged tails: rows past the end of a group are clamped on load and masked on store;
//     short tails use the 128/64/32-row variants so padded MFMA work stays small.
//
// Work distribution: a device-built list of m-tiles (ffn_plan) x n-tiles; workgroup ids are
// remapped so each XCD (ids are dealt round-robin over the 8 XCDs) receives runs of 32
// consecutive tiles, and consecutive tiles sweep `group_m` m-tiles before moving along n, so
// the tiles resident on one XCD share weight panels and X panels in its L2.
#include <type_traits>

#include "common.h"

namespace moe {
namespace {

constexpr int BK = 64;              // K elements per LDS stage
constexpr int WROWS = 256;          // W rows per macro tile
constexpr int MAX_LDS = 2 * (256 + WROWS) * BK * 2;  // 131072 bytes

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ void load16_to_lds(const char* g, char* lds_wave_base) {
    // 64 lanes x 16 bytes land at lds_wave_base + lane*16 (the LDS address is wave-uniform).
    __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)lds_wave_base, 16, 0, 0);
}

__device__ __forceinline__ void wait_loads_and_sync() {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's direct-to-LDS loads have landed
    __syncthreads();
}

// Scheduling pattern for one K sub-step: after each MFMA place (at most) one LDS read and, while
// direct-to-LDS loads remain, `VPER` of them.  Emitted through templates because the builtin
// only takes literal constants.
template <int N, int NMFMA, int NREAD, int NLOAD>
__device__ __forceinline__ void sched_substep() {
    if constexpr (N < NMFMA) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // 1 MFMA
        if constexpr (N < NREAD) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // 1 LDS read
        constexpr int VPER = (NLOAD + NMFMA - 1) / NMFMA;
        if constexpr (N * VPER < NLOAD)
            __builtin_amdgcn_sched_group_barrier(0x070, (N + 1) * VPER <= NLOAD ? VPER : NLOAD - N * VPER, 0);  // VMEM
        sched_substep<N + 1, NMFMA, NREAD, NLOAD>();
    }
}

// WM x (4/WM) wave grid; TI = 32-row X blocks per wave; GATED = GEMM 1.
template <int WM, int TI, bool GATED>
__device__ __forceinline__ void gemm_tile(const GemmArgs& p, const TileDesc d, const int n_tile, char* lds) {
    constexpr int WN = 4 / WM;
    constexpr int TJ = 8 / WN;               // 32-row W blocks per wave
    constexpr int BM = WM * TI * 32;
    constexpr int XBYTES = BM * BK * 2;
    constexpr int STAGE = XBYTES + WROWS * BK * 2;
    constexpr int NLX = BM / 32;             // direct-to-LDS loads per wave per stage, X part
    constexpr int NLW = WROWS / 32;          // ... W part
    constexpr int BN = GATED ? 128 : 256;    // output columns per macro tile
    constexpr int TJH = TJ / 2;              // GATED: gate blocks per wave (= up blocks per wave)

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int K = p.K, N = p.N;
    const int n0 = n_tile * BN;
    const bool shared = d.srow >= 0;
    const int nseg = (!GATED && shared) ? p.nseg_shared : 1;

    // ------------------------------------------------------------------ loader setup
    const int lrow = lane >> 3, lslot = lane & 7;
    uint32_t xoff[NLX], woff[NLW];
#pragma unroll
    for (int i = 0; i < NLX; ++i) {
        const int q = i * 4 + wave;               // wave-load index inside the X region
        int r = q * 8 + lrow;                     // tile row 0..BM-1
        if (r > d.nrows - 1) r = d.nrows - 1;     // clamp: padded rows re-read the last valid row
        int grow = d.row0 + r;
        if (GATED && !shared && p.row_token) grow = p.row_token[grow];
        const int c = lslot ^ ((lrow ^ q) & 7);   // logical 16-byte piece that lands in slot lslot
        xoff[i] = (uint32_t)grow * (uint32_t)(K * 2) + (uint32_t)(c * 16);
    }
#pragma unroll
    for (int i = 0; i < NLW; ++i) {
        const int q = i * 4 + wave;               // wave-load index inside the W region; block = i
        const int rho = wave * 8 + lrow;          // LDS row inside the 32-row block = MFMA row
        const int nloc = ((rho >> 2) & 1) * 16 + (rho >> 3) * 4 + (rho & 3);
        int n = n0 + (GATED ? (i & 3) : i) * 32 + nloc;
        if (n > N - 1) n = N - 1;
        const int c = lslot ^ ((lrow ^ q) & 7);
        woff[i] = (uint32_t)n * (uint32_t)(K * 2) + (uint32_t)(c * 16);
    }
    const char* const a_base = shared ? p.a_shared : p.a_routed;
    const size_t a_seg_stride = (size_t)p.T * (size_t)K * 2;
    const char* a_ptr = a_base;
    const char* wa_ptr = nullptr;
    const char* wb_ptr = nullptr;

    // Enqueues the direct-to-LDS loads of one K tile and moves the (wave-uniform) source
    // pointers to the next tile.  Branch-free, so the loads can be scheduled between MFMAs.
    auto issue = [&](const int stage) {
        char* xs = lds + stage * STAGE;
        char* ws = xs + XBYTES;
#pragma unroll
        for (int i = 0; i < NLX; ++i) load16_to_lds(a_ptr + xoff[i], xs + (i * 4 + wave) * 1024);
#pragma unroll
        for (int i = 0; i < NLW; ++i)
            load16_to_lds(((GATED && i >= 4) ? wb_ptr : wa_ptr) + woff[i], ws + (i * 4 + wave) * 1024);
        a_ptr += BK * 2;
        wa_ptr += BK * 2;
        if (GATED) wb_ptr += BK * 2;
    };

    // ------------------------------------------------------------------ reader setup
    const int rl = lane & 31, g = lane >> 5;
    const int tsw = (g ^ (rl & 7) ^ (rl >> 3)) & 7;
    // offU[u] : byte offset inside a 32-row block for swizzle selector u (piece = tsw ^ 2u)
    uint32_t offU[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) offU[u] = (uint32_t)(rl * 128 + ((tsw ^ (2 * u)) << 4));
    // first X / W block of this wave and its parity (parity flips the piece index by 4)
    const int bx0 = wm * TI;
    const int bw0 = GATED ? wn * TJH : wn * TJ;
    uint32_t offX[4], offW[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        offX[kk] = ((bx0 & 1) ? offU[kk ^ 2] : offU[kk]) + (uint32_t)(bx0 * 4096);
        offW[kk] = ((bw0 & 1) ? offU[kk ^ 2] : offU[kk]) + (uint32_t)(XBYTES + bw0 * 4096);
    }

    f32x16 acc[TJ][TI];
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.f;

    // Software pipeline (one K tile = 4 sub-steps kk of 16):
    //   top of iteration : direct-to-LDS loads of the NEXT tile go out, interleaved with the
    //                      MFMAs of kk = 0 so the matrix pipe never waits for their issue
    //   kk = 0..2        : LDS reads of kk+1 are interleaved with the MFMAs of kk
    //   before kk = 3    : vmcnt(0) + barrier (next tile landed, everyone is done reading this
    //                      one), then the kk = 0 fragments of the NEXT tile are read while the
    //                      MFMAs of kk = 3 run.
    // Fragments live in two register buffers that alternate per sub-step.
    auto load_frags = [&](const char* base, const int kk, bf16x8 (&xf)[TI], bf16x8 (&wf)[TJ]) {
#pragma unroll
        for (int i = 0; i < TI; ++i)
            xf[i] = *reinterpret_cast<const bf16x8*>(base + offX[kk ^ ((i & 1) << 1)] + i * 4096);
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            // relative W block: GEMM 2: j; GEMM 1: gate blocks j < TJH, up blocks 4 + (j - TJH)
            const int rel = GATED ? (j < TJH ? j : 4 + (j - TJH)) : j;
            wf[j] = *reinterpret_cast<const bf16x8*>(base + offW[kk ^ ((rel & 1) << 1)] + rel * 4096);
        }
    };
    auto mfmas = [&](const bf16x8 (&xf)[TI], const bf16x8 (&wf)[TJ]) {
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int i = 0; i < TI; ++i)
                acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], xf[i], acc[j][i], 0, 0, 0);
    };
    constexpr int NMFMA = TI * TJ;      // per sub-step
    constexpr int NREAD = TI + TJ;      // LDS reads per sub-step
    constexpr int NLOAD = NLX + NLW;    // direct-to-LDS loads per tile per wave

    const int KT = K / BK;
    bf16x8 xf0[TI], wf0[TJ], xf1[TI], wf1[TJ];
    // MORE = another K tile follows (the last iteration is peeled so the body has no branches).
    auto body = [&](auto more_tag, const int kt) {
        constexpr bool MORE = decltype(more_tag)::value;
        const char* cur = lds + (kt & 1) * STAGE;
        const char* nxt = lds + ((kt & 1) ^ 1) * STAGE;
        // ---- kk = 0 (+ global loads of the next tile, + LDS reads of kk = 1)
        if (MORE) issue((kt & 1) ^ 1);
        load_frags(cur, 1, xf1, wf1);
        mfmas(xf0, wf0);
        sched_substep<0, NMFMA, NREAD, MORE ? NLOAD : 0>();
        __builtin_amdgcn_sched_barrier(0);
        // ---- kk = 1
        load_frags(cur, 2, xf0, wf0);
        mfmas(xf1, wf1);
        sched_substep<0, NMFMA, NREAD, 0>();
        __builtin_amdgcn_sched_barrier(0);
        // ---- kk = 2
        load_frags(cur, 3, xf1, wf1);
        mfmas(xf0, wf0);
        sched_substep<0, NMFMA, NREAD, 0>();
        __builtin_amdgcn_sched_barrier(0);
        // ---- kk = 3: hand-over to the next tile
        wait_loads_and_sync();
        if (MORE) load_frags(nxt, 0, xf0, wf0);
        mfmas(xf1, wf1);
        sched_substep<0, NMFMA, MORE ? NREAD : 0, 0>();
        __builtin_amdgcn_sched_barrier(0);
    };
    // GEMM 2 on shared experts walks `nseg` K-concatenated segments (one per shared expert);
    // every other tile has one segment.  The pipeline drains and restarts between segments.
    for (int seg = 0; seg < nseg; ++seg) {
        a_ptr = a_base + (size_t)seg * a_seg_stride;
        wa_ptr = (const char*)p.w_a[d.group + seg];
        if (GATED) wb_ptr = (const char*)p.w_b[d.group];
        issue(0);
        wait_loads_and_sync();
        load_frags(lds, 0, xf0, wf0);
        for (int kt = 0; kt < KT - 1; ++kt) body(std::true_type{}, kt);
        body(std::false_type{}, KT - 1);
    }

    // ------------------------------------------------------------------ epilogue
    // lane: output row = block row (lane & 31); its 16 registers of block j are output columns
    // (block column base) + (lane >> 5) * 16 + 0..15.
    char* out = shared ? p.out_shared : p.out_routed;
    const int orow_base = (shared ? (GATED ? d.srow : 0) : 0) + d.row0;
#pragma unroll
    for (int i = 0; i < TI; ++i) {
        const int r = (bx0 + i) * 32 + rl;
        if (r >= d.nrows) continue;
        char* orow = out + (size_t)(orow_base + r) * (size_t)N * 2;
        if (GATED) {
#pragma unroll
            for (int j = 0; j < TJH; ++j) {
                const int col = n0 + (bw0 + j) * 32 + g * 16;
                if (col >= N) continue;
                bf16x8 o0, o1;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const float g0 = acc[j][i][q], u0 = acc[j + TJH][i][q];
                    const float g1 = acc[j][i][q + 8], u1 = acc[j + TJH][i][q + 8];
                    o0[q] = (__bf16)((g0 / (1.0f + __expf(-g0))) * u0);
                    o1[q] = (__bf16)((g1 / (1.0f + __expf(-g1))) * u1);
                }
                *reinterpret_cast<bf16x8*>(orow + (size_t)col * 2) = o0;
                *reinterpret_cast<bf16x8*>(orow + (size_t)col * 2 + 16) = o1;
            }
        } else if (p.out_fp32) {
            orow = out + (size_t)(orow_base + r) * (size_t)N * 4;
#pragma unroll
            for (int j = 0; j < TJ; ++j) {
                const int col = n0 + (bw0 + j) * 32 + g * 16;
                if (col >= N) continue;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = acc[j][i][q * 4 + e];
                    *reinterpret_cast<f32x4*>(orow + (size_t)col * 4 + q * 16) = o;
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < TJ; ++j) {
                const int col = n0 + (bw0 + j) * 32 + g * 16;
                if (col >= N) continue;
                bf16x8 o0, o1;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    o0[q] = (__bf16)acc[j][i][q];
                    o1[q] = (__bf16)acc[j][i][q + 8];
                }
                *reinterpret_cast<bf16x8*>(orow + (size_t)col * 2) = o0;
                *reinterpret_cast<bf16x8*>(orow + (size_t)col * 2 + 16) = o1;
            }
        }
    }
}

// Workgroup id -> position in the tile order.  Hardware deals consecutive workgroup ids to the
// 8 XCDs in turn; inside each run of 256 ids, XCD x is given tiles [32x, 32x+32).
__device__ __forceinline__ int tile_order(const int wg, const int total, const int remap) {
    if (!remap) return wg;
    const int full = total & ~255;
    if (wg >= full) return wg;
    const int q = wg >> 8, r = wg & 255;
    return (q << 8) + ((r & 7) << 5) + (r >> 3);
}

template <int WM, bool GATED>
__global__ __launch_bounds__(256, 1) void ffn_gemm_kernel(const GemmArgs p) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int L = tile_order(blockIdx.x, gridDim.x, p.xcd_remap);
    // consecutive positions: group_m m-tiles first, then along n
    const int per_super = p.group_m * p.n_tiles;
    const int sr = L / per_super;
    const int rem = L - sr * per_super;
    const int mt0 = sr * p.group_m;
    const int gm = min(p.group_m, p.max_mtiles - mt0);
    const int n_tile = rem / gm;
    const int mt = mt0 + (rem - n_tile * gm);
    const int count = GATED ? p.plan->n_gate_up : p.plan->n_down;
    if (mt >= count) return;  // uniform for the workgroup
    const TileDesc d = p.descs[mt];
    const int blocks = p.small_tiles ? (d.nrows + 31) >> 5 : 8;  // 32-row blocks that hold real rows
    if (WM == 2) {
        if (blocks > 4) gemm_tile<2, 4, GATED>(p, d, n_tile, lds);
        else if (blocks > 2) gemm_tile<2, 2, GATED>(p, d, n_tile, lds);
        else gemm_tile<2, 1, GATED>(p, d, n_tile, lds);
    } else {
        if (blocks > 4) gemm_tile<1, 8, GATED>(p, d, n_tile, lds);
        else if (blocks > 2) gemm_tile<1, 4, GATED>(p, d, n_tile, lds);
        else if (blocks > 1) gemm_tile<1, 2, GATED>(p, d, n_tile, lds);
        else gemm_tile<1, 1, GATED>(p, d, n_tile, lds);
    }
}

// Builds the m-tile list from expert_offsets.  Order: shared expert 0, routed experts, shared
// experts 1.. (GEMM 2 takes the first two parts: shared experts are concatenated along K there).
// A group of n rows becomes floor(n/256) full tiles plus one tail tile (small_tiles) or
// ceil(n/256) tiles of 256 rows (the kernel still picks a short variant for a short tail).
__global__ __launch_bounds__(256) void ffn_plan_kernel(const int32_t* __restrict__ offsets, int T, int E, int Ns,
                                                       PlanHeader* __restrict__ plan, TileDesc* __restrict__ descs) {
    __shared__ int first[256];
    const int tid = threadIdx.x;
    const int shared_tiles = (T + 255) / 256;
    // group order: g = 0 -> shared 0 (if any), then routed 0..E-1, then shared 1..Ns-1
    const int ngroups = E + Ns;
    int ntiles = 0, row_begin = 0, rows = 0, group = 0, srow = -1;
    if (tid < ngroups) {
        int pos = tid;
        if (Ns > 0 && pos == 0) { group = E; rows = T; row_begin = 0; srow = 0; }
        else {
            if (Ns > 0) pos -= 1;
            if (pos < E) { group = pos; row_begin = offsets[pos]; rows = offsets[pos + 1] - row_begin; srow = -1; }
            else { const int s = pos - E + 1; group = E + s; rows = T; row_begin = 0; srow = s * T; }
        }
        ntiles = (rows + 255) / 256;
    }
    first[tid] = ntiles;
    __syncthreads();
    if (tid == 0) {
        int run = 0, down = 0;
        for (int i = 0; i < ngroups && i < 256; ++i) {
            const int v = first[i];
            first[i] = run;
            run += v;
            if (i == (Ns > 0 ? E : E - 1)) down = run;  // end of (shared 0 +) routed part
        }
        if (Ns == 0) down = run;
        plan->n_gate_up = run;
        plan->n_down = down;
        plan->pad[0] = shared_tiles;
        plan->pad[1] = 0;
    }
    __syncthreads();
    if (tid < ngroups) {
        const int base = first[tid];
        for (int i = 0; i < ntiles; ++i) {
            TileDesc d;
            d.group = group;
            d.row0 = row_begin + i * 256;
            d.nrows = min(256, rows - i * 256);
            d.srow = srow;
            descs[base + i] = d;
        }
    }
}

}  // namespace

hipError_t ffn_gemm_init() {
    hipError_t e;
#define SET_LDS(K_)                                                                                            \
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&K_), hipFuncAttributeMaxDynamicSharedMemorySize,    \
                            MAX_LDS);                                                                          \
    if (e != hipSuccess) return e;
    SET_LDS((ffn_gemm_kernel<2, true>))
    SET_LDS((ffn_gemm_kernel<2, false>))
    SET_LDS((ffn_gemm_kernel<1, true>))
    SET_LDS((ffn_gemm_kernel<1, false>))
#undef SET_LDS
    return hipSuccess;
}

hipError_t launch_ffn_plan(const moe_shape& s, const int32_t* offsets, PlanHeader* plan, TileDesc* descs,
                           int small_tiles, int wave_rows, hipStream_t st) {
    (void)small_tiles;
    (void)wave_rows;
    hipLaunchKernelGGL(ffn_plan_kernel, dim3(1), dim3(256), 0, st, offsets, s.T, s.E, s.num_shared, plan, descs);
    return hipGetLastError();
}

hipError_t launch_ffn_gemm(bool gated, const GemmArgs& a, const GemmConfig& cfg, hipStream_t st) {
    const dim3 grid((unsigned)(a.max_mtiles * a.n_tiles)), block(256);
    if (cfg.wave_rows == 2) {
        if (gated) hipLaunchKernelGGL((ffn_gemm_kernel<2, true>), grid, block, MAX_LDS, st, a);
        else hipLaunchKernelGGL((ffn_gemm_kernel<2, false>), grid, block, MAX_LDS, st, a);
    } else {
        if (gated) hipLaunchKernelGGL((ffn_gemm_kernel<1, true>), grid, block, MAX_LDS, st, a);
        else hipLaunchKernelGGL((ffn_gemm_kernel<1, false>), grid, block, MAX_LDS, st, a);
    }
    return hipGetLastError();
}

}  // namespace moe
