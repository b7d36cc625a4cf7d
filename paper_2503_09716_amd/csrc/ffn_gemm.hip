// Grouped SwiGLU FFN as two grouped bf16 MFMA GEMMs with fp32 accumulation.
// (Sec. 2: each token is processed by its k selected experts; Sec. 4.2: experts see one large
// accumulated batch, so each expert's rows form a tall matrix and the GEMMs are compute bound.)
//
//   GEMM 1 (gated):  h[r, f]  = silu(X_e[r,:] . W1p_e[f,:]) * (X_e[r,:] . W3p_e[f,:])      -> bf16
//   GEMM 2        :  y[r, n]  = h[r,:] . W2p_e[n,:]                                        -> fp32 / bf16
// One tile routine serves both.  Weights and h are stored TILED: a matrix [N, K] is cut into
// blocks of 16 rows x 32 k (1 KiB) laid out block-row-major ([N/16][K/32] blocks), and the 64
// 16-byte pieces inside a block are in exactly the order the tile routine wants them in LDS
// (row-major rows of 64 bytes, piece slot = piece ^ ((row/4)&3)).  One direct-to-LDS load of a
// wavefront then reads 1 KiB of consecutive memory (8 full 128-byte lines) instead of 16
// half-lines from 16 distant rows, which halves the number of L1->L2 requests in flight; the
// L1's pending-request capacity, not bandwidth, is what the row-major form ran into
// (TCP_PENDING_STALL_CYCLES at half of all cycles).  x is read row-major through the gather
// unless a tiled copy exists.
//
// Tile routine (one workgroup = NW wavefronts in a WM x WN grid):
//   * macro tile: BM rows of X (320/288/256/128/64/32) x 256 rows of W (GEMM 1: 128 gate + 128
//     up rows, so the SiLU-gate product is formed in registers); K advances in sub-tiles of 32.
//     The 288- and 320-row tiles (4 waves side by side only) keep the accumulators of their last
//     2-4 X blocks in VGPRs, the 256 AGPRs being full; they serve as the standard tile of GEMM 1
//     for large experts (fewer bytes from L2 per FLOP) and take in an expert's short tail.
//   * global -> LDS with buffer_load_dwordx4 ... lds (no VGPR round trip) into a ring of NS = 4
//     LDS stages (4 x 32 KiB at BM = 256): the loads of sub-tile t+3 are issued while sub-tile t
//     is multiplied, so HBM latency has three sub-tiles of MFMA work to hide behind, and they
//     are spread between the MFMAs (one every few) instead of bursting after the barrier.
//     One barrier per sub-tile; s_waitcnt vmcnt(n) waits only for the sub-tile needed next.
//   * LDS layout: 64-byte rows (32 bf16), the four 16-byte pieces of a row XOR-swizzled by
//     (4 - row / 4) & 3 so that each of the four 16-lane passes in which the LDS serves a
//     16-byte MFMA operand read falls in distinct banks (block_swizzle).  The swizzle is applied by choosing which global piece each lane of the
//     direct-to-LDS load fetches, since the LDS side of that load is fixed (lane * 16 bytes).
//   * v_mfma_f32_16x16x32_bf16: one instruction multiplies a 16-row block of each operand over
//     the whole sub-tile.  In a register-only loop on this workload's data it sustains 1.98
//     PFLOP/s under the chip's power limit against 1.72 for v_mfma_f32_32x32x16_bf16 (both reach
//     2.47 on zeros): a quarter of the accumulator traffic per multiply-add.  GEMM 1 feeds W as
//     the row operand (a lane then owns 4 consecutive output columns of one row: 8-byte stores
//     of bf16 h), GEMM 2 feeds X as the row operand (a lane owns one output column: a store
//     instruction writes 4 rows x 64 contiguous bytes of fp32 y).
//   * each operand fragment has one register copy; it is refilled from the next LDS stage
//     right after its last use, so reads run half a sub-tile ahead of the MFMAs that need
//     them.  The instruction stream is laid out by hand in small groups {MFMAs of one X block,
//     one or two LDS reads, at most one global load} fenced by scheduling barriers, so the
//     matrix pipe always has independent work queued.
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

constexpr int BK = 32;              // K elements per LDS stage
constexpr int ROWB = BK * 2;        // bytes per LDS row
constexpr int WROWS = 256;          // W rows per macro tile
constexpr int NS = 4;               // LDS ring depth
constexpr int MAX_ROWS = 320;       // tallest macro tile: a full 256-row tile that also takes a short tail of its group
constexpr int MAX_STAGE = (MAX_ROWS + WROWS) * ROWB;     // 36 KiB
constexpr int MAX_LDS = NS * MAX_STAGE;

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;
typedef __attribute__((address_space(3))) char* lds_t;

// Buffer descriptor over [ptr, ptr + 4 GiB - 1) for raw (untyped) accesses.  The pointer is
// wave-uniform by construction; readfirstlane tells the compiler so (otherwise every load is
// wrapped in a waterfall loop).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t uniform_rsrc(const void* ptr) {
    const uint64_t v = (uint64_t)ptr;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return __builtin_amdgcn_make_buffer_rsrc((void*)(((uint64_t)hi << 32) | lo), 0, 0xFFFFFFFF, 0x00020000);
}

// 64 lanes x 16 bytes from (descriptor base + voff + soff) to LDS at l + lane*16 (l wave-uniform).
// The 16-byte form exists on gfx950 only; the host pass of hipcc must not see it.
__device__ __forceinline__ void buffer_load16_to_lds(__amdgpu_buffer_rsrc_t rsrc, lptr_t l, uint32_t voff, int soff) {
#if defined(__gfx950__)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, l, 16, voff, soff, 0, 0);
#endif
}

// Descriptor over exactly [ptr, ptr + bytes): accesses at offsets >= bytes are dropped by hardware.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const void* ptr, uint32_t bytes) {
    const uint64_t v = (uint64_t)ptr;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return __builtin_amdgcn_make_buffer_rsrc((void*)(((uint64_t)hi << 32) | lo), 0, __builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}

__device__ __forceinline__ void buffer_store_b32(__amdgpu_buffer_rsrc_t rsrc, uint32_t voff, float v) {
#if defined(__gfx950__)
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), rsrc, voff, 0, 0);
#endif
}

__device__ __forceinline__ void buffer_store_bf16(__amdgpu_buffer_rsrc_t rsrc, uint32_t voff, float v) {
#if defined(__gfx950__)
    const __bf16 b = (__bf16)v;
    __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, b), rsrc, voff, 0, 0);
#endif
}

// c += a (16 x 32, row operand) * b (32 x 16, column operand).  Written as inline assembly with
// the accumulator tied to an AGPR quad: left to itself the register allocator (all 256 AGPRs
// hold accumulators) routes part of them through temporaries, two to four copies per MFMA.
// Hazards the compiler would otherwise cover: the operands come from LDS reads it still
// tracks (s_waitcnt); an accumulator is re-used only a full sub-tile (>= 8 MFMAs) later; the
// epilogue waits mfma_drain() before it reads accumulators.
__device__ __forceinline__ void mfma_16x16x32(f32x4& c, const bf16x8& a, const bf16x8& b) {
#if defined(__gfx950__)
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
#endif
}
// The same with the accumulator in VGPRs: the X blocks of a tall tile that the 256 AGPRs do not hold.
__device__ __forceinline__ void mfma_16x16x32_v(f32x4& c, const bf16x8& a, const bf16x8& b) {
#if defined(__gfx950__)
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
#endif
}
__device__ __forceinline__ void mfma_drain() {
#if defined(__gfx950__)
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
#endif
}

// Hand-over point of the LDS ring: wait until at most N of this wave's direct-to-LDS loads
// are still in flight (they retire in order, so everything older has landed) and until this
// wave's own LDS reads have returned, then meet the other waves.  A bare s_barrier is used
// instead of __syncthreads(), whose release fence would drain ALL outstanding loads and so
// serialise the ring; the empty asm statements keep the compiler from moving LDS accesses
// across the barrier.
template <int N>
__device__ __forceinline__ void ring_sync() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0070);  // vmcnt(N) lgkmcnt(0), gfx9 encoding
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// NW wavefronts as a WM x (NW/WM) grid; TI = 32-row X blocks per wave; GATED = GEMM 1.
template <int NW, int WM, int TI, bool GATED, bool UNIFORM = false>
__device__ __forceinline__ void gemm_tile(const GemmArgs& p, const TileDesc d, const int n_tile, char* lds) {
    constexpr int WN = NW / WM;
    constexpr int TJ = 8 / WN;               // 32-row W blocks per wave
    constexpr int BM = WM * TI * 32;
    constexpr int NLX = (BM / 16 + NW - 1) / NW;   // X wave-loads (16 rows x 64 B) per wave per stage
    constexpr int NQX = NLX * NW;                  // X wave-loads per stage (region padded to a multiple of NW)
    constexpr int XBYTES = NQX * 1024;
    constexpr int NL = NLX + (WROWS / 16) / NW;    // all wave-loads per wave per stage
    constexpr int NL0 = NL / 2;                    // issued in the first half of an iteration
    constexpr int RING_STRIDE = NL * NW * 1024;    // bytes per ring stage
    static_assert(NS * RING_STRIDE <= MAX_LDS, "ring does not fit");
    constexpr int BN = GATED ? 128 : 256;    // output columns per macro tile
    constexpr int TJH = TJ / 2;              // GATED: 32-row gate blocks per wave (= up blocks per wave)
    // The MFMA works on 16-row blocks (v_mfma_f32_16x16x32_bf16: one instruction spans a whole
    // K sub-tile of 32).  Per wave: XB blocks of X and WB blocks of W, the latter in two halves
    // of WBH (GEMM 1: gate blocks | up blocks).
    constexpr int XB = 2 * TI;
    constexpr int WB = 2 * TJ;
    constexpr int WBH = WB / 2;
    constexpr int XB_A = 64 / WB;            // X blocks whose accumulators fit the 256 AGPRs; the rest live in VGPRs
    static_assert(TJ >= 1 && (!GATED || TJ >= 2), "wave grid too wide");
    static_assert(BM <= MAX_ROWS, "tile too tall");

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int K = p.K, N = p.N;
    const int n0 = n_tile * BN;
    const bool shared = d.srow >= 0;
    // K-split.  Router GEMM: srow = -1 - s, the operands of piece s start s*K further along and
    // its partial output goes to rows s*split_rows + ...  Down GEMM with tail_splits > 1: a short
    // tail is cut into tail_splits pieces along K; srow = -2 - u, u counting the pieces of all
    // split tails; piece u covers K range (u % tail_splits) * K/tail_splits .. and writes fp32
    // partials to rows u * SPLIT_TAIL_ROWS of out_partial.
    const bool tail_split = !GATED && p.tail_splits > 1 && d.srow <= -2;
    const int piece = tail_split ? -2 - d.srow : (shared ? 0 : -1 - d.srow);
    const int split = tail_split ? piece % p.tail_splits : piece;
    const int nseg = (!GATED && shared) ? p.nseg_shared : 1;
    const int KT = (tail_split ? K / p.tail_splits : K) / BK;   // sub-tiles per segment (>= 2)
    // K step in bytes: one 1 KiB block for tiled operands, 64 bytes along a row for row-major x
    constexpr int kstep_w = 1024;
    // A operand layout (bit 0: routed tiles, bit 1: shared tiles): h is tiled; x is row-major
    // (read through the gather, by shared experts and by the router) unless a tiled x_perm exists
    const bool a_tiled = ((shared ? p.a_tiled >> 1 : p.a_tiled) & 1) != 0;
    const int kstep_x = a_tiled ? 1024 : ROWB;
    const char* const a_base = shared ? p.a_shared : p.a_routed;
    const size_t a_seg_stride = (size_t)p.t_pad * (size_t)K * 2;   // one shared expert's block of h

    // ------------------------------------------------------------------ loader setup
    // Wave-load q fills LDS bytes [q*1024, q*1024+1024) of a stage: 16 rows x 4 pieces.
    // Lane l supplies row q*16 + l/4, slot l%4, which must hold logical piece (l%4) ^ block_swizzle(l/4).
    // This wave owns q = i*NW + wave; the X region is padded to a multiple of NW wave-loads so
    // that load i is an X load for i < NLX and a W load otherwise, for every wave.
    // Loads are buffer loads: address = operand base (SGPR descriptor) + per-lane offset (VGPR,
    // fixed for the whole tile) + K offset (SGPR, advanced per sub-tile), so the K loop needs no
    // vector address arithmetic at all.
    const int lrow = lane >> 2;
    const int lpiece = (lane & 3) ^ block_swizzle(lrow);
    uint32_t loff[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int q = i * NW + wave;
        if (i < NLX) {
            int r = q * 16 + lrow;
            if (r > d.nrows - 1) r = d.nrows - 1;     // padded rows re-read the last valid row
            int grow = d.row0 + r;
            if (!a_tiled) {
                // x: row-major [rows, K]
                if (!shared && p.row_token) grow = p.row_token[grow];
                loff[i] = (uint32_t)grow * (uint32_t)p.lda_bytes + (uint32_t)(lpiece * 16);
            } else {
                // h: tiled; the piece this lane needs sits at slot piece ^ block_swizzle(row%16) of its row
                const int rr = grow & 15;
                loff[i] = (uint32_t)(grow >> 4) * (uint32_t)(p.kt_a * 1024) + (uint32_t)(rr * 64 + ((lpiece ^ block_swizzle(rr)) << 4));
            }
        } else {
            // W: tiled by the pack step, so LDS rows (q-NQX)*16 .. +15 of the W region
            // are one 1 KiB block: group index n0/16 + (q-NQX), in lane order.
            const int qw = q - NQX;
            int grp = (n0 >> 4) + (GATED ? (qw & 7) : qw);
            if (grp > (N >> 4) - 1) grp = (N >> 4) - 1;
            loff[i] = (uint32_t)grp * (uint32_t)(p.kt_w * 1024) + (uint32_t)(lane * 16);
        }
    }
    lds_t const ring = (lds_t)lds;
    __amdgpu_buffer_rsrc_t rs_x, rs_w, rs_u;   // X, W (gate / down), W (up)
    int koff_x = 0, koff_w = 0;                // byte offsets along K of the sub-tile being loaded

    // Enqueues direct-to-LDS load i of the sub-tile at `koff` into ring stage `stage`.
    auto issue_one = [&](const int i, const int stage) __attribute__((always_inline)) {
        lptr_t dst = (lptr_t)(ring + stage * RING_STRIDE + (i * NW + wave) * 1024);
        if (i < NLX) buffer_load16_to_lds(rs_x, dst, loff[i], koff_x);
        else if (GATED && (i - NLX) * NW >= 8) buffer_load16_to_lds(rs_u, dst, loff[i], koff_w);
        else buffer_load16_to_lds(rs_w, dst, loff[i], koff_w);
    };

    // ------------------------------------------------------------------ reader setup
    // Lane l reads row (l & 15) of a 16-row block, logical piece l >> 4 (k = 8*(l>>4) .. +7),
    // stored at slot piece ^ block_swizzle(row).  Block bases are multiples of 16 rows, so the
    // swizzle term depends on the lane only.
    const int rl = lane & 15, g = lane >> 4;
    const int bx0 = wm * TI;                       // in 32-row units
    const int bw0 = GATED ? wn * TJH : wn * TJ;    // in 32-row units
    const uint32_t offL = (uint32_t)(rl * ROWB + ((g ^ block_swizzle(rl)) << 4));
    const uint32_t offX = offL + (uint32_t)(bx0 * 32 * ROWB);
    const uint32_t offW = offL + (uint32_t)(XBYTES + bw0 * 32 * ROWB);

    f32x4 acc[WB][XB];
#pragma unroll
    for (int j = 0; j < WB; ++j)
#pragma unroll
        for (int i = 0; i < XB; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[j][i][r] = 0.f;

    // Operand fragments of one sub-tile: all X blocks, and the W blocks in two halves.  wA is
    // used by the first half of a sub-tile and refilled (from the NEXT stage) during the second;
    // wB the other way round; X block i is refilled from the next stage right after its last
    // MFMA of the second half.  So no fragment needs a second copy.
    bf16x8 xf[XB], wA[WBH], wB[WBH];
    typedef __attribute__((address_space(3))) const bf16x8* frag_ptr_t;
    auto read_x = [&](const int stage, const int i) __attribute__((always_inline)) {
        xf[i] = *(frag_ptr_t)(ring + stage * RING_STRIDE + offX + i * 16 * ROWB);
    };
    // W block jj of half hf: GEMM 2: rows (hf*WBH + jj)*16; GEMM 1: gate rows jj*16 | up rows 128 + jj*16
    auto read_w = [&](const int stage, const int hf, const int jj) __attribute__((always_inline)) {
        const int rows = GATED ? hf * 128 + jj * 16 : (hf * WBH + jj) * 16;
        const bf16x8 v = *(frag_ptr_t)(ring + stage * RING_STRIDE + offW + rows * ROWB);
        if (hf == 0) wA[jj] = v;
        else wB[jj] = v;
    };

    // One half of a sub-tile: XB groups, group i = the WBH MFMAs of X block i with this half's W
    // blocks.  HF = 0 reads the second half's W blocks of the same stage; HF = 1 reads the
    // next sub-tile's X blocks and first-half W blocks from stage `rd_stage` (RD).  Direct-to-LDS
    // loads LD0..LD1-1 are spread over the groups (LD).
    auto half = [&](auto hf_tag, auto rd_tag, auto ld_tag, auto ld0_tag, auto ld1_tag, const int rd_stage,
                    const int ld_stage) __attribute__((always_inline)) {
        constexpr int HF = decltype(hf_tag)::value;
        constexpr bool RD = decltype(rd_tag)::value;
        constexpr bool LD = decltype(ld_tag)::value;
        constexpr int LD0 = decltype(ld0_tag)::value, LD1 = decltype(ld1_tag)::value;
        constexpr int NLD = LD1 - LD0;
#pragma unroll
        for (int i = 0; i < XB; ++i) {
#pragma unroll
            for (int jj = 0; jj < WBH; ++jj) {
                const int j = HF * WBH + jj;
                const bf16x8 w = HF == 0 ? wA[jj] : wB[jj];
                if (i < XB_A) {
                    if (GATED) mfma_16x16x32(acc[j][i], w, xf[i]);
                    else mfma_16x16x32(acc[j][i], xf[i], w);
                } else {
                    if (GATED) mfma_16x16x32_v(acc[j][i], w, xf[i]);
                    else mfma_16x16x32_v(acc[j][i], xf[i], w);
                }
            }
            if (RD) {
                if (HF == 1) read_x(rd_stage, i);
                // the WBH W reads of this half go out with the first groups
                constexpr int RPGW = (WBH + XB - 1) / XB;
#pragma unroll
                for (int jj = i * RPGW; jj < (i + 1) * RPGW && jj < WBH; ++jj) read_w(rd_stage, 1 - HF, jj);
            }
            if (LD) {
#pragma unroll
                for (int l = (i * NLD) / XB; l < ((i + 1) * NLD) / XB; ++l) issue_one(LD0 + l, ld_stage);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using T_ = std::true_type;
    using F_ = std::false_type;

    using I0 = std::integral_constant<int, 0>;
    // GEMM 2 on shared experts walks `nseg` K-concatenated segments (one per shared expert);
    // every other tile has one segment.  The pipeline drains and restarts between segments.
    for (int seg = 0; seg < nseg; ++seg) {
        // the descriptors span 4 GiB - 1; bounds are kept by the row clamps above
        // a K piece starts `split` pieces along: K*2 bytes per piece in a row-major row, KT blocks of
        // 1 KiB in a tiled operand (the packed W is always tiled)
        const size_t piece_shift = (size_t)split * (size_t)KT * 1024;
        rs_x = uniform_rsrc(a_base + (size_t)seg * a_seg_stride + (tail_split ? piece_shift : (size_t)split * (size_t)K * 2));
        // UNIFORM (router GEMM): one packed matrix, K-split s starts s * w_uniform_stride bytes along
        if (UNIFORM) rs_w = uniform_rsrc(p.w_uniform + (size_t)d.group * (size_t)p.w_uniform_stride);
        else rs_w = uniform_rsrc((const char*)p.w_a[d.group + seg] + (tail_split ? piece_shift : 0));
        if (GATED) rs_u = uniform_rsrc(p.w_b[d.group]);
        koff_x = 0;
        koff_w = 0;
        // prologue: sub-tiles 0 .. NS-2 go out, wait for sub-tile 0
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) {
            if (s < KT) {
#pragma unroll
                for (int i = 0; i < NL; ++i) issue_one(i, s);
                koff_x += kstep_x;
                koff_w += kstep_w;
            }
        }
        if (KT >= NS - 1) ring_sync<(NS - 2) * NL>();
        else ring_sync<0>();
        // Same order as the reads inside the loop (the first-half W blocks among the first X
        // blocks): LDS reads return in order, and where the two paths into the loop meet the
        // compiler waits for whichever leaves fewer reads outstanding behind the registers the
        // first MFMAs need.  With the W blocks read last here (where the scheduler puts them if
        // left alone), that was a wait for every read of the previous iteration at the top of
        // each sub-tile.
        constexpr int RPGW0 = (WBH + XB - 1) / XB;
#pragma unroll
        for (int i = 0; i < XB; ++i) {
            read_x(0, i);
#pragma unroll
            for (int jj = i * RPGW0; jj < (i + 1) * RPGW0 && jj < WBH; ++jj) read_w(0, 0, jj);
            __builtin_amdgcn_sched_barrier(0);   // keeps the compiler from moving the W reads to the end
        }

        using H0 = std::integral_constant<int, 0>;
        using H1 = std::integral_constant<int, 1>;
        int t = 0;
        // steady state: sub-tile t is multiplied, sub-tile t+NS-1 is loaded
        for (; t + NS - 1 < KT; ++t) {
            const int cur = t % NS, nxt = (t + 1) % NS, ld = (t + NS - 1) % NS;
            half(H0{}, T_{}, T_{}, I0{}, std::integral_constant<int, NL0>{}, cur, ld);
            // Sub-tile t+1 has landed once only the younger loads are outstanding.  The same
            // barrier frees stage `cur` for the loads of the NEXT iteration: its last reads were
            // issued above and have returned (lgkmcnt(0)) before any wave passes.
            ring_sync<(NS - 3) * NL + NL0>();
            half(H1{}, T_{}, T_{}, std::integral_constant<int, NL0>{}, std::integral_constant<int, NL>{}, nxt, ld);
            koff_x += kstep_x;
            koff_w += kstep_w;
        }
        // tail: nothing left to load; conservative waits
        for (; t < KT - 1; ++t) {
            const int cur = t % NS, nxt = (t + 1) % NS;
            half(H0{}, T_{}, F_{}, I0{}, I0{}, cur, 0);
            ring_sync<0>();
            half(H1{}, T_{}, F_{}, I0{}, I0{}, nxt, 0);
        }
        half(H0{}, T_{}, F_{}, I0{}, I0{}, t % NS, 0);
        ring_sync<0>();    // every wave is done reading the ring before the next segment refills it
        half(H1{}, F_{}, F_{}, I0{}, I0{}, 0, 0);
    }

    // ------------------------------------------------------------------ epilogue
    // Accumulator block (j, i) is 16 x 16; a lane holds 4 registers: the block's MFMA-row-operand
    // index 4*(lane/16) + r and column-operand index lane%16.
    mfma_drain();
    char* out = shared ? p.out_shared : (tail_split ? p.out_partial : p.out_routed);
    const int orow_base = tail_split ? piece * SPLIT_TAIL_ROWS
                                     : (shared ? (GATED ? d.srow : 0) : split * p.split_rows) + d.row0;
    if (GATED) {
        // W is the row operand: the lane owns output row (X row) lane%16 of block i and the 4
        // consecutive columns 4*(lane/16) .. +3 of gate block j; the up value of the same
        // element sits in the same lane and register of block WBH + j.  h is written tiled:
        // block (row/16, col/32), row%16 at 64 bytes each, piece slot = piece ^ block_swizzle(row%16);
        // a store instruction covers 16 rows x 32 contiguous bytes.
#pragma unroll
        for (int i = 0; i < XB; ++i) {
            const int r = bx0 * 32 + i * 16 + rl;
            const bool row_ok = r < d.nrows;
            const int ro = orow_base + r, rr = ro & 15, sw = block_swizzle(rr);
            char* hrow = out + ((size_t)(ro >> 4) * (size_t)(N >> 5)) * 1024 + rr * 64;
#pragma unroll
            for (int j = 0; j < WBH; ++j) {
                const int col = n0 + bw0 * 32 + j * 16 + g * 4;
                bf16x4 o;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float gv = acc[j][i][q], uv = acc[WBH + j][i][q];
                    // silu(g) * u with the hardware reciprocal (1 ulp): far below the bf16 rounding of h
                    o[q] = (__bf16)(gv * __builtin_amdgcn_rcpf(1.0f + __expf(-gv)) * uv);
                }
                if (row_ok && col < N)
                    *reinterpret_cast<bf16x4*>(hrow + (size_t)(col >> 5) * 1024 + ((((col & 31) >> 3) ^ sw) << 4) + (col & 7) * 2) = o;
            }
            __builtin_amdgcn_sched_barrier(0);   // one block row at a time: keeps accumulator reads from piling up
        }
    } else {
        // GEMM 2 / router GEMM: X is the row operand, so the lane owns output column lane%16 of W
        // block j and the 4 consecutive rows 4*(lane/16) .. +3 of X block i.  One store
        // instruction writes 4 rows x 64 contiguous bytes (fp32).  Rows past the end of the
        // group and columns past N fall outside the buffer descriptor, which spans exactly the
        // valid rows of the 16-row block being stored, and are dropped by hardware.
        // The descriptor is rebuilt (scalar work) for every 16-row block of X so that the row
        // part of the address is in its base and the 16 per-lane offsets {W block j, row r} are
        // computed once per tile: a store then needs no vector address arithmetic and no
        // registers beyond its data.
        auto store_tile = [&](auto f32_tag) __attribute__((always_inline)) {
            constexpr bool F32 = decltype(f32_tag)::value;
            constexpr int esz = F32 ? 4 : 2;
            const uint32_t rowbytes = (uint32_t)N * (uint32_t)esz;
            uint32_t vcol[WB][4];
#pragma unroll
            for (int j = 0; j < WB; ++j) {
                const int col = n0 + bw0 * 32 + j * 16 + rl;
                const uint32_t base = col < N ? (uint32_t)(g * 4) * rowbytes + (uint32_t)col * esz : 0x80000000u;
#pragma unroll
                for (int r = 0; r < 4; ++r) vcol[j][r] = base + (uint32_t)r * rowbytes;
            }
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const int r0 = bx0 * 32 + i * 16;                          // wave-uniform
                const int left = min(max(d.nrows - r0, 0), 16);            // valid rows of this block
                const __amdgpu_buffer_rsrc_t rs_o =
                    tile_rsrc(out + (size_t)(orow_base + r0) * rowbytes, (uint32_t)left * rowbytes);
#pragma unroll
                for (int j = 0; j < WB; ++j) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if (F32) {
                            buffer_store_b32(rs_o, vcol[j][r], acc[j][i][r]);
                        } else {
                            // read the accumulator here, not earlier: left alone the compiler copies all
                            // accumulators to VGPRs ahead of the first store and spills to make room
                            float v;
                            if (i < XB_A) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(acc[j][i][r]) : "memory");
                            else asm volatile("v_mov_b32 %0, %1" : "=v"(v) : "v"(acc[j][i][r]) : "memory");
                            buffer_store_bf16(rs_o, vcol[j][r], v);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);   // one block row at a time
            }
        };
        if (tail_split || ((shared ? p.out_fp32 >> 1 : p.out_fp32) & 1)) store_tile(T_{});
        else store_tile(F_{});
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

// Tile picked by this workgroup (false: nothing to do).  The first n_run entries of the m-tile
// list are cut into runs of group_m consecutive m-tiles; the tiles of a run are visited
// m-fastest, then along n, so tiles that run at the same time share W panels (same n, same
// group) and X panels (same m) in L2.  (Runs of a fixed length that cross group boundaries
// measured 5-12 % faster than runs fitted to each group.)  Entries past n_run are tail tiles
// of different groups: they are walked along n, which shares the X panel.
template <bool UNIFORM = false>
__device__ __forceinline__ bool pick_tile(const GemmArgs& p, const bool gated, TileDesc& d, int& n_tile) {
    if (UNIFORM) {
        // Router GEMM: every K-split s covers all T rows in tiles of uniform_tm rows; nothing to look up.
        const int L = blockIdx.x;
        const int mt = L / p.n_tiles;
        n_tile = L - mt * p.n_tiles;
        if (mt >= p.uniform_per * p.uniform_splits) return false;
        const int s = mt / p.uniform_per, m = mt - s * p.uniform_per;
        d.group = s;
        d.row0 = m * p.uniform_tm;
        d.nrows = min(p.uniform_tm, p.T - d.row0);
        d.srow = -1 - s;
        return true;
    }
    const int count = gated ? p.plan->n_gate_up : p.plan->n_down;
    const int n_run = gated ? p.plan->n_run_up : p.plan->n_run_down;
    // Only whole rounds of 256 REAL tiles are dealt to the XCDs in runs of 32 (the grid is an upper
    // bound of the tile count, and how far the runs reach must not depend on it); the last,
    // partial round keeps the hardware's own order, which spreads it over all eight XCDs.  In
    // runs it would sit on the first few XCDs and leave the L2s and fabric links of the others
    // idle: a launch of 128 tiles measured 251 us on four XCDs against 210 us on eight, the
    // second of two rounds 6 % more; over the Mixtral-shaped layer from 1024 to 8192 tokens the
    // gate/up GEMM is 0.7-2.6 % faster this way, the named workloads are unchanged.
    const int L = tile_order(blockIdx.x, count * p.n_tiles, p.xcd_remap);
    const int run_positions = n_run * p.n_tiles;
    int mt;
    if (L < run_positions) {
        const int per_super = p.group_m * p.n_tiles;
        const int sr = L / per_super;
        const int rem = L - sr * per_super;
        const int mt0 = sr * p.group_m;
        const int gm = min(p.group_m, n_run - mt0);
        n_tile = rem / gm;
        mt = mt0 + (rem - n_tile * gm);
    } else {
        const int rem = L - run_positions;
        mt = n_run + rem / p.n_tiles;
        n_tile = rem - (mt - n_run) * p.n_tiles;
    }
    if (mt >= count) return false;  // uniform for the workgroup
    d = p.descs[mt];
    return true;
}

// 4 wavefronts (one per SIMD, up to 512 registers each), wave grid WM x 4/WM.
template <int WM, bool GATED, bool UNIFORM = false>
__global__ __launch_bounds__(256, 1) void ffn_gemm_kernel(const GemmArgs p) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    TileDesc d;
    int n_tile;
    if (!pick_tile<UNIFORM>(p, GATED, d, n_tile)) return;
    // 32-row blocks that hold real rows; 9 or 10: a tall tile (the plan kernel makes them for this wave grid only)
    const int blocks = d.nrows > 256 ? (d.nrows + 31) >> 5 : (p.small_tiles ? (d.nrows + 31) >> 5 : 8);
    if (WM == 2) {
        if (blocks > 4) gemm_tile<4, 2, 4, GATED, UNIFORM>(p, d, n_tile, lds);
        else if (blocks > 2) gemm_tile<4, 2, 2, GATED, UNIFORM>(p, d, n_tile, lds);
        else gemm_tile<4, 2, 1, GATED, UNIFORM>(p, d, n_tile, lds);
    } else {
        if (blocks > 9) gemm_tile<4, 1, 10, GATED>(p, d, n_tile, lds);
        else if (blocks > 8) gemm_tile<4, 1, 9, GATED>(p, d, n_tile, lds);
        else if (blocks > 4) gemm_tile<4, 1, 8, GATED>(p, d, n_tile, lds);
        else if (blocks > 2) gemm_tile<4, 1, 4, GATED>(p, d, n_tile, lds);
        else if (blocks > 1) gemm_tile<4, 1, 2, GATED>(p, d, n_tile, lds);
        else gemm_tile<4, 1, 1, GATED>(p, d, n_tile, lds);
    }
}

// 8 wavefronts (two per SIMD, up to 256 registers each), wave grid WM x 8/WM: while one wave
// of a SIMD waits at the ring barrier or on LDS, the other keeps the matrix pipe fed.
template <int WM, bool GATED>
__global__ __launch_bounds__(512, 2) void ffn_gemm_kernel8(const GemmArgs p) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    TileDesc d;
    int n_tile;
    if (!pick_tile(p, GATED, d, n_tile)) return;
    const int blocks = p.small_tiles ? (d.nrows + 31) >> 5 : 8;
    if (WM == 2) {
        if (blocks > 4) gemm_tile<8, 2, 4, GATED>(p, d, n_tile, lds);
        else if (blocks > 2) gemm_tile<8, 2, 2, GATED>(p, d, n_tile, lds);
        else gemm_tile<8, 2, 1, GATED>(p, d, n_tile, lds);
    } else {
        if (blocks > 4) gemm_tile<8, 4, 2, GATED>(p, d, n_tile, lds);
        else gemm_tile<8, 4, 1, GATED>(p, d, n_tile, lds);
    }
}

// Exclusive prefix sums of three per-thread counters over the 256 threads of a workgroup, and
// their totals (every thread gets them): a wave-level scan, then the four wave sums through LDS.
__device__ __forceinline__ void block_scan3(int& a, int& b, int& c, int (&tot)[3], int (*wsum)[3], const int tid) {
    const int lane = tid & 63, w = tid >> 6;
    int ia = a, ib = b, ic = c;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int ta = __shfl_up(ia, d, 64), tb = __shfl_up(ib, d, 64), tc = __shfl_up(ic, d, 64);
        if (lane >= d) { ia += ta; ib += tb; ic += tc; }
    }
    if (lane == 63) { wsum[w][0] = ia; wsum[w][1] = ib; wsum[w][2] = ic; }
    __syncthreads();
    int oa = 0, ob = 0, oc = 0;
    tot[0] = tot[1] = tot[2] = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (i < w) { oa += wsum[i][0]; ob += wsum[i][1]; oc += wsum[i][2]; }
        tot[0] += wsum[i][0]; tot[1] += wsum[i][1]; tot[2] += wsum[i][2];
    }
    __syncthreads();   // wsum may be written again
    a = oa + ia - a;
    b = ob + ib - b;
    c = oc + ic - c;
}

// Builds the two m-tile lists (gate/up GEMM with tiles of tm_up rows, down GEMM with tm_down rows)
// from expert_offsets.  Group order: shared expert 0, routed experts, shared experts 1.. (the down
// GEMM takes the first two parts only: shared experts are concatenated along K there).
// A group of n rows gives floor(n/tm) full tiles and at most one tail tile.  A tail higher than
// half a tile runs the full-height variant and always stays with its group; a short tail runs
// a short variant.  tails_last = 0: the short tail, too, directly follows its group's tiles,
// which keeps the load-bound short tiles mixed with the compute-bound full ones (better when
// a launch has many rounds of tiles).  tails_last = 1: the short tails follow all other tiles,
// sorted by falling height, ties in group order, so a launch with few rounds ends on its
// smallest work items and its other tiles all take the same time (CUs that share operand
// panels in L2 stay in step).  n_run_* = number of entries listed in group order.
__global__ __launch_bounds__(256) void ffn_plan_kernel(const int32_t* __restrict__ offsets, int T, int t_pad, int E, int Ns,
                                                       int tm_up, int tm_down, int tails_last_up, int tails_last_down,
                                                       int small_tiles, int e_lo, int e_hi, int shared_on, int down_splits,
                                                       int split_max_blocks, int split_rule_tiles, int tall_up, int tall_down,
                                                       SplitTail* __restrict__ split_tails, PlanHeader* __restrict__ plan,
                                                       TileDesc* __restrict__ descs_up, TileDesc* __restrict__ descs_down) {
    __shared__ int wsum[4][3];
    const int tid = threadIdx.x;
    // group order: g = 0 -> shared 0 (if any), then routed 0..E-1, then shared 1..Ns-1
    const int ngroups = E + Ns;
    int row_begin = 0, rows = 0, group = 0, srow = -1;
    if (tid < ngroups) {
        int pos = tid;
        if (Ns > 0 && pos == 0) { group = E; rows = T; row_begin = 0; srow = 0; }
        else {
            if (Ns > 0) pos -= 1;
            if (pos < E) { group = pos; row_begin = offsets[pos]; rows = offsets[pos + 1] - row_begin; srow = -1; }
            else { const int s = pos - E + 1; group = E + s; rows = T; row_begin = 0; srow = s * t_pad; }
        }
        // a streamed pass covers routed experts [e_lo, e_hi) and, if shared_on, the shared experts
        if (group < E ? (group < e_lo || group >= e_hi) : !shared_on) rows = 0;
    }
    for (int which = 0; which < 2; ++which) {
        const int tm = which == 0 ? tm_up : tm_down;
        TileDesc* descs = which == 0 ? descs_up : descs_down;
        const int last = which == 0 ? ngroups - 1 : (Ns > 0 ? E : E - 1);  // last group of this list
        const bool mine = tid <= last;
        const bool tails_last = (which == 0 ? tails_last_up : tails_last_down) != 0;
        const int nfull = mine ? rows / tm : 0;
        int tail = mine ? rows - nfull * tm : 0;
        // Tall tiles: a tail of at most 64 rows joins the group's last full 256-row tile (288 or
        // 320 rows, 12-25 % more time for that tile) instead of costing a pass of its own over
        // the group's weights.
        const int joined = ((which == 0 ? tall_up : tall_down) && tm == 256 && nfull > 0 && tail <= MAX_ROWS - 256) ? tail : 0;
        tail -= joined;
        const int blocks = (tail + 31) >> 5;   // 32-row blocks of the tail tile, 0 = none
        // A tail higher than half a tile runs the full-height variant and takes as long as a full
        // tile, so it stays with its group (keeps the group's W panels shared and the CUs in
        // step); only a short tail is moved to the end of the list.
        // (A shared expert's tail is not moved in a down list with K pieces: the pieces' partial
        // sums are reduced into y_perm, while shared rows belong to y_shared.)
        // (at most 128 rows: the K pieces' partial buffers hold SPLIT_TAIL_ROWS rows)
        const bool moved = tails_last && blocks > 0 && small_tiles && blocks * 64 <= min(tm, 2 * SPLIT_TAIL_ROWS) &&
                           !(which == 1 && down_splits > 1 && group >= E);
        // tall_* = 2: the tall tile keeps its place in the group (it shares the W panels its
        // neighbours stream, which is the point when a group is only a few tiles).  tall_* = 1 and
        // tails_last: a tall tile takes longer than its neighbours and in a long launch puts the
        // CUs it runs on out of step for the rest of it, so it leaves the group order too: tall
        // tiles come first after the run region, one entry each, never cut along K.
        const bool tall_moved = tails_last && joined > 0 && (which == 0 ? tall_up : tall_down) == 1;
        const int nrun = nfull - (tall_moved ? 1 : 0) + (blocks > 0 && !moved);   // tiles listed in group order
        // Positions by prefix sums over the groups (at most 256, one per thread): tiles listed in
        // group order; tall tiles moved behind them; moved short tails, counted per height in
        // 32-row blocks (1..4), three 10-bit counters to a word.
        int base = nrun;
        int k2 = (tall_moved ? 1 : 0) | (moved && blocks == 1 ? 1 << 10 : 0) | (moved && blocks == 2 ? 1 << 20 : 0);
        int k3 = (moved && blocks == 3 ? 1 : 0) | (moved && blocks == 4 ? 1 << 10 : 0);
        int tot[3];
        block_scan3(base, k2, k3, tot, wsum, tid);
        const int n_run_s = tot[0], n_tall_s = tot[1] & 1023;
        const int cnt[5] = {0, (tot[1] >> 10) & 1023, (tot[1] >> 20) & 1023, tot[2] & 1023, (tot[2] >> 10) & 1023};
        const int pre[5] = {0, (k2 >> 10) & 1023, (k2 >> 20) & 1023, k3 & 1023, (k3 >> 10) & 1023};
        const int tails = cnt[1] + cnt[2] + cnt[3] + cnt[4];
        // Down list with K pieces: only the moved tails of at most split_max_blocks 32-row blocks are
        // cut (down_splits list entries each); the higher ones, which come first, stay whole.
        // Whether to cut at all is decided here, where the tile counts are known.  Pieces make a
        // launch faster in two cases only (measured on the Mixtral-shaped layer from 64 to 16384
        // tokens): when EVERY tile of the launch is a short tail (a few tokens per expert: the
        // pieces then shorten the longest tile and fill idle CUs, -10 %), and when the launch is
        // many rounds of tiles long (the tails at its end then finish sooner: -2 % on the
        // 16384-token, skewed workload).  In between, a launch of one to three rounds is as long
        // as its full tiles whatever happens to the tails, and pieces only add a round and
        // traffic (+6 ... +50 % measured).  split_rule_tiles: that many m-tiles or more count as
        // "many rounds"; 0: always cut.
        int n_whole = tails;
        bool cutting = which == 1 && down_splits > 1;
        if (cutting) {
            n_whole = 0;
            for (int b = split_max_blocks + 1; b <= 4; ++b) n_whole += cnt[b];
            const int others = n_run_s + n_tall_s + n_whole;
            cutting = split_rule_tiles == 0 || others == 0 || others + tails - n_whole >= split_rule_tiles;
            if (!cutting) n_whole = tails;
        }
        const int n_cut = tails - n_whole;
        if (tid == 0) {
            const int total = n_run_s + n_tall_s + n_whole + n_cut * (cutting ? down_splits : 1);
            if (which == 0) { plan->n_gate_up = total; plan->n_run_up = n_run_s; }
            else { plan->n_down = total; plan->n_run_down = n_run_s; plan->n_split_tails = n_cut; }
        }
        if (mine) {
            TileDesc d;
            d.group = group;
            d.srow = srow;
            const int nlisted = nfull - (tall_moved ? 1 : 0);   // full tiles listed in group order
            for (int i = 0; i < nrun; ++i) {
                // entry nlisted (if any) is a tail that stays with its group; it starts after all full tiles
                const int at = i < nlisted ? i : nfull;
                d.row0 = row_begin + at * tm;
                d.nrows = min(tm, rows - at * tm) + ((at == nfull - 1 && !tall_moved) ? joined : 0);
                descs[base + i] = d;
            }
            if (tall_moved) {
                const int before = k2 & 1023;   // tall tiles of the groups before this one
                d.row0 = row_begin + (nfull - 1) * tm;
                d.nrows = tm + joined;
                descs[n_run_s + before] = d;
            }
            if (moved) {
                // tails that come before this one: the higher ones, and those as high of earlier groups
                int rank = pre[blocks];
                for (int b = blocks + 1; b <= 4; ++b) rank += cnt[b];
                d.row0 = row_begin + nfull * tm;
                d.nrows = tail;
                const int tbase = n_run_s + n_tall_s;
                if (cutting && blocks <= split_max_blocks) {
                    // one entry per K piece; the pieces' partial sums are added up after the launch
                    const int q = rank - n_whole;   // falling height: the whole ones rank first
                    for (int sp = 0; sp < down_splits; ++sp) {
                        d.srow = -2 - (q * down_splits + sp);
                        descs[tbase + n_whole + q * down_splits + sp] = d;
                    }
                    split_tails[q].row0 = d.row0;
                    split_tails[q].nrows = tail;
                } else {
                    descs[tbase + rank] = d;
                }
            }
        }
    }
}

// y_perm[row0 + r, :] of split tail q = sum over its K pieces of the fp32 partials, added in
// piece order (one thread per 4 columns, one workgroup per row): deterministic.
__global__ __launch_bounds__(256) void split_tail_reduce_kernel(const PlanHeader* __restrict__ plan,
                                                                const SplitTail* __restrict__ tails,
                                                                const float* __restrict__ partial, int splits, int H,
                                                                char* __restrict__ y, int y_fp32) {
    const int q = blockIdx.x / SPLIT_TAIL_ROWS, r = blockIdx.x % SPLIT_TAIL_ROWS;
    if (q >= plan->n_split_tails) return;
    const SplitTail t = tails[q];
    if (r >= t.nrows) return;
    for (int c = threadIdx.x * 4; c < H; c += 256 * 4) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int sp = 0; sp < splits; ++sp) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(partial + ((size_t)(q * splits + sp) * SPLIT_TAIL_ROWS + r) * H + c);
            acc += v;
        }
        const size_t at = (size_t)(t.row0 + r) * H + c;
        if (y_fp32) {
            *reinterpret_cast<f32x4*>(y + at * 4) = acc;
        } else {
            bf16x4 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = (__bf16)acc[i];
            *reinterpret_cast<bf16x4*>(y + at * 2) = o;
        }
    }
}

}  // namespace

hipError_t launch_split_tail_reduce(const moe_shape& s, const PlanHeader* plan, const SplitTail* tails, const float* partial,
                                    int splits, void* y_perm, bool y_fp32, hipStream_t st) {
    hipLaunchKernelGGL(split_tail_reduce_kernel, dim3((unsigned)(s.E * SPLIT_TAIL_ROWS)), dim3(256), 0, st, plan, tails, partial,
                       splits, s.H, (char*)y_perm, y_fp32 ? 1 : 0);
    return hipGetLastError();
}

hipError_t ffn_gemm_init() {
    hipError_t e;
#define SET_LDS(K_)                                                                                            \
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&K_), hipFuncAttributeMaxDynamicSharedMemorySize,    \
                            MAX_LDS);                                                                          \
    if (e != hipSuccess) return e;
    SET_LDS((ffn_gemm_kernel<2, true>))
    SET_LDS((ffn_gemm_kernel<2, false>))
    SET_LDS((ffn_gemm_kernel<2, false, true>))
    SET_LDS((ffn_gemm_kernel<1, true>))
    SET_LDS((ffn_gemm_kernel<1, false>))
    SET_LDS((ffn_gemm_kernel8<2, true>))
    SET_LDS((ffn_gemm_kernel8<2, false>))
    SET_LDS((ffn_gemm_kernel8<4, true>))
    SET_LDS((ffn_gemm_kernel8<4, false>))
#undef SET_LDS
    return hipSuccess;
}

hipError_t launch_ffn_plan(const moe_shape& s, const int32_t* offsets, int tm_up, int tm_down, bool tails_last_up,
                           bool tails_last_down, bool small_tiles, int e_lo, int e_hi, bool shared_on,
                           int down_tail_splits, int split_max_blocks, int split_rule_tiles, int tall_up, int tall_down,
                           SplitTail* split_tails, PlanHeader* plan, TileDesc* descs_up, TileDesc* descs_down, hipStream_t st) {
    hipLaunchKernelGGL(ffn_plan_kernel, dim3(1), dim3(256), 0, st, offsets, s.T, (s.T + 15) & ~15, s.E, s.num_shared, tm_up, tm_down,
                       tails_last_up ? 1 : 0, tails_last_down ? 1 : 0, small_tiles ? 1 : 0, e_lo, e_hi, shared_on ? 1 : 0,
                       tails_last_down ? down_tail_splits : 1, split_max_blocks, split_rule_tiles, tall_up, tall_down, split_tails, plan, descs_up,
                       descs_down);
    return hipGetLastError();
}

hipError_t launch_ffn_gemm(bool gated, const GemmArgs& a, const GemmConfig& cfg, hipStream_t st) {
    const dim3 grid((unsigned)(a.max_mtiles * a.n_tiles));
#define LAUNCH(KERNEL, THREADS) hipLaunchKernelGGL((KERNEL), grid, dim3(THREADS), MAX_LDS, st, a)
    if (a.w_uniform) {   // router GEMM: 4 waves as 2 x 2, tiles by arithmetic
        LAUNCH((ffn_gemm_kernel<2, false, true>), 256);
        return hipGetLastError();
    }
    if (cfg.waves == 8) {
        if (cfg.wave_rows == 4) {
            if (gated) LAUNCH((ffn_gemm_kernel8<4, true>), 512);
            else LAUNCH((ffn_gemm_kernel8<4, false>), 512);
        } else {
            if (gated) LAUNCH((ffn_gemm_kernel8<2, true>), 512);
            else LAUNCH((ffn_gemm_kernel8<2, false>), 512);
        }
    } else if (cfg.wave_rows == 2) {
        if (gated) LAUNCH((ffn_gemm_kernel<2, true>), 256);
        else LAUNCH((ffn_gemm_kernel<2, false>), 256);
    } else {
        if (gated) LAUNCH((ffn_gemm_kernel<1, true>), 256);
        else LAUNCH((ffn_gemm_kernel<1, false>), 256);
    }
#undef LAUNCH
    return hipGetLastError();
}

}  // namespace moe
