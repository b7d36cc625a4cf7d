// Internal declarations shared by the kernels and the C-ABI layer (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe.h"

namespace moe {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// One m-tile of the grouped GEMMs: rows [row0, row0+nrows) of one group.
//   routed group : group = expert id, row0 = permuted row, srow = -1
//   router GEMM  : group = K-split index s, row0 = first token, srow = -1 - s
//   shared group : group = E + s,     row0 = first token,  srow = s * t_pad (row offset inside the shared region of h)
//   K-split piece of a short tail of the down GEMM: group = expert id, row0 = permuted row,
//                  srow = -2 - (q * splits + s) for piece s of the q-th split tail
struct TileDesc {
    int32_t group;
    int32_t row0;
    int32_t nrows;
    int32_t srow;
};

struct PlanHeader {
    int32_t n_gate_up;  // m-tiles of GEMM 1 (routed + every shared expert)
    int32_t n_down;     // m-tiles of GEMM 2 (routed + shared expert 0; shared experts are K-concatenated)
    int32_t n_run_up;   // the first n_run_* entries of each list are in group order; short tail tiles moved
    int32_t n_run_down; // to the end of the list (if any) follow them
    int32_t n_split_tails;  // down GEMM: short tails whose K range is cut into pieces (0 if that is off)
    int32_t pad[3];
};

// Rows of y_perm that the K-split pieces of one short tail add up to.
struct SplitTail {
    int32_t row0, nrows;
};
constexpr int SPLIT_TAIL_ROWS = 128;   // a split tail is at most half a 256-row tile high

struct GemmArgs {
    const char* a_routed;      // GEMM1: x_perm, or x when row_token != nullptr; GEMM2: h
    const char* a_shared;      // GEMM1: x; GEMM2: h + R*F
    const int32_t* row_token;  // GEMM1 gather map or nullptr
    const void* const* w_a;    // device table of packed weights: GEMM1 W1p, GEMM2 W2p
    const void* const* w_b;    // GEMM1 W3p
    char* out_routed;          // GEMM1: h; GEMM2: y_perm
    char* out_shared;          // GEMM1: h + R*F; GEMM2: y_shared
    const TileDesc* descs;
    const PlanHeader* plan;
    int32_t K, N;              // GEMM1: K=H, N=F; GEMM2: K=F, N=H
    int32_t T;
    int32_t nseg_shared;       // GEMM2: num_shared (K-concatenation); GEMM1: 1
    int32_t n_tiles;           // tiles along N
    int32_t max_mtiles;        // grid = max_mtiles * n_tiles
    int32_t group_m;
    int32_t xcd_remap;
    int32_t small_tiles;       // 1: a short tail tile runs the 128/64/32-row variant
    int32_t out_fp32;          // GEMM2: output stored as fp32 (else bf16): bit 0 routed tiles, bit 1 shared tiles (GEMM1 always stores bf16)
    int32_t lda_bytes;         // row stride of a row-major A operand
    int32_t kt_w;              // 1 KiB blocks per 16-row group of the packed W (its full K / 32)
    int32_t split_rows;        // router GEMM: output rows per K-split (partial s is written at rows s*split_rows + ...)
    int32_t kt_a;              // 1 KiB blocks per 16-row group of a tiled A operand (its full K / 32)
    int32_t tail_splits;       // down GEMM: K pieces per short tail (entries past n_run; 1 = not split)
    char* out_partial;         // down GEMM: fp32 partial results of split tails, SPLIT_TAIL_ROWS rows per piece
    int32_t a_tiled;           // A operand is in 16 x 32 blocks (else row-major): bit 0 routed tiles, bit 1 shared tiles
    int32_t t_pad;             // T rounded up to 16: rows of one shared expert's block of h
    // Router GEMM (w_uniform != nullptr): no tile list and no pointer table; K-split s multiplies the
    // packed gate matrix from byte w_uniform_stride * s on, over uniform_per tiles of uniform_tm rows.
    const char* w_uniform;
    uint32_t w_uniform_stride;
    int32_t uniform_tm, uniform_per, uniform_splits;
};

struct GemmConfig {
    int wave_rows;    // rows of the wave grid: 1 or 2 with 4 waves, 2 or 4 with 8 waves
    int waves;        // wavefronts per workgroup: 4 or 8
    int group_m;
    int xcd_remap;
    int small_tiles;
    int tile_rows_up;      // rows per m-tile of the gate/up GEMM: 0 = choose per launch, else 128 or 256
    int tile_rows_down;    // same for the down GEMM
    int x_tiled;           // moe_layer: 1 = gather x into a tiled x_perm first, 0 = gather inside GEMM 1, -1 = choose
    int tails_last;        // order of the m-tile lists: 1 = short tail tiles after all full tiles, 0 = in group order, -1 = choose
    int down_tail_splits;  // the down GEMM cuts the K range of short tail tiles into pieces (few experts only): 0 off,
                           // 1 where it pays (decided on the device from the tile counts), 2 always
    int tall_tiles;        // a tail of <= 64 rows joins its group's last full 256-row tile (4 waves x 1 wave row only):
                           // 0 off, 1 tall tiles after the run region, 2 in place, -1 choose
};

// Upper bound on the number of m-tiles of `tm` rows for any routing outcome.
inline int64_t max_mtiles(const moe_shape& s, int tm) {
    const int64_t R = (int64_t)s.T * s.top_k;
    return R / tm + s.E + (int64_t)s.num_shared * ((s.T + tm - 1) / tm);
}

// ---- launchers (each only enqueues on `st`; returns the launch status) ----
hipError_t launch_route_mfma(const moe_shape& s, const void* x, const void* wg_packed, const float* bias, int32_t* idx,
                             float* w, float* logits, hipStream_t st);   // E <= 16: one kernel, x against the packed gate matrix
// softmax + top-k from `splits` fp32 partial logit matrices [splits][T][ep]
hipError_t launch_route_topk(const moe_shape& s, const float* partial, int splits, int ep, const float* bias,
                             int32_t* idx, float* w, float* logits, hipStream_t st);

// Swizzle of the 1 KiB operand blocks (16 rows x 64 bytes, in LDS and in every tiled global
// layout): the logical 16-byte piece c of row r (0..15) sits at slot c ^ block_swizzle(r).
// ds_read_b128 serves a wave's 64 lanes in four passes of 16, and not 16 consecutive ones:
// lanes {0-3, 12-15, 20-27}, {4-11, 16-19, 28-31} and the same two sets + 32 (measured lane
// pair by lane pair with the LDS bank-conflict counter).  An MFMA operand read has lane l on
// row l % 16, piece l / 16, so a pass covers row quads {0, 3} of one piece and {1, 2} of the
// next: with (4 - r/4) % 4 the four quads of a pass land in four different slots and its 16
// lanes in 16 different 16-byte bank groups (r/4 itself puts quads 0 and 1, 2 and 3 of a pass
// in the same slot: every read took twice the cycles).
__host__ __device__ constexpr int block_swizzle(const int r) { return (0 - (r >> 2)) & 3; }

constexpr int PERMUTE_CHUNK_TOKENS = 256;
inline int permute_chunks(const moe_shape& s) { return (s.T + PERMUTE_CHUNK_TOKENS - 1) / PERMUTE_CHUNK_TOKENS; }
hipError_t launch_permute_index(const moe_shape& s, const int32_t* idx, int32_t* chunk_counts, int32_t* offsets,
                                int32_t* perm, int32_t* inv_perm, int32_t* row_token, hipStream_t st);
hipError_t launch_permute_gather(const moe_shape& s, const void* x, const int32_t* perm, void* x_perm,
                                 hipStream_t st);
hipError_t launch_zero_offsets(int E, int32_t* offsets, hipStream_t st);
// x_perm in 16-row x 32-column blocks (the layout of h), rows past T*k in the last block undefined
hipError_t launch_permute_gather_tiled(const moe_shape& s, const void* x, const int32_t* row_token, void* x_tiled,
                                       hipStream_t st);

// the lists cover routed experts [e_lo, e_hi) and, if shared_on, the shared experts
hipError_t launch_ffn_plan(const moe_shape& s, const int32_t* offsets, int tm_up, int tm_down, bool tails_last_up,
                           bool tails_last_down, bool small_tiles, int e_lo, int e_hi, bool shared_on,
                           int down_tail_splits, int split_max_blocks, int split_rule_tiles, int tall_up, int tall_down,
                           SplitTail* split_tails, PlanHeader* plan, TileDesc* descs_up, TileDesc* descs_down, hipStream_t st);
// y_perm rows of the split tails = sum over pieces of the fp32 partials, in y_perm's dtype
hipError_t launch_split_tail_reduce(const moe_shape& s, const PlanHeader* plan, const SplitTail* tails, const float* partial,
                                    int splits, void* y_perm, bool y_fp32, hipStream_t st);
hipError_t launch_ffn_gemm(bool gated, const GemmArgs& a, const GemmConfig& cfg, hipStream_t st);
hipError_t ffn_gemm_init();  // one-time function attributes (dynamic LDS size)

hipError_t launch_combine(const moe_shape& s, const void* y_perm, const int32_t* inv_perm, const float* w,
                          const void* y_shared, void* out, bool y_fp32, bool shared_fp32, bool out_fp32, hipStream_t st);
// in: logical [rows = K, cols] row-major; out: packed [cols_padded x K] (cols_padded % 32 == 0, columns >= cols are zero)
hipError_t launch_pack_weight(const void* in, int rows, int cols, int cols_padded, void* out, hipStream_t st);

// register-only MFMA loop (profile.hip): sink holds blocks*256 floats
constexpr int CEILING_BLOCKS = 1024;
double mfma_ceiling_flops(int blocks, int iters);
hipError_t launch_mfma_ceiling(const void* a, const void* b, size_t bytes, int blocks, int iters, float* sink, hipStream_t st);

// Rows of the h scratch: routed rows and each shared expert's rows start on a 16-row block boundary.
inline int64_t h_rows(const moe_shape& s) {
    const int64_t R = (int64_t)s.T * s.top_k;
    return ((R + 15) & ~(int64_t)15) + (int64_t)s.num_shared * ((s.T + 15) & ~15);
}

}  // namespace moe
