/*
 * moe.h -- C ABI of the MI355X (gfx950) MoE expert-module library.
 *
 * The library computes the sparse MoE layer of the paper's Sec. 2 ("MoE inference": a router
 * assigns each token to top-k experts, each token is processed by its k experts, the output
 * is the weighted sum of their outputs, optionally plus shared experts every token passes
 * through) on ONE large accumulated token batch, which is what module-based batching
 * (Sec. 4.2) hands to the expert module.  Experts are SwiGLU MLPs:
 *     expert_e(x) = ( silu(x W1_e) * (x W3_e) ) W2_e ,   silu(z) = z / (1 + exp(-z)).
 *
 * Conventions for every entry point
 *  - Plain C types only.  "device" pointers are HIP device memory on the context's GPU;
 *    "host" pointers are ordinary process memory.  bf16 data is passed as `void*`.
 *  - All matrices are dense, row-major, without padding.
 *  - Ownership: the caller owns every buffer, including the workspace.  The library
 *    allocates device memory only inside moe_create (small tables) and frees it in
 *    moe_destroy.  Nothing is retained from the caller's buffers after a call's kernels
 *    have run.
 *  - Asynchrony: a call validates its arguments, enqueues kernels on `hip_stream`
 *    (a hipStream_t, NULL = the default stream) and returns without synchronising.
 *    One context must be used from one host thread and one stream at a time.
 *  - Errors: every call returns a moe_status; nothing has been enqueued when the status is
 *    MOE_E_ARG / MOE_E_UNSUPPORTED / MOE_E_WORKSPACE.  moe_last_error gives the message.
 *  - Expert weight tables are HOST arrays of DEVICE pointers, read when the call is made,
 *    so that a weight streamer may repoint them between calls (sequential execution of
 *    experts with prefetched weights, Sec. 4.2).  The library copies them into one of 8
 *    device tables the context owns and re-uses the last copy while the pointers stay the same
 *    (a call on another stream first waits for that copy).  A HIP graph captured from a call
 *    refers to the table that was current at capture: it stays valid until 8 further tables
 *    have been uploaded on the context (calls with other weight pointers; every expert group of
 *    moe_layer_streamed is one), so give graphs that are replayed for long a context of their own.
 *  - Weight layout on the hot path is the PACKED one produced by moe_pack_weight from the
 *    logical [H,F] / [F,H] matrices (same number of bytes): the transposed matrix W[n][k]
 *    (k = contraction index) is cut into blocks of 16 rows x 32 k = 1 KiB, blocks ordered
 *    [N/16][K/32]; inside a block, row r (0..15) occupies bytes 64r..64r+63 and its 16-byte
 *    piece c (k = 8c..8c+7) sits at slot c ^ ((4 - r/4) & 3); rows keep their logical order.
 *    Weights are static, so packing is not part of the timed path.
 *  - Limits: H % 64 == 0, F % 64 == 0, 1 <= top_k <= E <= 256, top_k <= 64,
 *    0 <= num_shared <= 8, every matrix below 4 GiB.  Other shapes: MOE_E_UNSUPPORTED.
 *  - An empty batch (T = 0) is valid: the call returns MOE_OK, reads no buffer and enqueues
 *    nothing, except that moe_permute writes expert_offsets = 0 (every group is empty).
 */
#ifndef MOE_MI355_H
#define MOE_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct moe_ctx moe_ctx; /* opaque: device id, pointer-table slots, profiling events, error text */

typedef enum {
    MOE_OK = 0,
    MOE_E_ARG = 1,         /* null pointer, non-positive size, top_k > E, ... */
    MOE_E_UNSUPPORTED = 2, /* a shape outside the limits above */
    MOE_E_WORKSPACE = 3,   /* workspace_bytes smaller than moe_workspace_bytes(shape) */
    MOE_E_HIP = 4          /* a HIP runtime call or kernel launch failed */
} moe_status;

typedef struct {
    int32_t T;           /* tokens in the accumulated batch */
    int32_t H;           /* hidden size */
    int32_t F;           /* expert FFN width */
    int32_t E;           /* routed experts */
    int32_t top_k;       /* experts per token */
    int32_t num_shared;  /* always-on shared experts, each of width F */
    int32_t renormalize; /* 1: weights divided by their sum over the selected k; 0: raw softmax probabilities */
    float routed_scale;  /* multiplies the routed weights (1.0 in all reference workloads) */
} moe_shape;

/* Stage ids for the profiling interface. */
enum {
    MOE_STAGE_ROUTE = 0,
    MOE_STAGE_PERMUTE_INDEX = 1, /* histogram + scan + stable placement */
    MOE_STAGE_PERMUTE_GATHER = 2,
    MOE_STAGE_PLAN = 3,          /* tile work-list from expert_offsets */
    MOE_STAGE_FFN_GATE_UP = 4,   /* grouped GEMM 1 + SiLU-gate epilogue */
    MOE_STAGE_FFN_DOWN = 5,      /* grouped GEMM 2 */
    MOE_STAGE_COMBINE = 6,
    MOE_STAGE_COUNT = 7
};

/* Creates a context bound to HIP device `device` (host call; allocates the small device
 * tables).  *out is NULL on failure. */
moe_status moe_create(moe_ctx** out, int device);
void moe_destroy(moe_ctx* ctx);
/* Message of the last failing call on this context ("" if none); valid until the next call. */
const char* moe_last_error(const moe_ctx* ctx);

/* Bytes of device workspace that is enough for any call below with this shape, for ANY
 * routing outcome (per-expert token counts are unknown until run time, Sec. 4.3).
 * Returns 0 for an invalid shape. */
size_t moe_workspace_bytes(const moe_shape* shape);

/* Bytes of the h scratch that moe_grouped_ffn needs: (roundup16(T*k) + num_shared *
 * roundup16(T)) rows of F bf16 (h is kept in 16-row x 32-column blocks, and the routed rows
 * and each shared expert's rows start on a block boundary).  0 for an invalid shape. */
size_t moe_h_scratch_bytes(const moe_shape* shape);

/* Tuning knobs (host call).  Unknown key or out-of-range value: MOE_E_ARG.
 *   "gemm_waves"      4 | 8   wavefronts per GEMM workgroup (one or two per SIMD)
 *   "gemm_wave_rows"  1|2|4   rows of the wave grid (rows x waves/rows): 1 or 2 with 4 waves (4 rows
 *                             is treated as 1), 2 or 4 with 8 waves (1 row is treated as 2)
 *   "gemm_group_m"    0..64   m-tiles swept together along n (L2 reuse of weight panels); 0 (default) picks
 *                             the typical number of tiles per expert, between 4 and 8
 *   "xcd_remap"       0 | 1   give each XCD runs of consecutive tiles
 *   "small_tiles"     0 | 1   use 128/64/32-row tiles for the ragged tail of an expert
 *   "gemm_tile_rows_up" / "gemm_tile_rows_down"  0 | 128 | 256 | 320   rows per m-tile of the gate/up and
 *                             the down GEMM; 0 (default) picks per launch from the tile count and the mean
 *                             rows per expert (320: 4 waves x 1 wave row only, else treated as 256)
 *   "x_tiled"         -1|0|1  moe_layer: 1 gathers x once into a block-tiled x_perm that the gate/up GEMM
 *                             loads in 1 KiB pieces, 0 fuses the gather into that GEMM's loads, -1 (default)
 *                             chooses by expert width.  Same results bit for bit.
 *   "tails_last"      -1|0|1  order of a GEMM's tiles: 1 or -1 (default) = every expert's short tail tile (at most
 *                             half a tile high) after all other tiles, longest first; 0 = behind its own
 *                             expert's tiles.  Same results bit for bit.
 *   "down_tail_splits" 0|1|2  with at most 32 experts the down projection can cut the contraction range of an
 *                             expert's short tail tile into 2 or 4 pieces run by different CUs and add the fp32
 *                             partial sums afterwards in fixed order.  0: never; 2: every eligible tail;
 *                             1 (default): where it pays, decided on the device from the call's tile counts
 *                             (launches in which every tile is a short tail, i.e. a few tokens per expert, and
 *                             launches many rounds of tiles long).  Cutting changes the summation order of
 *                             those rows only: results are deterministic for given inputs and options, but not
 *                             bit-identical between the three settings, nor, under 1, between calls that
 *                             cover the same tokens in differently sized passes.
 *   "tall_tiles"    -1|0|1|2  an expert's tail of at most 64 rows joins its last full 256-row tile (a tile of up to
 *                             320 rows: 12-25 % more time for that tile) instead of costing a pass of its own
 *                             over the expert's weights; 4 waves x 1 wave row only.  2: the tall tile keeps its
 *                             place, 1: tall tiles run after the regular ones (when "tails_last"), 0: off,
 *                             -1 (default): 2 for up to 8 tiles per expert on average, else 1.  Same results
 *                             bit for bit.
 *   "y_fp32"          0 | 1   staged calls: dtype of y_perm / y_shared: 1 (default) fp32, 0 bf16.  bf16 halves the
 *                             traffic of the down projection's store and of the combine's loads, but
 *                             rounds each expert output to 8 mantissa bits before the weighted sum
 *   "layer_y_fp32"    -1|0|1  moe_layer: dtype of its internal y_perm: 1 fp32, 0 bf16, -1 (default) bf16 when
 *                             top_k >= 4 and shared experts exist (each rounded term then carries a small
 *                             share of the output), fp32 otherwise.
 *                             Its y_shared is always fp32.
 *   "out_fp32"        0 | 1   dtype of the layer output written by moe_combine / moe_layer:
 *                             0 (default) bf16 = round-to-nearest-even of the fp32 sum, 1 fp32
 *   "gate_packed"     0 | 1   1: the wg_bf16 argument of moe_route and of every moe_layer variant is the packed
 *                             gate matrix made by moe_pack_gate (the router then skips its per-call packing
 *                             launch).  Default 0. */
moe_status moe_set_option(moe_ctx* ctx, const char* key, int32_t value);

/* One-time weight packing: w_logical [rows, cols] bf16 (device; rows = contraction dimension)
 * -> w_packed, rows*cols bf16 in the packed layout described above (device, distinct buffer).
 * rows, cols multiples of 32. */
moe_status moe_pack_weight(moe_ctx* ctx, const void* w_logical, int32_t rows, int32_t cols,
                           void* w_packed, void* hip_stream);

/* One-time packing of the gate matrix (the router multiplies x with it on the matrix cores):
 * wg_bf16 [H,E] logical (device) -> wg_packed (device, moe_gate_packed_bytes(shape) bytes: the
 * expert count padded to a multiple of 32 with zero rows, in the packed weight layout).  The gate
 * matrix is static like the expert weights, so this cost is outside the timed path; pass the
 * result as wg_bf16 under option "gate_packed" = 1.  Without it every call packs the matrix into
 * its workspace first (one small launch). */
size_t moe_gate_packed_bytes(const moe_shape* shape);
moe_status moe_pack_gate(moe_ctx* ctx, const moe_shape* shape, const void* wg_bf16, void* wg_packed, void* hip_stream);

/* Router (Sec. 2 "MoE inference": every token is sent to its k best-scoring experts).
 * logit[t,e] = sum_h x[t,h] Wg[h,e] (+ gate_bias[e]) in fp32;
 * p = softmax over all E; the k largest logits are selected (ties: lower expert id),
 * listed in descending order; weight = p (divided by the sum over the selected k when
 * renormalize) * routed_scale.
 *   x_bf16 [T,H] device, wg_bf16 [H,E] device (logical layout; packed under option "gate_packed"),
 *   gate_bias [E] fp32 device or NULL
 *   topk_idx [T,k] int32 device out, topk_w [T,k] fp32 device out,
 *   logits_or_null [T,E] fp32 device out (for near-tie reports) or NULL
 *   workspace: device, at least moe_workspace_bytes(shape) (holds the packed gate matrix unless the
 *   caller passes it packed and, for E > 16, the partial logits of the gate GEMM). */
moe_status moe_route(moe_ctx* ctx, const moe_shape* shape, const void* x_bf16, const void* wg_bf16,
                     const float* gate_bias, int32_t* topk_idx, float* topk_w, float* logits_or_null,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/* Groups the T*k (token, rank) pairs by expert (Table 1 measures the expert module by the
 * tokens each expert receives; the counts are only known at run time, Sec. 4.3).  Order: ascending expert, then ascending
 * token.  expert_offsets[e] = first row of expert e (expert_offsets[E] = T*k);
 * perm[r] = t*k+j of the pair at row r; inv_perm[t*k+j] = r; x_perm[r,:] = x[t,:].
 *   topk_idx [T,k] int32 device in (every id in [0,E); not validated)
 *   x_perm_bf16 [T*k,H] device out, or NULL to skip the row gather
 *   expert_offsets [E+1], perm [T*k], inv_perm [T*k] int32 device out
 *   row_token_or_null [T*k] int32 device out: row_token[r] = perm[r] / k, or NULL
 *   workspace: device, at least moe_workspace_bytes(shape). */
moe_status moe_permute(moe_ctx* ctx, const moe_shape* shape, const void* x_bf16, const int32_t* topk_idx,
                       void* x_perm_bf16, int32_t* expert_offsets, int32_t* perm, int32_t* inv_perm,
                       int32_t* row_token_or_null, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Per-expert SwiGLU FFN over the grouped rows (Sec. 2: a token goes through each of its k
 * experts; experts with no rows are skipped, App. A), as two grouped bf16 GEMMs with fp32
 * accumulation: h = silu(X_e W1_e) * (X_e W3_e) rounded to bf16, then y = h W2_e kept in
 * fp32 (or rounded to bf16 under option "y_fp32" = 0).  Shared experts E..E+num_shared-1 run on all T tokens of x; their outputs are
 * summed (one GEMM over the concatenated contraction dimension) into y_shared.
 *   x_perm_bf16 [T*k,H] device in; ignored (may be NULL) when row_token is given
 *   row_token_or_null [T*k] int32 device: row r of the expert input is x[row_token[r],:]
 *   x_bf16 [T,H] device in: needed when num_shared > 0 or row_token is given, else may be NULL
 *   expert_offsets [E+1] int32 device in
 *   w1p, w3p, w2p: host arrays of E+num_shared device pointers; w1p[e] / w3p[e] = moe_pack_weight of
 *   the logical [H,F] gate / up matrix, w2p[e] = moe_pack_weight of the logical [F,H] down matrix
 *   h_scratch_bf16: device scratch of moe_h_scratch_bytes(shape) bytes
 *   y_perm [T*k,H] device out; y_shared [T,H] device out (NULL iff num_shared == 0); both fp32,
 *   or bf16 under option "y_fp32" = 0
 *   workspace: device, at least moe_workspace_bytes(shape). */
moe_status moe_grouped_ffn(moe_ctx* ctx, const moe_shape* shape, const void* x_perm_bf16,
                           const int32_t* row_token_or_null, const void* x_bf16,
                           const int32_t* expert_offsets, const void* const* w1p, const void* const* w3p,
                           const void* const* w2p, void* h_scratch_bf16, void* y_perm, void* y_shared,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/* Weighted sum back in token order (Sec. 2: the layer output is the weighted sum of the
 * selected experts' outputs, plus the shared expert every token goes through):
 *   out[t,:] = sum_{j<k} topk_w[t,j] * y_perm[inv_perm[t*k+j],:] (+ y_shared[t,:]),
 * fp32 accumulation in the order j = 0..k-1 then shared, one store per element, no atomics.
 *   y_perm [T*k,H] and y_shared_or_null [T,H]: fp32 (bf16 under "y_fp32" = 0); inv_perm [T*k];
 *   topk_w [T,k] fp32 (already carries routed_scale); out [T,H] bf16 (fp32 under "out_fp32" = 1):
 *   all device. */
moe_status moe_combine(moe_ctx* ctx, const moe_shape* shape, const void* y_perm, const int32_t* inv_perm,
                       const float* topk_w, const void* y_shared_or_null, void* out, void* hip_stream);

/* The whole expert module (Sec. 2 "MoE inference") on the one large batch that module-based
 * batching accumulates for it (Sec. 4.2), on one stream: route -> permute (indices; the row gather is fused
 * into the first GEMM's loads, or done once into a tiled x_perm: option "x_tiled") -> grouped
 * FFN -> combine.  Same results as the staged
 * calls bit for bit (options alike).  All intermediates live in `workspace`.  out [T,H] is bf16, or fp32
 * under option "out_fp32" = 1. */
moe_status moe_layer(moe_ctx* ctx, const moe_shape* shape, const void* x_bf16, const void* wg_bf16,
                     const float* gate_bias, const void* const* w1p, const void* const* w3p,
                     const void* const* w2p, void* out, void* workspace, size_t workspace_bytes,
                     void* hip_stream);

/* moe_layer for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same
 * results bit for bit; the intermediates live in a scratch array of MOE_STATIC_WORKSPACE_BYTES
 * that is part of the library's device image (each GPU the library runs on holds one copy until
 * the process ends).  The call allocates nothing and frees nothing.
 * Limit: moe_workspace_bytes(shape) <= MOE_STATIC_WORKSPACE_BYTES (small and decode-sized batches;
 * e.g. 256 tokens of H = 512, F = 1024 with 8 experts), else MOE_E_WORKSPACE and nothing is enqueued.
 * All contexts and calls on one GPU share that GPU's array: two calls that overlap in time on
 * one GPU (different streams, or different contexts) race; calls on one stream are safe.  The
 * array keeps the previous call's contents; the layer never reads a region before writing it. */
#define MOE_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)
moe_status moe_layer_static(moe_ctx* ctx, const moe_shape* shape, const void* x_bf16, const void* wg_bf16,
                            const float* gate_bias, const void* const* w1p, const void* const* w3p,
                            const void* const* w2p, void* out, void* hip_stream);

/* Accumulation of micro-batches (Sec. 4.2: the hidden states that leave attention in micro-batches
 * of b_a sequences are accumulated until the expert module's batch B is reached): appends
 * `rows` rows of x_microbatch [rows, H] bf16 (device) to staging [capacity_rows, H] bf16 (device)
 * at row *rows_filled and adds `rows` to *rows_filled (host counter owned by the caller).
 * An asynchronous device-to-device copy on hip_stream.  MOE_E_ARG if the rows do not fit. */
moe_status moe_accumulate(moe_ctx* ctx, void* staging, int32_t capacity_rows, int32_t H, int32_t* rows_filled,
                          const void* x_microbatch, int32_t rows, void* hip_stream);

/* moe_layer over at most max_tokens_per_pass tokens at a time (Sec. 4.3: the expert module
 * takes b_e tokens per pass so that its intermediates fit the memory left beside weights and
 * KV cache).  Tokens are independent, so the result equals moe_layer's: bit for bit with option
 * "down_tail_splits" = 0, otherwise up to the summation order of rows that fall into a K-split
 * tail tile in one run and not in the other.  `shape` describes all T tokens; the workspace only
 * has to hold one pass: moe_workspace_bytes of the same shape with T = min(T, max_tokens_per_pass). */
moe_status moe_layer_chunked(moe_ctx* ctx, const moe_shape* shape, const void* x_bf16, const void* wg_bf16,
                             const float* gate_bias, const void* const* w1p, const void* const* w3p,
                             const void* const* w2p, int32_t max_tokens_per_pass, void* out, void* workspace,
                             size_t workspace_bytes, void* hip_stream);

/* moe_layer with the expert weights in HOST memory (Sec. 4.2: experts are executed one after
 * another while the next expert's weights are prefetched into a second buffer; App. A: only
 * experts that received tokens are fetched).  Experts are taken in groups of
 * `experts_per_group` consecutive non-empty experts; group g is copied into staging slot
 * g % num_slots with hipMemcpyAsync on a stream the context owns while the GEMMs of earlier
 * groups run on `hip_stream`; events hand the slots back and forth.  The shared experts form
 * the last group.  Same kernels and same results as moe_layer, bit for bit (with option
 * "down_tail_splits" at 0 or 2; under its default rule a pass over one group of experts and a
 * pass over all of them may decide differently whether to cut a short tail, which changes the
 * summation order of that tail's rows).
 *   host_w1p / host_w3p / host_w2p: host arrays of E+num_shared HOST pointers to packed
 *   matrices (H*F bf16 each, moe_pack_weight layout), in pinned memory for the copies to overlap
 *   slots: device buffer of num_slots * slot_bytes bytes; a slot must hold
 *   max(experts_per_group, num_shared) experts, 3*H*F*2 bytes each; num_slots in 2..8
 * The call SYNCHRONISES hip_stream once (it needs the per-expert row counts on the host to
 * decide what to fetch); everything after that is enqueued asynchronously.
 * Errors: as moe_layer; MOE_E_ARG for a slot that is too small. */
moe_status moe_layer_streamed(moe_ctx* ctx, const moe_shape* shape, const void* x_bf16, const void* wg_bf16,
                              const float* gate_bias, const void* const* host_w1p, const void* const* host_w3p,
                              const void* const* host_w2p, void* slots, size_t slot_bytes, int32_t num_slots,
                              int32_t experts_per_group, void* out, void* workspace, size_t workspace_bytes,
                              void* hip_stream);

/* Counters of the last moe_layer_streamed call: bytes copied host -> device, expert groups run,
 * experts skipped because they had no rows.  Any out-pointer may be NULL. */
moe_status moe_stream_stats(const moe_ctx* ctx, uint64_t* bytes_copied, int32_t* groups, int32_t* experts_skipped);

/* Run-time estimate of moe_layer_streamed's expert phase, in milliseconds (host arithmetic only;
 * Sec. 4.4: the jobs of an offloaded layer form a DAG of copy and compute nodes, and the
 * earliest finishing time of each node follows in topological order from
 * finish[v] = cost[v] + max over predecessors finish[u]; the exit node's value is the estimate).
 * Nodes: copy(g) and compute(g) for every group g that moe_layer_streamed would form from
 * rows_per_expert (empty experts skipped, shared experts last).  Edges: copy(g) -> compute(g);
 * copy(g-1) -> copy(g) (one copy stream); compute(g-1) -> compute(g) (one compute stream);
 * compute(g-num_slots) -> copy(g) (the slot must be free).
 * cost(copy g) = bytes of the group's experts / link_gbs; cost(compute g) = 6 * rows * H * F /
 * ffn_tflops, both rates measured by the caller (e.g. bench.py --streamed, the sweep script).
 *   rows_per_expert [E] host.  Returns a negative value for invalid arguments. */
double moe_estimate_streamed_ms(const moe_shape* shape, const int32_t* rows_per_expert, int32_t experts_per_group,
                                int32_t num_slots, double link_gbs, double ffn_tflops);

/* Device pointers into a workspace last used by moe_layer with this shape, for inspection:
 * topk_idx [T,k] int32, topk_w [T,k] fp32, expert_offsets [E+1] int32, inv_perm [T*k] int32.
 * Any out-pointer may be NULL. */
moe_status moe_layer_views(const moe_shape* shape, void* workspace, int32_t** topk_idx, float** topk_w,
                           int32_t** expert_offsets, int32_t** inv_perm);

/* Profiling.  While enabled, every kernel group a call enqueues is bracketed by HIP events on
 * the call's stream.  moe_profile_read waits for the recorded events, adds the elapsed
 * milliseconds per stage into ms_sum[MOE_STAGE_COUNT] and the number of intervals into
 * launches[MOE_STAGE_COUNT], and clears the record.  At most 8192 intervals are kept
 * between reads (further ones are dropped). */
moe_status moe_profile_enable(moe_ctx* ctx, int32_t on);
moe_status moe_profile_read(moe_ctx* ctx, double* ms_sum, int32_t* launches);
/* The same record interval by interval, in the order the calls enqueued them: stage[i] is a
 * MOE_STAGE_* id, ms[i] its elapsed time.  At most `capacity` intervals are returned (the rest
 * are dropped); *count = number returned.  Waits for the events; clears the record. */
moe_status moe_profile_read_intervals(moe_ctx* ctx, int32_t* stage, float* ms, int32_t capacity, int32_t* count);

/* Measured ceiling of the matrix cores for the roofline report: one launch of a register-only loop
 * of the MFMA instruction the grouped GEMMs use (1024 workgroups x 4 wavefronts x iters x 64
 * instructions, no LDS or memory traffic inside the loop), timed with HIP events on hip_stream.
 * The sustained rate depends on the operand values (the chip is power-limited on dense bf16
 * work), so the operand fragments are read from a_bf16 / b_bf16 (device, `bytes` bytes each,
 * 16-byte aligned; e.g. a packed weight matrix and the activations of the workload); NULL for
 * both = all-zero operands.  sink: device scratch of at least 1 MiB (receives checksums).
 * SYNCHRONISES the stream.  *tflops = 2*16*16*32 FLOP per instruction / elapsed time. */
moe_status moe_profile_mfma_ceiling(moe_ctx* ctx, const void* a_bf16, const void* b_bf16, size_t bytes, int32_t iters,
                                    void* sink, size_t sink_bytes, double* tflops, double* ms_or_null, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_MI355_H */
