// C-ABI layer: argument validation, workspace carving, weight pointer tables, profiling events.
// Every step of the path runs in the kernels of this library; this file only enqueues them.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "common.h"

using namespace moe;

// Scratch for moe_layer_static: callers that must not allocate get their workspace from here.
// Every GPU the library runs on holds its own copy of the array until the process ends.  In
// host code the array's name is only a handle for hipGetSymbolAddress (done once per context
// in moe_create, with the context's device current); kernels are given the address it returns.
constexpr size_t STATIC_SCRATCH_BYTES = MOE_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

constexpr int TABLE_SLOTS = 8;
constexpr int MAX_GROUPS = 256;
constexpr int PROF_MAX = 8192;
constexpr int MAX_SLOTS = 8;

struct ProfRec {
    int stage;
    hipEvent_t a, b;
};

}  // namespace

struct moe_ctx {
    int device = 0;
    char err[512] = {0};
    GemmConfig gemm{1, 4, 0, 1, 1, 0, 0, -1, -1, 1, -1};
    bool y_fp32 = true;    // dtype of y_perm / y_shared in the staged calls
    int layer_y = -1;      // moe_layer's y_perm: 1 fp32, 0 bf16, -1 choose (its y_shared is always fp32)
    bool out_fp32 = false; // dtype of the layer output
    bool gate_packed = false;  // E > 16: the wg argument is already in the packed layout (moe_pack_gate)
    char* static_ws = nullptr;  // this device's address of `scratch`
    // Ring of device pointer tables [3][MAX_GROUPS] (W1p, W3p, W2p), each with a pinned host
    // staging copy and an event marking the end of its upload.
    void** d_tab[TABLE_SLOTS] = {nullptr};
    void** h_tab[TABLE_SLOTS] = {nullptr};
    hipEvent_t tab_done[TABLE_SLOTS] = {nullptr};
    int tab_next = 0;
    int tab_cur = -1;
    int tab_n = 0;
    hipStream_t tab_stream = nullptr;     // stream of the current table's upload
    std::vector<const void*> tab_shadow;  // contents of slot tab_cur
    // streamed weights: copy stream, slot hand-over events, pinned copy of expert_offsets, counters
    hipStream_t copy_stream = nullptr;
    hipEvent_t slot_ready[MAX_SLOTS] = {nullptr};
    hipEvent_t slot_free[MAX_SLOTS] = {nullptr};
    int32_t* h_offsets = nullptr;
    uint64_t stream_bytes = 0;
    int stream_groups = 0, stream_skipped = 0;
    // profiling
    bool prof = false;
    std::vector<ProfRec> recs;
    std::vector<hipEvent_t> pool;
};

namespace {

moe_status fail(moe_ctx* c, moe_status st, const char* fmt, ...) {
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->err, sizeof(c->err), fmt, ap);
        va_end(ap);
    }
    return st;
}

#define HIP_TRY(ctx, expr)                                                                      \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess) return fail(ctx, MOE_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

const char* shape_problem(const moe_shape* s, moe_status* st) {
    *st = MOE_E_ARG;
    if (!s) return "shape is NULL";
    if (s->T < 0 || s->H < 1 || s->F < 1 || s->E < 1 || s->top_k < 1) return "T must be >= 0; H, F, E, top_k >= 1";
    if (s->top_k > s->E) return "top_k > E";
    if (s->num_shared < 0) return "num_shared < 0";
    if (s->renormalize != 0 && s->renormalize != 1) return "renormalize must be 0 or 1";
    *st = MOE_E_UNSUPPORTED;
    if (s->H % 64 || s->F % 64) return "H and F must be multiples of 64";
    if (s->E > 256 || s->top_k > 64) return "E <= 256 and top_k <= 64 required";
    if (s->num_shared > 8 || s->E + s->num_shared > MAX_GROUPS) return "num_shared <= 8 and E + num_shared <= 256 required";
    const int64_t lim = (int64_t)1 << 32;
    const int64_t R = (int64_t)s->T * s->top_k, Rs = (int64_t)s->T * s->num_shared;
    if (R >= ((int64_t)1 << 31) / 2) return "T * top_k too large";
    if (R * s->H * 2 >= lim || (R + Rs + 16 * (1 + s->num_shared)) * s->F * 2 >= lim || (int64_t)s->H * s->F * 2 >= lim)
        return "a matrix reaches 4 GiB";
    *st = MOE_OK;
    return nullptr;
}

inline size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

// Router through the GEMM tile routine (E > 16): experts padded to 32, K cut into `splits`
// independent accumulation chains (shorter fp32 sums, and more tiles to fill the CUs), tiles
// of `tm` tokens.  splits == 0 (E <= 16): one kernel does the contraction and the selection; `ep`
// (rows of the packed gate matrix) is valid for every shape.
struct RouteGemm {
    int splits, ep, tm;
};
RouteGemm route_gemm_config(const moe_shape& s) {
    RouteGemm r{0, 0, 0};
    r.ep = (s.E + 31) & ~31;   // rows of the packed gate matrix (zero rows past E)
    if (s.E <= 16) return r;   // splits = 0: no gate GEMM launch, route_mfma_kernel does it all
    // K pieces: a divisor of H/32 (a piece is a whole number of K sub-tiles, at least two), at most 8:
    // the smallest that keeps a chain of fp32 additions at or under 1536 terms (the logits'
    // rounding error grows with the chain: a single chain over H = 6336 measured 7e-6 against
    // the fp64 reference, over half the near-tie margin), and from H = 1024 on at least 4
    // (enough tiles to fill the chip at the batch sizes this is for).  If no divisor reaches that
    // count, the largest one below it.
    const int kt = s.H / 32;
    int want = (s.H + 1535) / 1536;
    if (s.H >= 1024 && want < 4) want = 4;
    int below = 1, pick = 0;
    for (int n = 1; n <= 8 && !pick; ++n) {
        if (kt % n != 0 || kt / n < 2) continue;
        if (n >= want) pick = n;
        else below = n;
    }
    r.splits = pick ? pick : below;
    r.tm = (int64_t)r.splits * ((s.T + 255) / 256) >= 512 ? 256 : 128;
    return r;
}

// K pieces per short tail tile of the down GEMM.  A short tail of the down projection streams a
// whole 256-row panel of W2 for a few rows of work, and few of them run at a time at the end of
// the launch, each limited by what one CU can load; cutting K spreads that over more CUs.  The
// partial sums need E * pieces * 128 fp32 rows of workspace, so this is for few experts only.
int down_tail_splits(const moe_shape& s) {
    if (s.E > 32) return 1;
    for (int sp : {4, 2})
        if (s.F % (32 * sp) == 0 && s.F / (32 * sp) >= 8) return sp;
    return 1;
}

// Workspace layout: fixed order, every region 256-byte aligned.
struct Layout {
    size_t topk_idx, topk_w, offsets, perm, inv_perm, row_token, chunk_counts, plan, descs_up, descs_down,
        split_tails, split_partial, rt_wg, rt_logits, x_tiled, h, y_perm, y_shared, total;
};

Layout make_layout(const moe_shape& s) {
    Layout L;
    const size_t R = (size_t)s.T * s.top_k, Rs = (size_t)s.T * s.num_shared;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    L.topk_idx = take(R * 4);
    L.topk_w = take(R * 4);
    L.offsets = take(((size_t)s.E + 1) * 4);
    L.perm = take(R * 4);
    L.inv_perm = take(R * 4);
    L.row_token = take(R * 4);
    L.chunk_counts = take((size_t)permute_chunks(s) * s.E * 4);
    L.plan = take(sizeof(PlanHeader));
    L.descs_up = take((size_t)max_mtiles(s, 128) * sizeof(TileDesc));
    const int dsp = down_tail_splits(s);
    L.descs_down = take(((size_t)max_mtiles(s, 128) + (size_t)s.E * (dsp - 1)) * sizeof(TileDesc));
    L.split_tails = take((size_t)s.E * sizeof(SplitTail));
    L.split_partial = take(dsp > 1 ? (size_t)s.E * dsp * SPLIT_TAIL_ROWS * s.H * 4 : 0);
    // router: packed gate matrix (unless the caller passes it packed); E > 16: partial logits of the gate GEMM
    const RouteGemm rg = route_gemm_config(s);
    L.rt_wg = take((size_t)rg.ep * s.H * 2);
    L.rt_logits = take(rg.splits ? (size_t)rg.splits * s.T * rg.ep * 4 : 0);
    L.x_tiled = take(((R + 15) & ~(size_t)15) * s.H * 2);
    L.h = take((size_t)h_rows(s) * s.F * 2);
    L.y_perm = take(R * s.H * 4);  // sized for fp32 y
    L.y_shared = take(Rs ? (size_t)s.T * s.H * 4 : 0);
    L.total = o;
    return L;
}

moe_status check_common(moe_ctx* c, const moe_shape* s) {
    if (!c) return MOE_E_ARG;
    c->err[0] = 0;
    moe_status st;
    if (const char* why = shape_problem(s, &st)) return fail(c, st, "%s", why);
    HIP_TRY(c, hipSetDevice(c->device));
    return MOE_OK;
}

moe_status check_ws(moe_ctx* c, const moe_shape* s, const void* ws, size_t bytes) {
    if (!ws) return fail(c, MOE_E_ARG, "workspace is NULL");
    if ((uintptr_t)ws & 255) return fail(c, MOE_E_ARG, "workspace must be 256-byte aligned");
    const size_t need = make_layout(*s).total;
    if (bytes < need) return fail(c, MOE_E_WORKSPACE, "workspace %zu bytes < required %zu", bytes, need);
    return MOE_OK;
}

// ---- profiling helpers --------------------------------------------------------------------
hipEvent_t get_event(moe_ctx* c) {
    if (!c->pool.empty()) { hipEvent_t e = c->pool.back(); c->pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

struct StageTimer {
    moe_ctx* c; hipStream_t st; int stage; hipEvent_t a = nullptr, b = nullptr;
    StageTimer(moe_ctx* c_, hipStream_t st_, int stage_) : c(c_), st(st_), stage(stage_) {
        if (c->prof && (int)c->recs.size() < PROF_MAX) {
            a = get_event(c); b = get_event(c);
            if (a && b) (void)hipEventRecord(a, st);
        }
    }
    ~StageTimer() {
        if (a && b) { (void)hipEventRecord(b, st); c->recs.push_back({stage, a, b}); }
    }
};

// ---- weight pointer tables ----------------------------------------------------------------
// Returns the device table holding [w1p | w3p | w2p] (MAX_GROUPS entries each); uploads only
// when the caller's pointers differ from the last upload.
moe_status weight_table(moe_ctx* c, int n, const void* const* w1, const void* const* w3, const void* const* w2,
                        hipStream_t st, void*** out) {
    if (!w1 || !w3 || !w2) return fail(c, MOE_E_ARG, "weight pointer table is NULL");
    for (int i = 0; i < n; ++i)
        if (!w1[i] || !w3[i] || !w2[i]) return fail(c, MOE_E_ARG, "weight pointer %d is NULL", i);
    bool same = c->tab_cur >= 0 && c->tab_n == n;
    if (same)
        for (int i = 0; i < n && same; ++i)
            same = c->tab_shadow[i] == w1[i] && c->tab_shadow[MAX_GROUPS + i] == w3[i] &&
                   c->tab_shadow[2 * MAX_GROUPS + i] == w2[i];
    if (!same) {
        const int slot = c->tab_next;
        c->tab_next = (slot + 1) % TABLE_SLOTS;
        HIP_TRY(c, hipEventSynchronize(c->tab_done[slot]));  // the slot's previous upload has finished
        for (int i = 0; i < n; ++i) {
            c->h_tab[slot][i] = const_cast<void*>(w1[i]);
            c->h_tab[slot][MAX_GROUPS + i] = const_cast<void*>(w3[i]);
            c->h_tab[slot][2 * MAX_GROUPS + i] = const_cast<void*>(w2[i]);
            c->tab_shadow[i] = w1[i];
            c->tab_shadow[MAX_GROUPS + i] = w3[i];
            c->tab_shadow[2 * MAX_GROUPS + i] = w2[i];
        }
        HIP_TRY(c, hipMemcpyAsync(c->d_tab[slot], c->h_tab[slot], 3 * MAX_GROUPS * sizeof(void*),
                                  hipMemcpyHostToDevice, st));
        HIP_TRY(c, hipEventRecord(c->tab_done[slot], st));
        c->tab_cur = slot;
        c->tab_n = n;
        c->tab_stream = st;
    } else if (st != c->tab_stream) {
        // the cached table was uploaded on another stream: this stream's kernels must not overtake that copy
        HIP_TRY(c, hipStreamWaitEvent(st, c->tab_done[c->tab_cur], 0));
    }
    *out = c->d_tab[c->tab_cur];
    return MOE_OK;
}

moe_status run_route(moe_ctx* c, const moe_shape& s, const void* x, const void* wg, const float* bias, int32_t* idx,
                     float* w, float* logits, char* ws, hipStream_t st) {
    const RouteGemm rg = route_gemm_config(s);
    const Layout L = make_layout(s);
    // The gate matrix is static: a caller that packs it once (moe_pack_gate, option "gate_packed")
    // spares every call this launch.
    const char* wg_packed = (const char*)wg;
    if (!c->gate_packed) {
        HIP_TRY(c, launch_pack_weight(wg, s.H, s.E, rg.ep, ws + L.rt_wg, st));
        wg_packed = ws + L.rt_wg;
    }
    if (!rg.splits) {
        // E <= 16: one kernel, logits on the matrix cores and the selection in the same workgroup
        HIP_TRY(c, launch_route_mfma(s, x, wg_packed, bias, idx, w, logits, st));
        return MOE_OK;
    }
    const int k_split = s.H / rg.splits;
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.a_routed = (const char*)x;
    a.a_shared = (const char*)x;
    a.w_uniform = wg_packed;
    a.w_uniform_stride = (uint32_t)(k_split / 32) * 1024u;   // K-split s starts s * (k_split / 32) blocks of 1 KiB along
    a.uniform_tm = rg.tm;
    a.uniform_per = (s.T + rg.tm - 1) / rg.tm;
    a.uniform_splits = rg.splits;
    a.out_routed = ws + L.rt_logits;
    a.out_shared = ws + L.rt_logits;
    a.K = k_split;
    a.N = rg.ep;
    a.T = s.T;
    a.nseg_shared = 1;
    a.n_tiles = (rg.ep + 255) / 256;
    a.max_mtiles = rg.splits * ((s.T + rg.tm - 1) / rg.tm);
    a.group_m = 8;
    a.xcd_remap = 0;
    a.small_tiles = 1;
    a.out_fp32 = 3;
    a.lda_bytes = s.H * 2;
    a.kt_w = s.H / 32;
    a.split_rows = s.T;
    a.a_tiled = 0;
    a.t_pad = (s.T + 15) & ~15;
    a.kt_a = 0;
    a.tail_splits = 1;
    GemmConfig cfg = c->gemm;
    cfg.waves = 4;
    cfg.wave_rows = 2;
    HIP_TRY(c, launch_ffn_gemm(false, a, cfg, st));
    HIP_TRY(c, launch_route_topk(s, (const float*)(ws + L.rt_logits), rg.splits, rg.ep, bias, idx, w, logits, st));
    return MOE_OK;
}

// Rows per m-tile for one GEMM.  Tiles of 256 rows are the efficient shape (measured: the
// 128-row shape runs at ~0.75 of their rate); 128 rows only win when a launch has so few
// 256-row tiles that most CUs would idle in its last round.
double expected_tiles(const moe_shape& s, int tm, int n_tiles, int nseg) {
    return ((double)s.T * s.top_k / tm + 0.5 * s.E + (double)nseg * ((s.T + tm - 1) / tm)) * n_tiles;
}

int pick_tile_rows(const moe_shape& s, int n_tiles, int nseg) {
    double best = 0;
    int best_tm = 256;
    for (int tm : {256, 128}) {
        const double tiles = expected_tiles(s, tm, n_tiles, nseg);
        const double rounds = (double)(int64_t)((tiles + 255) / 256);
        const double cost = rounds * tm * (tm == 128 ? 1.35 : 1.0);
        if (best == 0 || cost < best) { best = cost; best_tm = tm; }
    }
    return best_tm;
}

// m-tiles swept together before moving along n.  Tiles of one expert share W panels, so runs
// that match the typical number of tiles per expert (when that is below 8) keep an XCD's 32
// concurrent tiles on fewer distinct panels (measured: C4 with 6 instead of 8: down GEMM +2 %).
int pick_group_m(const moe_ctx* c, const moe_shape& s, int tm) {
    if (c->gemm.group_m > 0) return c->gemm.group_m;
    const double per_expert = (double)s.T * s.top_k / ((double)s.E * tm);
    int g = (int)(per_expert + 0.5);
    return g < 4 ? 4 : (g > 8 ? 8 : g);
}

// Which groups one pass of the two GEMMs covers (streamed weights run several passes), and how
// many m-tiles it can have at most (0 = the bound for any routing).
struct FfnPass {
    int e_lo, e_hi;
    bool shared_on;
    int mtiles_up, mtiles_down;
};

// x_perm_tiled: when non-null, the routed rows of GEMM 1 are read from it (tiled layout) and
// x_perm / row_token are not used for them.
moe_status run_ffn(moe_ctx* c, const moe_shape& s, const void* x_perm, const int32_t* row_token, const void* x,
                   const void* x_perm_tiled, const int32_t* offsets, void** tab, char* ws, void* h, void* y_perm,
                   void* y_shared, bool y_fp32, bool shared_fp32, hipStream_t st, const FfnPass* pass = nullptr) {
    const FfnPass all{0, s.E, true, 0, 0};
    const FfnPass& ps = pass ? *pass : all;
    const Layout L = make_layout(s);
    PlanHeader* plan = (PlanHeader*)(ws + L.plan);
    TileDesc* descs_up = (TileDesc*)(ws + L.descs_up);
    TileDesc* descs_down = (TileDesc*)(ws + L.descs_down);
    const size_t Rpad = ((size_t)s.T * s.top_k + 15) & ~(size_t)15;   // shared experts' rows of h start block-aligned
    const int nt_up = (s.F + 127) / 128, nt_down = (s.H + 255) / 256;
    int tm_up = c->gemm.tile_rows_up ? c->gemm.tile_rows_up : pick_tile_rows(s, nt_up, s.num_shared);
    int tm_down = c->gemm.tile_rows_down ? c->gemm.tile_rows_down : pick_tile_rows(s, nt_down, s.num_shared ? 1 : 0);
    // tiles above 256 rows exist for the 4-wave, 1-wave-row kernel only
    const bool tall_kernel = c->gemm.waves == 4 && c->gemm.wave_rows == 1;
    // Gate/up GEMM: 320-row tiles move 10 % fewer bytes per FLOP from L2 to LDS (the chip is
    // power-limited, and what the loads cost is clock), measured -1.3 % (C3) to -3.9 % (C4, C5) on
    // that GEMM; not when an expert is only about four tiles (C2: 1024 rows = 3 tiles + a tail
    // that needs a pass of its own, +10 %).  In the down GEMM the 320-row variant measures within
    // 1 % of the 256-row one either way, so it keeps 256.
    if (!c->gemm.tile_rows_up && tall_kernel && tm_up == 256 && (double)s.T * s.top_k / s.E >= 1200.0) tm_up = 320;
    if (!tall_kernel && tm_up > 256) tm_up = 256;
    if (!tall_kernel && tm_down > 256) tm_down = 256;
    // Short tail tiles go last by default: the other tiles of a launch then all take the same
    // time, which keeps the CUs that share operand panels in L2 in step (measured: the L2 miss
    // traffic of the gate/up GEMM doubles when short tiles are mixed in), and the launch ends on
    // its smallest work items.
    const bool tl_up = c->gemm.tails_last != 0;
    const bool tl_down = c->gemm.tails_last != 0;
    // K pieces for short tails of the down GEMM: the device-side plan decides from the real tile
    // counts whether to cut (ffn_plan_kernel); here only what the shape alone rules out, which
    // spares the launch of the reduction: tiny matrices (a launch costs more than it can save).
    int dsp = (tl_down && c->gemm.small_tiles && c->gemm.down_tail_splits != 0) ? down_tail_splits(s) : 1;
    if (c->gemm.down_tail_splits == 1 && (int64_t)s.F * s.H < ((int64_t)1 << 21)) dsp = 1;
    // "many rounds" for the plan's rule: eight rounds of 256 tiles (at two to three rounds pieces
    // measured +6 %, at four to five +-0, at thirteen -2 %)
    const int split_rule_tiles = c->gemm.down_tail_splits == 2 ? 0 : (2048 + nt_down - 1) / nt_down;
    SplitTail* split_tails = (SplitTail*)(ws + L.split_tails);
    {
        StageTimer tm(c, st, MOE_STAGE_PLAN);
        // tall tiles exist for the 4-wave, 1-wave-row kernel only
        // In place when a group is at most one run of m-tiles (the tall tile then shares its
        // group's W panels in L2: C2 step -4 %, against -0.5 % after the run region); after the run
        // region for longer groups (C3: in place +5 %, after -0.7 %).
        const double per_expert = (double)s.T * s.top_k / ((double)s.E * 256);
        int tall = c->gemm.tall_tiles >= 0 ? c->gemm.tall_tiles : (per_expert <= 8.0 ? 2 : 1);
        if (!tall_kernel) tall = 0;
        HIP_TRY(c, launch_ffn_plan(s, offsets, tm_up, tm_down, tl_up, tl_down, c->gemm.small_tiles != 0, ps.e_lo, ps.e_hi,
                                   ps.shared_on, dsp, 4, split_rule_tiles, tall, tall, split_tails, plan, descs_up,
                                   descs_down, st));
    }
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.plan = plan;
    a.T = s.T;
    a.xcd_remap = c->gemm.xcd_remap;
    a.small_tiles = c->gemm.small_tiles;
    a.out_fp32 = 0;
    a.t_pad = (s.T + 15) & ~15;
    a.split_rows = 0;
    // GEMM 1: [rows, H] x W1p/W3p [F, H] -> h [rows, F]
    a.descs = descs_up;
    a.group_m = pick_group_m(c, s, tm_up);
    a.max_mtiles = ps.mtiles_up > 0 ? ps.mtiles_up : (int)max_mtiles(s, tm_up);
    a.a_routed = (const char*)(x_perm_tiled ? x_perm_tiled : (row_token ? x : x_perm));
    a.a_shared = (const char*)x;
    a.row_token = x_perm_tiled ? nullptr : row_token;
    a.a_tiled = x_perm_tiled ? 1 : 0;
    a.w_a = (const void* const*)tab;
    a.w_b = (const void* const*)(tab + MAX_GROUPS);
    a.out_routed = (char*)h;
    a.out_shared = (char*)h + Rpad * s.F * 2;
    a.K = s.H;
    a.N = s.F;
    a.lda_bytes = s.H * 2;
    a.kt_w = s.H / 32;
    a.kt_a = s.H / 32;
    a.tail_splits = 1;
    a.nseg_shared = 1;
    a.n_tiles = nt_up;
    {
        StageTimer tm(c, st, MOE_STAGE_FFN_GATE_UP);
        HIP_TRY(c, launch_ffn_gemm(true, a, c->gemm, st));
    }
    // GEMM 2: h [rows, F] x W2p [H, F] -> y [rows, H]
    a.descs = descs_down;
    a.group_m = pick_group_m(c, s, tm_down);
    a.max_mtiles = (ps.mtiles_down > 0 ? ps.mtiles_down : (int)max_mtiles(s, tm_down)) + s.E * (dsp - 1);
    a.a_routed = (const char*)h;
    a.a_shared = (const char*)h + Rpad * s.F * 2;
    a.row_token = nullptr;
    a.a_tiled = 3;
    a.w_a = (const void* const*)(tab + 2 * MAX_GROUPS);
    a.w_b = nullptr;
    a.out_routed = (char*)y_perm;
    a.out_shared = (char*)y_shared;
    a.K = s.F;
    a.N = s.H;
    a.lda_bytes = s.F * 2;
    a.kt_w = s.F / 32;
    a.kt_a = s.F / 32;
    a.tail_splits = dsp;
    a.out_partial = ws + L.split_partial;
    a.nseg_shared = s.num_shared > 0 ? s.num_shared : 1;
    a.out_fp32 = (y_fp32 ? 1 : 0) | (shared_fp32 ? 2 : 0);
    a.n_tiles = nt_down;
    {
        StageTimer tm(c, st, MOE_STAGE_FFN_DOWN);
        HIP_TRY(c, launch_ffn_gemm(false, a, c->gemm, st));
        if (dsp > 1)
            HIP_TRY(c, launch_split_tail_reduce(s, plan, split_tails, (const float*)(ws + L.split_partial), dsp, y_perm, y_fp32, st));
    }
    return MOE_OK;
}

// Route, permutation indices and (for wide experts) the tiled gather of moe_layer; the pointers
// into the workspace that the rest of the layer uses.
struct LayerFront {
    int32_t *topk_idx, *offsets, *perm, *inv_perm, *row_token;
    float* topk_w;
    const void* x_tiled;   // nullptr: the gather is fused into GEMM 1's loads
    void *h, *y_perm, *y_shared;
    bool y32;              // dtype of y_perm
};

moe_status run_front(moe_ctx* c, const moe_shape& s, const void* x, const void* wg, const float* bias, char* w8,
                     hipStream_t hs, LayerFront* f) {
    const Layout L = make_layout(s);
    f->topk_idx = (int32_t*)(w8 + L.topk_idx);
    f->topk_w = (float*)(w8 + L.topk_w);
    f->offsets = (int32_t*)(w8 + L.offsets);
    f->perm = (int32_t*)(w8 + L.perm);
    f->inv_perm = (int32_t*)(w8 + L.inv_perm);
    f->row_token = (int32_t*)(w8 + L.row_token);
    f->h = w8 + L.h;
    f->y_perm = w8 + L.y_perm;
    f->y_shared = s.num_shared > 0 ? (void*)(w8 + L.y_shared) : nullptr;
    {
        StageTimer tm(c, hs, MOE_STAGE_ROUTE);
        if (moe_status st = run_route(c, s, x, wg, bias, f->topk_idx, f->topk_w, nullptr, w8, hs)) return st;
    }
    {
        StageTimer tm(c, hs, MOE_STAGE_PERMUTE_INDEX);
        HIP_TRY(c, launch_permute_index(s, f->topk_idx, (int32_t*)(w8 + L.chunk_counts), f->offsets, f->perm, f->inv_perm,
                                        f->row_token, hs));
    }
    // The gather is either fused into GEMM 1's loads (row-major x, 64-byte pieces from 16 distant
    // rows per load) or done once into a tiled x_perm (one extra pass over T*k*H*2 bytes, after
    // which GEMM 1 loads whole 1 KiB blocks).  The extra pass pays off when each x row is re-read
    // by many n-tiles, i.e. for wide experts.
    const bool tiled = c->gemm.x_tiled == 1 || (c->gemm.x_tiled < 0 && s.F >= 4096);
    f->x_tiled = nullptr;
    if (tiled) {
        StageTimer tm(c, hs, MOE_STAGE_PERMUTE_GATHER);
        HIP_TRY(c, launch_permute_gather_tiled(s, x, f->row_token, w8 + L.x_tiled, hs));
        f->x_tiled = w8 + L.x_tiled;
    }
    // y_perm in bf16 halves the down projection's stores and the combine's loads.  Its rounding
    // moves out[t] by at most sum_j w_j * 2^-8 * |y_j|.  Chosen when that is small against the
    // output: at least 4 routed terms next to shared experts of weight 1, which then carry most
    // of the output (measured at full size: no change of the error).  Without shared experts the
    // routed terms are the whole output and their rounding would use up most of the error bar
    // whatever their weights: fp32 there (measured on the Mixtral-shaped workloads against the
    // oracle, every token: bf16 y_perm would take 1 % off the step and move the worst element
    // from 1.04e-2 to 1.97e-2 x RMS on the 8x7B shape and to 2.1e-2, past the bar, on the 8x22B shape).
    // y_shared (weight 1) is always fp32.
    f->y32 = c->layer_y >= 0 ? c->layer_y != 0 : !(s.top_k >= 4 && s.num_shared > 0);
    return MOE_OK;
}

// The whole layer with its intermediates in `ws` (validated by the caller).
moe_status layer_with_workspace(moe_ctx* c, const moe_shape* s, const void* x, const void* wg, const float* bias,
                                const void* const* w1p, const void* const* w3p, const void* const* w2p, void* out,
                                char* ws, hipStream_t hs) {
    void** tab = nullptr;
    if (moe_status st = weight_table(c, s->E + s->num_shared, w1p, w3p, w2p, hs, &tab)) return st;
    LayerFront f;
    if (moe_status st = run_front(c, *s, x, wg, bias, ws, hs, &f)) return st;
    if (moe_status st = run_ffn(c, *s, nullptr, f.row_token, x, f.x_tiled, f.offsets, tab, ws, f.h, f.y_perm,
                                f.y_shared, f.y32, true, hs))
        return st;
    {
        StageTimer tm(c, hs, MOE_STAGE_COMBINE);
        HIP_TRY(c, launch_combine(*s, f.y_perm, f.inv_perm, f.topk_w, f.y_shared, out, f.y32, true, c->out_fp32, hs));
    }
    return MOE_OK;
}

}  // namespace

extern "C" {

moe_status moe_create(moe_ctx** out, int device) {
    if (!out) return MOE_E_ARG;
    *out = nullptr;
    if (hipSetDevice(device) != hipSuccess) return MOE_E_HIP;
    moe_ctx* c = new moe_ctx();
    c->device = device;
    c->tab_shadow.assign(3 * MAX_GROUPS, nullptr);
    bool ok = ffn_gemm_init() == hipSuccess;
    ok = ok && hipGetSymbolAddress((void**)&c->static_ws, HIP_SYMBOL(scratch)) == hipSuccess && c->static_ws != nullptr &&
         ((uintptr_t)c->static_ws & 255) == 0;
    ok = ok && hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking) == hipSuccess &&
         hipHostMalloc((void**)&c->h_offsets, (MAX_GROUPS + 1) * sizeof(int32_t), hipHostMallocDefault) == hipSuccess;
    for (int i = 0; i < MAX_SLOTS && ok; ++i)
        ok = hipEventCreateWithFlags(&c->slot_ready[i], hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&c->slot_free[i], hipEventDisableTiming) == hipSuccess;
    for (int i = 0; i < TABLE_SLOTS && ok; ++i) {
        ok = hipMalloc((void**)&c->d_tab[i], 3 * MAX_GROUPS * sizeof(void*)) == hipSuccess &&
             hipHostMalloc((void**)&c->h_tab[i], 3 * MAX_GROUPS * sizeof(void*), hipHostMallocDefault) == hipSuccess &&
             hipEventCreateWithFlags(&c->tab_done[i], hipEventDisableTiming) == hipSuccess;
    }
    if (!ok) { moe_destroy(c); return MOE_E_HIP; }
    *out = c;
    return MOE_OK;
}

void moe_destroy(moe_ctx* c) {
    if (!c) return;
    (void)hipSetDevice(c->device);
    (void)hipDeviceSynchronize();
    for (int i = 0; i < TABLE_SLOTS; ++i) {
        if (c->d_tab[i]) (void)hipFree(c->d_tab[i]);
        if (c->h_tab[i]) (void)hipHostFree(c->h_tab[i]);
        if (c->tab_done[i]) (void)hipEventDestroy(c->tab_done[i]);
    }
    for (int i = 0; i < MAX_SLOTS; ++i) {
        if (c->slot_ready[i]) (void)hipEventDestroy(c->slot_ready[i]);
        if (c->slot_free[i]) (void)hipEventDestroy(c->slot_free[i]);
    }
    if (c->copy_stream) (void)hipStreamDestroy(c->copy_stream);
    if (c->h_offsets) (void)hipHostFree(c->h_offsets);
    for (auto& r : c->recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (auto e : c->pool) (void)hipEventDestroy(e);
    delete c;
}

const char* moe_last_error(const moe_ctx* c) { return c ? c->err : "context is NULL"; }

size_t moe_h_scratch_bytes(const moe_shape* s) {
    moe_status st;
    if (shape_problem(s, &st)) return 0;
    return (size_t)h_rows(*s) * s->F * 2;
}

size_t moe_workspace_bytes(const moe_shape* s) {
    moe_status st;
    if (shape_problem(s, &st)) return 0;
    return make_layout(*s).total;
}

moe_status moe_set_option(moe_ctx* c, const char* key, int32_t v) {
    if (!c || !key) return MOE_E_ARG;
    c->err[0] = 0;
    if (!strcmp(key, "gemm_wave_rows") && (v == 1 || v == 2 || v == 4)) { c->gemm.wave_rows = v; return MOE_OK; }
    if (!strcmp(key, "gemm_waves") && (v == 4 || v == 8)) { c->gemm.waves = v; return MOE_OK; }
    if (!strcmp(key, "gemm_group_m") && v >= 0 && v <= 64) { c->gemm.group_m = v; return MOE_OK; }
    if (!strcmp(key, "xcd_remap") && (v == 0 || v == 1)) { c->gemm.xcd_remap = v; return MOE_OK; }
    if (!strcmp(key, "small_tiles") && (v == 0 || v == 1)) { c->gemm.small_tiles = v; return MOE_OK; }
    if (!strcmp(key, "gemm_tile_rows_up") && (v == 0 || v == 128 || v == 256 || v == 320)) { c->gemm.tile_rows_up = v; return MOE_OK; }
    if (!strcmp(key, "gemm_tile_rows_down") && (v == 0 || v == 128 || v == 256 || v == 320)) { c->gemm.tile_rows_down = v; return MOE_OK; }
    if (!strcmp(key, "x_tiled") && v >= -1 && v <= 1) { c->gemm.x_tiled = v; return MOE_OK; }
    if (!strcmp(key, "down_tail_splits") && v >= 0 && v <= 2) { c->gemm.down_tail_splits = v; return MOE_OK; }
    if (!strcmp(key, "tails_last") && v >= -1 && v <= 1) { c->gemm.tails_last = v; return MOE_OK; }
    if (!strcmp(key, "tall_tiles") && v >= -1 && v <= 2) { c->gemm.tall_tiles = v; return MOE_OK; }
    if (!strcmp(key, "y_fp32") && (v == 0 || v == 1)) { c->y_fp32 = v != 0; return MOE_OK; }
    if (!strcmp(key, "layer_y_fp32") && v >= -1 && v <= 1) { c->layer_y = v; return MOE_OK; }
    if (!strcmp(key, "out_fp32") && (v == 0 || v == 1)) { c->out_fp32 = v != 0; return MOE_OK; }
    if (!strcmp(key, "gate_packed") && (v == 0 || v == 1)) { c->gate_packed = v != 0; return MOE_OK; }
    return fail(c, MOE_E_ARG, "unknown option or value out of range: %s=%d", key, (int)v);
}

moe_status moe_pack_weight(moe_ctx* c, const void* w, int32_t rows, int32_t cols, void* packed, void* stream) {
    if (!c) return MOE_E_ARG;
    c->err[0] = 0;
    if (!w || !packed || w == packed) return fail(c, MOE_E_ARG, "pack: NULL or aliased buffers");
    if (rows < 32 || cols < 32 || rows % 32 || cols % 32) return fail(c, MOE_E_ARG, "pack: rows, cols must be positive multiples of 32");
    if ((int64_t)rows * cols * 2 >= ((int64_t)1 << 32)) return fail(c, MOE_E_UNSUPPORTED, "pack: matrix reaches 4 GiB");
    HIP_TRY(c, hipSetDevice(c->device));
    HIP_TRY(c, launch_pack_weight(w, rows, cols, cols, packed, (hipStream_t)stream));
    return MOE_OK;
}

size_t moe_gate_packed_bytes(const moe_shape* s) {
    moe_status st;
    if (shape_problem(s, &st)) return 0;
    return (size_t)route_gemm_config(*s).ep * s->H * 2;
}

moe_status moe_pack_gate(moe_ctx* c, const moe_shape* s, const void* wg, void* wg_packed, void* stream) {
    if (moe_status st = check_common(c, s)) return st;
    const RouteGemm rg = route_gemm_config(*s);
    if (!wg || !wg_packed || wg == wg_packed) return fail(c, MOE_E_ARG, "pack_gate: NULL or aliased buffers");
    HIP_TRY(c, launch_pack_weight(wg, s->H, s->E, rg.ep, wg_packed, (hipStream_t)stream));
    return MOE_OK;
}

moe_status moe_route(moe_ctx* c, const moe_shape* s, const void* x, const void* wg, const float* bias,
                     int32_t* idx, float* w, float* logits, void* ws, size_t ws_bytes, void* stream) {
    if (moe_status st = check_common(c, s)) return st;
    if (s->T == 0) return MOE_OK;   // an empty batch: nothing to do
    if (!x || !wg || !idx || !w) return fail(c, MOE_E_ARG, "route: NULL pointer");
    if (moe_status st = check_ws(c, s, ws, ws_bytes)) return st;
    hipStream_t hs = (hipStream_t)stream;
    StageTimer tm(c, hs, MOE_STAGE_ROUTE);
    return run_route(c, *s, x, wg, bias, idx, w, logits, (char*)ws, hs);
}

moe_status moe_permute(moe_ctx* c, const moe_shape* s, const void* x, const int32_t* idx, void* x_perm,
                       int32_t* offsets, int32_t* perm, int32_t* inv_perm, int32_t* row_token, void* ws,
                       size_t ws_bytes, void* stream) {
    if (moe_status st = check_common(c, s)) return st;
    if (s->T == 0) {   // an empty batch: every group is empty
        if (!offsets) return fail(c, MOE_E_ARG, "permute: NULL pointer");
        HIP_TRY(c, launch_zero_offsets(s->E, offsets, (hipStream_t)stream));
        return MOE_OK;
    }
    if (!idx || !offsets || !perm || !inv_perm) return fail(c, MOE_E_ARG, "permute: NULL pointer");
    if (x_perm && !x) return fail(c, MOE_E_ARG, "permute: x is NULL but x_perm was requested");
    if (moe_status st = check_ws(c, s, ws, ws_bytes)) return st;
    hipStream_t hs = (hipStream_t)stream;
    const Layout L = make_layout(*s);
    {
        StageTimer tm(c, hs, MOE_STAGE_PERMUTE_INDEX);
        HIP_TRY(c, launch_permute_index(*s, idx, (int32_t*)((char*)ws + L.chunk_counts), offsets, perm, inv_perm,
                                        row_token, hs));
    }
    if (x_perm) {
        StageTimer tm(c, hs, MOE_STAGE_PERMUTE_GATHER);
        HIP_TRY(c, launch_permute_gather(*s, x, perm, x_perm, hs));
    }
    return MOE_OK;
}

moe_status moe_grouped_ffn(moe_ctx* c, const moe_shape* s, const void* x_perm, const int32_t* row_token,
                           const void* x, const int32_t* offsets, const void* const* w1p, const void* const* w3p,
                           const void* const* w2p, void* h, void* y_perm, void* y_shared, void* ws, size_t ws_bytes,
                           void* stream) {
    if (moe_status st = check_common(c, s)) return st;
    if (s->T == 0) return MOE_OK;   // an empty batch: nothing to do
    if (!offsets || !h || !y_perm) return fail(c, MOE_E_ARG, "grouped_ffn: NULL pointer");
    if (!row_token && !x_perm) return fail(c, MOE_E_ARG, "grouped_ffn: need x_perm or row_token");
    if ((row_token || s->num_shared > 0) && !x) return fail(c, MOE_E_ARG, "grouped_ffn: x is NULL");
    if ((s->num_shared > 0) != (y_shared != nullptr)) return fail(c, MOE_E_ARG, "grouped_ffn: y_shared must be given iff num_shared > 0");
    if (moe_status st = check_ws(c, s, ws, ws_bytes)) return st;
    hipStream_t hs = (hipStream_t)stream;
    void** tab = nullptr;
    if (moe_status st = weight_table(c, s->E + s->num_shared, w1p, w3p, w2p, hs, &tab)) return st;
    return run_ffn(c, *s, x_perm, row_token, x, nullptr, offsets, tab, (char*)ws, h, y_perm, y_shared, c->y_fp32,
                   c->y_fp32, hs);
}

moe_status moe_combine(moe_ctx* c, const moe_shape* s, const void* y_perm, const int32_t* inv_perm, const float* w,
                       const void* y_shared, void* out, void* stream) {
    if (moe_status st = check_common(c, s)) return st;
    if (s->T == 0) return MOE_OK;   // an empty batch: nothing to do
    if (!y_perm || !inv_perm || !w || !out) return fail(c, MOE_E_ARG, "combine: NULL pointer");
    hipStream_t hs = (hipStream_t)stream;
    StageTimer tm(c, hs, MOE_STAGE_COMBINE);
    HIP_TRY(c, launch_combine(*s, y_perm, inv_perm, w, y_shared, out, c->y_fp32, c->y_fp32, c->out_fp32, hs));
    return MOE_OK;
}

moe_status moe_layer(moe_ctx* c, const moe_shape* s, const void* x, const void* wg, const float* bias,
                     const void* const* w1p, const void* const* w3p, const void* const* w2p, void* out, void* ws,
                     size_t ws_bytes, void* stream) {
    if (moe_status st = check_common(c, s)) return st;
    if (s->T == 0) return MOE_OK;   // an empty batch: nothing to do
    if (!x || !wg || !out) return fail(c, MOE_E_ARG, "layer: NULL pointer");
    if (moe_status st = check_ws(c, s, ws, ws_bytes)) return st;
    return layer_with_workspace(c, s, x, wg, bias, w1p, w3p, w2p, out, (char*)ws, (hipStream_t)stream);
}

moe_status moe_layer_static(moe_ctx* c, const moe_shape* s, const void* x, const void* wg, const float* bias,
                            const void* const* w1p, const void* const* w3p, const void* const* w2p, void* out,
                            void* stream) {
    if (moe_status st = check_common(c, s)) return st;
    if (s->T == 0) return MOE_OK;   // an empty batch: nothing to do
    if (!x || !wg || !out) return fail(c, MOE_E_ARG, "layer_static: NULL pointer");
    const size_t need = make_layout(*s).total;
    if (need > STATIC_SCRATCH_BYTES)
        return fail(c, MOE_E_WORKSPACE, "layer_static: this shape needs %zu bytes of workspace, the built-in scratch holds %zu; "
                                        "use moe_layer with a caller-owned workspace", need, STATIC_SCRATCH_BYTES);
    // Nothing in the layer relies on the workspace's previous contents: every region is written
    // by the kernel that precedes its first reader, so the last call's leftovers need no clearing.
    return layer_with_workspace(c, s, x, wg, bias, w1p, w3p, w2p, out, c->static_ws, (hipStream_t)stream);
}

moe_status moe_accumulate(moe_ctx* c, void* staging, int32_t capacity, int32_t H, int32_t* filled, const void* x_mb,
                          int32_t rows, void* stream) {
    if (!c) return MOE_E_ARG;
    c->err[0] = 0;
    if (!staging || !filled || !x_mb || rows < 0 || H < 1 || capacity < 0) return fail(c, MOE_E_ARG, "accumulate: bad argument");
    if (*filled < 0 || (int64_t)*filled + rows > capacity)
        return fail(c, MOE_E_ARG, "accumulate: %d rows do not fit (%d of %d filled)", rows, *filled, capacity);
    HIP_TRY(c, hipSetDevice(c->device));
    if (rows > 0)
        HIP_TRY(c, hipMemcpyAsync((char*)staging + (size_t)*filled * H * 2, x_mb, (size_t)rows * H * 2, hipMemcpyDeviceToDevice,
                                  (hipStream_t)stream));
    *filled += rows;
    return MOE_OK;
}

moe_status moe_layer_chunked(moe_ctx* c, const moe_shape* s, const void* x, const void* wg, const float* bias,
                             const void* const* w1p, const void* const* w3p, const void* const* w2p, int32_t max_tokens,
                             void* out, void* ws, size_t ws_bytes, void* stream) {
    if (moe_status st = check_common(c, s)) return st;
    if (s->T == 0) return MOE_OK;   // an empty batch: nothing to do
    if (max_tokens < 1) return fail(c, MOE_E_ARG, "layer_chunked: max_tokens_per_pass must be >= 1");
    if (!x || !out) return fail(c, MOE_E_ARG, "layer_chunked: NULL pointer");
    const size_t out_row = (size_t)s->H * (c->out_fp32 ? 4 : 2);
    for (int t0 = 0; t0 < s->T; t0 += max_tokens) {
        moe_shape part = *s;
        part.T = s->T - t0 < max_tokens ? s->T - t0 : max_tokens;
        if (moe_status st = moe_layer(c, &part, (const char*)x + (size_t)t0 * s->H * 2, wg, bias, w1p, w3p, w2p,
                                      (char*)out + (size_t)t0 * out_row, ws, ws_bytes, stream))
            return st;
    }
    return MOE_OK;
}

moe_status moe_layer_streamed(moe_ctx* c, const moe_shape* s, const void* x, const void* wg, const float* bias,
                              const void* const* hw1, const void* const* hw3, const void* const* hw2, void* slots,
                              size_t slot_bytes, int32_t num_slots, int32_t per_group, void* out, void* ws,
                              size_t ws_bytes, void* stream) {
    if (moe_status st = check_common(c, s)) return st;
    if (s->T == 0) return MOE_OK;   // an empty batch: nothing to do
    if (!x || !wg || !out || !slots || !hw1 || !hw3 || !hw2) return fail(c, MOE_E_ARG, "layer_streamed: NULL pointer");
    if (moe_status st = check_ws(c, s, ws, ws_bytes)) return st;
    const int E = s->E, Ns = s->num_shared;
    const size_t mat_bytes = (size_t)s->H * s->F * 2, expert_bytes = 3 * mat_bytes;
    if (num_slots < 2 || num_slots > MAX_SLOTS) return fail(c, MOE_E_ARG, "layer_streamed: num_slots must be 2..%d", MAX_SLOTS);
    if (per_group < 1 || per_group > E) return fail(c, MOE_E_ARG, "layer_streamed: experts_per_group must be 1..E");
    const int cap = per_group > Ns ? per_group : Ns;
    if (slot_bytes < (size_t)cap * expert_bytes || ((uintptr_t)slots & 255) || (slot_bytes & 255))
        return fail(c, MOE_E_ARG, "layer_streamed: a slot needs %zu bytes (256-byte aligned), got %zu", (size_t)cap * expert_bytes, slot_bytes);
    for (int e = 0; e < E + Ns; ++e)
        if (!hw1[e] || !hw3[e] || !hw2[e]) return fail(c, MOE_E_ARG, "layer_streamed: host weight pointer %d is NULL", e);
    hipStream_t hs = (hipStream_t)stream;
    LayerFront f;
    if (moe_status st = run_front(c, *s, x, wg, bias, (char*)ws, hs, &f)) return st;
    // the per-expert row counts decide what is fetched: one synchronising read-back
    HIP_TRY(c, hipMemcpyAsync(c->h_offsets, f.offsets, (size_t)(E + 1) * sizeof(int32_t), hipMemcpyDeviceToHost, hs));
    HIP_TRY(c, hipStreamSynchronize(hs));
    c->stream_bytes = 0;
    c->stream_groups = 0;
    c->stream_skipped = 0;

    // groups: runs of up to per_group non-empty routed experts (a group spans [lo, hi) and the
    // empty experts inside it are neither copied nor given tiles), then the shared experts
    struct Group { int lo, hi; bool shared; };
    std::vector<Group> groups;
    for (int e = 0; e < E;) {
        while (e < E && c->h_offsets[e + 1] == c->h_offsets[e]) { ++e; ++c->stream_skipped; }
        if (e >= E) break;
        int lo = e, n = 0;
        while (e < E && n < per_group) {
            if (c->h_offsets[e + 1] > c->h_offsets[e]) ++n;
            else ++c->stream_skipped;
            ++e;
        }
        groups.push_back({lo, e, false});
    }
    if (Ns > 0) groups.push_back({E, E, true});

    std::vector<const void*> t1(E + Ns), t3(E + Ns), t2(E + Ns);
    for (size_t g = 0; g < groups.size(); ++g) {
        const Group& G = groups[g];
        const int slot = (int)(g % (size_t)num_slots);
        char* base = (char*)slots + (size_t)slot * slot_bytes;
        if (g >= (size_t)num_slots) HIP_TRY(c, hipStreamWaitEvent(c->copy_stream, c->slot_free[slot], 0));
        // every table entry must be a valid pointer; experts outside the group get no tiles
        for (int e = 0; e < E + Ns; ++e) { t1[e] = base; t3[e] = base; t2[e] = base; }
        int member = 0, mt = 0;
        const int e0 = G.shared ? E : G.lo, e1 = G.shared ? E + Ns : G.hi;
        for (int e = e0; e < e1; ++e) {
            const int rows = e < E ? c->h_offsets[e + 1] - c->h_offsets[e] : s->T;
            if (rows == 0) continue;
            char* dst = base + (size_t)member * expert_bytes;
            HIP_TRY(c, hipMemcpyAsync(dst, hw1[e], mat_bytes, hipMemcpyHostToDevice, c->copy_stream));
            HIP_TRY(c, hipMemcpyAsync(dst + mat_bytes, hw3[e], mat_bytes, hipMemcpyHostToDevice, c->copy_stream));
            HIP_TRY(c, hipMemcpyAsync(dst + 2 * mat_bytes, hw2[e], mat_bytes, hipMemcpyHostToDevice, c->copy_stream));
            t1[e] = dst; t3[e] = dst + mat_bytes; t2[e] = dst + 2 * mat_bytes;
            c->stream_bytes += expert_bytes;
            mt += (rows + 127) / 128;
            ++member;
        }
        HIP_TRY(c, hipEventRecord(c->slot_ready[slot], c->copy_stream));
        HIP_TRY(c, hipStreamWaitEvent(hs, c->slot_ready[slot], 0));
        void** tab = nullptr;
        if (moe_status st = weight_table(c, E + Ns, t1.data(), t3.data(), t2.data(), hs, &tab)) return st;
        const FfnPass pass{G.shared ? 0 : G.lo, G.shared ? 0 : G.hi, G.shared, mt, G.shared ? (s->T + 127) / 128 : mt};
        if (moe_status st = run_ffn(c, *s, nullptr, f.row_token, x, f.x_tiled, f.offsets, tab, (char*)ws, f.h, f.y_perm,
                                    f.y_shared, f.y32, true, hs, &pass))
            return st;
        HIP_TRY(c, hipEventRecord(c->slot_free[slot], hs));
        ++c->stream_groups;
    }
    {
        StageTimer tm(c, hs, MOE_STAGE_COMBINE);
        HIP_TRY(c, launch_combine(*s, f.y_perm, f.inv_perm, f.topk_w, f.y_shared, out, f.y32, true, c->out_fp32, hs));
    }
    return MOE_OK;
}

double moe_estimate_streamed_ms(const moe_shape* s, const int32_t* rows, int32_t per_group, int32_t num_slots,
                                double link_gbs, double ffn_tflops) {
    moe_status st;
    if (shape_problem(s, &st) || !rows || per_group < 1 || num_slots < 2 || num_slots > MAX_SLOTS || !(link_gbs > 0) ||
        !(ffn_tflops > 0))
        return -1.0;
    const double expert_ms = 3.0 * s->H * s->F * 2 / (link_gbs * 1e9) * 1e3;
    const double row_ms = 6.0 * s->H * s->F / (ffn_tflops * 1e12) * 1e3;
    // job costs per group, formed exactly as moe_layer_streamed forms them
    std::vector<double> copy_ms, comp_ms;
    for (int e = 0; e < s->E;) {
        while (e < s->E && rows[e] <= 0) ++e;
        if (e >= s->E) break;
        int n = 0;
        double r = 0;
        while (e < s->E && n < per_group) {
            if (rows[e] > 0) { ++n; r += rows[e]; }
            ++e;
        }
        copy_ms.push_back(n * expert_ms);
        comp_ms.push_back(r * row_ms);
    }
    if (s->num_shared > 0) {
        copy_ms.push_back(s->num_shared * expert_ms);
        comp_ms.push_back((double)s->num_shared * s->T * row_ms);
    }
    // longest path: nodes in topological order copy(0), compute(0), copy(1), compute(1), ...
    const size_t G = copy_ms.size();
    std::vector<double> f_copy(G, 0.0), f_comp(G, 0.0);
    for (size_t g = 0; g < G; ++g) {
        double ready = g > 0 ? f_copy[g - 1] : 0.0;
        if (g >= (size_t)num_slots && f_comp[g - num_slots] > ready) ready = f_comp[g - num_slots];
        f_copy[g] = ready + copy_ms[g];
        double start = f_copy[g];
        if (g > 0 && f_comp[g - 1] > start) start = f_comp[g - 1];
        f_comp[g] = start + comp_ms[g];
    }
    return G ? f_comp[G - 1] : 0.0;
}

moe_status moe_stream_stats(const moe_ctx* c, uint64_t* bytes, int32_t* groups, int32_t* skipped) {
    if (!c) return MOE_E_ARG;
    if (bytes) *bytes = c->stream_bytes;
    if (groups) *groups = c->stream_groups;
    if (skipped) *skipped = c->stream_skipped;
    return MOE_OK;
}

moe_status moe_layer_views(const moe_shape* s, void* ws, int32_t** idx, float** w, int32_t** offsets,
                           int32_t** inv_perm) {
    moe_status st;
    if (shape_problem(s, &st)) return st;
    if (!ws) return MOE_E_ARG;
    const Layout L = make_layout(*s);
    char* w8 = (char*)ws;
    if (idx) *idx = (int32_t*)(w8 + L.topk_idx);
    if (w) *w = (float*)(w8 + L.topk_w);
    if (offsets) *offsets = (int32_t*)(w8 + L.offsets);
    if (inv_perm) *inv_perm = (int32_t*)(w8 + L.inv_perm);
    return MOE_OK;
}

moe_status moe_profile_enable(moe_ctx* c, int32_t on) {
    if (!c) return MOE_E_ARG;
    c->prof = on != 0;
    return MOE_OK;
}

moe_status moe_profile_read_intervals(moe_ctx* c, int32_t* stage, float* ms, int32_t capacity, int32_t* count) {
    if (!c || !stage || !ms || !count || capacity < 0) return MOE_E_ARG;
    c->err[0] = 0;
    int n = 0;
    for (auto& r : c->recs) {
        HIP_TRY(c, hipEventSynchronize(r.b));
        float v = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&v, r.a, r.b));
        if (n < capacity) { stage[n] = r.stage; ms[n] = v; ++n; }
        c->pool.push_back(r.a);
        c->pool.push_back(r.b);
    }
    c->recs.clear();
    *count = n;
    return MOE_OK;
}

moe_status moe_profile_mfma_ceiling(moe_ctx* c, const void* a, const void* b, size_t bytes, int32_t iters, void* sink,
                                    size_t sink_bytes, double* tflops, double* ms_out, void* stream) {
    if (!c) return MOE_E_ARG;
    c->err[0] = 0;
    if (!sink || !tflops || iters < 1 || iters > (1 << 22)) return fail(c, MOE_E_ARG, "mfma_ceiling: bad argument");
    if ((a || b) && (bytes < 16 || bytes >= ((size_t)1 << 35))) return fail(c, MOE_E_ARG, "mfma_ceiling: operand buffers need 16 bytes .. 32 GiB");
    if (((uintptr_t)a | (uintptr_t)b) & 15) return fail(c, MOE_E_ARG, "mfma_ceiling: operand buffers must be 16-byte aligned");
    if (sink_bytes < (size_t)CEILING_BLOCKS * 256 * sizeof(float)) return fail(c, MOE_E_WORKSPACE, "mfma_ceiling: sink needs %zu bytes", (size_t)CEILING_BLOCKS * 256 * sizeof(float));
    HIP_TRY(c, hipSetDevice(c->device));
    hipStream_t hs = (hipStream_t)stream;
    hipEvent_t e0 = get_event(c), e1 = get_event(c);
    if (!e0 || !e1) return fail(c, MOE_E_HIP, "mfma_ceiling: no event");
    HIP_TRY(c, hipEventRecord(e0, hs));
    HIP_TRY(c, launch_mfma_ceiling(a, b, bytes, CEILING_BLOCKS, iters, (float*)sink, hs));
    HIP_TRY(c, hipEventRecord(e1, hs));
    HIP_TRY(c, hipEventSynchronize(e1));
    float ms = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&ms, e0, e1));
    c->pool.push_back(e0);
    c->pool.push_back(e1);
    *tflops = mfma_ceiling_flops(CEILING_BLOCKS, iters) / ((double)ms * 1e-3) / 1e12;
    if (ms_out) *ms_out = ms;
    return MOE_OK;
}

moe_status moe_profile_read(moe_ctx* c, double* ms_sum, int32_t* launches) {
    if (!c || !ms_sum || !launches) return MOE_E_ARG;
    c->err[0] = 0;
    for (int i = 0; i < MOE_STAGE_COUNT; ++i) { ms_sum[i] = 0.0; launches[i] = 0; }
    for (auto& r : c->recs) {
        HIP_TRY(c, hipEventSynchronize(r.b));
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, r.a, r.b));
        ms_sum[r.stage] += ms;
        launches[r.stage] += 1;
        c->pool.push_back(r.a);
        c->pool.push_back(r.b);
    }
    c->recs.clear();
    return MOE_OK;
}

}  // extern "C"
