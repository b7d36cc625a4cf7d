/* A plain C caller of the library: shows that the boundary is a C ABI (no C++ types, no
 * Python) and checks, without any reference implementation, properties that must hold
 * bit for bit: moe_layer equals the staged calls; every token appears top_k times in the
 * permutation; the routing weights sum to 1 under renormalisation; zero input gives zero
 * output.  Built by paper_2503_09716_amd/build.py with gcc; run by tests/test_gpu_c_abi.py. */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "moe.h"

#define CHECK_HIP(e) do { hipError_t e_ = (e); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define CHECK_MOE(e) do { moe_status s_ = (e); if (s_ != MOE_OK) { printf("moe status %d at line %d: %s\n", (int)s_, __LINE__, moe_last_error(ctx)); return 3; } } while (0)

static uint32_t rng_state = 12345u;
static uint32_t rng(void) { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }
/* bf16 bits of a small pseudo-random value: sign, exponent of 2^-3..2^0 scaled, 7 mantissa bits */
static uint16_t small_bf16(float scale_pow2) {
    uint32_t r = rng();
    uint32_t sign = (r & 1u) << 15, mant = (r >> 1) & 0x7fu, e = 124u + ((r >> 8) & 3u);   /* 2^-3 .. 2^0 */
    e = (uint32_t)((int)e + (int)scale_pow2);
    return (uint16_t)(sign | (e << 7) | mant);
}

int main(void) {
    enum { T = 300, H = 128, F = 192, E = 6, K = 2, NS = 1, R = T * K };
    moe_shape s = {T, H, F, E, K, NS, 1, 1.0f};
    moe_ctx* ctx = NULL;
    if (moe_create(&ctx, 0) != MOE_OK) { printf("moe_create failed\n"); return 1; }
    const size_t ws_bytes = moe_workspace_bytes(&s), h_bytes = moe_h_scratch_bytes(&s);
    if (!ws_bytes || !h_bytes) { printf("shape refused\n"); return 1; }

    /* host data */
    uint16_t* hx = malloc((size_t)T * H * 2); uint16_t* hwg = malloc((size_t)H * E * 2);
    uint16_t* hw = malloc((size_t)H * F * 2);
    for (int i = 0; i < T * H; ++i) hx[i] = small_bf16(2);
    for (int i = 0; i < H * E; ++i) hwg[i] = small_bf16(-2);

    void *x, *wg, *ws, *ws2, *hscr, *out, *out2, *logical, *xperm, *y, *ysh;
    int32_t *idx, *off, *perm, *inv;
    float* w;
    CHECK_HIP(hipMalloc(&x, (size_t)T * H * 2)); CHECK_HIP(hipMalloc(&wg, (size_t)H * E * 2));
    CHECK_HIP(hipMalloc(&ws, ws_bytes)); CHECK_HIP(hipMalloc(&ws2, ws_bytes)); CHECK_HIP(hipMalloc(&hscr, h_bytes));
    CHECK_HIP(hipMalloc(&out, (size_t)T * H * 2)); CHECK_HIP(hipMalloc(&out2, (size_t)T * H * 2));
    CHECK_HIP(hipMalloc(&logical, (size_t)H * F * 2)); CHECK_HIP(hipMalloc(&xperm, (size_t)R * H * 2));
    CHECK_HIP(hipMalloc(&y, (size_t)R * H * 4)); CHECK_HIP(hipMalloc(&ysh, (size_t)T * H * 4));
    CHECK_HIP(hipMalloc((void**)&idx, (size_t)R * 4)); CHECK_HIP(hipMalloc((void**)&w, (size_t)R * 4));
    CHECK_HIP(hipMalloc((void**)&off, (E + 1) * 4)); CHECK_HIP(hipMalloc((void**)&perm, (size_t)R * 4));
    CHECK_HIP(hipMalloc((void**)&inv, (size_t)R * 4));
    CHECK_HIP(hipMemcpy(x, hx, (size_t)T * H * 2, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(wg, hwg, (size_t)H * E * 2, hipMemcpyHostToDevice));

    /* expert weights: logical [H,F] / [F,H] -> packed */
    const void *w1p[E + NS], *w3p[E + NS], *w2p[E + NS];
    for (int e = 0; e < E + NS; ++e)
        for (int m = 0; m < 3; ++m) {
            void* packed;
            for (int i = 0; i < H * F; ++i) hw[i] = small_bf16(-3);
            CHECK_HIP(hipMalloc(&packed, (size_t)H * F * 2));
            CHECK_HIP(hipMemcpy(logical, hw, (size_t)H * F * 2, hipMemcpyHostToDevice));
            CHECK_MOE(moe_pack_weight(ctx, logical, m < 2 ? H : F, m < 2 ? F : H, packed, NULL));
            CHECK_HIP(hipDeviceSynchronize());
            if (m == 0) w1p[e] = packed; else if (m == 1) w3p[e] = packed; else w2p[e] = packed;
        }

    /* fused */
    CHECK_MOE(moe_layer(ctx, &s, x, wg, NULL, w1p, w3p, w2p, out, ws, ws_bytes, NULL));
    /* staged */
    CHECK_MOE(moe_route(ctx, &s, x, wg, NULL, idx, w, NULL, ws2, ws_bytes, NULL));
    CHECK_MOE(moe_permute(ctx, &s, x, idx, xperm, off, perm, inv, NULL, ws2, ws_bytes, NULL));
    CHECK_MOE(moe_grouped_ffn(ctx, &s, xperm, NULL, x, off, w1p, w3p, w2p, hscr, y, ysh, ws2, ws_bytes, NULL));
    CHECK_MOE(moe_combine(ctx, &s, y, inv, w, ysh, out2, NULL));
    CHECK_HIP(hipDeviceSynchronize());

    uint16_t* o1 = malloc((size_t)T * H * 2); uint16_t* o2 = malloc((size_t)T * H * 2);
    int32_t* hperm = malloc((size_t)R * 4); int32_t* hoff = malloc((E + 1) * 4); float* hwt = malloc((size_t)R * 4);
    CHECK_HIP(hipMemcpy(o1, out, (size_t)T * H * 2, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(o2, out2, (size_t)T * H * 2, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hperm, perm, (size_t)R * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hoff, off, (E + 1) * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hwt, w, (size_t)R * 4, hipMemcpyDeviceToHost));
    int bad = 0, nonzero = 0;
    if (memcmp(o1, o2, (size_t)T * H * 2) != 0) { printf("FAIL: fused and staged outputs differ\n"); bad = 1; }
    for (int i = 0; i < T * H; ++i) nonzero += (o1[i] & 0x7fff) != 0;
    if (nonzero < T * H / 2) { printf("FAIL: output mostly zero (%d of %d)\n", nonzero, T * H); bad = 1; }
    int* seen = calloc(T, sizeof(int));
    for (int r = 0; r < R; ++r) {
        if (hperm[r] < 0 || hperm[r] >= R) { printf("FAIL: perm out of range\n"); bad = 1; break; }
        seen[hperm[r] / K]++;
    }
    for (int t = 0; t < T; ++t) if (seen[t] != K) { printf("FAIL: token %d appears %d times\n", t, seen[t]); bad = 1; break; }
    if (hoff[0] != 0 || hoff[E] != R) { printf("FAIL: expert_offsets ends %d %d\n", hoff[0], hoff[E]); bad = 1; }
    for (int t = 0; t < T; ++t) {
        float sum = 0; for (int j = 0; j < K; ++j) sum += hwt[t * K + j];
        if (sum < 0.99999f || sum > 1.00001f) { printf("FAIL: weights of token %d sum to %g\n", t, sum); bad = 1; break; }
    }
    /* zero input -> zero output */
    CHECK_HIP(hipMemset(x, 0, (size_t)T * H * 2));
    CHECK_MOE(moe_layer(ctx, &s, x, wg, NULL, w1p, w3p, w2p, out, ws, ws_bytes, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(o1, out, (size_t)T * H * 2, hipMemcpyDeviceToHost));
    for (int i = 0; i < T * H; ++i) if (o1[i] & 0x7fff) { printf("FAIL: zero input gave non-zero output\n"); bad = 1; break; }
    /* error path: a workspace that is too small is refused before anything runs */
    if (moe_layer(ctx, &s, x, wg, NULL, w1p, w3p, w2p, out, ws, 256, NULL) != MOE_E_WORKSPACE) { printf("FAIL: small workspace accepted\n"); bad = 1; }
    moe_destroy(ctx);
    printf(bad ? "C ABI check FAILED\n" : "C ABI check passed\n");
    return bad;
}
