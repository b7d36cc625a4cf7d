/*
 * CPU oracle for the MoE expert module (router -> top-k experts -> weighted sum, plus
 * always-on shared experts), the sparse MoE layer of the paper's Sec. 2 "MoE inference".
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition written out per token; it
 * is what the HIP library is checked against.  It shares no code with the HIP path and
 * nothing in the product path may call it.
 *
 * Precision: every stored value and every element-wise operation is fp32; inputs are bf16
 * bit patterns widened exactly; every dot product is accumulated in fp64 and rounded to
 * fp32 once.  There is no intermediate bf16 rounding anywhere.
 *
 * Module-based batching (Sec. 4.2) changes how many tokens are processed at once, never the
 * per-token result, so the oracle needs no permutation to compute the layer output: each
 * token is handled on its own.  oracle_permute is the separate plain definition (a stable
 * counting sort) of the per-expert grouping the GPU path materialises.
 *
 * Parity pins: see tests/test_oracle_pins.py (brute force, closed forms, dense SwiGLU per
 * expert against an independent library routine, two hand-computed examples, fp32 and bf16
 * inputs of the combine against a float64 sum).  tests/test_oracle_mutations.py plants single
 * mistakes into scratch copies of this file and requires those pins to fail on each.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline float bf16_to_f32(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* ---------------------------------------------------------------------------------------
 * Router (Sec. 2 "MoE inference": every token is sent to its k best-scoring experts).
 * Reading: linear gate with optional additive bias, softmax
 * over ALL E experts in fp32, top-k chosen on the logits (ties -> lower expert index),
 * selected list in descending logit order; weights are the softmax probabilities of the
 * selected experts, divided by their sum when `renormalize`, then times routed_scale.
 *
 * x      [T,H] bf16 bits, row-major        wg    [H,E] bf16 bits, row-major
 * bias   [E] fp32 or NULL                  tokens[ntok] token ids to evaluate (NULL: 0..ntok-1)
 * idx    [ntok,k] int32 out                w     [ntok,k] fp32 out
 * logits [ntok,E] fp32 out or NULL         probs [ntok,E] fp32 out or NULL
 * ------------------------------------------------------------------------------------- */
void oracle_route(const uint16_t* x, const uint16_t* wg, const float* bias,
                  int T, int H, int E, int k, int renormalize, float routed_scale,
                  const int32_t* tokens, int ntok,
                  int32_t* idx, float* w, float* logits, float* probs)
{
    (void)T;
#pragma omp parallel
    {
        double* acc = (double*)malloc(sizeof(double) * (size_t)E);
        float* lg = (float*)malloc(sizeof(float) * (size_t)E);
        float* p = (float*)malloc(sizeof(float) * (size_t)E);
        char* taken = (char*)malloc((size_t)E);
#pragma omp for schedule(dynamic, 8)
        for (int n = 0; n < ntok; ++n) {
            const int t = tokens ? tokens[n] : n;
            const uint16_t* xr = x + (size_t)t * H;
            for (int e = 0; e < E; ++e) acc[e] = bias ? (double)bias[e] : 0.0;
            for (int h = 0; h < H; ++h) {
                const double xv = (double)bf16_to_f32(xr[h]);
                const uint16_t* wr = wg + (size_t)h * E;
                for (int e = 0; e < E; ++e) acc[e] += xv * (double)bf16_to_f32(wr[e]);
            }
            float m = -INFINITY;
            for (int e = 0; e < E; ++e) { lg[e] = (float)acc[e]; if (lg[e] > m) m = lg[e]; }
            double Z = 0.0;
            for (int e = 0; e < E; ++e) { p[e] = expf(lg[e] - m); Z += (double)p[e]; }
            for (int e = 0; e < E; ++e) p[e] = (float)((double)p[e] / Z);
            memset(taken, 0, (size_t)E);
            double wsum = 0.0;
            for (int j = 0; j < k; ++j) {
                int best = -1;
                for (int e = 0; e < E; ++e)
                    if (!taken[e] && (best < 0 || lg[e] > lg[best])) best = e;
                taken[best] = 1;
                idx[(size_t)n * k + j] = best;
                w[(size_t)n * k + j] = p[best];
                wsum += (double)p[best];
            }
            for (int j = 0; j < k; ++j) {
                float v = w[(size_t)n * k + j];
                if (renormalize) v = (float)((double)v / wsum);
                w[(size_t)n * k + j] = v * routed_scale;
            }
            if (logits) memcpy(logits + (size_t)n * E, lg, sizeof(float) * (size_t)E);
            if (probs) memcpy(probs + (size_t)n * E, p, sizeof(float) * (size_t)E);
        }
        free(acc); free(lg); free(p); free(taken);
    }
}

/* ---------------------------------------------------------------------------------------
 * Per-expert grouping of the T*k (token, rank) pairs (Table 1 measures the expert module by
 * the number of tokens each expert receives; the counts are only known at run time, Sec. 4.3).
 * Canonical order: ascending expert id, inside an expert ascending token id (a token never
 * picks an expert twice).  Stable counting sort:
 *   offsets[e]      first row of expert e, offsets[E] = T*k
 *   perm[r]         = t*k + j of the pair placed at row r
 *   inv_perm[t*k+j] = r
 * ------------------------------------------------------------------------------------- */
void oracle_permute(const int32_t* idx, int T, int k, int E,
                    int32_t* offsets, int32_t* perm, int32_t* inv_perm)
{
    int64_t* cursor = (int64_t*)calloc((size_t)E + 1, sizeof(int64_t));
    for (int64_t i = 0; i < (int64_t)T * k; ++i) cursor[idx[i] + 1]++;
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) { cursor[e + 1] += cursor[e]; offsets[e + 1] = (int32_t)cursor[e + 1]; }
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) {
            const int e = idx[(size_t)t * k + j];
            const int32_t r = (int32_t)cursor[e]++;
            perm[r] = t * k + j;
            inv_perm[(size_t)t * k + j] = r;
        }
    free(cursor);
}

/* One token through one SwiGLU expert: y = (silu(x W1) * (x W3)) W2, silu(z) = z/(1+e^-z).
 * W1, W3: [H,F] bf16 bits row-major; W2: [F,H].  xr: H bf16 bits.  y: H fp32.
 * scratch: 2*F + H doubles, F floats (caller-provided). */
static void expert_row(const uint16_t* xr, const uint16_t* w1, const uint16_t* w3, const uint16_t* w2,
                       int H, int F, double* g, double* u, double* y64, float* a, float* y)
{
    for (int f = 0; f < F; ++f) { g[f] = 0.0; u[f] = 0.0; }
    for (int h = 0; h < H; ++h) {
        const double xv = (double)bf16_to_f32(xr[h]);
        const uint16_t* r1 = w1 + (size_t)h * F;
        const uint16_t* r3 = w3 + (size_t)h * F;
        for (int f = 0; f < F; ++f) {
            g[f] += xv * (double)bf16_to_f32(r1[f]);
            u[f] += xv * (double)bf16_to_f32(r3[f]);
        }
    }
    for (int f = 0; f < F; ++f) {
        const float gf = (float)g[f], uf = (float)u[f];
        a[f] = (gf / (1.0f + expf(-gf))) * uf;
    }
    for (int h = 0; h < H; ++h) y64[h] = 0.0;
    for (int f = 0; f < F; ++f) {
        const double av = (double)a[f];
        const uint16_t* r2 = w2 + (size_t)f * H;
        for (int h = 0; h < H; ++h) y64[h] += av * (double)bf16_to_f32(r2[h]);
    }
    for (int h = 0; h < H; ++h) y[h] = (float)y64[h];
}

/* Rows through given experts: y[n,:] = expert_{eid[n]}(xrows[n,:]).  Used to check the
 * grouped FFN stage on its own.  xrows [n,H] bf16 bits; w1/w3/w2: arrays of per-expert
 * pointers; y [n,H] fp32. */
void oracle_expert_rows(const uint16_t* xrows, const int32_t* eid, int nrows,
                        const uint16_t* const* w1, const uint16_t* const* w3, const uint16_t* const* w2,
                        int H, int F, float* y)
{
#pragma omp parallel
    {
        double* g = (double*)malloc(sizeof(double) * (size_t)(2 * F + H));
        float* a = (float*)malloc(sizeof(float) * (size_t)F);
#pragma omp for schedule(dynamic, 1)
        for (int n = 0; n < nrows; ++n) {
            const int e = eid[n];
            expert_row(xrows + (size_t)n * H, w1[e], w3[e], w2[e], H, F, g, g + F, g + 2 * F, a,
                       y + (size_t)n * H);
        }
        free(g); free(a);
    }
}

/* ---------------------------------------------------------------------------------------
 * Whole layer for a list of tokens (Sec. 2): out[t] = sum_j w[t,j] * expert_{idx[t,j]}(x[t])
 * + sum_s shared_s(x[t]).  idx/w [ntok,k] are inputs (from oracle_route, or the routing
 * under test when a near-tie was excused).  Shared experts are w1[E+s] etc., weight 1, not
 * scaled.  The routed sum is taken in rank order j = 0..k-1 in fp32; shared outputs are
 * added afterwards in order s = 0..Ns-1.  out [ntok,H] fp32.
 * ------------------------------------------------------------------------------------- */
void oracle_layer(const uint16_t* x, const int32_t* tokens, int ntok,
                  const int32_t* idx, const float* w,
                  const uint16_t* const* w1, const uint16_t* const* w3, const uint16_t* const* w2,
                  int H, int F, int E, int k, int num_shared, float* out)
{
#pragma omp parallel
    {
        double* g = (double*)malloc(sizeof(double) * (size_t)(2 * F + H));
        float* a = (float*)malloc(sizeof(float) * (size_t)F);
        float* y = (float*)malloc(sizeof(float) * (size_t)H);
#pragma omp for schedule(dynamic, 1)
        for (int n = 0; n < ntok; ++n) {
            const int t = tokens ? tokens[n] : n;
            const uint16_t* xr = x + (size_t)t * H;
            float* o = out + (size_t)n * H;
            for (int h = 0; h < H; ++h) o[h] = 0.0f;
            for (int j = 0; j < k; ++j) {
                const int e = idx[(size_t)n * k + j];
                const float wj = w[(size_t)n * k + j];
                expert_row(xr, w1[e], w3[e], w2[e], H, F, g, g + F, g + 2 * F, a, y);
                for (int h = 0; h < H; ++h) o[h] += wj * y[h];
            }
            for (int s = 0; s < num_shared; ++s) {
                expert_row(xr, w1[E + s], w3[E + s], w2[E + s], H, F, g, g + F, g + 2 * F, a, y);
                for (int h = 0; h < H; ++h) o[h] += y[h];
            }
        }
        free(g); free(a); free(y);
    }
}

/* Weighted combine on its own (Sec. 2: the layer output is the weighted sum of the selected
 * experts' outputs): out[t,:] = sum_j w[t,j] * y_perm[inv_perm[t*k+j],:] (+ y_shared[t,:]).
 * y_perm [R,H] and y_shared [T,H] are the stage's inputs, fp32 when y_is_f32 else bf16 bits;
 * products and sums in fp32 in rank order, shared added last.  out [T,H] fp32. */
static inline float y_at(const void* y, int y_is_f32, size_t i)
{
    return y_is_f32 ? ((const float*)y)[i] : bf16_to_f32(((const uint16_t*)y)[i]);
}

void oracle_combine(const void* y_perm, int y_is_f32, const int32_t* inv_perm, const float* w,
                    const void* y_shared, int T, int H, int k, float* out)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        float* o = out + (size_t)t * H;
        for (int h = 0; h < H; ++h) o[h] = 0.0f;
        for (int j = 0; j < k; ++j) {
            const size_t r = (size_t)inv_perm[(size_t)t * k + j];
            const float wj = w[(size_t)t * k + j];
            for (int h = 0; h < H; ++h) o[h] += wj * y_at(y_perm, y_is_f32, r * H + h);
        }
        if (y_shared)
            for (int h = 0; h < H; ++h) o[h] += y_at(y_shared, y_is_f32, (size_t)t * H + h);
    }
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
