/*
 * CPU oracle for one Mixture-of-Experts layer — TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, per-definition implementation used to check the HIP library and to time
 * a host-core baseline. It shares no code, header, table or helper with the HIP path, and
 * nothing in the product path may call it (only tests, the smoke check and the bench's
 * cpu_baseline leg do).
 *
 * What it computes (all pointers are HOST pointers; bf16 values travel as raw uint16 bits):
 *
 *   y[t] = sum_{e in topk(t)} g[t,e] * Expert_e(x[t]),
 *   Expert_e(x) = W2_e ( SiLU(W1_e x) (.) W3_e x ),   SiLU(a) = a / (1 + exp(-a)).
 *
 * Paper passages followed: top-k routing over N experts with uneven per-expert load
 * (Section 2.1); the expert stage OP_3 is a gated FFN per expert with three d_h x d_e bf16
 * matrices and 6*rows*d_h*d_e FLOPs (Section 4.1, Table 1 row 3); coalesced execution runs
 * the expert stage once over the whole batch, m_exp = B (Section 4.1.1, Eq. 7-9), while the
 * prior strategy runs micro-batches one after the other through the same weights
 * (Section 2.3, Section 3.1). The paper never prints the layer's equation; the SwiGLU form,
 * "softmax over the selected k logits" and fp32 gates are the benchmark's statement of it.
 *
 * Precision: floating point in double unless stated. Two places are fp32 on purpose because
 * an integer decision hangs on them and both sides must take it in the same precision:
 *   - router logits are the canonical fp32 value defined at moe_ref_logits (fixed
 *     fused-multiply-add order and a fixed 64-leaf butterfly), and top-k compares those;
 *   - gates are rounded to fp32 after being computed in double.
 * No blocking, fusion or reordering beyond the definitions (the order of a double dot
 * product is left to the compiler's SIMD reduction; it does not matter at 2^-53).
 *
 * Parity pins live in tests/test_oracle_pins.py. Unpinned by the paper: *which* fp32
 * summation tree the router logits use (the paper is silent; the tree below is this
 * repository's reading, pinned only by hand-derived order-sensitive cases).
 *
 * Build: gcc -O3 -march=x86-64-v3 -ffp-contract=off -fopenmp -shared -fPIC (oracle/build.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_OK 0
#define REF_ERR_ARG (-1)
#define REF_MAX_E 1024

static inline float bf16_val(uint16_t bits) {
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

int moe_ref_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void moe_ref_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---------------------------------------------------------------------------------------
 * Router logits, canonical fp32 (Section 2.1 routing function; logits = x . W_r (+ bias)).
 *
 * The paper does not say in which order the d products are summed, and a 1-ulp change can
 * flip a near-tie in top-k, so the order is part of this repository's definition:
 * 64 partial sums p[0..63]; element i = 512*j + 8*l + v (j chunk, l in [0,64), v in [0,8))
 * belongs to p[l]; p[l] starts at +0.0f and takes p[l] = fma(x_i, w_i, p[l]) for j
 * ascending, then v ascending. The 64 partials are combined by a butterfly:
 * for s = 32,16,8,4,2,1: p[l] <- p[l] + p[l xor s] (all l at once). The logit is p[0]
 * (every p[l] is then equal); the optional bias is added last, in fp32.
 * d must be a multiple of 512.  One row t -> logits_row[E].
 * ------------------------------------------------------------------------------------- */
static void logits_row(const uint16_t* xrow, const float* wr, const float* bias, int d, int E,
                       float* out) {
    for (int e = 0; e < E; ++e) {
        float p[64], q[64];
        for (int l = 0; l < 64; ++l) p[l] = 0.0f;
        for (int j = 0; j < d / 512; ++j)
            for (int l = 0; l < 64; ++l)
                for (int v = 0; v < 8; ++v) {
                    int i = 512 * j + 8 * l + v;
                    p[l] = fmaf(bf16_val(xrow[i]), wr[(size_t)i * E + e], p[l]);
                }
        for (int s = 32; s >= 1; s >>= 1) {
            for (int l = 0; l < 64; ++l) q[l] = p[l] + p[l ^ s];
            memcpy(p, q, sizeof p);
        }
        out[e] = bias ? p[0] + bias[e] : p[0];
    }
}

int moe_ref_logits(const uint16_t* x, const float* w_router, const float* bias, int T, int d,
                   int E, float* logits) {
    if (T < 0 || d <= 0 || d % 512 != 0 || E <= 0) return REF_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        logits_row(x + (size_t)t * d, w_router, bias, d, E, logits + (size_t)t * E);
    return REF_OK;
}

/* The same logits in double, plain ascending-i sum: a diagnostic to bound the fp32 value. */
int moe_ref_logits_f64(const uint16_t* x, const float* w_router, const float* bias, int T, int d,
                       int E, double* logits) {
    if (T < 0 || d <= 0 || E <= 0) return REF_ERR_ARG;
    for (int t = 0; t < T; ++t)
        for (int e = 0; e < E; ++e) {
            double s = 0.0;
            for (int i = 0; i < d; ++i)
                s += (double)bf16_val(x[(size_t)t * d + i]) * (double)w_router[(size_t)i * E + e];
            logits[(size_t)t * E + e] = s + (bias ? (double)bias[e] : 0.0);
        }
    return REF_OK;
}

/* ---------------------------------------------------------------------------------------
 * Top-k selection and gates (Section 2.1: each token goes to the top-k of N experts).
 * Slot s holds the expert with the (s+1)-th largest logit; equal logits go to the lower
 * expert index (-0.0 and +0.0 compare equal); a NaN logit ranks below every number.
 * Gates are the softmax over the k selected logits (identical to a softmax over all E
 * followed by renormalisation over the selected ones):
 *   g[s] = exp(l_s - l_0) / sum_{s'} exp(l_s' - l_0),  computed in double, stored as fp32.
 * ------------------------------------------------------------------------------------- */
static void topk_row(const float* l, int E, int k, int32_t* idx, float* g) {
    unsigned char taken[REF_MAX_E];
    memset(taken, 0, (size_t)E);
    for (int s = 0; s < k; ++s) {
        int best = -1;
        float bestv = 0.0f;
        for (int e = 0; e < E; ++e) {
            if (taken[e]) continue;
            float v = isnan(l[e]) ? -INFINITY : l[e];
            if (best < 0 || v > bestv) { best = e; bestv = v; }
        }
        taken[best] = 1;
        idx[s] = best;
    }
    double w[REF_MAX_E], den = 0.0;
    for (int s = 0; s < k; ++s) {
        w[s] = exp((double)l[idx[s]] - (double)l[idx[0]]);
        den += w[s];
    }
    for (int s = 0; s < k; ++s) g[s] = (float)(w[s] / den);
}

int moe_ref_topk(const float* logits, int T, int E, int k, int32_t* topk_idx, float* topk_w) {
    if (T < 0 || E <= 0 || E > REF_MAX_E || k <= 0 || k > E) return REF_ERR_ARG;
    for (int t = 0; t < T; ++t)
        topk_row(logits + (size_t)t * E, E, k, topk_idx + (size_t)t * k, topk_w + (size_t)t * k);
    return REF_OK;
}

/* ---------------------------------------------------------------------------------------
 * Permutation that groups routed rows by expert (the "per-expert inputs" of Section 3.1).
 * Flat id i = t*k + s. counts[e] = #{i : idx[i] = e}; offsets = exclusive prefix sum with
 * offsets[E] = R; rows of one expert keep ascending i (a stable counting sort), so
 * perm[p] = i and inv_perm[i] = p are unique.
 * ------------------------------------------------------------------------------------- */
int moe_ref_permute(const int32_t* topk_idx, int R, int E, int32_t* counts, int32_t* offsets,
                    int32_t* perm, int32_t* inv_perm) {
    if (R < 0 || E <= 0) return REF_ERR_ARG;
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int i = 0; i < R; ++i) {
        if (topk_idx[i] < 0 || topk_idx[i] >= E) return REF_ERR_ARG;
        counts[topk_idx[i]]++;
    }
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
    int32_t* cursor = (int32_t*)malloc(sizeof(int32_t) * (size_t)E);
    if (!cursor) return REF_ERR_ARG;
    memcpy(cursor, offsets, sizeof(int32_t) * (size_t)E);
    for (int i = 0; i < R; ++i) {
        int p = cursor[topk_idx[i]]++;
        perm[p] = i;
        inv_perm[i] = p;
    }
    free(cursor);
    return REF_OK;
}

/* Row gather: x_perm[p,:] = x[perm[p] / k, :]  (raw bf16 bits, exact copy). */
int moe_ref_gather(const uint16_t* x, const int32_t* perm, int R, int d, int k, uint16_t* x_perm) {
    if (R < 0 || d <= 0 || k <= 0) return REF_ERR_ARG;
    for (int p = 0; p < R; ++p)
        memcpy(x_perm + (size_t)p * d, x + (size_t)(perm[p] / k) * d, sizeof(uint16_t) * (size_t)d);
    return REF_OK;
}

/* ---------------------------------------------------------------------------------------
 * One expert applied to one row (Table 1 row 3: three d_h x d_e matrices; Section 4.1:
 * a gated FFN):  a = W1 x, b = W3 x, h = SiLU(a) * b, o = W2 h.
 * W1, W3 are [f, d] row-major (out, in); W2 is [d, f] row-major. All sums in double.
 * ------------------------------------------------------------------------------------- */
static void expert_row(const double* xd, const uint16_t* W1e, const uint16_t* W3e,
                       const uint16_t* W2e, int d, int f, double* h, double* o) {
    for (int j = 0; j < f; ++j) {
        const uint16_t* w1 = W1e + (size_t)j * d;
        const uint16_t* w3 = W3e + (size_t)j * d;
        double a = 0.0, b = 0.0;
#pragma omp simd reduction(+ : a, b)
        for (int i = 0; i < d; ++i) {
            a += xd[i] * (double)bf16_val(w1[i]);
            b += xd[i] * (double)bf16_val(w3[i]);
        }
        h[j] = a / (1.0 + exp(-a)) * b;
    }
    for (int c = 0; c < d; ++c) {
        const uint16_t* w2 = W2e + (size_t)c * f;
        double s = 0.0;
#pragma omp simd reduction(+ : s)
        for (int j = 0; j < f; ++j) s += h[j] * (double)bf16_val(w2[j]);
        o[c] = s;
    }
}

/* ---------------------------------------------------------------------------------------
 * The layer by its definition, one token at a time:  y[t] = sum_s g[t,s] * Expert_{idx[t,s]}(x[t]),
 * slots added in order s = 0..k-1. Tokens are independent of one another, which is why the
 * coalesced batch and any split into micro-batches give the same y (Section 3.1,
 * Opportunity 1), and why a subset of tokens can be evaluated alone.
 * tokens[n] lists the token ids to evaluate (NULL = 0..n-1); y_out is [n, d] double.
 * Optional outputs (may be NULL): idx_out[n,k], g_out[n,k].
 * ------------------------------------------------------------------------------------- */
int moe_ref_layer_tokens(const uint16_t* x, const float* w_router, const float* bias,
                         const uint16_t* W1, const uint16_t* W3, const uint16_t* W2, int T, int d,
                         int f, int E, int k, const int32_t* tokens, int n, double* y_out,
                         int32_t* idx_out, float* g_out) {
    if (T < 0 || n < 0 || d <= 0 || d % 512 != 0 || f <= 0 || E <= 0 || E > REF_MAX_E || k <= 0 ||
        k > E)
        return REF_ERR_ARG;
    for (int q = 0; q < n; ++q) {
        int t = tokens ? tokens[q] : q;
        if (t < 0 || t >= T) return REF_ERR_ARG;
    }
    int fail = 0;
#pragma omp parallel
    {
        double* xd = (double*)malloc(sizeof(double) * (size_t)d);
        double* h = (double*)malloc(sizeof(double) * (size_t)f);
        double* o = (double*)malloc(sizeof(double) * (size_t)d);
        float* l = (float*)malloc(sizeof(float) * (size_t)E);
        int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)k);
        float* g = (float*)malloc(sizeof(float) * (size_t)k);
        if (!xd || !h || !o || !l || !idx || !g) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int q = 0; q < n; ++q) {
                int t = tokens ? tokens[q] : q;
                const uint16_t* xr = x + (size_t)t * d;
                logits_row(xr, w_router, bias, d, E, l);
                topk_row(l, E, k, idx, g);
                for (int i = 0; i < d; ++i) xd[i] = (double)bf16_val(xr[i]);
                double* y = y_out + (size_t)q * d;
                for (int c = 0; c < d; ++c) y[c] = 0.0;
                for (int s = 0; s < k; ++s) {
                    size_t e = (size_t)idx[s];
                    expert_row(xd, W1 + e * f * d, W3 + e * f * d, W2 + e * d * f, d, f, h, o);
                    for (int c = 0; c < d; ++c) y[c] += (double)g[s] * o[c];
                }
                if (idx_out) memcpy(idx_out + (size_t)q * k, idx, sizeof(int32_t) * (size_t)k);
                if (g_out) memcpy(g_out + (size_t)q * k, g, sizeof(float) * (size_t)k);
            }
        }
        free(xd); free(h); free(o); free(l); free(idx); free(g);
    }
    return fail ? REF_ERR_ARG : REF_OK;
}

/* ---------------------------------------------------------------------------------------
 * Stage form of the expert FFN: rows already grouped by expert. Row p belongs to the expert
 * e with offsets[e] <= p < offsets[e+1].  rows[n] lists the permuted rows to evaluate
 * (NULL = 0..n-1);  y_perm_out is [n, d] double; h_out (may be NULL) is [n, f] double.
 * ------------------------------------------------------------------------------------- */
int moe_ref_expert_ffn(const uint16_t* x_perm, const int32_t* offsets, int R, int d, int f, int E,
                       const uint16_t* W1, const uint16_t* W3, const uint16_t* W2,
                       const int32_t* rows, int n, double* y_perm_out, double* h_out) {
    if (R < 0 || n < 0 || d <= 0 || f <= 0 || E <= 0) return REF_ERR_ARG;
    if (offsets[0] != 0 || offsets[E] != R) return REF_ERR_ARG;
    for (int e = 0; e < E; ++e)
        if (offsets[e + 1] < offsets[e]) return REF_ERR_ARG;
    for (int q = 0; q < n; ++q) {
        int p = rows ? rows[q] : q;
        if (p < 0 || p >= R) return REF_ERR_ARG;
    }
    int fail = 0;
#pragma omp parallel
    {
        double* xd = (double*)malloc(sizeof(double) * (size_t)d);
        double* h = (double*)malloc(sizeof(double) * (size_t)f);
        if (!xd || !h) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int q = 0; q < n; ++q) {
                int p = rows ? rows[q] : q;
                size_t e = 0;
                while (!(offsets[e] <= p && p < offsets[e + 1])) ++e;
                for (int i = 0; i < d; ++i) xd[i] = (double)bf16_val(x_perm[(size_t)p * d + i]);
                expert_row(xd, W1 + e * f * d, W3 + e * f * d, W2 + e * d * f, d, f, h,
                           y_perm_out + (size_t)q * d);
                if (h_out) memcpy(h_out + (size_t)q * f, h, sizeof(double) * (size_t)f);
            }
        }
        free(xd); free(h);
    }
    return fail ? REF_ERR_ARG : REF_OK;
}

/* Stage form of the combine:  y[t,:] = sum_{s<k} g[t,s] * y_perm[inv_perm[t*k+s], :],
 * slots added in order; y_perm given as double [R, d]; y double [T, d]. */
int moe_ref_combine(const double* y_perm, const int32_t* inv_perm, const float* topk_w, int T,
                    int d, int k, double* y) {
    if (T < 0 || d <= 0 || k <= 0) return REF_ERR_ARG;
    for (int t = 0; t < T; ++t) {
        double* yr = y + (size_t)t * d;
        for (int c = 0; c < d; ++c) yr[c] = 0.0;
        for (int s = 0; s < k; ++s) {
            const double* src = y_perm + (size_t)inv_perm[(size_t)t * k + s] * d;
            double g = (double)topk_w[(size_t)t * k + s];
            for (int c = 0; c < d; ++c) yr[c] += g * src[c];
        }
    }
    return REF_OK;
}

/* The same combine for a bf16 y_perm (raw bits), as the library's stage receives it. */
int moe_ref_combine_bf16(const uint16_t* y_perm, const int32_t* inv_perm, const float* topk_w,
                         int T, int d, int k, double* y) {
    if (T < 0 || d <= 0 || k <= 0) return REF_ERR_ARG;
    for (int t = 0; t < T; ++t) {
        double* yr = y + (size_t)t * d;
        for (int c = 0; c < d; ++c) yr[c] = 0.0;
        for (int s = 0; s < k; ++s) {
            const uint16_t* src = y_perm + (size_t)inv_perm[(size_t)t * k + s] * d;
            double g = (double)topk_w[(size_t)t * k + s];
            for (int c = 0; c < d; ++c) yr[c] += g * (double)bf16_val(src[c]);
        }
    }
    return REF_OK;
}

/* ---------------------------------------------------------------------------------------
 * The layer through its stages on consecutive micro-batches of m tokens (Section 2.3: the
 * micro-batches run one after the other through the same expert weights): for each chunk
 * [c*m, min(T,(c+1)*m)) route, build that chunk's own permutation, gather, run the grouped
 * expert FFN, combine. m = T is the coalesced batch (m_exp = B, Section 4.1.1).
 * y is [T, d] double.
 * ------------------------------------------------------------------------------------- */
int moe_ref_layer_staged(const uint16_t* x, const float* w_router, const float* bias,
                         const uint16_t* W1, const uint16_t* W3, const uint16_t* W2, int T, int d,
                         int f, int E, int k, int m, double* y) {
    if (T < 0 || m <= 0 || d <= 0 || d % 512 != 0 || f <= 0 || E <= 0 || E > REF_MAX_E || k <= 0 ||
        k > E)
        return REF_ERR_ARG;
    int rc = REF_OK;
    for (int t0 = 0; t0 < T && rc == REF_OK; t0 += m) {
        int Tc = (T - t0 < m) ? T - t0 : m;
        int Rc = Tc * k;
        float* l = (float*)malloc(sizeof(float) * (size_t)Tc * E);
        int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)Rc);
        float* g = (float*)malloc(sizeof(float) * (size_t)Rc);
        int32_t* counts = (int32_t*)malloc(sizeof(int32_t) * (size_t)E);
        int32_t* offsets = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E + 1));
        int32_t* perm = (int32_t*)malloc(sizeof(int32_t) * (size_t)Rc);
        int32_t* inv = (int32_t*)malloc(sizeof(int32_t) * (size_t)Rc);
        uint16_t* xp = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)Rc * d);
        double* yp = (double*)malloc(sizeof(double) * (size_t)Rc * d);
        if (!l || !idx || !g || !counts || !offsets || !perm || !inv || !xp || !yp) {
            rc = REF_ERR_ARG;
        } else {
            const uint16_t* xc = x + (size_t)t0 * d;
            rc = moe_ref_logits(xc, w_router, bias, Tc, d, E, l);
            if (rc == REF_OK) rc = moe_ref_topk(l, Tc, E, k, idx, g);
            if (rc == REF_OK) rc = moe_ref_permute(idx, Rc, E, counts, offsets, perm, inv);
            if (rc == REF_OK) rc = moe_ref_gather(xc, perm, Rc, d, k, xp);
            if (rc == REF_OK)
                rc = moe_ref_expert_ffn(xp, offsets, Rc, d, f, E, W1, W3, W2, NULL, Rc, yp, NULL);
            if (rc == REF_OK) rc = moe_ref_combine(yp, inv, g, Tc, d, k, y + (size_t)t0 * d);
        }
        free(l); free(idx); free(g); free(counts); free(offsets); free(perm); free(inv);
        free(xp); free(yp);
    }
    return rc;
}
