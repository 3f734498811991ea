/*
 * Runs entry points of oracle/moe_oracle.c on inputs read from a text file, with every buffer
 * allocated on the heap at exactly the size the entry point's contract states, and prints the
 * outputs as text. tests/test_oracle_sanitizers.py compiles this file together with the oracle
 * under -fsanitize=address,undefined (no recovery) and compares the printed values with the
 * hand-derived pins: an out-of-bounds access, a signed overflow or a misaligned or
 * uninitialised-size access in the oracle ends the run with a non-zero status.
 *
 * Input: first token = operation; then the integers and values it needs (floats as C99 hex or
 * decimal, bf16 as raw bit patterns in decimal).
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int moe_ref_logits(const uint16_t*, const float*, const float*, int, int, int, float*);
int moe_ref_topk(const float*, int, int, int, int32_t*, float*);
int moe_ref_permute(const int32_t*, int, int, int32_t*, int32_t*, int32_t*, int32_t*);
int moe_ref_gather(const uint16_t*, const int32_t*, int, int, int, uint16_t*);
int moe_ref_layer_tokens(const uint16_t*, const float*, const float*, const uint16_t*,
                         const uint16_t*, const uint16_t*, int, int, int, int, int, const int32_t*,
                         int, double*, int32_t*, float*);
int moe_ref_layer_staged(const uint16_t*, const float*, const float*, const uint16_t*,
                         const uint16_t*, const uint16_t*, int, int, int, int, int, int, double*);
int moe_ref_expert_ffn(const uint16_t*, const int32_t*, int, int, int, int, const uint16_t*,
                       const uint16_t*, const uint16_t*, const int32_t*, int, double*, double*);

static FILE* in;

static int rd_int(void) {
    int v;
    if (fscanf(in, "%d", &v) != 1) { fprintf(stderr, "driver: expected an integer\n"); exit(3); }
    return v;
}
static float* rd_f32(size_t n) {
    float* p = (float*)malloc(sizeof(float) * (n ? n : 1));
    char tok[64];
    for (size_t i = 0; i < n; ++i) {
        if (fscanf(in, "%63s", tok) != 1) { fprintf(stderr, "driver: expected a float\n"); exit(3); }
        p[i] = strtof(tok, NULL);
    }
    return p;
}
static uint16_t* rd_u16(size_t n) {
    uint16_t* p = (uint16_t*)malloc(sizeof(uint16_t) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = (uint16_t)rd_int();
    return p;
}
static int32_t* rd_i32(size_t n) {
    int32_t* p = (int32_t*)malloc(sizeof(int32_t) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = rd_int();
    return p;
}
static void pr_i32(const char* name, const int32_t* p, size_t n) {
    printf("%s", name);
    for (size_t i = 0; i < n; ++i) printf(" %d", p[i]);
    printf("\n");
}
static void pr_f32(const char* name, const float* p, size_t n) {
    printf("%s", name);
    for (size_t i = 0; i < n; ++i) printf(" %a", (double)p[i]);
    printf("\n");
}
static void pr_f64(const char* name, const double* p, size_t n) {
    printf("%s", name);
    for (size_t i = 0; i < n; ++i) printf(" %a", p[i]);
    printf("\n");
}

int main(int argc, char** argv) {
    if (argc != 2 || !(in = fopen(argv[1], "r"))) { fprintf(stderr, "usage: driver FILE\n"); return 2; }
    char op[32];
    if (fscanf(in, "%31s", op) != 1) return 2;
    int rc = 0;
    if (!strcmp(op, "topk")) {
        int T = rd_int(), E = rd_int(), k = rd_int();
        float* lg = rd_f32((size_t)T * E);
        int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)T * k);
        float* g = (float*)malloc(sizeof(float) * (size_t)T * k);
        rc = moe_ref_topk(lg, T, E, k, idx, g);
        pr_i32("idx", idx, (size_t)T * k);
        pr_f32("gates", g, (size_t)T * k);
        free(lg); free(idx); free(g);
    } else if (!strcmp(op, "permute")) {
        int R = rd_int(), E = rd_int();
        int32_t* idx = rd_i32((size_t)R);
        int32_t* counts = (int32_t*)malloc(sizeof(int32_t) * (size_t)E);
        int32_t* offsets = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E + 1));
        int32_t* perm = (int32_t*)malloc(sizeof(int32_t) * (size_t)(R ? R : 1));
        int32_t* inv = (int32_t*)malloc(sizeof(int32_t) * (size_t)(R ? R : 1));
        rc = moe_ref_permute(idx, R, E, counts, offsets, perm, inv);
        pr_i32("counts", counts, (size_t)E);
        pr_i32("offsets", offsets, (size_t)E + 1);
        pr_i32("perm", perm, (size_t)R);
        pr_i32("inv_perm", inv, (size_t)R);
        free(idx); free(counts); free(offsets); free(perm); free(inv);
    } else if (!strcmp(op, "logits")) {
        int T = rd_int(), d = rd_int(), E = rd_int(), has_bias = rd_int();
        uint16_t* x = rd_u16((size_t)T * d);
        float* w = rd_f32((size_t)d * E);
        float* b = has_bias ? rd_f32((size_t)E) : NULL;
        float* lg = (float*)malloc(sizeof(float) * (size_t)T * E);
        rc = moe_ref_logits(x, w, b, T, d, E, lg);
        pr_f32("logits", lg, (size_t)T * E);
        free(x); free(w); free(b); free(lg);
    } else if (!strcmp(op, "layer")) {
        /* the layer by its definition on a token subset, and through its stages for micro-batch m */
        int T = rd_int(), d = rd_int(), f = rd_int(), E = rd_int(), k = rd_int(), m = rd_int(), n = rd_int();
        int32_t* tokens = rd_i32((size_t)n);
        uint16_t* x = rd_u16((size_t)T * d);
        float* w = rd_f32((size_t)d * E);
        uint16_t* W1 = rd_u16((size_t)E * f * d);
        uint16_t* W3 = rd_u16((size_t)E * f * d);
        uint16_t* W2 = rd_u16((size_t)E * d * f);
        double* y = (double*)malloc(sizeof(double) * (size_t)n * d);
        int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)n * k);
        float* g = (float*)malloc(sizeof(float) * (size_t)n * k);
        rc = moe_ref_layer_tokens(x, w, NULL, W1, W3, W2, T, d, f, E, k, tokens, n, y, idx, g);
        pr_i32("idx", idx, (size_t)n * k);
        pr_f64("y_tokens", y, (size_t)n * d);
        double* ys = (double*)malloc(sizeof(double) * (size_t)T * d);
        if (rc == 0) rc = moe_ref_layer_staged(x, w, NULL, W1, W3, W2, T, d, f, E, k, m, ys);
        pr_f64("y_staged", ys, (size_t)T * d);
        free(tokens); free(x); free(w); free(W1); free(W3); free(W2); free(y); free(idx); free(g); free(ys);
    } else if (!strcmp(op, "ffn")) {
        int R = rd_int(), d = rd_int(), f = rd_int(), E = rd_int();
        int32_t* offsets = rd_i32((size_t)E + 1);
        uint16_t* xp = rd_u16((size_t)R * d);
        uint16_t* W1 = rd_u16((size_t)E * f * d);
        uint16_t* W3 = rd_u16((size_t)E * f * d);
        uint16_t* W2 = rd_u16((size_t)E * d * f);
        double* y = (double*)malloc(sizeof(double) * (size_t)(R ? R : 1) * d);
        double* h = (double*)malloc(sizeof(double) * (size_t)(R ? R : 1) * f);
        rc = moe_ref_expert_ffn(xp, offsets, R, d, f, E, W1, W3, W2, NULL, R, y, h);
        pr_f64("y_perm", y, (size_t)R * d);
        pr_f64("h", h, (size_t)R * f);
        free(offsets); free(xp); free(W1); free(W3); free(W2); free(y); free(h);
    } else {
        fprintf(stderr, "driver: unknown operation %s\n", op);
        return 2;
    }
    fclose(in);
    printf("rc %d\n", rc);
    return rc == 0 ? 0 : 1;
}
