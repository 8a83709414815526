/*
 * sanitize_oracle.c - TEST INFRASTRUCTURE.  Walks every function of the CPU oracle over small,
 * deliberately ragged shapes (widths that are no power of two, empty expert groups, k = E, one
 * token, weight-decomposed experts with and without a shared base, both storage types) so that an
 * AddressSanitizer / UndefinedBehaviorSanitizer build of the oracle's source reads and writes every
 * buffer at its edges.  Buffers are allocated at their exact sizes: one element past any of them
 * is a sanitizer report.  A few cheap invariants are checked on the way (gates sum to one, the
 * permutation is a permutation, the staged pipeline equals the direct definition); the numerical
 * pins proper live in the Python tests.  Exit status 0 = no report and no failed check.
 */
#include <stdio.h>

#include "moe_oracle.c"

static uint32_t lcg_state = 12345u;
static double lcg_unit(void) { /* uniform in (-1, 1) */
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return ((double)(lcg_state >> 8) / 8388608.0) - 1.0;
}

static uint16_t to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

/* n stored values of the given type, exactly n elements long */
static void* stored(size_t n, int dtype, double scale) {
    if (dtype == DT_F32) {
        float* p = (float*)malloc(sizeof(float) * (n ? n : 1));
        for (size_t i = 0; i < n; ++i) p[i] = (float)(scale * lcg_unit());
        return p;
    }
    uint16_t* p = (uint16_t*)malloc(sizeof(uint16_t) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = to_bf16((float)(scale * lcg_unit()));
    return p;
}

static int failures = 0;
#define CHECK(cond, what)                                              \
    do {                                                               \
        if (!(cond)) {                                                 \
            fprintf(stderr, "check failed (%s): %s\n", what, #cond); \
            failures += 1;                                             \
        }                                                              \
    } while (0)

static void one_layer(int d, int F, int E, int k, int r, int base, int dtype, int T, const char* what) {
    oracle_layer L;
    memset(&L, 0, sizeof L);
    L.d = d; L.F = F; L.E = E; L.k = k; L.r = r; L.dtype = dtype;
    L.flags = base && r > 0 ? FLAG_SHARED_BASE : 0;
    float* rw = (float*)stored((size_t)E * d, DT_F32, 0.3);
    float* rb = (float*)stored((size_t)E, DT_F32, 0.5);
    L.router_w = rw;
    L.router_b = rb;
    const int dense = (r == 0) || base;
    const size_t eb = base ? 1 : (size_t)E;
    void *wg = NULL, *wu = NULL, *wd = NULL, *f[6] = {0};
    if (dense) {
        wg = stored(eb * F * d, dtype, 0.2);
        wu = stored(eb * F * d, dtype, 0.2);
        wd = stored(eb * d * F, dtype, 0.2);
    }
    if (r > 0) {
        f[0] = stored((size_t)E * r * d, dtype, 0.3); /* rg */
        f[1] = stored((size_t)E * r * d, dtype, 0.3); /* ru */
        f[2] = stored((size_t)E * r * F, dtype, 0.3); /* rd */
        f[3] = stored((size_t)E * F * r, dtype, 0.3); /* lg */
        f[4] = stored((size_t)E * F * r, dtype, 0.3); /* lu */
        f[5] = stored((size_t)E * d * r, dtype, 0.3); /* ld */
    }
    L.w_gate = wg; L.w_up = wu; L.w_down = wd;
    L.rg = f[0]; L.ru = f[1]; L.rd = f[2]; L.lg = f[3]; L.lu = f[4]; L.ld = f[5];
    void* x = stored((size_t)T * d, dtype, 1.0);
    const size_t P = (size_t)T * k;

    /* router */
    int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (P ? P : 1));
    double* gate = (double*)malloc(sizeof(double) * (P ? P : 1));
    double* probs = (double*)malloc(sizeof(double) * ((size_t)T * E ? (size_t)T * E : 1));
    double* logits = (double*)malloc(sizeof(double) * ((size_t)T * E ? (size_t)T * E : 1));
    CHECK(oracle_route(T, d, E, k, dtype, x, rw, rb, idx, gate, probs, logits) == 0, what);
    for (int t = 0; t < T; ++t) {
        double s = 0;
        for (int j = 0; j < k; ++j) s += gate[(size_t)t * k + j];
        CHECK(fabs(s - 1.0) < 1e-12, what);
    }
    /* dispatch */
    int32_t* off = (int32_t*)malloc(sizeof(int32_t) * (size_t)(E + 1));
    int32_t* perm = (int32_t*)malloc(sizeof(int32_t) * (P ? P : 1));
    int32_t* inv = (int32_t*)malloc(sizeof(int32_t) * (P ? P : 1));
    CHECK(oracle_permute((int)P, E, idx, off, perm, inv) == 0, what);
    CHECK(off[E] == (int32_t)P, what);
    for (size_t s = 0; s < P; ++s) CHECK(inv[perm[s]] == (int32_t)s, what);
    /* staged experts + combine against the direct per-token definition */
    size_t esz = dtype == DT_F32 ? 4 : 2;
    char* xp = (char*)malloc(esz * (P * d ? P * d : 1));
    for (size_t s = 0; s < P; ++s) memcpy(xp + s * d * esz, (char*)x + (size_t)(perm[s] / k) * d * esz, d * esz);
    double* yp = (double*)malloc(sizeof(double) * (P * d ? P * d : 1));
    CHECK(oracle_expert_ffn(&L, (int)P, xp, off, yp) == 0, what);
    double* y1 = (double*)malloc(sizeof(double) * ((size_t)T * d ? (size_t)T * d : 1));
    CHECK(oracle_combine(T, d, k, dtype, yp, inv, gate, x, y1) == 0, what);
    L.flags |= FLAG_RESIDUAL;
    double* y2 = (double*)malloc(sizeof(double) * ((size_t)T * d ? (size_t)T * d : 1));
    int32_t* idx2 = (int32_t*)malloc(sizeof(int32_t) * (P ? P : 1));
    double* gate2 = (double*)malloc(sizeof(double) * (P ? P : 1));
    CHECK(oracle_forward(&L, T, x, y2, idx2, gate2) == 0, what);
    for (size_t i = 0; i < (size_t)T * d; ++i) CHECK(fabs(y1[i] - y2[i]) <= 1e-9 * (1.0 + fabs(y2[i])), what);
    for (size_t i = 0; i < P; ++i) CHECK(idx[i] == idx2[i], what);
    /* a stack of three such layers, with every optional output */
    oracle_layer stack[3] = {L, L, L};
    double* ys = (double*)malloc(sizeof(double) * ((size_t)T * d ? (size_t)T * d : 1));
    int32_t* trace = (int32_t*)malloc(sizeof(int32_t) * (3 * P ? 3 * P : 1));
    double* xs = (double*)malloc(sizeof(double) * (4 * (size_t)T * d ? 4 * (size_t)T * d : 1));
    CHECK(oracle_stack_forward(stack, 3, T, x, ys, trace, xs) == 0, what);
    /* trace statistics on that trace: [3 layers, T, k] */
    if (T > 0) {
        int64_t* He = (int64_t*)malloc(sizeof(int64_t) * (size_t)E);
        int64_t H = oracle_expert_replacements(3, T, k, E, trace, He);
        CHECK(H >= 0, what);
        float* W32 = (float*)malloc(sizeof(float) * (size_t)T * E);
        for (size_t i = 0; i < (size_t)T * E; ++i) W32[i] = (float)probs[i];
        double out[5];
        CHECK(oracle_bles_loss(1, T, k, E, W32, idx, out) == 0, what);
        int64_t* ch = (int64_t*)malloc(sizeof(int64_t) * 3);
        int64_t* ld = (int64_t*)malloc(sizeof(int64_t) * 3);
        CHECK(oracle_offload_counters(3, T, k, E, trace, ch, ld) == 0, what);
        int64_t* cnt = (int64_t*)malloc(sizeof(int64_t) * 3 * (size_t)E);
        double* dl = (double*)malloc(sizeof(double) * 3);
        double mean;
        CHECK(oracle_delta_uniform(3, T, k, E, trace, cnt, dl, &mean) == 0, what);
        CHECK(mean >= 0.0 && mean <= 2.0, what);
        free(He); free(W32); free(ch); free(ld); free(cnt); free(dl);
    }
    free(rw); free(rb); free(wg); free(wu); free(wd);
    for (int i = 0; i < 6; ++i) free(f[i]);
    free(x); free(idx); free(gate); free(probs); free(logits); free(off); free(perm); free(inv);
    free(xp); free(yp); free(y1); free(y2); free(idx2); free(gate2); free(ys); free(trace); free(xs);
}

int main(void) {
    /*        d   F   E  k  r  base dtype    T */
    one_layer(24, 40, 5, 3, 0, 0, DT_BF16, 9, "dense bf16, ragged widths");
    one_layer(17, 33, 4, 4, 0, 0, DT_F32, 7, "dense fp32, odd widths, k = E");
    one_layer(24, 40, 6, 2, 8, 0, DT_BF16, 11, "pure L R");
    one_layer(16, 24, 3, 1, 5, 1, DT_F32, 13, "shared base + L R, k = 1");
    one_layer(8, 8, 1, 1, 0, 0, DT_BF16, 1, "one expert, one token");
    one_layer(32, 264, 9, 2, 0, 0, DT_BF16, 300, "rows >= 256: OpenMP inside a product; T >= 8: over tokens");
    one_layer(8, 16, 64, 8, 0, 0, DT_F32, 3, "64 experts, most groups empty");
    one_layer(8, 16, 4, 2, 0, 0, DT_BF16, 0, "no tokens");
    /* argument checks */
    int32_t bad[2] = {0, 7};
    int32_t o[5], p2[2], i2[2];
    CHECK(oracle_permute(2, 4, bad, o, p2, i2) == -1, "out-of-range expert");
    CHECK(oracle_route(1, 8, 4, 5, DT_F32, NULL, NULL, NULL, NULL, NULL, NULL, NULL) == -1, "k > E");
    if (failures) {
        fprintf(stderr, "%d check(s) failed\n", failures);
        return 1;
    }
    printf("sanitized oracle walk: ok\n");
    return 0;
}
