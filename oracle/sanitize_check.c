/*
 * Sanitizer run of the CPU oracle.  TEST INFRASTRUCTURE: compiled together with aride_oracle.c
 * under -fsanitize=address,undefined by tests/test_oracle_sanitizers.py and executed once.  It
 * calls every oracle routine on small inputs with exactly sized heap buffers -- ragged and empty
 * trajectories, padding rows, rows with a stride, repeated and out-of-range indices, a buffer with
 * no mass, an insert longer than the buffer -- so that a read or write one element past an
 * array, an uninitialised read that reaches a branch, a signed overflow or a bad shift aborts
 * the run.  It checks no values (the pins in tests/test_oracle_*.py do); it prints "ok".
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_score_logits(const uint16_t*, int64_t, int64_t, int64_t, const int32_t*, int32_t, double*, double*,
                        double*, double*, int);
int oracle_retrace_targets(const double*, const double*, const double*, const double*, const double*, const double*,
                           const int32_t*, int64_t, int64_t, double, double, double*, double*, double*);
int oracle_vtrace_targets(const double*, const double*, const double*, const double*, const double*, const double*,
                          const int32_t*, int64_t, int64_t, double, double, double, double, double*, double*, double*);
int oracle_mc_returns(const double*, const int32_t*, int64_t, int64_t, double, double*, double*);
int oracle_compute_priorities(const double*, const double*, const double*, const int32_t*, int64_t, int64_t, double,
                              double, double, double, double, double, int, double*, double*);
int64_t oracle_update_priorities(float*, int64_t, const int64_t*, const float*, int64_t, float);
uint64_t oracle_quantise_weights(const float*, int64_t, uint64_t*);
int oracle_sample_prioritized(const float*, int64_t, const double*, int64_t, int64_t*, double*);
int64_t oracle_replay_insert(float*, int64_t, int64_t, const float*, int64_t, float, int64_t*);
int oracle_actor_loss_grad(const uint16_t*, int64_t, int64_t, int64_t, const int32_t*, int32_t, const double*,
                           const double*, const double*, const double*, double, double, double, double*, double*);

static uint32_t state = 20241014u;
static double unit(void) {            /* a small linear congruential generator: values only need variety */
    state = state * 1664525u + 1013904223u;
    return (double)(state >> 8) / 16777216.0;
}
static double* doubles(int64_t n, double lo, double hi) {
    double* p = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    for (int64_t i = 0; i < n; ++i) p[i] = lo + (hi - lo) * unit();
    return p;
}
#define FAIL(msg) do { fprintf(stderr, "sanitize_check: %s\n", msg); return 1; } while (0)

int main(void) {
    /* ---- logits: R rows of V columns inside a wider stride, bf16 bit patterns */
    const int64_t N = 7, A = 3, R = N * A, V = 37, stride = 41;
    uint16_t* logits = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)(R * stride));
    for (int64_t i = 0; i < R * stride; ++i) {
        const float f = (float)(4.0 * unit() - 2.0);
        uint32_t bits;
        __builtin_memcpy(&bits, &f, 4);
        logits[i] = (uint16_t)(bits >> 16);
    }
    logits[5] = 0xFF80;                                   /* -inf: a masked vocabulary entry */
    int32_t* tokens = (int32_t*)malloc(sizeof(int32_t) * (size_t)R);
    for (int64_t r = 0; r < R; ++r) tokens[r] = (int32_t)(unit() * V) % (int32_t)V;
    tokens[4] = -1;                                       /* a padding row */
    double *tl = doubles(R, 0, 0), *te = doubles(R, 0, 0), *sl = doubles(N, 0, 0), *se = doubles(N, 0, 0);
    if (oracle_score_logits(logits, R, V, stride, tokens, (int32_t)A, tl, te, sl, se, 1) != 0) FAIL("score");
    if (oracle_score_logits(logits, R, V, stride, tokens, (int32_t)A, tl, te, sl, se, 3) != 0) FAIL("score, threads");
    if (oracle_score_logits(logits, R, V, stride, tokens, (int32_t)A, NULL, NULL, sl, NULL, 1) != 0) FAIL("score, nulls");
    if (oracle_score_logits(logits, 0, V, stride, tokens, (int32_t)A, tl, te, sl, se, 1) != 0) FAIL("score, no rows");

    /* ---- scans over ragged trajectories with empty ones at the front, inside and at the back */
    const int32_t off[] = {0, 0, 3, 3, 4, 7, 7};
    const int64_t B = 6;
    double *lm = doubles(N, -3, 0), *rw = doubles(N, 0, 1), *v = doubles(N, -1, 1), *q = doubles(N, -1, 1);
    double *boot = doubles(B, -1, 1), *tg = doubles(N, 0, 0), *td = doubles(N, 0, 0), *rho = doubles(N, 0, 0);
    if (oracle_retrace_targets(sl, lm, rw, v, q, boot, off, B, N, 0.9, 0.95, tg, td, rho) != 0) FAIL("retrace");
    if (oracle_retrace_targets(sl, lm, rw, v, NULL, NULL, off, B, N, 0.9, 0.95, tg, NULL, NULL) != 0) FAIL("retrace, nulls");
    if (oracle_vtrace_targets(sl, lm, rw, v, q, boot, off, B, N, 0.9, 0.95, 1.3, 0.9, tg, td, rho) != 0) FAIL("vtrace");
    if (oracle_retrace_targets(sl, lm, rw, v, q, boot, off, 0, 0, 0.9, 0.95, tg, td, rho) != 0) FAIL("retrace, empty batch");
    double *ret = doubles(N, 0, 0), *lab = doubles(N, 0, 0);
    if (oracle_mc_returns(rw, off, B, N, 0.99, ret, lab) != 0) FAIL("mc returns");
    double *sp = doubles(N, 0, 0), *tp = doubles(B, 0, 0);
    if (oracle_compute_priorities(td, rho, se, off, B, N, 1.0, 0.5, 0.1, 2.0, 8.0, 1e-3, 1, sp, tp) != 0) FAIL("priorities");
    if (oracle_compute_priorities(td, rho, se, off, B, N, 1.0, 0.5, 0.1, 2.0, 8.0, 0.0, 0, NULL, tp) != 0) FAIL("priorities, nulls");

    /* ---- replay: update with repeated and out-of-range indices, quantise, draw, insert */
    const int64_t M = 29, K = 11;
    float* w = (float*)malloc(sizeof(float) * (size_t)M);
    for (int64_t i = 0; i < M; ++i) w[i] = (float)unit();
    w[3] = 0.f; w[7] = NAN; w[8] = -1.f; w[9] = INFINITY;
    int64_t idx[] = {0, 5, 5, 28, -1, 29, 5, 1, 1LL << 40, 2, 28};
    float* pr = (float*)malloc(sizeof(float) * (size_t)K);
    for (int64_t k = 0; k < K; ++k) pr[k] = (float)(3.0 * unit());
    pr[2] = NAN; pr[3] = -2.f;
    if (oracle_update_priorities(w, M, idx, pr, K, 0.6f) != 3) FAIL("update: three indices lie outside the buffer");
    uint64_t* quant = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)M);
    if (oracle_quantise_weights(w, M, quant) == 0) FAIL("quantise");
    double* u = doubles(K, 0, 1);
    u[0] = 0.0; u[1] = nextafter(1.0, 0.0); u[2] = -0.5; u[3] = 2.0; u[4] = NAN;
    int64_t* drawn = (int64_t*)malloc(sizeof(int64_t) * (size_t)K);
    double* prob = doubles(K, 0, 0);
    if (oracle_sample_prioritized(w, M, u, K, drawn, prob) != 0) FAIL("sample");
    if (oracle_sample_prioritized(w, M, u, K, drawn, NULL) != 0) FAIL("sample, no probabilities");
    float* none = (float*)calloc((size_t)M, sizeof(float));
    if (oracle_sample_prioritized(none, M, u, K, drawn, prob) != -5) FAIL("sample: a buffer without mass");
    int64_t* slots = (int64_t*)malloc(sizeof(int64_t) * 70);
    float* many = (float*)malloc(sizeof(float) * 70);
    for (int k = 0; k < 70; ++k) many[k] = (float)unit();
    if (oracle_replay_insert(w, M, 27, many, 5, 0.6f, slots) != (27 + 5) % M) FAIL("insert, wrapping");
    if (oracle_replay_insert(w, M, 3, many, 70, 0.6f, slots) != (3 + 70) % M) FAIL("insert, longer than the buffer");
    if (oracle_replay_insert(w, M, 3, many, 0, 0.6f, NULL) != 3) FAIL("insert, nothing");

    /* ---- actor loss and gradient */
    double *tgt = doubles(N, -1, 1), *base = doubles(N, -1, 1), *pen = doubles(N, 0, 1);
    double* grad = doubles(R * V, 0, 0);
    double loss = 0.0;
    if (oracle_actor_loss_grad(logits, R, V, stride, tokens, (int32_t)A, rho, tgt, base, pen, 0.01, 0.25, 1.0 / N, grad, &loss) != 0)
        FAIL("actor");
    if (oracle_actor_loss_grad(logits, R, V, stride, tokens, (int32_t)A, rho, tgt, base, NULL, 0.01, 0.0, 1.0 / N, NULL, &loss) != 0)
        FAIL("actor, loss only");

    free(logits); free(tokens); free(tl); free(te); free(sl); free(se); free(lm); free(rw); free(v); free(q);
    free(boot); free(tg); free(td); free(rho); free(ret); free(lab); free(sp); free(tp); free(w); free(pr);
    free(quant); free(u); free(drawn); free(prob); free(none); free(slots); free(many); free(tgt); free(base);
    free(pen); free(grad);
    puts("ok");
    return 0;
}
