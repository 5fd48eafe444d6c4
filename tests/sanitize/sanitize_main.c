/*
 * Driver for a sanitizer build of the host-side code: calls every function of the CPU oracle
 * (specee_ref.c) and the host-side scheduler of the library (csrc/sched.cpp) on small seeded inputs, so that
 * AddressSanitizer / UndefinedBehaviorSanitizer see every loop and index computation run.  TEST INFRASTRUCTURE
 * ONLY.  It checks no values (the pin tests do that); it succeeds when the sanitizers stay silent.
 * Built and run by build_and_run.py beside this file.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/specee.h"

/* oracle entry points (specee_ref.c has no header: it shares nothing with the library) */
int specee_predict_ref(int, int, int, int, double, float, int, const uint16_t *, const uint16_t *, const uint16_t *,
                       const int32_t *, const float *, const uint16_t *, const uint16_t *, const uint16_t *,
                       const uint16_t *, double *, double *, double *, double *, int32_t *);
int specee_predict_q4_ref(int, int, int, int, double, float, int, const uint16_t *, const uint16_t *, const uint32_t *,
                          const uint16_t *, const uint16_t *, int, const int32_t *, const float *, const uint16_t *,
                          const uint16_t *, const uint16_t *, const uint16_t *, double *, double *, double *, double *,
                          int32_t *);
int specee_predict_sweep_ref(int, int, int, int, double, float, int, int, const uint16_t *, const uint16_t *,
                             const uint16_t *, const int32_t *, const float *, const uint16_t *, const uint16_t *,
                             const uint16_t *, const uint16_t *, const int32_t *, double *, double *, double *,
                             int32_t *, int32_t *);
int specee_merge_ref(const int32_t *, int, int32_t *, int, int32_t *, int32_t *);
int specee_predict_tree_ref(int, int, int, int, double, float, int, int, int, const uint16_t *, const uint16_t *,
                            const uint16_t *, const int32_t *, const int32_t *, const float *, const uint16_t *,
                            const uint16_t *, const uint16_t *, const uint16_t *, int32_t *, int32_t *, int32_t *,
                            double *, double *, double *, double *, int32_t *, int32_t *);
int lm_head_gemv_ref(int, int, double, int, const uint16_t *, const uint16_t *, const uint16_t *, double *);
int lm_head_rows_ref(int, int, double, int, const uint16_t *, const uint16_t *, const uint16_t *, const int32_t *, int,
                     double *);
int specee_verify_ref(int, int, int, double, int, const uint16_t *, const uint16_t *, const uint16_t *,
                      const int32_t *, int32_t *, double *, int32_t *);
int lm_head_gemv_q4_ref(int, int, double, int, const uint16_t *, const uint16_t *, const uint32_t *, const uint16_t *,
                        const uint16_t *, int, double *);
int specee_verify_q4_ref(int, int, int, double, int, const uint16_t *, const uint16_t *, const uint32_t *,
                         const uint16_t *, const uint16_t *, int, const int32_t *, int32_t *, double *, int32_t *);
int specee_predict_tree_q4_ref(int, int, int, int, double, float, int, int, int, const uint16_t *, const uint16_t *,
                               const uint32_t *, const uint16_t *, const uint16_t *, int, const int32_t *,
                               const int32_t *, const float *, const uint16_t *, const uint16_t *, const uint16_t *,
                               const uint16_t *, int32_t *, int32_t *, int32_t *, double *, double *, double *,
                               int32_t *, int32_t *);
int specee_layer_loop_ref(int, int, int, int, double, float, int, int, const uint16_t *, const uint16_t *,
                          const uint16_t *, const int32_t *, const float *, const uint16_t *, const uint16_t *,
                          const uint16_t *, const uint16_t *, const int32_t *, double *, double *, double *, int32_t *,
                          int32_t *, int32_t *, int32_t *, int32_t *);
int specee_layer_loop_q4_ref(int, int, int, int, double, float, int, int, const uint16_t *, const uint16_t *,
                             const uint32_t *, const uint16_t *, const uint16_t *, int, const int32_t *, const float *,
                             const uint16_t *, const uint16_t *, const uint16_t *, const uint16_t *, const int32_t *,
                             double *, double *, double *, int32_t *, int32_t *, int32_t *, int32_t *, int32_t *);
int specee_schedule_ref(int, int, int, int, const int32_t *, const int32_t *, int32_t *, int32_t *);
void specee_ref_set_threads(int);

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) {
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state >> 8;
}
/* a finite half-precision pattern of moderate magnitude (exponent 11..15: 2^-4 .. 2) */
static uint16_t rnd_half(void) {
    return (uint16_t)(((rnd() & 1u) << 15) | ((11u + rnd() % 5u) << 10) | (rnd() & 0x3ffu));
}
static uint16_t *halves(size_t n) {
    uint16_t *p = (uint16_t *)malloc(sizeof(uint16_t) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) p[i] = rnd_half();
    return p;
}
#define CHECK(call)                                                        \
    do {                                                                   \
        int rc_ = (call);                                                  \
        if (rc_ != 0) {                                                    \
            fprintf(stderr, "%s returned %d\n", #call, rc_);               \
            return 1;                                                      \
        }                                                                  \
    } while (0)

int main(void) {
    enum { d = 64, V = 37, K = 3, H = 20, B = 5, L = 4, N = 9, G = 2, Mcap = 27, group = 16 };
    specee_ref_set_threads(2);
    uint16_t *hidden = halves((size_t)L * B * d), *gamma = halves(d), *lm = halves((size_t)V * d);
    uint16_t *W1 = halves((size_t)L * H * 3 * K), *b1 = halves((size_t)L * H), *w2 = halves((size_t)L * H), *b2 = halves(L);
    uint16_t *hid_tree = halves((size_t)G * N * d);
    uint32_t *qw = (uint32_t *)malloc(sizeof(uint32_t) * V * d / 8);
    for (int i = 0; i < V * d / 8; ++i) qw[i] = rnd() * 2654435761u;
    uint16_t *qs = halves((size_t)V * d / group), *qz = halves((size_t)V * d / group);
    int32_t ids[B * K], tids[G * N * K], parent[G * N];
    float prev[B * K], tprev[G * N * K];
    for (int i = 0; i < B * K; ++i) ids[i] = (int32_t)(rnd() % V), prev[i] = 1.0f / K;
    for (int i = 0; i < G * N * K; ++i) tids[i] = (int32_t)(rnd() % V), tprev[i] = 1.0f / K;
    for (int g = 0; g < G; ++g)
        for (int n = 0; n < N; ++n) parent[g * N + n] = n == 0 ? -1 : (int32_t)(rnd() % (uint32_t)n);
    double logits[L * B * K], probs[L * B * K], feats[B * 3 * K], scores[L * B], mx[B];
    int32_t ex[L * B], first[B], vt[L * B], hit[L * B], el[B], tok[B];
    CHECK(specee_predict_ref(d, V, K, H, 1e-5, 0.5f, B, hidden, gamma, lm, ids, prev, W1, b1, w2, b2, logits, probs, feats,
                             scores, ex));
    CHECK(specee_predict_ref(d, V, K, H, 1e-5, 0.5f, B, hidden, gamma, lm, ids, prev, W1, NULL, w2, NULL, logits, probs,
                             NULL, scores, ex));
    CHECK(specee_predict_q4_ref(d, V, K, H, 1e-5, 0.5f, B, hidden, gamma, qw, qs, qz, group, ids, prev, W1, b1, w2, b2,
                                logits, probs, feats, scores, ex));
    int32_t active[L] = {1, 0, 1, 1};
    CHECK(specee_predict_sweep_ref(d, V, K, H, 1e-5, 0.5f, L, B, hidden, gamma, lm, ids, NULL, W1, b1, w2, b2, active,
                                   logits, probs, scores, ex, first));
    CHECK(specee_layer_loop_ref(d, V, K, H, 1e-5, -1.0f, L, B, hidden, gamma, lm, ids, prev, W1, b1, w2, b2, active,
                                logits, probs, scores, ex, vt, hit, el, tok));
    CHECK(specee_layer_loop_q4_ref(d, V, K, H, 1e-5, -1.0f, L, B, hidden, gamma, qw, qs, qz, group, ids, prev, W1, b1,
                                   w2, b2, active, logits, probs, scores, ex, vt, hit, el, tok));
    int32_t merged[G * Mcap], M[G], cols[G * N * K], texit[G * N], tpath[G * N];
    double Z[G * N * Mcap], tl[G * N * K], tp[G * N * K], ts[G * N];
    CHECK(specee_merge_ref(tids, N * K, merged, Mcap, M, cols));
    CHECK(specee_predict_tree_ref(d, V, K, H, 1e-5, 0.5f, G, N, Mcap, hid_tree, gamma, lm, tids, parent, tprev, W1, b1,
                                  w2, b2, merged, M, cols, Z, tl, tp, ts, texit, tpath));
    CHECK(specee_predict_tree_q4_ref(d, V, K, H, 1e-5, 0.5f, G, N, Mcap, hid_tree, gamma, qw, qs, qz, group, tids, parent,
                                     tprev, W1, b1, w2, b2, merged, M, cols, tl, tp, ts, texit, tpath));
    double *full = (double *)malloc(sizeof(double) * B * V);
    CHECK(lm_head_gemv_ref(d, V, 1e-5, B, hidden, gamma, lm, full));
    CHECK(lm_head_gemv_q4_ref(d, V, 1e-5, B, hidden, gamma, qw, qs, qz, group, full));
    int32_t rows[4] = {0, V - 1, 5, 5};
    CHECK(lm_head_rows_ref(d, V, 1e-5, B, hidden, gamma, lm, rows, 4, full));
    CHECK(specee_verify_ref(d, V, K, 1e-5, B, hidden, gamma, lm, ids, tok, mx, hit));
    CHECK(specee_verify_q4_ref(d, V, K, 1e-5, B, hidden, gamma, qw, qs, qz, group, ids, tok, mx, hit));
    /* the oracle's scheduler and the library's, step by step */
    enum { T = 40, SL = 12 };
    int32_t seq[T], act[T * SL], cnt[T * SL], mask[SL] = {0}, now[SL];
    for (int t = 0; t < T; ++t) seq[t] = (int32_t)(rnd() % SL);
    mask[3] = 1;
    CHECK(specee_schedule_ref(SL, 5, 2, T, seq, mask, act, cnt));
    specee_sched s;
    CHECK(specee_sched_init(&s, SL, 5, 2));
    for (int t = 0; t < T; ++t) {
        if (specee_sched_active(&s, mask, now) < 0) return 1;
        if (memcmp(now, act + t * SL, sizeof(now)) != 0) {
            fprintf(stderr, "scheduler mismatch at token %d\n", t);
            return 1;
        }
        CHECK(specee_sched_push(&s, seq[t]));
    }
    free(hidden); free(gamma); free(lm); free(W1); free(b1); free(w2); free(b2); free(hid_tree); free(qw); free(qs);
    free(qz); free(full);
    puts("sanitized host code: ok");
    return 0;
}
