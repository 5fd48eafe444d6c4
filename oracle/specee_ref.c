/*
 * specee_ref.c -- CPU oracle for the SpecEE speculative early-exit predictor.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what
 * the GPU library computes.  It shares no code, header, table or helper with
 * the HIP path and must never be called from the product path: only the test
 * suite, the smoke check and the benchmark's cpu_baseline leg may load it.
 *
 * Everything is written out as the paper states it, in double precision, with
 * no blocking, fusion or reordering:
 *
 *   - "Feature Selection" (Sec. 4.3.1 of the paper, Speculation-based
 *     Lightweight Predictor / Approach): (1) speculative token logits are the
 *     1 x hidden_dim x num_speculatives product of the layer's hidden state
 *     with the LM-head rows of the speculative tokens; (2) local probabilities
 *     are the softmax over those logits only; (3) probability variation is the
 *     difference between this layer's local probabilities and the last layer's.
 *   - "Judgment Mechanism" (Sec. 4.3.2): a two-layer MLP (3K -> H, ReLU,
 *     H -> 1, sigmoid), exit iff the output passes the threshold (0.5).
 *   - "Verification Algorithm" (Sec. 4.3.3): full-vocabulary logits, exit iff
 *     the arg-max token is one of the speculative tokens.
 *   - "Context-aware Merged Mapping" (Sec. 6.2): all tree nodes are mapped
 *     onto one merged set of speculative tokens; a token path exits at the
 *     rearmost exit position of its tokens.
 *   - "Online Scheduling" (Sec. 5.3): circular queue of the last exit layers
 *     plus a per-layer neighbourhood counter.
 *   - the same predictor on a 4-bit group-quantised LM head (the quantised
 *     setting of the cloud evaluation, Sec. 7.1 / 7.3; the format is a reading).
 *
 * Readings where the paper is silent (each is a stated convention, not a
 * quotation): the model's final RMSNorm (weight gamma, epsilon eps) is applied
 * to the hidden state before the projection, as the LM head of a Llama model
 * expects; fp16 inputs are widened exactly and nothing is rounded in between;
 * the 3K features are laid out block-wise [logits | probs | variation] in the
 * caller's token order; the exit test is strict (score > threshold) and is
 * taken in single precision because that is the precision the scores are
 * delivered in; merged token ids are in ascending order.
 *
 * Parity pins (tests/test_oracle_*.py): every function below is checked
 * against something other than itself -- numpy/scipy library routines on the
 * same inputs, closed forms, brute force on tiny shapes and the structural
 * invariants the paper fixes (reduced logits == full-vocabulary logits at the
 * ids, softmax sums to one, merged tree == independent nodes, the predictor
 * parameter count of Sec. 7.4.2).  The paper prints no numeric example of a
 * feature vector or score, so no end-to-end printed value exists to pin to.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_OK 0
#define REF_EINVAL (-1)

/* Number of threads used by the loops over independent tokens / vocabulary
 * rows.  Threads only split independent outputs; each output's arithmetic and
 * summation order are unchanged. */
static int g_threads = 1;

void specee_ref_set_threads(int n) {
    g_threads = n < 1 ? 1 : n;
}

int specee_ref_get_threads(void) {
#ifdef _OPENMP
    return g_threads;
#else
    return 1;
#endif
}

/* IEEE 754 binary16 bit pattern -> double (exact). */
double specee_ref_half_to_double(uint16_t bits) {
    int sign = (bits >> 15) & 1;
    int exponent = (bits >> 10) & 0x1f;
    int mantissa = bits & 0x3ff;
    double v;
    if (exponent == 0) {
        v = ldexp((double)mantissa, -24); /* zero and subnormals */
    } else if (exponent == 31) {
        v = mantissa ? NAN : INFINITY;
    } else {
        v = ldexp(1.0 + (double)mantissa / 1024.0, exponent - 15);
    }
    return sign ? -v : v;
}

#define H2D(x) specee_ref_half_to_double(x)

/* Final RMSNorm scale of one hidden state: 1 / sqrt(mean(h^2) + eps). */
double specee_ref_rms_scale(const uint16_t *h, int d, double eps) {
    double ss = 0.0;
    for (int i = 0; i < d; ++i) {
        double v = H2D(h[i]);
        ss += v * v;
    }
    return 1.0 / sqrt(ss / (double)d + eps);
}

/* One logit: <RMSNorm(h) , w> = sum_i (h_i * r * gamma_i) * w_i. */
static double normed_dot(const uint16_t *h, const uint16_t *gamma, const uint16_t *w, int d, double r) {
    double acc = 0.0;
    for (int i = 0; i < d; ++i) {
        double x = H2D(h[i]) * r * H2D(gamma[i]);
        acc += x * H2D(w[i]);
    }
    return acc;
}

/* Softmax over K values (Sec. 4.3.1, feature (2)). */
static void local_softmax(const double *z, int K, double *p) {
    double m = z[0];
    for (int k = 1; k < K; ++k)
        if (z[k] > m) m = z[k];
    double s = 0.0;
    for (int k = 0; k < K; ++k) {
        p[k] = exp(z[k] - m);
        s += p[k];
    }
    for (int k = 0; k < K; ++k) p[k] /= s;
}

/* Features + MLP + judgment for one token whose K logits are known.
 * W1 is [H][3K] row-major (output x input), b1 [H] or NULL, w2 [H], b2 [1] or
 * NULL.  feat (3K doubles) may be NULL. */
static void score_token(const double *z, const float *prev, int K, int H, const uint16_t *W1, const uint16_t *b1,
                        const uint16_t *w2, const uint16_t *b2, float threshold, double *probs, double *feat_out,
                        double *score, int32_t *exit_flag) {
    double f[3 * 64];
    local_softmax(z, K, probs);
    for (int k = 0; k < K; ++k) {
        f[k] = z[k];
        f[K + k] = probs[k];
        f[2 * K + k] = probs[k] - (double)prev[k]; /* Sec. 4.3.1, feature (3) */
    }
    if (feat_out) memcpy(feat_out, f, sizeof(double) * 3 * K);
    double u = b2 ? H2D(b2[0]) : 0.0;
    for (int j = 0; j < H; ++j) {
        double a = b1 ? H2D(b1[j]) : 0.0;
        for (int t = 0; t < 3 * K; ++t) a += H2D(W1[(size_t)j * 3 * K + t]) * f[t];
        if (a < 0.0) a = 0.0; /* ReLU */
        u += H2D(w2[j]) * a;
    }
    double s = 1.0 / (1.0 + exp(-u)); /* sigmoid */
    *score = s;
    *exit_flag = ((float)s > threshold) ? 1 : 0;
}

static int check_dims(int d, int V, int K, int H, int n) {
    if (d < 1 || V < 1 || K < 1 || K > 64 || H < 1 || n < 0) return REF_EINVAL;
    return REF_OK;
}

/*
 * Predictor for B independent tokens at one layer (Sec. 4.3.1 + 4.3.2).
 *   hidden [B][d] fp16, gamma [d] fp16, lm_head [V][d] fp16 (row v = token v),
 *   ids [B][K], prev_probs [B][K] float.
 * Outputs (double): logits [B][K], probs [B][K], features [B][3K] (may be
 * NULL), scores [B]; exit_flags [B] int32.
 */
int specee_predict_ref(int d, int V, int K, int H, double eps, float threshold, int B, const uint16_t *hidden,
                       const uint16_t *gamma, const uint16_t *lm_head, const int32_t *ids, const float *prev_probs,
                       const uint16_t *W1, const uint16_t *b1, const uint16_t *w2, const uint16_t *b2,
                       double *logits, double *probs, double *features, double *scores, int32_t *exit_flags) {
    if (check_dims(d, V, K, H, B)) return REF_EINVAL;
    for (int i = 0; i < B * K; ++i)
        if (ids[i] < 0 || ids[i] >= V) return REF_EINVAL;
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int n = 0; n < B; ++n) {
        const uint16_t *h = hidden + (size_t)n * d;
        double r = specee_ref_rms_scale(h, d, eps);
        for (int k = 0; k < K; ++k) {
            const uint16_t *row = lm_head + (size_t)ids[n * K + k] * d; /* speculative LM-head row */
            logits[n * K + k] = normed_dot(h, gamma, row, d, r);
        }
        score_token(logits + n * K, prev_probs + n * K, K, H, W1, b1, w2, b2, threshold, probs + n * K,
                    features ? features + (size_t)n * 3 * K : NULL, scores + n, exit_flags + n);
    }
    return REF_OK;
}

/*
 * All layers of B tokens (the per-layer predictor applied down the stack; the
 * features of a layer use the local probabilities of the previous layer that
 * ran a predictor, Sec. 4.3.1 feature (3)).
 *   hidden [L][B][d]; ids [B][K] (fixed per token); prev0 [B][K] or NULL (= 0);
 *   W1 [L][H][3K], b1 [L][H] or NULL, w2 [L][H], b2 [L] or NULL;
 *   active [L] or NULL: layers with active[l]==0 run no predictor (outputs 0,
 *   exit 0) and leave the carried probabilities untouched.
 * The carried probabilities are rounded to float between layers because that
 * is the precision in which a caller hands them back.
 * first_exit [B]: smallest active layer with exit==1, or -1.
 */
/*
 * The predictor on a 4-bit group-quantised LM head (the paper combines SpecEE
 * with a weight-quantised model in its cloud evaluation, Sec. 7.1 "Quantization"
 * and Sec. 7.3; it fixes no storage format, so this is a stated reading):
 * element i of row v is stored as a code c in 0..15 -- bits 4*(i%8)..4*(i%8)+3
 * of 32-bit word i/8 of the row -- and stands for the weight
 *     w[v][i] = scale[v][i/group] * (c - zero[v][i/group]),
 * scale and zero being fp16 numbers per group of `group` consecutive elements.
 * Everything else is specee_predict_ref: the logits are taken against these
 * weights, nothing is rounded in between.
 */
/* One logit against row v of the quantised head: <RMSNorm(h), w_v> with
 * w_v[i] = scale[v][i/group] * (code[v][i] - zero[v][i/group]). */
static double normed_dot_q4(const uint16_t *h, const uint16_t *gamma, const uint32_t *qweight, const uint16_t *scales,
                            const uint16_t *zeros, int group, size_t v, int d, double r) {
    const int ng = d / group;
    double acc = 0.0;
    for (int i = 0; i < d; ++i) {
        const uint32_t word = qweight[v * (size_t)(d / 8) + (size_t)(i / 8)];
        const double code = (double)((word >> (4 * (i % 8))) & 15u);
        const double w = H2D(scales[v * ng + i / group]) * (code - H2D(zeros[v * ng + i / group]));
        const double x = H2D(h[i]) * r * H2D(gamma[i]);
        acc += x * w;
    }
    return acc;
}

int specee_predict_q4_ref(int d, int V, int K, int H, double eps, float threshold, int B, const uint16_t *hidden,
                          const uint16_t *gamma, const uint32_t *qweight, const uint16_t *scales,
                          const uint16_t *zeros, int group, const int32_t *ids, const float *prev_probs,
                          const uint16_t *W1, const uint16_t *b1, const uint16_t *w2, const uint16_t *b2,
                          double *logits, double *probs, double *features, double *scores, int32_t *exit_flags) {
    if (check_dims(d, V, K, H, B)) return REF_EINVAL;
    if (group < 8 || group % 8 != 0 || d % group != 0) return REF_EINVAL;
    for (int i = 0; i < B * K; ++i)
        if (ids[i] < 0 || ids[i] >= V) return REF_EINVAL;
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int n = 0; n < B; ++n) {
        const uint16_t *h = hidden + (size_t)n * d;
        double r = specee_ref_rms_scale(h, d, eps);
        for (int k = 0; k < K; ++k) {
            logits[n * K + k] = normed_dot_q4(h, gamma, qweight, scales, zeros, group, (size_t)ids[n * K + k], d, r);
        }
        score_token(logits + n * K, prev_probs + n * K, K, H, W1, b1, w2, b2, threshold, probs + n * K,
                    features ? features + (size_t)n * 3 * K : NULL, scores + n, exit_flags + n);
    }
    return REF_OK;
}

int specee_predict_sweep_ref(int d, int V, int K, int H, double eps, float threshold, int L, int B,
                             const uint16_t *hidden, const uint16_t *gamma, const uint16_t *lm_head,
                             const int32_t *ids, const float *prev0, const uint16_t *W1, const uint16_t *b1,
                             const uint16_t *w2, const uint16_t *b2, const int32_t *active, double *logits,
                             double *probs, double *scores, int32_t *exit_flags, int32_t *first_exit) {
    if (check_dims(d, V, K, H, B) || L < 0) return REF_EINVAL;
    float *carry = (float *)malloc(sizeof(float) * (size_t)(B * K > 0 ? B * K : 1));
    if (!carry) return REF_EINVAL;
    for (int i = 0; i < B * K; ++i) carry[i] = prev0 ? prev0[i] : 0.0f;
    for (int b = 0; b < B; ++b) first_exit[b] = -1;
    int rc = REF_OK;
    for (int l = 0; l < L && rc == REF_OK; ++l) {
        size_t o1 = (size_t)l * B;
        if (active && !active[l]) {
            for (int i = 0; i < B * K; ++i) logits[o1 * K + i] = probs[o1 * K + i] = 0.0;
            for (int b = 0; b < B; ++b) {
                scores[o1 + b] = 0.0;
                exit_flags[o1 + b] = 0;
            }
            continue;
        }
        rc = specee_predict_ref(d, V, K, H, eps, threshold, B, hidden + o1 * d, gamma, lm_head, ids, carry,
                                W1 + (size_t)l * H * 3 * K, b1 ? b1 + (size_t)l * H : NULL, w2 + (size_t)l * H,
                                b2 ? b2 + l : NULL, logits + o1 * K, probs + o1 * K, NULL, scores + o1,
                                exit_flags + o1);
        if (rc != REF_OK) break;
        for (int i = 0; i < B * K; ++i) carry[i] = (float)probs[o1 * K + i];
        for (int b = 0; b < B; ++b)
            if (exit_flags[o1 + b] && first_exit[b] < 0) first_exit[b] = l;
    }
    free(carry);
    return rc;
}

static int cmp_i32(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Merged speculative-token set of a token tree (Sec. 6.2): the distinct ids of
 * all nodes in ascending order, and for every (node, slot) the column of its
 * id in that set.  merged has room for cap entries; unused tail is -1.
 * Returns REF_EINVAL if the number of distinct ids exceeds cap (M_out is still
 * the true count).
 */
int specee_merge_ref(const int32_t *ids, int n, int32_t *merged, int cap, int32_t *M_out, int32_t *cols) {
    if (n < 0 || cap < 0) return REF_EINVAL;
    int32_t *tmp = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    if (!tmp) return REF_EINVAL;
    memcpy(tmp, ids, sizeof(int32_t) * (size_t)n);
    qsort(tmp, (size_t)n, sizeof(int32_t), cmp_i32);
    int M = 0;
    for (int i = 0; i < n; ++i)
        if (i == 0 || tmp[i] != tmp[i - 1]) tmp[M++] = tmp[i];
    *M_out = M;
    if (M > cap) {
        free(tmp);
        return REF_EINVAL;
    }
    for (int m = 0; m < cap; ++m) merged[m] = m < M ? tmp[m] : -1;
    for (int i = 0; i < n; ++i) {
        int c = -1;
        for (int m = 0; m < M; ++m)
            if (tmp[m] == ids[i]) c = m;
        cols[i] = c;
    }
    free(tmp);
    return REF_OK;
}

/*
 * Token tree under the merged mapping (Sec. 6.2).  G independent trees of N
 * nodes each:
 *   hidden [G][N][d], ids [G][N][K], parent [G][N] or NULL (-1 = root,
 *   parent < own index), prev_probs [G][N][K].
 * Every node is projected onto all M merged tokens of its tree
 * (Zfull [G][N][Mcap], may be NULL), then reads its own K columns.
 * path_exit [G][N] (may be NULL; requires parent): a path exits only when
 * every token on it exits (the rearmost exit position decides), i.e. the AND
 * of exit flags from the root down to the node.
 */
int specee_predict_tree_ref(int d, int V, int K, int H, double eps, float threshold, int G, int N, int Mcap,
                            const uint16_t *hidden, const uint16_t *gamma, const uint16_t *lm_head,
                            const int32_t *ids, const int32_t *parent, const float *prev_probs, const uint16_t *W1,
                            const uint16_t *b1, const uint16_t *w2, const uint16_t *b2, int32_t *merged,
                            int32_t *M_out, int32_t *cols, double *Zfull, double *logits, double *probs,
                            double *scores, int32_t *exit_flags, int32_t *path_exit) {
    if (check_dims(d, V, K, H, N) || G < 0 || Mcap < 1) return REF_EINVAL;
    if (path_exit && !parent) return REF_EINVAL;
    for (size_t i = 0; i < (size_t)G * N * K; ++i)
        if (ids[i] < 0 || ids[i] >= V) return REF_EINVAL;
    if (parent)
        for (int g = 0; g < G; ++g)
            for (int n = 0; n < N; ++n) {
                int32_t p = parent[(size_t)g * N + n];
                if (p < -1 || p >= n) return REF_EINVAL;
            }
    for (int g = 0; g < G; ++g) {
        const int32_t *gids = ids + (size_t)g * N * K;
        int32_t *gmerged = merged + (size_t)g * Mcap;
        int32_t *gcols = cols + (size_t)g * N * K;
        int rc = specee_merge_ref(gids, N * K, gmerged, Mcap, M_out + g, gcols);
        if (rc != REF_OK) return rc;
        int M = M_out[g];
        double *Z = (double *)malloc(sizeof(double) * (size_t)N * (size_t)(M > 0 ? M : 1));
        if (!Z) return REF_EINVAL;
#pragma omp parallel for num_threads(g_threads) schedule(static)
        for (int n = 0; n < N; ++n) {
            const uint16_t *h = hidden + ((size_t)g * N + n) * d;
            double r = specee_ref_rms_scale(h, d, eps);
            for (int m = 0; m < M; ++m)
                Z[(size_t)n * M + m] = normed_dot(h, gamma, lm_head + (size_t)gmerged[m] * d, d, r);
        }
        for (int n = 0; n < N; ++n) {
            size_t gn = (size_t)g * N + n;
            if (Zfull)
                for (int m = 0; m < Mcap; ++m) Zfull[gn * Mcap + m] = m < M ? Z[(size_t)n * M + m] : 0.0;
            for (int k = 0; k < K; ++k) logits[gn * K + k] = Z[(size_t)n * M + gcols[n * K + k]];
            score_token(logits + gn * K, prev_probs + gn * K, K, H, W1, b1, w2, b2, threshold, probs + gn * K,
                        NULL, scores + gn, exit_flags + gn);
        }
        free(Z);
        if (path_exit)
            for (int n = 0; n < N; ++n) {
                size_t gn = (size_t)g * N + n;
                int32_t p = parent[gn];
                path_exit[gn] = exit_flags[gn] && (p < 0 ? 1 : path_exit[(size_t)g * N + p]);
            }
    }
    return REF_OK;
}

/*
 * Full-vocabulary LM head on N hidden states: the search space the predictor
 * avoids and the verification step needs (Sec. 4.1 and 4.3.3).
 * out [N][V] double.
 */
int lm_head_gemv_ref(int d, int V, double eps, int N, const uint16_t *hidden, const uint16_t *gamma,
                     const uint16_t *lm_head, double *out) {
    if (d < 1 || V < 1 || N < 0) return REF_EINVAL;
    for (int n = 0; n < N; ++n) {
        const uint16_t *h = hidden + (size_t)n * d;
        double r = specee_ref_rms_scale(h, d, eps);
#pragma omp parallel for num_threads(g_threads) schedule(static)
        for (int v = 0; v < V; ++v) out[(size_t)n * V + v] = normed_dot(h, gamma, lm_head + (size_t)v * d, d, r);
    }
    return REF_OK;
}

/* The same, for a chosen list of vocabulary rows only: out [N][R]. */
int lm_head_rows_ref(int d, int V, double eps, int N, const uint16_t *hidden, const uint16_t *gamma,
                     const uint16_t *lm_head, const int32_t *rows, int R, double *out) {
    if (d < 1 || V < 1 || N < 0 || R < 0) return REF_EINVAL;
    for (int i = 0; i < R; ++i)
        if (rows[i] < 0 || rows[i] >= V) return REF_EINVAL;
    for (int n = 0; n < N; ++n) {
        const uint16_t *h = hidden + (size_t)n * d;
        double r = specee_ref_rms_scale(h, d, eps);
#pragma omp parallel for num_threads(g_threads) schedule(static)
        for (int i = 0; i < R; ++i)
            out[(size_t)n * R + i] = normed_dot(h, gamma, lm_head + (size_t)rows[i] * d, d, r);
    }
    return REF_OK;
}

/*
 * Verification (Sec. 4.3.3): global logits over the whole vocabulary; the
 * token with the highest logit (lowest id on ties) is accepted iff it is one
 * of the K speculative tokens.
 *   token [N] = arg-max id, max_logit [N], hit [N] = 1 iff token in ids[n][:].
 */
int specee_verify_ref(int d, int V, int K, double eps, int N, const uint16_t *hidden, const uint16_t *gamma,
                      const uint16_t *lm_head, const int32_t *ids, int32_t *token, double *max_logit,
                      int32_t *hit) {
    if (d < 1 || V < 1 || N < 0 || K < 1) return REF_EINVAL;
    double *y = (double *)malloc(sizeof(double) * (size_t)V);
    if (!y) return REF_EINVAL;
    for (int n = 0; n < N; ++n) {
        int rc = lm_head_gemv_ref(d, V, eps, 1, hidden + (size_t)n * d, gamma, lm_head, y);
        if (rc != REF_OK) {
            free(y);
            return rc;
        }
        int best = 0;
        for (int v = 1; v < V; ++v)
            if (y[v] > y[best]) best = v;
        token[n] = best;
        max_logit[n] = y[best];
        hit[n] = 0;
        for (int k = 0; k < K; ++k)
            if (ids[n * K + k] == best) hit[n] = 1;
    }
    free(y);
    return REF_OK;
}

/*
 * The full-vocabulary head, the verification and the token tree on the 4-bit
 * group-quantised LM head (the quantised setting of Sec. 7.1 / 7.3 runs the whole
 * predict -> verify loop, and the tree mapping, on the quantised model): the
 * definitions above with every LM-head row replaced by its dequantised weights
 * scale * (code - zero); nothing else changes and nothing is rounded.
 */
int lm_head_gemv_q4_ref(int d, int V, double eps, int N, const uint16_t *hidden, const uint16_t *gamma,
                        const uint32_t *qweight, const uint16_t *scales, const uint16_t *zeros, int group,
                        double *out) {
    if (d < 1 || V < 1 || N < 0) return REF_EINVAL;
    if (group < 8 || group % 8 != 0 || d % group != 0) return REF_EINVAL;
    for (int n = 0; n < N; ++n) {
        const uint16_t *h = hidden + (size_t)n * d;
        double r = specee_ref_rms_scale(h, d, eps);
#pragma omp parallel for num_threads(g_threads) schedule(static)
        for (int v = 0; v < V; ++v)
            out[(size_t)n * V + v] = normed_dot_q4(h, gamma, qweight, scales, zeros, group, (size_t)v, d, r);
    }
    return REF_OK;
}

int specee_verify_q4_ref(int d, int V, int K, double eps, int N, const uint16_t *hidden, const uint16_t *gamma,
                         const uint32_t *qweight, const uint16_t *scales, const uint16_t *zeros, int group,
                         const int32_t *ids, int32_t *token, double *max_logit, int32_t *hit) {
    if (d < 1 || V < 1 || N < 0 || K < 1) return REF_EINVAL;
    double *y = (double *)malloc(sizeof(double) * (size_t)V);
    if (!y) return REF_EINVAL;
    for (int n = 0; n < N; ++n) {
        int rc = lm_head_gemv_q4_ref(d, V, eps, 1, hidden + (size_t)n * d, gamma, qweight, scales, zeros, group, y);
        if (rc != REF_OK) {
            free(y);
            return rc;
        }
        int best = 0;
        for (int v = 1; v < V; ++v)
            if (y[v] > y[best]) best = v; /* strict: the lowest id wins a tie */
        token[n] = best;
        max_logit[n] = y[best];
        hit[n] = 0;
        for (int k = 0; k < K; ++k)
            if (ids[n * K + k] == best) hit[n] = 1;
    }
    free(y);
    return REF_OK;
}

int specee_predict_tree_q4_ref(int d, int V, int K, int H, double eps, float threshold, int G, int N, int Mcap,
                               const uint16_t *hidden, const uint16_t *gamma, const uint32_t *qweight,
                               const uint16_t *scales, const uint16_t *zeros, int group, const int32_t *ids,
                               const int32_t *parent, const float *prev_probs, const uint16_t *W1,
                               const uint16_t *b1, const uint16_t *w2, const uint16_t *b2, int32_t *merged,
                               int32_t *M_out, int32_t *cols, double *logits, double *probs, double *scores,
                               int32_t *exit_flags, int32_t *path_exit) {
    if (check_dims(d, V, K, H, N) || G < 0 || Mcap < 1) return REF_EINVAL;
    if (group < 8 || group % 8 != 0 || d % group != 0) return REF_EINVAL;
    if (path_exit && !parent) return REF_EINVAL;
    for (size_t i = 0; i < (size_t)G * N * K; ++i)
        if (ids[i] < 0 || ids[i] >= V) return REF_EINVAL;
    if (parent)
        for (int g = 0; g < G; ++g)
            for (int n = 0; n < N; ++n) {
                int32_t p = parent[(size_t)g * N + n];
                if (p < -1 || p >= n) return REF_EINVAL;
            }
    for (int g = 0; g < G; ++g) {
        int32_t *gmerged = merged + (size_t)g * Mcap;
        int32_t *gcols = cols + (size_t)g * N * K;
        int rc = specee_merge_ref(ids + (size_t)g * N * K, N * K, gmerged, Mcap, M_out + g, gcols);
        if (rc != REF_OK) return rc;
        const int M = M_out[g];
        double *Z = (double *)malloc(sizeof(double) * (size_t)N * (size_t)(M > 0 ? M : 1));
        if (!Z) return REF_EINVAL;
#pragma omp parallel for num_threads(g_threads) schedule(static)
        for (int n = 0; n < N; ++n) { /* every node against every merged token of its tree */
            const uint16_t *h = hidden + ((size_t)g * N + n) * d;
            double r = specee_ref_rms_scale(h, d, eps);
            for (int m = 0; m < M; ++m)
                Z[(size_t)n * M + m] = normed_dot_q4(h, gamma, qweight, scales, zeros, group, (size_t)gmerged[m], d, r);
        }
        for (int n = 0; n < N; ++n) { /* each node reads back its own K columns */
            size_t gn = (size_t)g * N + n;
            for (int k = 0; k < K; ++k) logits[gn * K + k] = Z[(size_t)n * M + gcols[n * K + k]];
            score_token(logits + gn * K, prev_probs + gn * K, K, H, W1, b1, w2, b2, threshold, probs + gn * K,
                        NULL, scores + gn, exit_flags + gn);
        }
        free(Z);
        if (path_exit)
            for (int n = 0; n < N; ++n) {
                size_t gn = (size_t)g * N + n;
                int32_t p = parent[gn];
                path_exit[gn] = exit_flags[gn] && (p < 0 ? 1 : path_exit[(size_t)g * N + p]);
            }
    }
    return REF_OK;
}

/*
 * The early-exit decode loop of one token down the layer stack (dataflow of
 * Sec. 4.3.3 with the active-predictor set of Sec. 5.3): at every layer whose
 * predictor is active the features are computed and scored; a positive
 * prediction is followed by verification on the full vocabulary; the token
 * leaves the model at the first layer where the verification accepts one of
 * the speculative tokens, and nothing is evaluated after that layer.
 *   hidden [L][B][d], ids [B][K] (fixed per token), prev0 [B][K] or NULL (= 0),
 *   W1 [L][H][3K], b1 [L][H] or NULL, w2 [L][H], b2 [L] or NULL,
 *   active [L] or NULL (= every layer).
 * Outputs per layer and token ([L][B]...; zero for layers that were not
 * evaluated -- inactive, or after the token's exit; ver_token is -1 where no
 * verification ran): logits, probs [L][B][K], scores, exit_flags, ver_token,
 * hit [L][B]; per token: exit_layer [B] (-1: the token ran the whole stack),
 * token [B] (the accepted token, or -1).
 * The probabilities carried to the next active layer are rounded to float, as
 * in the layer-by-layer sweep above.
 */
int specee_layer_loop_ref(int d, int V, int K, int H, double eps, float threshold, int L, int B,
                          const uint16_t *hidden, const uint16_t *gamma, const uint16_t *lm_head, const int32_t *ids,
                          const float *prev0, const uint16_t *W1, const uint16_t *b1, const uint16_t *w2,
                          const uint16_t *b2, const int32_t *active, double *logits, double *probs, double *scores,
                          int32_t *exit_flags, int32_t *ver_token, int32_t *hit, int32_t *exit_layer,
                          int32_t *token) {
    if (check_dims(d, V, K, H, B) || L < 0) return REF_EINVAL;
    for (size_t i = 0; i < (size_t)L * B * K; ++i) logits[i] = probs[i] = 0.0;
    for (size_t i = 0; i < (size_t)L * B; ++i) {
        scores[i] = 0.0;
        exit_flags[i] = 0;
        ver_token[i] = -1;
        hit[i] = 0;
    }
    int rc_all = REF_OK;
    /* threads split the tokens; a single token leaves them to the vocabulary loop of its verifications */
#pragma omp parallel for num_threads(g_threads) schedule(dynamic, 1) if (B > 1)
    for (int b = 0; b < B; ++b) {
        float carry[64];
        for (int k = 0; k < K; ++k) carry[k] = prev0 ? prev0[b * K + k] : 0.0f;
        exit_layer[b] = -1;
        token[b] = -1;
        for (int l = 0; l < L; ++l) {
            if (active && !active[l]) continue;
            const size_t o = (size_t)l * B + b;
            int rc = specee_predict_ref(d, V, K, H, eps, threshold, 1, hidden + o * d, gamma, lm_head, ids + b * K,
                                        carry, W1 + (size_t)l * H * 3 * K, b1 ? b1 + (size_t)l * H : NULL,
                                        w2 + (size_t)l * H, b2 ? b2 + l : NULL, logits + o * K, probs + o * K, NULL,
                                        scores + o, exit_flags + o);
            if (rc != REF_OK) {
                rc_all = rc;
                break;
            }
            for (int k = 0; k < K; ++k) carry[k] = (float)probs[o * K + k];
            if (!exit_flags[o]) continue;
            double mx;
            rc = specee_verify_ref(d, V, K, eps, 1, hidden + o * d, gamma, lm_head, ids + b * K, ver_token + o, &mx,
                                   hit + o);
            if (rc != REF_OK) {
                rc_all = rc;
                break;
            }
            if (hit[o]) {
                exit_layer[b] = l;
                token[b] = ver_token[o];
                break;
            }
        }
    }
    return rc_all;
}

/*
 * The early-exit decode loop on the 4-bit group-quantised LM head (Sec. 4.3.3 and 5.3 in the
 * weight-quantised setting of Sec. 7.1 / 7.3): specee_layer_loop_ref with the predictor and the
 * verification taken on rows scale * (code - zero).  Same outputs, same not-evaluated values.
 */
int specee_layer_loop_q4_ref(int d, int V, int K, int H, double eps, float threshold, int L, int B,
                             const uint16_t *hidden, const uint16_t *gamma, const uint32_t *qweight,
                             const uint16_t *scales, const uint16_t *zeros, int group, const int32_t *ids,
                             const float *prev0, const uint16_t *W1, const uint16_t *b1, const uint16_t *w2,
                             const uint16_t *b2, const int32_t *active, double *logits, double *probs,
                             double *scores, int32_t *exit_flags, int32_t *ver_token, int32_t *hit,
                             int32_t *exit_layer, int32_t *token) {
    if (check_dims(d, V, K, H, B) || L < 0) return REF_EINVAL;
    for (size_t i = 0; i < (size_t)L * B * K; ++i) logits[i] = probs[i] = 0.0;
    for (size_t i = 0; i < (size_t)L * B; ++i) {
        scores[i] = 0.0;
        exit_flags[i] = 0;
        ver_token[i] = -1;
        hit[i] = 0;
    }
    int rc_all = REF_OK;
#pragma omp parallel for num_threads(g_threads) schedule(dynamic, 1) if (B > 1)
    for (int b = 0; b < B; ++b) {
        float carry[64];
        for (int k = 0; k < K; ++k) carry[k] = prev0 ? prev0[b * K + k] : 0.0f;
        exit_layer[b] = -1;
        token[b] = -1;
        for (int l = 0; l < L; ++l) {
            if (active && !active[l]) continue;
            const size_t o = (size_t)l * B + b;
            int rc = specee_predict_q4_ref(d, V, K, H, eps, threshold, 1, hidden + o * d, gamma, qweight, scales, zeros,
                                           group, ids + b * K, carry, W1 + (size_t)l * H * 3 * K,
                                           b1 ? b1 + (size_t)l * H : NULL, w2 + (size_t)l * H, b2 ? b2 + l : NULL,
                                           logits + o * K, probs + o * K, NULL, scores + o, exit_flags + o);
            if (rc != REF_OK) {
                rc_all = rc;
                break;
            }
            for (int k = 0; k < K; ++k) carry[k] = (float)probs[o * K + k];
            if (!exit_flags[o]) continue;
            double mx;
            rc = specee_verify_q4_ref(d, V, K, eps, 1, hidden + o * d, gamma, qweight, scales, zeros, group,
                                      ids + b * K, ver_token + o, &mx, hit + o);
            if (rc != REF_OK) {
                rc_all = rc;
                break;
            }
            if (hit[o]) {
                exit_layer[b] = l;
                token[b] = ver_token[o];
                break;
            }
        }
    }
    return rc_all;
}

/*
 * Online scheduling (Sec. 5.3): a circular queue holds the exit layers of the
 * last Q tokens; counter[i] is the number of queued exit layers within
 * `radius` of layer i (itself included).  A layer's predictor is active when
 * the offline selection marks it or its counter is positive.
 *   exit_layers [T]: exit layer of token t (the layer whose predictor fired,
 *   or L-1 when the token ran the whole stack).
 *   offline_mask [L] or NULL.
 * Outputs: active [T][L] = predictor set used while decoding token t (built
 * from tokens before t); counters [T][L] the counter array at that moment.
 */
int specee_schedule_ref(int L, int Q, int radius, int T, const int32_t *exit_layers, const int32_t *offline_mask,
                        int32_t *active, int32_t *counters) {
    if (L < 1 || Q < 1 || radius < 0 || T < 0) return REF_EINVAL;
    for (int t = 0; t < T; ++t)
        if (exit_layers[t] < 0 || exit_layers[t] >= L) return REF_EINVAL;
    int32_t *queue = (int32_t *)malloc(sizeof(int32_t) * (size_t)Q);
    if (!queue) return REF_EINVAL;
    int filled = 0, head = 0;
    for (int t = 0; t < T; ++t) {
        for (int i = 0; i < L; ++i) {
            int c = 0;
            for (int q = 0; q < filled; ++q)
                if (abs(queue[q] - i) <= radius) ++c;
            counters[(size_t)t * L + i] = c;
            active[(size_t)t * L + i] = (c > 0 || (offline_mask && offline_mask[i])) ? 1 : 0;
        }
        queue[head] = exit_layers[t]; /* overwrite the oldest entry */
        head = (head + 1) % Q;
        if (filled < Q) ++filled;
    }
    free(queue);
    return REF_OK;
}
