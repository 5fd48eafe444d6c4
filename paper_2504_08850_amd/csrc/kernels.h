// Host-visible launch interface of the gfx950 kernels.  The C ABI in
// specee_api.hip validates arguments and lays out the workspace; the launchers
// declared here only choose a specialisation and enqueue.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace specee {

typedef _Float16 half_t;

struct PredictParams {
    int d, V, K, H;
    float eps, threshold;
    int B, L;
    const half_t *hidden;   // [L][B][d]
    const half_t *gamma;    // [d]
    const half_t *lm_head;  // [V][d]
    const int32_t *ids;     // [B][K] (shared by all layers)
    const float *prev;      // [B][K] or null
    const half_t *W1, *b1, *w2, *b2;  // leading layer dimension L
    const int32_t *active;  // [L] or null (sweep only)
    float *logits, *probs, *scores;
    int32_t *exit_flags;
};

hipError_t launch_predict(const PredictParams &p, hipStream_t s);
hipError_t launch_predict_sweep(const PredictParams &p, int32_t *first_exit, hipStream_t s);

// Full-vocabulary head, one hidden state per grid.y: out[n][v] = RMSNorm(h_n) . W[v]
hipError_t launch_lm_head_gemv(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                               const half_t *lm_head, float *out, hipStream_t s);

}  // namespace specee
