// Per-node tail of the token-tree predictor, shared by the stand-alone finish
// kernels and by the whole-tree contraction kernel: given a node's K logits it
// runs the feature/MLP/judgment tail (paper Sec. 4.3.1-4.3.2) on one wavefront
// and writes the node's outputs.  Eight hidden units per lane stay in registers
// across nodes when the predictor has the common shape (K in {4, 8}, H <= 512).
#pragma once
#include "device_utils.h"
#include "kernels.h"
#include "predictor_tail.h"

namespace specee {

constexpr int kFinishUnits = 8;  // hidden units per lane held in registers (H <= 512)

template <int KC>
struct FinishRows {
    MlpRow<KC> rows[KC <= 8 ? kFinishUnits : 1];
    bool regs;
    float b2;
};

template <int KC>
__device__ __forceinline__ void finish_load_rows(FinishRows<KC> &fr, const TreeFinishParams &p, int lane) {
    fr.regs = (p.K == KC) && (p.H <= kFinishUnits * kWave) && KC <= 8;
    if (fr.regs) {
#pragma unroll
        for (int u = 0; u < kFinishUnits; ++u)
            mlp_row_load<KC>(fr.rows[u], p.W1, p.b1, p.w2, p.K, p.H, lane + u * kWave);
    }
    fr.b2 = p.b2 ? (float)p.b2[0] : 0.f;
}

// One wavefront scores node gn from its normalised logits z (NaN = invalid) and previous
// probabilities; writes logits, probs, score and exit flag; returns the exit flag (all lanes).
template <int KC>
__device__ __forceinline__ int finish_score_node(FinishRows<KC> &fr, const TreeFinishParams &p, size_t gn,
                                                 const float (&z)[KC], const float (&prev)[KC], int lane) {
    const int K = p.K, H = p.H;
    float pr[KC];
    local_softmax<KC>(z, K, pr);
    bool poisoned = false;  // a NaN logit (invalid id / overflowing merged set) poisons the whole node
#pragma unroll
    for (int k = 0; k < KC; ++k)
        if (k < K && z[k] != z[k]) poisoned = true;

    float part = 0.f;
    if (fr.regs) {
        // keep the rows packed as fp16 across nodes: without this the compiler widens all of them to
        // fp32 outside the node loop and runs out of registers
#pragma unroll
        for (int u = 0; u < kFinishUnits; ++u)
#pragma unroll
            for (int q = 0; q < (3 * KC) / 4; ++q)
                asm volatile("" : "+v"(fr.rows[u].w1[q].x), "+v"(fr.rows[u].w1[q].y));
#pragma unroll
        for (int u = 0; u < kFinishUnits; ++u)
            if (lane + u * kWave < H) part += mlp_unit<KC>(fr.rows[u], p.W1, K, lane + u * kWave, z, pr, prev);
    } else {
        for (int j = lane; j < H; j += kWave) {
            MlpRow<KC> row;
            mlp_row_load<KC>(row, p.W1, p.b1, p.w2, K, H, j);
            part += mlp_unit<KC>(row, p.W1, K, j, z, pr, prev);
        }
    }
    part = wave_sum(part);
    const float sc = sigmoidf(fr.b2 + part);
    const int ex = (sc > p.threshold) ? 1 : 0;
    if (lane == 0) {
        p.scores[gn] = sc;
        p.exit_flags[gn] = ex;
    }
    if (lane < K) {
        float zl = 0.f, pl = 0.f;
#pragma unroll
        for (int k = 0; k < KC; ++k)
            if (k == lane) {
                zl = z[k];
                pl = pr[k];
            }
        p.logits[gn * K + lane] = poisoned ? quiet_nan() : zl;
        p.probs[gn * K + lane] = pl;
    }
    return ex;
}

// Path rule from exit flags in LDS (paper Sec. 6.2): a token path exits only if every token on it
// exits.  Parents precede children, so at most N steps; a malformed parent refuses the path.
__device__ __forceinline__ void finish_paths(const int32_t *exit_lds, const int32_t *par, int N, int tid,
                                             int threads, int32_t *path_out) {
    for (int n = tid; n < N; n += threads) {
        int cur = n, ok = 1;
        for (int step = 0; step < N && cur >= 0; ++step) {
            ok &= exit_lds[cur];
            int up = par[cur];
            if (up >= cur) {
                ok = 0;
                break;
            }
            cur = up;
        }
        path_out[n] = ok;
    }
}

}  // namespace specee
