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
    const int32_t *done;    // [B] or null (single layer only): tokens to skip
    // 4-bit group-quantised head (predict_q4 only; lm_head is then null): codes, per-group scale and zero-point
    const uint32_t *qweight;  // [V][d/8], element i in bits 4*(i%8).. of word i/8
    const half_t *qscales;    // [V][d/group]
    const half_t *qzeros;     // [V][d/group]
    int group;
    float *logits, *probs, *scores;
    int32_t *exit_flags;
};

hipError_t launch_predict(const PredictParams &p, hipStream_t s);
hipError_t launch_predict_q4(const PredictParams &p, hipStream_t s);
hipError_t launch_predict_sweep(const PredictParams &p, int32_t *first_exit, hipStream_t s);

// Persistent early-exit loop over the layers of B tokens (layer_loop.hip)
struct LoopParams {
    int d, V, K, H, L, B;
    float eps, threshold;
    const half_t *hidden;   // [L][B][d]
    const half_t *gamma;    // [d]
    const half_t *lm_head;  // [V][d] (fp16 head), or null with the quantised head below
    const uint32_t *qweight;            // [V][d/8] 4-bit codes, or null
    const half_t *qscales, *qzeros;     // [V][d/group]
    int group;
    const int32_t *ids;     // [B][K]
    const float *prev0;     // [B][K] or null
    const half_t *W1, *b1, *w2, *b2;  // leading layer dimension L
    const int32_t *active;  // [L] or null
    float *logits, *probs, *scores;            // [L][B][K], [L][B][K], [L][B]
    int32_t *exit_flags, *ver_token, *hit;     // [L][B]
    int32_t *exit_layer, *token, *status;      // [B]
    int rows_per_wg;        // LM-head rows per workgroup in a verification pass (set by the launcher)
    int32_t *arrive;        // [B] arrival counters of the groups, zero at launch
    int32_t *abort;         // [1] zero at launch; set by a group that could not meet
    float *cand_val;        // [2][B][workgroups per token] arg-max candidates
    int32_t *cand_idx;
    long long spin_limit;   // polls of the arrival counter before a meeting is given up
};
hipError_t launch_layer_loop(const LoopParams &p, int max_wgs, hipStream_t s);

#define SPECEE_KMAX_INTERNAL 16

// MFMA gather-contraction (gemm_kernels.hip)
struct GemmParams {
    int d, V, N;             // N hidden states per group
    float eps;
    const half_t *hidden;    // [G][N][d]
    const half_t *gamma;     // [d]
    const half_t *lm_head;   // [V][d]
    const int32_t *rowlist;  // [G][Mcap] LM-head row of output column m, or null (row = m)
    const int32_t *Mptr;     // [G] number of valid columns (device), or null (= Mcap)
    int Mcap;
    int dslice, S;           // k-range per workgroup (multiple of 64) and number of ranges
    float *out;              // FINAL: [N][V] logits; else partial sums [G][S][Npad][Mpad]
    float *ssq_part;         // [G][S][Npad] partial sums of h^2 (tree only)
    int Mpad, Npad;
    float *best_val;         // arg-max mode: [N][gridDim.x] candidates
    int32_t *best_idx;
    const int32_t *gate;     // arg-max mode: [N] or null; states with gate == 0 are not verified
    const int32_t *done;     // arg-max mode: [N] or null; states with done != 0 are not verified
    // fused merge (tree, N*K <= 1024): the kernel merges ids itself and workgroup (0,0) of each tree
    // publishes the results
    const int32_t *ids;      // [G][N][K] or null (rowlist / Mptr are then inputs)
    int K;
    int32_t *merged_out, *M_out, *cols_out;
    // whole-tree kernel with S > 1: the S workgroups of a tree leave their accumulators in `out`
    // ([G][S][256 threads][row tiles] quads) and `ssq_part` ([G][S][64]); the one that draws the last
    // ticket adds them up in slice order and scores the tree.  tickets [G] must be zero at launch.
    int32_t *tickets;
};

struct TreeFinishParams {
    int d, V, K, H, N, S, Mcap, Mpad, Npad;
    float eps, threshold;
    const float *partial;    // [G][S][Npad][Mpad]
    const float *ssq_part;   // [G][S][Npad]
    const int32_t *ids;      // [G][N][K]
    const int32_t *cols;     // [G][N][K]
    const int32_t *M_out;    // [G]
    const float *prev;       // [G][N][K]
    const half_t *W1, *b1, *w2, *b2;
    float *logits, *probs, *scores;
    int32_t *exit_flags;
    const int32_t *parent;   // [G][N] or null
    int32_t *path_exit;      // [G][N] or null
};

hipError_t launch_zero_i32(int32_t *p, int n, hipStream_t st);
hipError_t launch_merge(const int32_t *ids, int n, int G, int Mcap, int32_t *merged, int32_t *M_out, int32_t *cols,
                        hipStream_t st);
bool tree_gemm_can_fuse_merge(int n_ids);
hipError_t launch_tree_gemm(const GemmParams &p, int G, hipStream_t st);
hipError_t launch_tree_finish(const TreeFinishParams &p, int G, hipStream_t st);
bool tree_whole_supported(int N, int K, int Mcap);
int tree_whole_row_tiles(int Mcap);
hipError_t launch_tree_whole(const GemmParams &p, const TreeFinishParams &f, int G, hipStream_t st);
// Full-vocabulary head for several hidden states on the matrix cores
hipError_t launch_lm_head_gemm(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                               const half_t *lm_head, float *out, hipStream_t st);

// Full-vocabulary head, one hidden state per grid.y: out[n][v] = RMSNorm(h_n) . W[v]
hipError_t launch_lm_head_gemv(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                               const half_t *lm_head, float *out, hipStream_t s);

// Verification: arg-max candidates per workgroup, then the combining tail
int lm_head_gemv_workgroups(int V);
int lm_head_gemm_workgroups(int V);
hipError_t launch_lm_head_argmax_gemv(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                                      const half_t *lm_head, float *best_val, int32_t *best_idx, const int32_t *gate,
                                      const int32_t *done, hipStream_t s);
hipError_t launch_lm_head_argmax_gemm(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                                      const half_t *lm_head, float *best_val, int32_t *best_idx, const int32_t *gate,
                                      const int32_t *done, hipStream_t s);
hipError_t launch_verify_finish(const float *best_val, const int32_t *best_idx, int P, int N, const int32_t *ids,
                                int K, const int32_t *gate, int32_t *done, int32_t *token, float *max_logit,
                                int32_t *hit, hipStream_t s);

// Token trees on a 4-bit group-quantised head, one workgroup per tree (tree_q4.hip)
struct TreeQ4Params {
    int d, V, N, K, Mcap, group;
    float eps;
    const half_t *hidden;     // [G][N][d]
    const half_t *gamma;      // [d]
    const uint32_t *qweight;  // [V][d/8]
    const half_t *qscales;    // [V][d/group]
    const half_t *qzeros;     // [V][d/group]
    const int32_t *ids;       // [G][N][K]
    int32_t *merged_out, *M_out, *cols_out;
};
bool tree_q4_supported(int d, int N, int K, int Mcap, int group);
size_t tree_q4_lds_bytes(int d, int Mcap, int group);
hipError_t launch_tree_q4(const TreeQ4Params &p, const TreeFinishParams &f, int G, hipStream_t st);

// Full-vocabulary head on a 4-bit group-quantised head (lm_head_q4_kernels.hip): all logits, or arg-max
// candidates per workgroup for verification (combined by launch_verify_finish)
int lm_head_q4_workgroups(int V);
hipError_t launch_lm_head_q4(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                             const uint32_t *qweight, const half_t *scales, const half_t *zeros, int group,
                             float *out, hipStream_t s);
hipError_t launch_lm_head_q4_argmax(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                                    const uint32_t *qweight, const half_t *scales, const half_t *zeros, int group,
                                    float *best_val, int32_t *best_idx, const int32_t *gate, const int32_t *done,
                                    hipStream_t s);

}  // namespace specee
