/*
 * specee.h -- C ABI of the MI355X (gfx950) SpecEE speculative early-exit
 * predictor library, libspecee.so.
 *
 * The library implements the per-layer predictor of SpecEE ("Speculation-based
 * Lightweight Predictor", Sec. 4.3 of the paper), its token-tree variant
 * ("Context-aware Merged Mapping", Sec. 6.2), the full-vocabulary LM head the
 * predictor replaces (Sec. 4.1) with the verification step that follows a
 * positive prediction (Sec. 4.3.3), and the online half of the two-level
 * scheduler (Sec. 5.3).
 *
 * Conventions for every entry point
 * ---------------------------------
 *  - Half-precision tensors are IEEE binary16, passed as `specee_half`
 *    (a 16-bit pattern); all are row-major and must be 16-byte aligned.
 *  - Unless a parameter says HOST, pointers are DEVICE pointers owned by the
 *    caller.  Inputs are only read, outputs only written; the library never
 *    allocates or frees device memory and keeps no state between calls
 *    (one documented exception: specee_predict_tree_static).
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *    default stream) and the call returns without synchronising.  Outputs are
 *    valid once the stream has reached the end of the enqueued work.
 *  - Return value: SPECEE_OK or a negative specee_status.  Argument checks are
 *    made on the host before anything is enqueued.  Conditions only the device
 *    can see are reported in the outputs themselves: a speculative id outside
 *    [0, V) makes that token's logits, probs and score NaN and its exit flag 0;
 *    a tree whose merged set exceeds Mcap reports the true size in M_out and
 *    NaN / 0 in that tree's other outputs.  No kernel reads out of bounds in
 *    either case.  specee_status_word() folds these reports into one word.
 *  - Arithmetic: fp16 inputs are widened exactly; products and sums are fp32;
 *    outputs are fp32 / int32.  Reductions have a fixed order, so results are
 *    bit-identical from run to run.
 *  - Range: the matrix-core paths (token trees, the full head for more than
 *    two hidden states) form hidden * gamma in fp16 before splitting it exactly
 *    into two halves, so |hidden[i] * gamma[i]| must stay below 65504 there
 *    (beyond that the logits are inf / NaN); the other paths form it in fp32.
 *  - Calls that share a workspace must not overlap in time.
 */
#ifndef SPECEE_H
#define SPECEE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t specee_half;

#define SPECEE_KMAX 16    /* speculative tokens per token / node */
#define SPECEE_HMAX 2048  /* predictor hidden width */

typedef enum specee_status {
    SPECEE_OK = 0,
    SPECEE_EINVAL = -1,     /* bad size, NULL required pointer, aliasing outputs */
    SPECEE_EALIGN = -2,     /* a tensor pointer is not 16-byte aligned */
    SPECEE_EWORKSPACE = -3, /* workspace missing or smaller than specee_workspace_bytes() */
    SPECEE_EHIP = -4,       /* the HIP runtime refused a launch */
    SPECEE_ESCRATCH = -5    /* the call needs more scratch than specee_predict_tree_static owns */
} specee_status;

/* Model and predictor shape.  d: hidden size (multiple of 8), V: vocabulary,
 * K: speculative tokens per token (1..SPECEE_KMAX), H: predictor hidden width
 * (1..SPECEE_HMAX), eps: RMSNorm epsilon, threshold: exit iff score > threshold
 * (Sec. 4.3.2 uses 0.5). */
typedef struct specee_dims {
    int32_t d, V, K, H;
    float eps, threshold;
} specee_dims;

/* One predictor (Sec. 4.3.2: two-layer MLP, ReLU, sigmoid output).
 * W1 [H][3K] (output x input), w2 [H]; b1 [H] and b2 [1] may be NULL (the
 * parameter count of Sec. 7.4.2 has no bias terms).  The 3K inputs are
 * [K logits | K local probabilities | K probability variations], each block in
 * the caller's order of the K speculative tokens (Sec. 4.3.1).
 * For the multi-layer entry point every array has a leading layer dimension:
 * W1 [L][H][3K], w2 [L][H], b1 [L][H], b2 [L]. */
typedef struct specee_mlp {
    const specee_half *W1, *b1, *w2, *b2;
} specee_mlp;

/* Operation selector for specee_workspace_bytes(). */
typedef enum specee_op {
    SPECEE_OP_PREDICT = 0,
    SPECEE_OP_PREDICT_SWEEP = 1,
    SPECEE_OP_PREDICT_TREE = 2,
    SPECEE_OP_LM_HEAD = 3,
    SPECEE_OP_VERIFY = 4,
    SPECEE_OP_LAYER_LOOP = 5,
    SPECEE_OP_VERIFY_Q4 = 6,
    SPECEE_OP_PREDICT_TREE_Q4 = 7
} specee_op;

/*
 * Per-layer predictor for B independent tokens (Sec. 4.3.1 features, Sec. 4.3.2
 * judgment).  For each token: final RMSNorm of the hidden state (weight gamma),
 * logits against the K LM-head rows named by ids, softmax over those K logits,
 * variation against prev_probs, MLP, sigmoid, threshold.
 *   hidden [B][d], gamma [d], lm_head [V][d] (row v = token v), ids [B][K],
 *   prev_probs [B][K] fp32 (local probabilities of the last layer that ran a
 *   predictor; zeros for the first).
 *   logits [B][K], probs [B][K], scores [B] fp32; exit_flags [B] int32 (0/1).
 * done (optional, device, [B]): tokens that already left the model at an earlier
 * layer (done[b] != 0, as maintained by specee_verify) are skipped on the device:
 * their LM-head rows are not read, logits are 0, probs repeat prev_probs (so the
 * layer-to-layer chain stays defined), score 0 and exit flag 0.  With done and
 * the gate of specee_verify a whole layer loop (predict -> verify -> next layer)
 * runs from one HIP graph without the host looking at a flag.
 * probs must not alias prev_probs.  Needs no workspace.
 */
int specee_predict(const specee_dims *dims, int B, const specee_half *hidden, const specee_half *gamma,
                   const specee_half *lm_head, const int32_t *ids, const float *prev_probs,
                   const specee_mlp *mlp /* HOST struct of device pointers */, const int32_t *done /* [B] or NULL */,
                   float *logits, float *probs, float *scores, int32_t *exit_flags, void *stream);

/*
 * specee_predict on a 4-bit group-quantised LM head (the paper runs SpecEE on
 * top of a weight-quantised model in its cloud evaluation, Sec. 7.1
 * "Quantization" and Sec. 7.3; it fixes no storage format, this one is the
 * library's reading).  Element i of row v is a code c in 0..15, stored in bits
 * 4*(i%8) .. 4*(i%8)+3 of 32-bit word i/8 of the row, and stands for the weight
 *     scales[v][i/group] * (c - zeros[v][i/group]).
 *   qweight [V][d/8] uint32, scales and zeros [V][d/group] fp16 (device);
 *   group: a multiple of 8 that divides d.  Everything else, including `done`,
 *   is as for specee_predict.  A speculative row is d/2 bytes instead of 2d.
 * Needs no workspace.
 */
int specee_predict_q4(const specee_dims *dims, int B, const specee_half *hidden, const specee_half *gamma,
                      const uint32_t *qweight, const specee_half *scales, const specee_half *zeros, int group,
                      const int32_t *ids, const float *prev_probs, const specee_mlp *mlp,
                      const int32_t *done /* [B] or NULL */, float *logits, float *probs, float *scores,
                      int32_t *exit_flags, void *stream);

/*
 * All L layers of B tokens in one call: layer l uses hidden[l], predictor l and
 * the local probabilities of the nearest earlier active layer (prev0, or zeros
 * if NULL, before the first).  Used when every layer's hidden state already
 * exists (collecting predictor training data or exit statistics, Sec. 5.3
 * offline scheduling and Sec. 7.4.4; benchmarking).
 *   hidden [L][B][d], ids [B][K], prev0 [B][K] or NULL, mlp with leading L,
 *   active [L] int32 or NULL (all active): inactive layers output zeros.
 *   logits/probs [L][B][K], scores/exit_flags [L][B],
 *   first_exit [B]: first active layer whose exit flag is 1, else -1.
 * Needs no workspace.
 */
int specee_predict_sweep(const specee_dims *dims, int L, int B, const specee_half *hidden,
                         const specee_half *gamma, const specee_half *lm_head, const int32_t *ids,
                         const float *prev0, const specee_mlp *mlp /* HOST */, const int32_t *active,
                         float *logits, float *probs, float *scores, int32_t *exit_flags, int32_t *first_exit,
                         void *stream);

/*
 * Token trees under the merged mapping (Sec. 6.2).  G independent trees of N
 * nodes; the N*K speculative ids of a tree are merged into their sorted
 * distinct set (M <= Mcap entries), all N nodes are projected onto the M
 * LM-head rows in one contraction, and each node reads back its K columns and
 * is scored like a single token.
 *   hidden [G][N][d], ids [G][N][K], prev_probs [G][N][K],
 *   parent [G][N] or NULL: -1 for a root, otherwise an index smaller than the
 *   node's own.
 *   merged_ids [G][Mcap] ascending, tail -1; M_out [G]; cols [G][N][K] with
 *   merged_ids[g][cols[g][n][k]] == ids[g][n][k];
 *   logits/probs [G][N][K], scores/exit_flags [G][N];
 *   path_exit [G][N] or NULL (needs parent): 1 iff the node and all its
 *   ancestors exit -- a token path exits at the rearmost exit of its tokens.
 * Limits: N*K <= 4096, Mcap <= 4096.  Workspace: SPECEE_OP_PREDICT_TREE with
 * n = G*N.
 */
int specee_predict_tree(const specee_dims *dims, int G, int N, int Mcap, const specee_half *hidden,
                        const specee_half *gamma, const specee_half *lm_head, const int32_t *ids,
                        const int32_t *parent, const float *prev_probs, const specee_mlp *mlp /* HOST */,
                        int32_t *merged_ids, int32_t *M_out, int32_t *cols, float *logits, float *probs,
                        float *scores, int32_t *exit_flags, int32_t *path_exit, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * specee_predict_tree for callers that cannot allocate device memory or hand in a
 * workspace -- code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, outputs and results as specee_predict_tree,
 * without `workspace`: partial sums, tickets and the like live in an array of
 * SPECEE_STATIC_SCRATCH_BYTES that is part of the library's device code (every GPU
 * the library runs on holds its own copy until the process ends).  The call
 * allocates and frees nothing, on the host or on the device, and enqueues kernels
 * only (what must start at zero is cleared by a kernel).
 * A call whose launch shape needs more scratch than that returns SPECEE_ESCRATCH
 * and enqueues nothing.  What a call needs: nothing with 20 or more trees of at
 * most 64 nodes, N*K <= 1024 and Mcap <= 256 when there is no room for d-slices;
 * otherwise about 4 * ceil(d/256) * G*N * (Mcap rounded up to 16) bytes or less
 * (one 60-node tree at d = 4096, Mcap = 64: 0.25 MB; one 64-node tree at
 * d = 8192, Mcap = 256: 2.1 MB).
 * This is the one entry point with state: the per-device address of that array
 * is looked up on the first call on a device (that device must be current, as
 * for any call) and kept.  All calls on one GPU share the array, which keeps the
 * previous call's contents: calls on the same GPU must not overlap in time (two
 * streams, two threads), or they race on it.
 */
#define SPECEE_STATIC_SCRATCH_BYTES (18u << 20)
int specee_predict_tree_static(const specee_dims *dims, int G, int N, int Mcap, const specee_half *hidden,
                               const specee_half *gamma, const specee_half *lm_head, const int32_t *ids,
                               const int32_t *parent, const float *prev_probs,
                               const specee_mlp *mlp /* HOST */, int32_t *merged_ids, int32_t *M_out,
                               int32_t *cols, float *logits, float *probs, float *scores, int32_t *exit_flags,
                               int32_t *path_exit, void *stream);

/*
 * Full-vocabulary LM head with the final RMSNorm: the search space of earlier
 * early-exit predictors (Sec. 4.1) and the first half of verification
 * (Sec. 4.3.3).  out [N][V] fp32 = RMSNorm(hidden[n]) . lm_head[v].
 * dims->K and dims->H are ignored.  Workspace: SPECEE_OP_LM_HEAD with n = N.
 */
int lm_head_gemv(const specee_dims *dims, int N, const specee_half *hidden, const specee_half *gamma,
                 const specee_half *lm_head, float *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Verification (Sec. 4.3.3): arg-max of the full-vocabulary logits (lowest id
 * on ties) without materialising them, and whether it is one of the K
 * speculative ids.  token [N], max_logit [N] fp32, hit [N] int32.
 * gate (optional): verification follows a positive prediction only, so the exit
 * flags of specee_predict can be passed here; hidden states with gate[n] == 0
 * are skipped on the device -- token -1, max_logit 0, hit 0 -- and when no state
 * of a launch is gated in, the pass over the LM head is not made at all.  This
 * keeps the predict -> verify sequence free of host round trips.
 * done (optional, in/out): states with done[n] != 0 are skipped like gated-off
 * ones; where the verification hits, done[n] is set to 1 (the token leaves the
 * model here, Sec. 4.3.3), which switches off this token's later predict and
 * verify calls that are given the same array.
 * Workspace: SPECEE_OP_VERIFY with n = N.
 */
int specee_verify(const specee_dims *dims, int N, const specee_half *hidden, const specee_half *gamma,
                  const specee_half *lm_head, const int32_t *ids, const int32_t *gate /* [N] or NULL */,
                  int32_t *done /* [N] or NULL */, int32_t *token, float *max_logit, int32_t *hit, void *workspace,
                  size_t workspace_bytes, void *stream);

/*
 * lm_head_gemv and specee_verify on the 4-bit group-quantised LM head of
 * specee_predict_q4 (same format, same reading): the weight-quantised setting of
 * the paper's cloud evaluation runs the whole predict -> verify loop on the
 * quantised model (Sec. 7.1 "Quantization", Sec. 7.3).  Every LM-head row is
 * scale * (code - zero) per group; nothing else changes, and the dequantised
 * weights are never formed or rounded.  One pass over the head per hidden state
 * (d/2 + 4*d/group bytes per row).
 *   lm_head_gemv_q4: out [N][V] fp32.  Needs no workspace.
 *   specee_verify_q4: arguments and outputs as specee_verify (gate, done, token,
 *   max_logit, hit).  Workspace: SPECEE_OP_VERIFY_Q4 with n = N.
 * group: a multiple of 8 that divides d; qweight 4-byte aligned (16-byte aligned
 * rows and group % 32 == 0 take the faster path).
 */
int lm_head_gemv_q4(const specee_dims *dims, int N, const specee_half *hidden, const specee_half *gamma,
                    const uint32_t *qweight, const specee_half *scales, const specee_half *zeros, int group,
                    float *out, void *stream);
int specee_verify_q4(const specee_dims *dims, int N, const specee_half *hidden, const specee_half *gamma,
                     const uint32_t *qweight, const specee_half *scales, const specee_half *zeros, int group,
                     const int32_t *ids, const int32_t *gate /* [N] or NULL */, int32_t *done /* [N] or NULL */,
                     int32_t *token, float *max_logit, int32_t *hit, void *workspace, size_t workspace_bytes,
                     void *stream);

/*
 * specee_predict_tree on the 4-bit group-quantised LM head (Sec. 6.2 in the
 * quantised setting of Sec. 7.1 / 7.3): arguments, outputs and conventions as
 * specee_predict_tree, the head given as for specee_predict_q4.  The merged
 * contraction runs on the codes themselves (exact), each quantisation group's
 * sums being scaled and shifted by that group's scale and zero-point.
 * One workgroup per tree, so the call is meant for batches of trees; a single
 * tree is correct but takes one CU's time.  Needs no workspace.
 * Limits: N <= 64, N*K <= 1024, Mcap <= 128, group a multiple of 32 that divides
 * d, qweight 8-byte aligned; d and group such that the staged scales and
 * zero-points fit in LDS (d / group <= 128 at Mcap <= 64).  Other shapes return
 * SPECEE_EINVAL.
 */
int specee_predict_tree_q4(const specee_dims *dims, int G, int N, int Mcap, const specee_half *hidden,
                           const specee_half *gamma, const uint32_t *qweight, const specee_half *scales,
                           const specee_half *zeros, int group, const int32_t *ids, const int32_t *parent,
                           const float *prev_probs, const specee_mlp *mlp /* HOST */, int32_t *merged_ids,
                           int32_t *M_out, int32_t *cols, float *logits, float *probs, float *scores,
                           int32_t *exit_flags, int32_t *path_exit, void *stream);

/*
 * The early-exit decode loop of B tokens down L layers in one launch (Sec. 4.3.3:
 * a positive prediction is followed by verification, and the token leaves the
 * model at the first layer whose verification accepts a speculative token;
 * Sec. 5.3: only the layers of the active set run their predictor).  For each
 * token, layer by layer: specee_predict with the local probabilities of the
 * token's previous active layer; if the exit flag is set, specee_verify on the
 * same hidden state; on a hit the loop ends for that token.  Nothing is
 * evaluated after a token's exit, and the host takes no part in any decision.
 *   hidden [L][B][d] (every layer's hidden state exists before the call),
 *   ids [B][K], prev0 [B][K] or NULL (zeros), mlp with leading L (as for
 *   specee_predict_sweep), active [L] int32 or NULL (all layers active).
 *   logits/probs [L][B][K], scores/exit_flags [L][B]: as specee_predict wrote
 *   them; ver_token/hit [L][B]: arg-max token and hit flag where a verification
 *   ran, -1 / 0 elsewhere.  Layers that were not evaluated for a token
 *   (inactive, or after its exit) hold zeros (ver_token -1).
 *   exit_layer [B]: layer at which the token left the model, -1 if it ran the
 *   whole stack; token [B]: the accepted token or -1.
 *   status [B]: 0, or 1 if the token's workgroups could not meet (see below);
 *   its outputs from the failing layer on are then the not-evaluated values.
 * One group of workgroups per token stays on the GPU for the whole call and meets
 * once per verification, so the call needs every one of its workgroups resident
 * at once: the grid is sized to what the device holds, B must not exceed 64, and
 * the GPU should not be shared with other kernels while it runs.  Every wait in
 * the kernel is bounded: spin_limit polls (0: a default worth a few seconds), after
 * which the token is given up with status 1 -- the call never hangs.
 * Limits: d <= 8192, B <= 64.  Workspace: SPECEE_OP_LAYER_LOOP with n = B.
 */
int specee_layer_loop(const specee_dims *dims, int L, int B, const specee_half *hidden, const specee_half *gamma,
                      const specee_half *lm_head, const int32_t *ids, const float *prev0,
                      const specee_mlp *mlp /* HOST */, const int32_t *active, float *logits, float *probs,
                      float *scores, int32_t *exit_flags, int32_t *ver_token, int32_t *hit, int32_t *exit_layer,
                      int32_t *token, int32_t *status, long long spin_limit, void *workspace,
                      size_t workspace_bytes, void *stream);

/*
 * specee_layer_loop on the 4-bit group-quantised LM head of specee_predict_q4 (same
 * format, same reading): the weight-quantised setting of the paper's cloud
 * evaluation runs the whole predict -> verify loop on the quantised model
 * (Sec. 7.1 "Quantization", Sec. 7.3; loop: Sec. 4.3.3, Sec. 5.3).  Arguments,
 * outputs, status, bounded waits and residency requirements as specee_layer_loop;
 * the predictor is specee_predict_q4's and the verification specee_verify_q4's.
 * Limits: d <= 8192, B <= 64, K <= 8; group a multiple of 8 that divides d, qweight
 * 4-byte aligned.  Workspace: SPECEE_OP_LAYER_LOOP with n = B.
 */
int specee_layer_loop_q4(const specee_dims *dims, int L, int B, const specee_half *hidden, const specee_half *gamma,
                         const uint32_t *qweight, const specee_half *scales, const specee_half *zeros, int group,
                         const int32_t *ids, const float *prev0, const specee_mlp *mlp /* HOST */,
                         const int32_t *active, float *logits, float *probs, float *scores, int32_t *exit_flags,
                         int32_t *ver_token, int32_t *hit, int32_t *exit_layer, int32_t *token, int32_t *status,
                         long long spin_limit, void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of device workspace `op` needs for n tokens / nodes (Mcap: tree only).
 * Pure host function; 0 means none; (size_t)-1 means invalid arguments. */
size_t specee_workspace_bytes(int op, const specee_dims *dims, int n, int Mcap);

/*
 * Online scheduling (Sec. 5.3), host-side and allocation-free: the caller owns
 * the state.  A circular queue keeps the exit layers of the last Q tokens;
 * counter[i] counts queued exit layers within `radius` of layer i.  A layer's
 * predictor is active iff offline_mask[i] != 0 or counter[i] > 0.
 * All pointers are HOST pointers.
 */
#define SPECEE_SCHED_MAXQ 64
#define SPECEE_SCHED_MAXL 256
typedef struct specee_sched {
    int32_t L, Q, radius, filled, head;
    int32_t queue[SPECEE_SCHED_MAXQ];
    int32_t counter[SPECEE_SCHED_MAXL];
} specee_sched;

int specee_sched_init(specee_sched *s, int L, int Q, int radius);
/* Record the exit layer of the token just decoded (0..L-1). */
int specee_sched_push(specee_sched *s, int exit_layer);
/* active [L] (0/1) for the next token; offline_mask [L] or NULL. Returns the number of active layers. */
int specee_sched_active(const specee_sched *s, const int32_t *offline_mask, int32_t *active);

/*
 * Device status word.  What only the device can see is reported in the outputs
 * (see the conventions at the top): this call folds those reports into one
 * int32 on the device, enqueued on `stream` like everything else, so that a
 * caller reads one word after synchronising instead of scanning outputs:
 *   bit SPECEE_STATUS_INVALID_ID      some score is NaN: a speculative id of that
 *                                     token / node lies outside [0, V);
 *   bit SPECEE_STATUS_MERGE_OVERFLOW  some M_out[g] > Mcap (trees only).
 * scores [n_scores] fp32 as written by any predictor entry point; M_out [G] or
 * NULL (then G and Mcap are ignored); status [1] int32 is overwritten.
 */
#define SPECEE_STATUS_INVALID_ID 1
#define SPECEE_STATUS_MERGE_OVERFLOW 2
int specee_status_word(const float *scores, size_t n_scores, const int32_t *M_out, int G, int Mcap,
                       int32_t *status, void *stream);

/*
 * Measurement aid, not part of the method: copies `bytes` (multiple of 16,
 * 16-byte aligned device pointers) with a plain streaming kernel, so that
 * per-dispatch hardware byte counters can be calibrated against a transfer of
 * known size.
 */
int specee_calib_copy(void *dst, const void *src, size_t bytes, void *stream);

const char *specee_strerror(int status);
int specee_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPECEE_H */
