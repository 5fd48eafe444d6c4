// C ABI of libspecee.so: host-side argument checks, workspace layout and
// kernel launches.  See include/specee.h for the contract of every entry point.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/specee.h"
#include "kernels.h"

using namespace specee;

namespace {

inline bool misaligned(const void *p) {
    return (reinterpret_cast<uintptr_t>(p) & 15u) != 0;
}

int check_dims(const specee_dims *dm, bool need_predictor) {
    if (!dm) return SPECEE_EINVAL;
    if (dm->d < 8 || (dm->d & 7) || dm->d > 16384 || dm->V < 1) return SPECEE_EINVAL;
    if (need_predictor) {
        if (dm->K < 1 || dm->K > SPECEE_KMAX || dm->H < 1 || dm->H > SPECEE_HMAX) return SPECEE_EINVAL;
    }
    if (!(dm->eps >= 0.f)) return SPECEE_EINVAL;
    return SPECEE_OK;
}

int check_mlp(const specee_mlp *m) {
    if (!m || !m->W1 || !m->w2) return SPECEE_EINVAL;
    if (misaligned(m->W1) || misaligned(m->w2) || misaligned(m->b1)) return SPECEE_EALIGN;
    return SPECEE_OK;
}

const half_t *H(const specee_half *p) {
    return reinterpret_cast<const half_t *>(p);
}

// d-slices of the tree contraction.  A single tree is latency-bound: slices of ~256 elements spread
// it over many CUs.  With many trees per call the grid is already full, and fewer, longer slices
// mean fewer partial sums to write and re-read.  Slices are multiples of 64; at most 128 of them.
struct TreeSplit {
    int S, dslice;
};
int tree_max_slices(int d) {
    int max_S = (d + 255) / 256;
    return max_S > 128 ? 128 : max_S;
}
TreeSplit tree_split(int d, int n_total, int N, int Mcap) {
    const int max_S = tree_max_slices(d);
    const int G = N > 0 ? (n_total + N - 1) / N : 1;
    const long long wgs_per_slice = (long long)G * ((Mcap + 63) / 64) * ((N + 63) / 64);
    int S = (int)((768 + wgs_per_slice - 1) / wgs_per_slice);
    if (S > max_S) S = max_S;
    if (S < 1) S = 1;
    int dslice = (((d + S - 1) / S + 63) / 64) * 64;
    S = (d + dslice - 1) / dslice;
    return {S, dslice};
}

// Trees per launch from which one workgroup (or a few, see below) per tree beats spreading every
// tree over the whole GPU, and the workgroups per launch the ticketed d-slices aim for (one
// 512-thread workgroup per CU).  With more slices than kWholeMaxSlices the serial hand-off to the
// last workgroup costs more than the slices save.  Measured on MI355X with 60-node trees.
constexpr int kWholeTreeMinTrees = 20;
constexpr int kWholeTargetWgs = 256;
constexpr int kWholeMaxSlices = 8;

inline size_t align256(size_t b) {
    return (b + 255) & ~(size_t)255;
}

struct TreeLayout {
    int Mpad;
    size_t partial_off, ssq_off, total;
};
TreeLayout tree_layout(int S, int n_total, int Mcap) {
    TreeLayout L;
    L.Mpad = ((Mcap + 15) / 16) * 16;
    L.partial_off = 0;
    L.ssq_off = align256((size_t)S * n_total * L.Mpad * sizeof(float));
    L.total = L.ssq_off + align256((size_t)S * n_total * sizeof(float));
    return L;
}

// Workspace of the persistent layer loop: arrival counters [B] and the abort flag (cleared at every call),
// then two buffers of arg-max candidates, one (value, row) pair per workgroup.
constexpr int kLoopMaxTokens = 64;
constexpr int kLoopMaxWgs = 1024;
struct LoopLayout {
    size_t flags_off, val_off, idx_off, total;
    int flag_ints;
};
LoopLayout loop_layout(int B) {
    LoopLayout l;
    l.flag_ints = B + 1;
    l.flags_off = 0;
    l.val_off = align256((size_t)l.flag_ints * sizeof(int32_t));
    l.idx_off = l.val_off + align256((size_t)2 * kLoopMaxWgs * sizeof(float));
    l.total = l.idx_off + align256((size_t)2 * kLoopMaxWgs * sizeof(int32_t));
    return l;
}

// Workspace of the whole-tree kernel when S > 1 workgroups share a tree: accumulators
// [G][S][256 threads x row tiles] quads, sums of squares [G][S][64], tickets [G].
size_t whole_tree_part_bytes(int G, int S, int Mcap) {
    return align256((size_t)G * S * 256 * tree_whole_row_tiles(Mcap) * 16);
}
size_t whole_tree_ssq_bytes(int G, int S) {
    return align256((size_t)G * S * 64 * sizeof(float));
}
size_t whole_tree_bytes(int G, int S, int Mcap) {
    return whole_tree_part_bytes(G, S, Mcap) + whole_tree_ssq_bytes(G, S) + align256((size_t)G * sizeof(int32_t));
}

}  // namespace

// Scratch memory of specee_predict_tree_static, the entry point for callers that cannot allocate.
// Every GPU that the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the address
// that kernels may use is looked up once per device, with that device current, and kept below.
static __device__ __align__(256) unsigned char scratch[SPECEE_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_ptr[kMaxDevices] = {nullptr};

// Device address of the current device's scratch array (looked up on the first call per device).
int static_scratch(void **base) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SPECEE_EHIP;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SPECEE_EHIP;
        scratch_ptr[dev] = ptr;
    }
    *base = scratch_ptr[dev];
    return SPECEE_OK;
}

}  // namespace

extern "C" {

int specee_version(void) {
    return 100;
}

const char *specee_strerror(int status) {
    switch (status) {
        case SPECEE_OK: return "success";
        case SPECEE_EINVAL: return "invalid argument";
        case SPECEE_EALIGN: return "tensor pointer is not 16-byte aligned";
        case SPECEE_EWORKSPACE: return "workspace missing or too small";
        case SPECEE_EHIP: return "HIP runtime refused the launch";
        case SPECEE_ESCRATCH: return "the call needs more scratch than the static buffer holds";
        default: return "unknown status";
    }
}

size_t specee_workspace_bytes(int op, const specee_dims *dm, int n, int Mcap) {
    if (n < 0) return (size_t)-1;
    switch (op) {
        case SPECEE_OP_PREDICT:
        case SPECEE_OP_PREDICT_SWEEP:
            return check_dims(dm, true) ? (size_t)-1 : 0;
        case SPECEE_OP_LM_HEAD:
            return check_dims(dm, false) ? (size_t)-1 : 0;
        case SPECEE_OP_VERIFY: {
            if (check_dims(dm, false)) return (size_t)-1;
            int P = n <= 2 ? lm_head_gemv_workgroups(dm->V) : lm_head_gemm_workgroups(dm->V);
            return 2 * align256((size_t)n * P * sizeof(float));
        }
        case SPECEE_OP_PREDICT_TREE_Q4:
            return check_dims(dm, true) ? (size_t)-1 : 0;
        case SPECEE_OP_VERIFY_Q4:
            if (check_dims(dm, false)) return (size_t)-1;
            return 2 * align256((size_t)n * lm_head_q4_workgroups(dm->V) * sizeof(float));
        case SPECEE_OP_LAYER_LOOP:
            if (check_dims(dm, true) || n > kLoopMaxTokens) return (size_t)-1;
            return loop_layout(n).total;
        case SPECEE_OP_PREDICT_TREE:
            if (check_dims(dm, true) || Mcap < 1 || Mcap > 4096) return (size_t)-1;
        {
            // the split depends on how n divides into trees: size for the finest one
            size_t need = tree_layout(tree_max_slices(dm->d), n, Mcap).total;
            // batches of small trees may run as a few d-slice workgroups per tree, at most
            // kWholeTargetWgs in all, each leaving its accumulators behind, plus one ticket per tree
            if (n >= kWholeTreeMinTrees && Mcap <= 256) {
                const size_t whole = whole_tree_bytes(kWholeTargetWgs, 1, Mcap) + align256((size_t)n * sizeof(int32_t));
                if (whole > need) need = whole;
            }
            return need;
        }
        default:
            return (size_t)-1;
    }
}

int specee_predict(const specee_dims *dm, int B, const specee_half *hidden, const specee_half *gamma,
                   const specee_half *lm_head, const int32_t *ids, const float *prev_probs, const specee_mlp *mlp,
                   const int32_t *done, float *logits, float *probs, float *scores, int32_t *exit_flags,
                   void *stream) {
    int rc = check_dims(dm, true);
    if (rc) return rc;
    if (B < 0) return SPECEE_EINVAL;
    if (B == 0) return SPECEE_OK;  // nothing to read or write: pointers may be NULL
    if ((rc = check_mlp(mlp))) return rc;
    if (!hidden || !gamma || !lm_head || !ids || !prev_probs || !logits || !probs || !scores || !exit_flags)
        return SPECEE_EINVAL;
    if (probs == prev_probs) return SPECEE_EINVAL;
    if (misaligned(hidden) || misaligned(gamma) || misaligned(lm_head)) return SPECEE_EALIGN;
    PredictParams p{};
    p.d = dm->d; p.V = dm->V; p.K = dm->K; p.H = dm->H; p.eps = dm->eps; p.threshold = dm->threshold;
    p.B = B; p.L = 1;
    p.hidden = H(hidden); p.gamma = H(gamma); p.lm_head = H(lm_head); p.ids = ids; p.prev = prev_probs;
    p.W1 = H(mlp->W1); p.b1 = H(mlp->b1); p.w2 = H(mlp->w2); p.b2 = H(mlp->b2);
    p.active = nullptr;
    p.done = done;
    p.logits = logits; p.probs = probs; p.scores = scores; p.exit_flags = exit_flags;
    return launch_predict(p, static_cast<hipStream_t>(stream)) == hipSuccess ? SPECEE_OK : SPECEE_EHIP;
}

int specee_predict_q4(const specee_dims *dm, int B, const specee_half *hidden, const specee_half *gamma,
                      const uint32_t *qweight, const specee_half *scales, const specee_half *zeros, int group,
                      const int32_t *ids, const float *prev_probs, const specee_mlp *mlp, const int32_t *done,
                      float *logits, float *probs, float *scores, int32_t *exit_flags, void *stream) {
    int rc = check_dims(dm, true);
    if (rc) return rc;
    if (B < 0 || group < 8 || group % 8 != 0 || dm->d % group != 0) return SPECEE_EINVAL;
    if (B == 0) return SPECEE_OK;
    if ((rc = check_mlp(mlp))) return rc;
    if (!hidden || !gamma || !qweight || !scales || !zeros || !ids || !prev_probs || !logits || !probs || !scores ||
        !exit_flags)
        return SPECEE_EINVAL;
    if (probs == prev_probs) return SPECEE_EINVAL;
    if (misaligned(hidden) || misaligned(gamma) || (reinterpret_cast<uintptr_t>(qweight) & 3) != 0)
        return SPECEE_EALIGN;
    PredictParams p{};
    p.d = dm->d; p.V = dm->V; p.K = dm->K; p.H = dm->H; p.eps = dm->eps; p.threshold = dm->threshold;
    p.B = B; p.L = 1;
    p.hidden = H(hidden); p.gamma = H(gamma); p.lm_head = nullptr; p.ids = ids; p.prev = prev_probs;
    p.qweight = qweight; p.qscales = H(scales); p.qzeros = H(zeros); p.group = group;
    p.W1 = H(mlp->W1); p.b1 = H(mlp->b1); p.w2 = H(mlp->w2); p.b2 = H(mlp->b2);
    p.active = nullptr;
    p.done = done;
    p.logits = logits; p.probs = probs; p.scores = scores; p.exit_flags = exit_flags;
    return launch_predict_q4(p, static_cast<hipStream_t>(stream)) == hipSuccess ? SPECEE_OK : SPECEE_EHIP;
}

int specee_predict_sweep(const specee_dims *dm, int L, int B, const specee_half *hidden, const specee_half *gamma,
                         const specee_half *lm_head, const int32_t *ids, const float *prev0, const specee_mlp *mlp,
                         const int32_t *active, float *logits, float *probs, float *scores, int32_t *exit_flags,
                         int32_t *first_exit, void *stream) {
    int rc = check_dims(dm, true);
    if (rc) return rc;
    if (B < 0 || L < 0 || L > 65535) return SPECEE_EINVAL;
    if (B == 0) return SPECEE_OK;
    if (L > 0 && (rc = check_mlp(mlp))) return rc;
    if (!first_exit) return SPECEE_EINVAL;
    if (L > 0 && (!hidden || !gamma || !lm_head || !ids || !logits || !probs || !scores || !exit_flags))
        return SPECEE_EINVAL;
    if (misaligned(hidden) || misaligned(gamma) || misaligned(lm_head)) return SPECEE_EALIGN;
    PredictParams p{};
    p.d = dm->d; p.V = dm->V; p.K = dm->K; p.H = dm->H; p.eps = dm->eps; p.threshold = dm->threshold;
    p.B = B; p.L = L;
    p.hidden = H(hidden); p.gamma = H(gamma); p.lm_head = H(lm_head); p.ids = ids; p.prev = prev0;
    p.W1 = H(mlp->W1); p.b1 = H(mlp->b1); p.w2 = H(mlp->w2); p.b2 = H(mlp->b2);
    p.active = active;
    p.logits = logits; p.probs = probs; p.scores = scores; p.exit_flags = exit_flags;
    return launch_predict_sweep(p, first_exit, static_cast<hipStream_t>(stream)) == hipSuccess ? SPECEE_OK
                                                                                              : SPECEE_EHIP;
}

int lm_head_gemv(const specee_dims *dm, int N, const specee_half *hidden, const specee_half *gamma,
                 const specee_half *lm_head, float *out, void *workspace, size_t workspace_bytes, void *stream) {
    (void)workspace;
    (void)workspace_bytes;
    int rc = check_dims(dm, false);
    if (rc) return rc;
    if (N < 0 || N > 65535) return SPECEE_EINVAL;
    if (N == 0) return SPECEE_OK;
    if (!hidden || !gamma || !lm_head || !out) return SPECEE_EINVAL;
    if (misaligned(hidden) || misaligned(gamma) || misaligned(lm_head)) return SPECEE_EALIGN;
    if (misaligned(out)) return SPECEE_EALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // one or two hidden states: stream the head once per state on the vector units;
    // more: one pass over the head on the matrix cores
    hipError_t e = (N <= 2) ? launch_lm_head_gemv(dm->d, dm->V, dm->eps, N, H(hidden), H(gamma), H(lm_head), out, st)
                            : launch_lm_head_gemm(dm->d, dm->V, dm->eps, N, H(hidden), H(gamma), H(lm_head), out, st);
    return e == hipSuccess ? SPECEE_OK : SPECEE_EHIP;
}

// Host-side checks shared by the tree entry points; nothing is dereferenced.
static int check_tree_args(const specee_dims *dm, int G, int N, int Mcap, const specee_half *hidden,
                           const specee_half *gamma, const specee_half *lm_head, const int32_t *ids,
                           const int32_t *parent, const float *prev_probs, const specee_mlp *mlp,
                           const int32_t *merged_ids, const int32_t *M_out, const int32_t *cols, const float *logits,
                           const float *probs, const float *scores, const int32_t *exit_flags,
                           const int32_t *path_exit) {
    int rc = check_dims(dm, true);
    if (rc) return rc;
    if (G < 0 || N < 1 || Mcap < 1 || Mcap > 4096 || (long long)N * dm->K > 4096) return SPECEE_EINVAL;
    if ((long long)G * N > (1 << 24) || G > 65535) return SPECEE_EINVAL;
    if (G == 0) return SPECEE_OK;
    if ((rc = check_mlp(mlp))) return rc;
    if (!hidden || !gamma || !lm_head || !ids || !prev_probs || !merged_ids || !M_out || !cols || !logits ||
        !probs || !scores || !exit_flags)
        return SPECEE_EINVAL;
    if (path_exit && !parent) return SPECEE_EINVAL;
    if (probs == prev_probs) return SPECEE_EINVAL;
    if (misaligned(hidden) || misaligned(gamma) || misaligned(lm_head)) return SPECEE_EALIGN;
    return SPECEE_OK;
}

// Shared body of the two tree entry points.  exact_fit: the workspace only has to hold what the
// launch shape chosen for this call needs (the static-scratch entry point); otherwise it has to be as
// large as specee_workspace_bytes() says, which covers every shape.
static int predict_tree_common(const specee_dims *dm, int G, int N, int Mcap, const specee_half *hidden,
                               const specee_half *gamma, const specee_half *lm_head, const int32_t *ids,
                               const int32_t *parent, const float *prev_probs, const specee_mlp *mlp,
                               int32_t *merged_ids, int32_t *M_out, int32_t *cols, float *logits, float *probs,
                               float *scores, int32_t *exit_flags, int32_t *path_exit, void *workspace,
                               size_t workspace_bytes, bool exact_fit, void *stream) {
    const int rc = check_tree_args(dm, G, N, Mcap, hidden, gamma, lm_head, ids, parent, prev_probs, mlp, merged_ids,
                                   M_out, cols, logits, probs, scores, exit_flags, path_exit);
    if (rc) return rc;
    if (G == 0) return SPECEE_OK;
    if (misaligned(workspace)) return SPECEE_EALIGN;
    const TreeSplit ts = tree_split(dm->d, G * N, N, Mcap);
    const TreeLayout lay = tree_layout(ts.S, G * N, Mcap);
    if (!exact_fit) {
        const size_t need = tree_layout(tree_max_slices(dm->d), G * N, Mcap).total;
        if (!workspace || workspace_bytes < need) return SPECEE_EWORKSPACE;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    float *partial = reinterpret_cast<float *>(ws + lay.partial_off);
    float *ssq_part = reinterpret_cast<float *>(ws + lay.ssq_off);

    GemmParams gp{};
    gp.d = dm->d; gp.V = dm->V; gp.N = N; gp.eps = dm->eps;
    gp.hidden = H(hidden); gp.gamma = H(gamma); gp.lm_head = H(lm_head);
    gp.rowlist = merged_ids; gp.Mptr = M_out; gp.Mcap = Mcap;
    gp.out = partial; gp.ssq_part = ssq_part; gp.Mpad = lay.Mpad; gp.Npad = N;
    gp.K = dm->K;
    gp.merged_out = merged_ids; gp.M_out = M_out; gp.cols_out = cols;

    TreeFinishParams fp{};
    fp.d = dm->d; fp.V = dm->V; fp.K = dm->K; fp.H = dm->H; fp.N = N; fp.Mcap = Mcap;
    fp.Mpad = lay.Mpad; fp.Npad = N; fp.eps = dm->eps; fp.threshold = dm->threshold;
    fp.partial = partial; fp.ssq_part = ssq_part; fp.ids = ids; fp.cols = cols; fp.M_out = M_out;
    fp.prev = prev_probs;
    fp.W1 = H(mlp->W1); fp.b1 = H(mlp->b1); fp.w2 = H(mlp->w2); fp.b2 = H(mlp->b2);
    fp.logits = logits; fp.probs = probs; fp.scores = scores; fp.exit_flags = exit_flags;
    fp.parent = parent; fp.path_exit = path_exit;

    // enough small trees to occupy the GPU with one workgroup each: a single launch does merge,
    // contraction over all of d, scoring and the path rule, and no partial sums touch memory
    if (G >= kWholeTreeMinTrees && tree_whole_supported(N, dm->K, Mcap)) {
        gp.ids = ids;
        // fewer trees than the GPU holds workgroups: S workgroups per tree, one d-slice each, and the
        // last to finish adds the slices up and scores the tree
        int S = kWholeTargetWgs / G;
        if (S > kWholeMaxSlices) S = kWholeMaxSlices;
        if (S < 1) S = 1;
        int dslice = (((dm->d + S - 1) / S + 127) / 128) * 128;
        S = (dm->d + dslice - 1) / dslice;
        const size_t part_bytes = whole_tree_part_bytes(G, S, Mcap), ssq_bytes = whole_tree_ssq_bytes(G, S);
        if (S > 1 && (!workspace || whole_tree_bytes(G, S, Mcap) > workspace_bytes)) {
            S = 1;  // one workgroup per tree over all of d needs no workspace at all
            dslice = ((dm->d + 127) / 128) * 128;
        }
        gp.dslice = dslice; gp.S = S;
        gp.out = reinterpret_cast<float *>(ws);
        gp.ssq_part = S > 1 ? reinterpret_cast<float *>(ws + part_bytes) : nullptr;
        gp.tickets = S > 1 ? reinterpret_cast<int32_t *>(ws + part_bytes + ssq_bytes) : nullptr;
        if (S > 1 && launch_zero_i32(gp.tickets, G, st) != hipSuccess) return SPECEE_EHIP;
        return launch_tree_whole(gp, fp, G, st) == hipSuccess ? SPECEE_OK : SPECEE_EHIP;
    }

    if (exact_fit && (!workspace || workspace_bytes < lay.total)) return SPECEE_EWORKSPACE;
    // few trees: split d over many workgroups; merge inside the contraction kernel (one launch less on the
    // latency path) unless that would repeat it too often
    const bool fuse = tree_gemm_can_fuse_merge(N * dm->K) && (long long)G * ts.S <= 64;
    if (!fuse && launch_merge(ids, N * dm->K, G, Mcap, merged_ids, M_out, cols, st) != hipSuccess) return SPECEE_EHIP;
    gp.ids = fuse ? ids : nullptr;
    gp.dslice = ts.dslice; gp.S = ts.S;
    if (launch_tree_gemm(gp, G, st) != hipSuccess) return SPECEE_EHIP;
    fp.S = ts.S;
    if (launch_tree_finish(fp, G, st) != hipSuccess) return SPECEE_EHIP;
    return SPECEE_OK;
}

int specee_predict_tree(const specee_dims *dm, int G, int N, int Mcap, const specee_half *hidden,
                        const specee_half *gamma, const specee_half *lm_head, const int32_t *ids,
                        const int32_t *parent, const float *prev_probs, const specee_mlp *mlp, int32_t *merged_ids,
                        int32_t *M_out, int32_t *cols, float *logits, float *probs, float *scores,
                        int32_t *exit_flags, int32_t *path_exit, void *workspace, size_t workspace_bytes,
                        void *stream) {
    return predict_tree_common(dm, G, N, Mcap, hidden, gamma, lm_head, ids, parent, prev_probs, mlp, merged_ids, M_out,
                               cols, logits, probs, scores, exit_flags, path_exit, workspace, workspace_bytes, false,
                               stream);
}

int specee_predict_tree_static(const specee_dims *dm, int G, int N, int Mcap, const specee_half *hidden,
                               const specee_half *gamma, const specee_half *lm_head, const int32_t *ids,
                               const int32_t *parent, const float *prev_probs, const specee_mlp *mlp,
                               int32_t *merged_ids, int32_t *M_out, int32_t *cols, float *logits, float *probs,
                               float *scores, int32_t *exit_flags, int32_t *path_exit, void *stream) {
    // argument errors first (they need no GPU), then the address of this device's scratch array
    int rc = check_tree_args(dm, G, N, Mcap, hidden, gamma, lm_head, ids, parent, prev_probs, mlp, merged_ids, M_out,
                             cols, logits, probs, scores, exit_flags, path_exit);
    if (rc) return rc;
    if (G == 0) return SPECEE_OK;
    void *base = nullptr;
    if ((rc = static_scratch(&base))) return rc;
    const int r = predict_tree_common(dm, G, N, Mcap, hidden, gamma, lm_head, ids, parent, prev_probs, mlp, merged_ids,
                                      M_out, cols, logits, probs, scores, exit_flags, path_exit, base,
                                      SPECEE_STATIC_SCRATCH_BYTES, true, stream);
    return r == SPECEE_EWORKSPACE ? SPECEE_ESCRATCH : r;
}

static int check_q4(const specee_dims *dm, const uint32_t *qweight, const specee_half *scales,
                    const specee_half *zeros, int group) {
    if (group < 8 || group % 8 != 0 || dm->d % group != 0) return SPECEE_EINVAL;
    if (!qweight || !scales || !zeros) return SPECEE_EINVAL;
    if ((reinterpret_cast<uintptr_t>(qweight) & 3) != 0) return SPECEE_EALIGN;
    return SPECEE_OK;
}

int lm_head_gemv_q4(const specee_dims *dm, int N, const specee_half *hidden, const specee_half *gamma,
                    const uint32_t *qweight, const specee_half *scales, const specee_half *zeros, int group,
                    float *out, void *stream) {
    int rc = check_dims(dm, false);
    if (rc) return rc;
    if (N < 0 || N > 65535) return SPECEE_EINVAL;
    if (group < 8 || group % 8 != 0 || dm->d % group != 0) return SPECEE_EINVAL;
    if (N == 0) return SPECEE_OK;
    if ((rc = check_q4(dm, qweight, scales, zeros, group))) return rc;
    if (!hidden || !gamma || !out) return SPECEE_EINVAL;
    if (misaligned(hidden) || misaligned(gamma)) return SPECEE_EALIGN;
    return launch_lm_head_q4(dm->d, dm->V, dm->eps, N, H(hidden), H(gamma), qweight, H(scales), H(zeros), group, out,
                             static_cast<hipStream_t>(stream)) == hipSuccess
               ? SPECEE_OK
               : SPECEE_EHIP;
}

int specee_verify_q4(const specee_dims *dm, int N, const specee_half *hidden, const specee_half *gamma,
                     const uint32_t *qweight, const specee_half *scales, const specee_half *zeros, int group,
                     const int32_t *ids, const int32_t *gate, int32_t *done, int32_t *token, float *max_logit,
                     int32_t *hit, void *workspace, size_t workspace_bytes, void *stream) {
    int rc = check_dims(dm, false);
    if (rc) return rc;
    if (N < 0 || N > 65535 || dm->K < 1 || dm->K > SPECEE_KMAX) return SPECEE_EINVAL;
    if (group < 8 || group % 8 != 0 || dm->d % group != 0) return SPECEE_EINVAL;
    if (N == 0) return SPECEE_OK;
    if ((rc = check_q4(dm, qweight, scales, zeros, group))) return rc;
    if (!hidden || !gamma || !ids || !token || !max_logit || !hit) return SPECEE_EINVAL;
    if (misaligned(hidden) || misaligned(gamma) || misaligned(workspace)) return SPECEE_EALIGN;
    const int P = lm_head_q4_workgroups(dm->V);
    const size_t half_ws = align256((size_t)N * P * sizeof(float));
    if (!workspace || workspace_bytes < 2 * half_ws) return SPECEE_EWORKSPACE;
    float *best_val = static_cast<float *>(workspace);
    int32_t *best_idx = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + half_ws);
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (launch_lm_head_q4_argmax(dm->d, dm->V, dm->eps, N, H(hidden), H(gamma), qweight, H(scales), H(zeros), group,
                                 best_val, best_idx, gate, done, st) != hipSuccess)
        return SPECEE_EHIP;
    return launch_verify_finish(best_val, best_idx, P, N, ids, dm->K, gate, done, token, max_logit, hit, st) ==
                   hipSuccess
               ? SPECEE_OK
               : SPECEE_EHIP;
}

int specee_predict_tree_q4(const specee_dims *dm, int G, int N, int Mcap, const specee_half *hidden,
                           const specee_half *gamma, const uint32_t *qweight, const specee_half *scales,
                           const specee_half *zeros, int group, const int32_t *ids, const int32_t *parent,
                           const float *prev_probs, const specee_mlp *mlp, int32_t *merged_ids, int32_t *M_out,
                           int32_t *cols, float *logits, float *probs, float *scores, int32_t *exit_flags,
                           int32_t *path_exit, void *stream) {
    // the head pointer of the fp16 entry point is not used here: any aligned non-null value passes its check
    int rc = check_tree_args(dm, G, N, Mcap, hidden, gamma, reinterpret_cast<const specee_half *>(gamma), ids, parent,
                             prev_probs, mlp, merged_ids, M_out, cols, logits, probs, scores, exit_flags, path_exit);
    if (rc) return rc;
    if (group < 8 || group % 8 != 0 || dm->d % group != 0) return SPECEE_EINVAL;
    if (G == 0) return SPECEE_OK;
    if ((rc = check_q4(dm, qweight, scales, zeros, group))) return rc;
    if ((reinterpret_cast<uintptr_t>(qweight) & 7) != 0) return SPECEE_EALIGN;
    if (!tree_q4_supported(dm->d, N, dm->K, Mcap, group)) return SPECEE_EINVAL;
    TreeQ4Params tp{};
    tp.d = dm->d; tp.V = dm->V; tp.N = N; tp.K = dm->K; tp.Mcap = Mcap; tp.group = group; tp.eps = dm->eps;
    tp.hidden = H(hidden); tp.gamma = H(gamma); tp.qweight = qweight; tp.qscales = H(scales); tp.qzeros = H(zeros);
    tp.ids = ids; tp.merged_out = merged_ids; tp.M_out = M_out; tp.cols_out = cols;
    TreeFinishParams fp{};
    fp.d = dm->d; fp.V = dm->V; fp.K = dm->K; fp.H = dm->H; fp.N = N; fp.Mcap = Mcap;
    fp.eps = dm->eps; fp.threshold = dm->threshold;
    fp.prev = prev_probs;
    fp.W1 = H(mlp->W1); fp.b1 = H(mlp->b1); fp.w2 = H(mlp->w2); fp.b2 = H(mlp->b2);
    fp.logits = logits; fp.probs = probs; fp.scores = scores; fp.exit_flags = exit_flags;
    fp.parent = parent; fp.path_exit = path_exit;
    return launch_tree_q4(tp, fp, G, static_cast<hipStream_t>(stream)) == hipSuccess ? SPECEE_OK : SPECEE_EHIP;
}

}  // extern "C" (the common body below is internal)

// specee_layer_loop and specee_layer_loop_q4: lm_head, or the quantised head (qweight non-null)
static int layer_loop_common(const specee_dims *dm, int L, int B, const specee_half *hidden, const specee_half *gamma,
                             const specee_half *lm_head, const uint32_t *qweight, const specee_half *scales,
                             const specee_half *zeros, int group, const int32_t *ids, const float *prev0,
                             const specee_mlp *mlp, const int32_t *active, float *logits, float *probs, float *scores,
                             int32_t *exit_flags, int32_t *ver_token, int32_t *hit, int32_t *exit_layer,
                             int32_t *token, int32_t *status, long long spin_limit, void *workspace,
                             size_t workspace_bytes, void *stream, bool q4) {
    int rc = check_dims(dm, true);
    if (rc) return rc;
    if (dm->d > 8192 || B < 0 || B > kLoopMaxTokens || L < 0 || L > 65535 || spin_limit < 0) return SPECEE_EINVAL;
    if (q4 && (dm->K > 8 || group < 8 || group % 8 != 0 || dm->d % group != 0)) return SPECEE_EINVAL;
    if (B == 0) return SPECEE_OK;
    if (L > 0 && (rc = check_mlp(mlp))) return rc;
    if (!exit_layer || !token || !status) return SPECEE_EINVAL;
    if (L > 0 && (!hidden || !gamma || !ids || !logits || !probs || !scores || !exit_flags || !ver_token || !hit))
        return SPECEE_EINVAL;
    if (L > 0 && !q4 && !lm_head) return SPECEE_EINVAL;
    if (L > 0 && q4 && (rc = check_q4(dm, qweight, scales, zeros, group))) return rc;
    if (misaligned(hidden) || misaligned(gamma) || misaligned(lm_head) || misaligned(workspace)) return SPECEE_EALIGN;
    const LoopLayout lay = loop_layout(B);
    if (!workspace || workspace_bytes < lay.total) return SPECEE_EWORKSPACE;
    char *ws = static_cast<char *>(workspace);
    LoopParams p{};
    p.d = dm->d; p.V = dm->V; p.K = dm->K; p.H = dm->H; p.L = L; p.B = B;
    p.eps = dm->eps; p.threshold = dm->threshold;
    p.hidden = H(hidden); p.gamma = H(gamma); p.lm_head = q4 ? nullptr : H(lm_head); p.ids = ids; p.prev0 = prev0;
    if (q4) {
        p.qweight = qweight; p.qscales = H(scales); p.qzeros = H(zeros); p.group = group;
    }
    if (mlp) {
        p.W1 = H(mlp->W1); p.b1 = H(mlp->b1); p.w2 = H(mlp->w2); p.b2 = H(mlp->b2);
    }
    p.active = active;
    p.logits = logits; p.probs = probs; p.scores = scores; p.exit_flags = exit_flags;
    p.ver_token = ver_token; p.hit = hit; p.exit_layer = exit_layer; p.token = token; p.status = status;
    p.arrive = reinterpret_cast<int32_t *>(ws + lay.flags_off);
    p.abort = p.arrive + B;
    p.cand_val = reinterpret_cast<float *>(ws + lay.val_off);
    p.cand_idx = reinterpret_cast<int32_t *>(ws + lay.idx_off);
    p.spin_limit = spin_limit > 0 ? spin_limit : (1ll << 20);
    hipStream_t st = static_cast<hipStream_t>(stream);
    // (an empty stack is handled by the launcher without touching any input: they may all be null then)
    if (L > 0 && launch_zero_i32(p.arrive, lay.flag_ints, st) != hipSuccess) return SPECEE_EHIP;
    // the launcher caps the grid at kLoopMaxWgs workgroups; each candidate buffer holds one entry per workgroup
    return launch_layer_loop(p, kLoopMaxWgs, st) == hipSuccess ? SPECEE_OK : SPECEE_EHIP;
}

extern "C" {

int specee_layer_loop(const specee_dims *dm, int L, int B, const specee_half *hidden, const specee_half *gamma,
                      const specee_half *lm_head, const int32_t *ids, const float *prev0, const specee_mlp *mlp,
                      const int32_t *active, float *logits, float *probs, float *scores, int32_t *exit_flags,
                      int32_t *ver_token, int32_t *hit, int32_t *exit_layer, int32_t *token, int32_t *status,
                      long long spin_limit, void *workspace, size_t workspace_bytes, void *stream) {
    return layer_loop_common(dm, L, B, hidden, gamma, lm_head, nullptr, nullptr, nullptr, 0, ids, prev0, mlp, active,
                             logits, probs, scores, exit_flags, ver_token, hit, exit_layer, token, status, spin_limit,
                             workspace, workspace_bytes, stream, false);
}

int specee_layer_loop_q4(const specee_dims *dm, int L, int B, const specee_half *hidden, const specee_half *gamma,
                         const uint32_t *qweight, const specee_half *scales, const specee_half *zeros, int group,
                         const int32_t *ids, const float *prev0, const specee_mlp *mlp, const int32_t *active,
                         float *logits, float *probs, float *scores, int32_t *exit_flags, int32_t *ver_token,
                         int32_t *hit, int32_t *exit_layer, int32_t *token, int32_t *status, long long spin_limit,
                         void *workspace, size_t workspace_bytes, void *stream) {
    return layer_loop_common(dm, L, B, hidden, gamma, nullptr, qweight, scales, zeros, group, ids, prev0, mlp, active,
                             logits, probs, scores, exit_flags, ver_token, hit, exit_layer, token, status, spin_limit,
                             workspace, workspace_bytes, stream, true);
}

int specee_verify(const specee_dims *dm, int N, const specee_half *hidden, const specee_half *gamma,
                  const specee_half *lm_head, const int32_t *ids, const int32_t *gate, int32_t *done,
                  int32_t *token, float *max_logit, int32_t *hit, void *workspace, size_t workspace_bytes,
                  void *stream) {
    int rc = check_dims(dm, false);
    if (rc) return rc;
    if (N < 0 || N > 65535 || dm->K < 1 || dm->K > SPECEE_KMAX) return SPECEE_EINVAL;
    if (N == 0) return SPECEE_OK;
    if (!hidden || !gamma || !lm_head || !ids || !token || !max_logit || !hit) return SPECEE_EINVAL;
    if (misaligned(hidden) || misaligned(gamma) || misaligned(lm_head) || misaligned(workspace)) return SPECEE_EALIGN;
    const bool vec = N <= 2;
    const int P = vec ? lm_head_gemv_workgroups(dm->V) : lm_head_gemm_workgroups(dm->V);
    const size_t half_ws = align256((size_t)N * P * sizeof(float));
    if (!workspace || workspace_bytes < 2 * half_ws) return SPECEE_EWORKSPACE;
    float *best_val = static_cast<float *>(workspace);
    int32_t *best_idx = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + half_ws);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = vec ? launch_lm_head_argmax_gemv(dm->d, dm->V, dm->eps, N, H(hidden), H(gamma), H(lm_head),
                                                    best_val, best_idx, gate, done, st)
                       : launch_lm_head_argmax_gemm(dm->d, dm->V, dm->eps, N, H(hidden), H(gamma), H(lm_head),
                                                    best_val, best_idx, gate, done, st);
    if (e != hipSuccess) return SPECEE_EHIP;
    e = launch_verify_finish(best_val, best_idx, P, N, ids, dm->K, gate, done, token, max_logit, hit, st);
    return e == hipSuccess ? SPECEE_OK : SPECEE_EHIP;
}

}  // extern "C"
