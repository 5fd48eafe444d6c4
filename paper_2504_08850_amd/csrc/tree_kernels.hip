// Token-tree side kernels of the merged mapping (paper Sec. 6.2):
//   merge_kernel        sorted distinct set of a tree's N*K speculative ids and
//                       the column of every (node, slot) in it (integer work,
//                       one workgroup per tree; the contraction kernel can run
//                       the same merge in its own prologue instead);
//   tree_finish_kernel  one wavefront per node: sums the d-slice partials of its
//                       K columns in fixed order, applies the RMSNorm scale and
//                       runs the same feature/MLP tail as the single-token
//                       predictor, eight hidden units per lane in registers;
//   path_kernel         the path rule: a token path exits only if every token
//                       on it exits (the rearmost exit decides), i.e. the AND of
//                       exit flags up to the root.
#include "device_utils.h"
#include "kernels.h"
#include "merge_block.h"
#include "predictor_tail.h"

namespace specee {

constexpr int kMergeThreads = 1024;

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(const int32_t *ids, int n, int Mcap, int32_t *merged,
                                                              int32_t *M_out, int32_t *cols) {
    extern __shared__ __attribute__((aligned(16))) int32_t merge_lds[];
    const int g = blockIdx.x, tid = threadIdx.x;
    int32_t *uniq;
    int col_of[kMergePerThread];
    const int M = merge_block(ids + (size_t)g * n, n, merge_lds, uniq, col_of);
    if (tid == 0) M_out[g] = M;
    for (int m = tid; m < Mcap; m += kMergeThreads) merged[(size_t)g * Mcap + m] = m < M ? uniq[m] : -1;
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        int i = tid + e * kMergeThreads;
        if (i < n) cols[(size_t)g * n + i] = col_of[e];
    }
}

constexpr int kFinishThreads = 256;
constexpr int kFinishWaves = kFinishThreads / kWave;  // nodes per workgroup: one per wavefront
constexpr int kFinishUnits = 8;                       // hidden units per lane held in registers (H <= 512)

template <int KC>
__global__ __launch_bounds__(kFinishThreads) void tree_finish_kernel(TreeFinishParams p) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.y;
    const int n = blockIdx.x * kFinishWaves + wave;
    const int K = p.K, H = p.H, S = p.S, N = p.N;
    if (n >= N) return;  // no barriers below: wavefronts are independent
    const bool regs = (K == KC) && (H <= kFinishUnits * kWave) && KC <= 8;

    MlpRow<KC> rows[KC <= 8 ? kFinishUnits : 1];
    if (regs) {
#pragma unroll
        for (int u = 0; u < kFinishUnits; ++u) mlp_row_load<KC>(rows[u], p.W1, p.b1, p.w2, K, H, lane + u * kWave);
    }
    const size_t gn = (size_t)g * N + n;
    // independent requests first: merged size, this node's ids, columns and previous probabilities
    const int M = p.M_out[g];
    const float b2 = p.b2 ? (float)p.b2[0] : 0.f;
    int id = 0, col = 0;
    if (lane < K) {
        id = p.ids[gn * K + lane];
        col = p.cols[gn * K + lane];
    }
    float prev[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) prev[k] = (k < K) ? p.prev[gn * K + k] : 0.f;

    // lanes 0..K-1: one logit each; lane K: the sum of squares.  Slices are summed in ascending
    // order, sixteen loads in flight at a time.
    float a = 0.f;
    bool bad = M > p.Mcap;
    const float *src = nullptr;
    size_t stride = 0;
    if (lane < K) {
        if (id < 0 || id >= p.V) bad = true;
        col = (col >= 0 && col < p.Mpad) ? col : 0;
        src = p.partial + ((size_t)g * S * p.Npad + n) * p.Mpad + col;
        stride = (size_t)p.Npad * p.Mpad;
    } else if (lane == K) {
        src = p.ssq_part + (size_t)g * S * p.Npad + n;
        stride = (size_t)p.Npad;
    }
    if (src) {
        int s = 0;
        for (; s + 16 <= S; s += 16) {
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = src[(size_t)(s + u) * stride];
#pragma unroll
            for (int u = 0; u < 16; ++u) a += v[u];
        }
        for (; s + 4 <= S; s += 4) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = src[(size_t)(s + u) * stride];
#pragma unroll
            for (int u = 0; u < 4; ++u) a += v[u];
        }
        for (; s < S; ++s) a += src[(size_t)s * stride];
    }
    bad = __any(bad);
    const float r = 1.0f / sqrtf(__shfl(a, K, kWave) / (float)p.d + p.eps);
    float z[KC], pr[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        float v = __shfl(a, k < K ? k : 0, kWave);
        z[k] = (k < K) ? (bad ? quiet_nan() : v * r) : 0.f;
    }
    local_softmax<KC>(z, K, pr);

    float part = 0.f;
    if (regs) {
#pragma unroll
        for (int u = 0; u < kFinishUnits; ++u)
            if (lane + u * kWave < H) part += mlp_unit<KC>(rows[u], p.W1, K, lane + u * kWave, z, pr, prev);
    } else {
        for (int j = lane; j < H; j += kWave) {
            MlpRow<KC> row;
            mlp_row_load<KC>(row, p.W1, p.b1, p.w2, K, H, j);
            part += mlp_unit<KC>(row, p.W1, K, j, z, pr, prev);
        }
    }
    part = wave_sum(part);
    const float sc = sigmoidf(b2 + part);
    if (lane == 0) {
        p.scores[gn] = sc;
        p.exit_flags[gn] = (sc > p.threshold) ? 1 : 0;
    }
    if (lane < K) {
        p.logits[gn * K + lane] = bad ? quiet_nan() : a * r;
        float mine = 0.f;
#pragma unroll
        for (int k = 0; k < KC; ++k)
            if (k == lane) mine = pr[k];
        p.probs[gn * K + lane] = mine;
    }
}

__global__ void path_kernel(const int32_t *exit_flags, const int32_t *parent, int N, int total, int32_t *path_exit) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int g = i / N;
    const int32_t *ex = exit_flags + (size_t)g * N;
    const int32_t *par = parent + (size_t)g * N;
    int cur = i - g * N;
    int ok = 1;
    for (int step = 0; step < N && cur >= 0; ++step) {  // parents precede children: at most N steps
        ok &= (ex[cur] != 0);
        int up = par[cur];
        if (up >= cur) {  // malformed tree: refuse the path rather than loop
            ok = 0;
            break;
        }
        cur = up;
    }
    path_exit[i] = ok;
}

hipError_t launch_merge(const int32_t *ids, int n, int G, int Mcap, int32_t *merged, int32_t *M_out, int32_t *cols,
                        hipStream_t st) {
    size_t lds = (size_t)merge_lds_ints(n) * sizeof(int32_t);
    hipLaunchKernelGGL(merge_kernel, dim3(G), dim3(kMergeThreads), lds, st, ids, n, Mcap, merged, M_out, cols);
    return hipGetLastError();
}

hipError_t launch_tree_finish(const TreeFinishParams &p, int G, hipStream_t st) {
    dim3 grid((p.N + kFinishWaves - 1) / kFinishWaves, G), block(kFinishThreads);
    if (p.K <= 4)
        hipLaunchKernelGGL((tree_finish_kernel<4>), grid, block, 0, st, p);
    else if (p.K <= 8)
        hipLaunchKernelGGL((tree_finish_kernel<8>), grid, block, 0, st, p);
    else
        hipLaunchKernelGGL((tree_finish_kernel<16>), grid, block, 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !p.path_exit) return e;
    const int total = p.N * G;
    hipLaunchKernelGGL(path_kernel, dim3((total + 255) / 256), dim3(256), 0, st, p.exit_flags, p.parent, p.N, total,
                       p.path_exit);
    return hipGetLastError();
}

}  // namespace specee
