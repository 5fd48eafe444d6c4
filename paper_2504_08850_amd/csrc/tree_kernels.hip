// Token-tree side kernels of the merged mapping (paper Sec. 6.2):
//   merge_kernel   sorted distinct set of a tree's N*K speculative ids and the
//                  column of every (node, slot) in it -- pure integer work, one
//                  workgroup per tree, bitonic sort + scan + binary search in LDS;
//   finish_kernel  per node: fixed-order sum of the d-slice partials of its K
//                  columns, RMSNorm scale, then the same feature/MLP tail as the
//                  single-token predictor;
//   path_kernel    a token path exits only if every token on it exits (the
//                  rearmost exit decides): AND of exit flags up to the root.
#include "device_utils.h"
#include "kernels.h"
#include "predictor_tail.h"

namespace specee {

constexpr int kMergeThreads = 1024;
constexpr int kMergeMax = 4096;           // N*K limit
constexpr int kPadKey = 0x7fffffff;       // sorts after every valid or invalid id

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(const int32_t *ids, int n, int P, int Mcap,
                                                              int32_t *merged, int32_t *M_out, int32_t *cols) {
    __shared__ int32_t key[kMergeMax];
    __shared__ int32_t pos[kMergeMax];
    __shared__ int32_t uniq[kMergeMax];
    const int tid = threadIdx.x;
    const int g = blockIdx.x;
    const int32_t *gids = ids + (size_t)g * n;

    for (int i = tid; i < P; i += kMergeThreads) key[i] = i < n ? gids[i] : kPadKey;
    __syncthreads();
    // bitonic sort, ascending (signed compare: negative, i.e. invalid, ids sort first)
    for (int k = 2; k <= P; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = tid; t < (P >> 1); t += kMergeThreads) {
                int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                int hi = lo | j;
                bool up = (lo & k) == 0;
                int32_t a = key[lo], b = key[hi];
                if ((a > b) == up) {
                    key[lo] = b;
                    key[hi] = a;
                }
            }
            __syncthreads();
        }
    // head-of-run flags and their inclusive scan (Hillis-Steele over P entries)
    for (int i = tid; i < P; i += kMergeThreads)
        pos[i] = (i < n && (i == 0 || key[i] != key[i - 1])) ? 1 : 0;
    __syncthreads();
    for (int off = 1; off < P; off <<= 1) {
        int32_t v[kMergeMax / kMergeThreads];
        int cnt = 0;
        for (int i = tid; i < P; i += kMergeThreads) v[cnt++] = pos[i] + (i >= off ? pos[i - off] : 0);
        __syncthreads();
        cnt = 0;
        for (int i = tid; i < P; i += kMergeThreads) pos[i] = v[cnt++];
        __syncthreads();
    }
    const int M = n > 0 ? pos[n - 1] : 0;
    for (int i = tid; i < n; i += kMergeThreads)
        if (i == 0 || key[i] != key[i - 1]) uniq[pos[i] - 1] = key[i];
    __syncthreads();
    if (tid == 0) M_out[g] = M;
    for (int m = tid; m < Mcap; m += kMergeThreads) merged[(size_t)g * Mcap + m] = m < M ? uniq[m] : -1;
    // column of every id: binary search in the distinct set
    for (int i = tid; i < n; i += kMergeThreads) {
        int32_t id = gids[i];
        int lo = 0, hi = M - 1;
        while (lo < hi) {
            int mid = (lo + hi) >> 1;
            if (uniq[mid] < id) lo = mid + 1;
            else hi = mid;
        }
        cols[(size_t)g * n + i] = lo;
    }
}

constexpr int kFinishThreads = 512;
constexpr int kFinishWaves = kFinishThreads / kWave;
constexpr int kFinishSMax = 128;  // d-slices

template <int KC>
__global__ __launch_bounds__(kFinishThreads) void tree_finish_kernel(TreeFinishParams p) {
    __shared__ float part[SPECEE_KMAX_INTERNAL * kFinishSMax];
    __shared__ float ssqp[kFinishSMax];
    __shared__ float zs[KC + 1];
    __shared__ float red_u[kFinishWaves];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = blockIdx.x, g = blockIdx.y;
    const int K = p.K, H = p.H, S = p.S;
    const size_t gn = (size_t)g * p.N + n;

    MlpRow<KC> row0;
    mlp_row_load<KC>(row0, p.W1, p.b1, p.w2, K, H, tid);
    float prev[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) prev[k] = k < K ? p.prev[gn * K + k] : 0.f;

    const int M = p.M_out[g];
    const bool overflow = M > p.Mcap;
    bool bad = overflow;
#pragma unroll
    for (int k = 0; k < KC; ++k)
        if (k < K) {
            int id = p.ids[gn * K + k];
            if (id < 0 || id >= p.V) bad = true;
        }
    // gather this node's K columns from every d-slice partial
    for (int t = tid; t < K * S; t += kFinishThreads) {
        int k = t / S, s = t - k * S;
        int col = p.cols[gn * K + k];
        col = (col >= 0 && col < p.Mpad) ? col : 0;
        part[k * S + s] = p.partial[(((size_t)g * S + s) * p.Npad + n) * p.Mpad + col];
    }
    for (int s = tid; s < S; s += kFinishThreads) ssqp[s] = p.ssq_part[((size_t)g * S + s) * p.Npad + n];
    __syncthreads();
    if (tid <= K) {  // threads 0..K-1: one logit each, ascending slice order; thread K: sum of squares
        float a = 0.f;
        const float *src = tid < K ? part + tid * S : ssqp;
        for (int s = 0; s < S; ++s) a += src[s];
        zs[tid < K ? tid : KC] = a;
    }
    __syncthreads();
    const float r = 1.0f / sqrtf(zs[KC] / (float)p.d + p.eps);
    float z[KC], pr[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) z[k] = (k < K) ? (bad ? quiet_nan() : zs[k] * r) : 0.f;
    local_softmax<KC>(z, K, pr);

    float partu = mlp_partial<KC, kFinishThreads>(row0, p.W1, p.b1, p.w2, K, H, tid, z, pr, prev);
    partu = wave_sum(partu);
    if (lane == 0) red_u[wave] = partu;
    __syncthreads();
    if (tid == 0) {
        float u = p.b2 ? (float)p.b2[0] : 0.f;
#pragma unroll
        for (int w = 0; w < kFinishWaves; ++w) u += red_u[w];
        float sc = sigmoidf(u);
        p.scores[gn] = sc;
        p.exit_flags[gn] = (sc > p.threshold) ? 1 : 0;
#pragma unroll
        for (int k = 0; k < KC; ++k)
            if (k < K) {
                p.logits[gn * K + k] = z[k];
                p.probs[gn * K + k] = pr[k];
            }
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
    int P = 64;
    while (P < n) P <<= 1;
    hipLaunchKernelGGL(merge_kernel, dim3(G), dim3(kMergeThreads), 0, st, ids, n, P, Mcap, merged, M_out, cols);
    return hipGetLastError();
}

hipError_t launch_tree_finish(const TreeFinishParams &p, int G, hipStream_t st) {
    dim3 grid(p.N, G), block(kFinishThreads);
    if (p.K <= 4)
        hipLaunchKernelGGL((tree_finish_kernel<4>), grid, block, 0, st, p);
    else if (p.K <= 8)
        hipLaunchKernelGGL((tree_finish_kernel<8>), grid, block, 0, st, p);
    else
        hipLaunchKernelGGL((tree_finish_kernel<16>), grid, block, 0, st, p);
    return hipGetLastError();
}

hipError_t launch_path(const int32_t *exit_flags, const int32_t *parent, int N, int G, int32_t *path_exit,
                       hipStream_t st) {
    int total = N * G;
    hipLaunchKernelGGL(path_kernel, dim3((total + 255) / 256), dim3(256), 0, st, exit_flags, parent, N, total,
                       path_exit);
    return hipGetLastError();
}

}  // namespace specee
