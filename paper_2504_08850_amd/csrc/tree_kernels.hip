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
#include "tree_finish.h"

namespace specee {

constexpr int kMergeThreads = 1024;

__global__ __launch_bounds__(kMergeThreads) void merge_kernel(const int32_t *ids, int n, int Mcap, int32_t *merged,
                                                              int32_t *M_out, int32_t *cols) {
    extern __shared__ __attribute__((aligned(16))) int32_t merge_lds[];
    const int g = blockIdx.x, tid = threadIdx.x;
    int32_t *uniq;
    int col_of[kMergePerThread];
    const int M = merge_block<kMergeThreads>(ids + (size_t)g * n, n, merge_lds, uniq, col_of);
    if (tid == 0) M_out[g] = M;
    for (int m = tid; m < Mcap; m += kMergeThreads) merged[(size_t)g * Mcap + m] = m < M ? uniq[m] : -1;
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        int i = tid + e * kMergeThreads;
        if (i < n) cols[(size_t)g * n + i] = col_of[e];
    }
}

// Sum over the S d-slices of one partial value, ascending slice order, sixteen loads in flight.
__device__ __forceinline__ float sum_slices(const float *src, size_t stride, int S) {
    float a = 0.f;
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
    return a;
}

// WHOLE = false: 256 threads, one node per wavefront, a few nodes per workgroup -- the latency
// shape (many CUs busy; the path rule runs in its own kernel).
// WHOLE = true: 512 threads, one workgroup per tree -- the throughput shape.  All threads first
// gather and sum every node's partials into LDS in one sweep (two dependent memory trips for the
// whole tree), then the wavefronts take nodes in turn with the predictor rows held in registers,
// and the path rule runs on the exit flags in LDS.
template <int KC, bool WHOLE>
__global__ __launch_bounds__(WHOLE ? 512 : 256) void tree_finish_kernel(TreeFinishParams p, int nodes_per_wg) {
    extern __shared__ float finish_lds[];  // WHOLE: zsum [N][K+1] | prev [N][K] | exit [N]
    constexpr int THREADS = WHOLE ? 512 : 256;
    constexpr int kWaves = THREADS / kWave;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.y;
    const int K = p.K, S = p.S, N = p.N;
    const int n_begin = blockIdx.x * nodes_per_wg;
    const int n_end = min(N, n_begin + nodes_per_wg);
    float *zsum = finish_lds;
    float *prevl = zsum + (size_t)N * (K + 1);
    int32_t *exit_lds = reinterpret_cast<int32_t *>(prevl + (size_t)N * K);

    const bool use_mfma = WHOLE && KC <= 8 && mlp_mfma_ok(K, p.H);
    FinishRows<KC> fr;
    TreeFinishParams pl = p;  // predictor pointers redirected to the LDS copy when the matrix cores are used
    if (use_mfma) {
        // [zsum | prev | exit | features] then the predictor copy, 16-byte aligned
        size_t off = ((size_t)N * (K + 1) + (size_t)N * K + N + 8 * 16 * kMlpFeat) * sizeof(float);
        off = (off + 15) & ~(size_t)15;
        pl = stage_mlp_to_lds(reinterpret_cast<half_t *>(reinterpret_cast<char *>(finish_lds) + off), p, tid, THREADS);
    }
    const int M = p.M_out[g];
    const size_t pstride = (size_t)p.Npad * p.Mpad;
    // WHOLE = false: the chain columns -> partial sums -> logits is the long one, so the first node's
    // ids, columns and previous probabilities are requested before the predictor rows, which are
    // not needed until the MLP (clamped lane index: the loads are unconditional)
    int id_next = 0, col_next = 0;
    float prev_next[KC];
    auto request_node = [&](int n) {
        const size_t gn = (size_t)g * N + min(n, N - 1);
        const int kk = min(lane, K - 1);
        id_next = p.ids[gn * K + kk];
        col_next = p.cols[gn * K + kk];
#pragma unroll
        for (int k = 0; k < KC; ++k) prev_next[k] = p.prev[gn * K + min(k, K - 1)];
    };
    if (!WHOLE) request_node(n_begin + wave);
    if (!use_mfma) finish_load_rows<KC>(fr, p, lane);

    if (WHOLE) {
        const int total = N * (K + 1);
        for (int idx = tid; idx < total; idx += THREADS) {
            const int n = idx / (K + 1), k = idx - n * (K + 1);
            const size_t gn = (size_t)g * N + n;
            float v;
            if (k < K) {
                const int id = p.ids[gn * K + k];
                int col = p.cols[gn * K + k];
                prevl[n * K + k] = p.prev[gn * K + k];
                col = (col >= 0 && col < p.Mpad) ? col : 0;
                v = sum_slices(p.partial + ((size_t)g * S * p.Npad + n) * p.Mpad + col, pstride, S);
                if (id < 0 || id >= p.V || M > p.Mcap) v = quiet_nan();
            } else {
                v = sum_slices(p.ssq_part + (size_t)g * S * p.Npad + n, (size_t)p.Npad, S);
            }
            zsum[idx] = v;
        }
        __syncthreads();
    }

    if (use_mfma) {
        // sixteen nodes per wavefront and round: lanes q == 0 build the features of node c, then the
        // whole wavefront evaluates the MLP on the matrix cores
        float *feat = reinterpret_cast<float *>(exit_lds + N);  // [kWaves][16][kMlpFeat]
        float *F = feat + wave * 16 * kMlpFeat;
        const int c = lane & 15, q = lane >> 4;
        const int ntiles = (N + 15) >> 4;
        const float b2 = p.b2 ? (float)p.b2[0] : 0.f;
        for (int t0 = 0; t0 < ntiles; t0 += kWaves) {  // same trip count for every wavefront
            const int n = (t0 + wave) * 16 + c;
            const bool live = n < N;
            const size_t gn = (size_t)g * N + (live ? n : 0);
            float z[KC], pr[KC];
            if (q == 0) {
                const float r = live ? 1.0f / sqrtf(zsum[n * (K + 1) + K] / (float)p.d + p.eps) : 0.f;
#pragma unroll
                for (int k = 0; k < KC; ++k) z[k] = (k < K && live) ? zsum[n * (K + 1) + k] * r : 0.f;
                local_softmax<KC>(z, K, pr);
#pragma unroll
                for (int k = 0; k < KC; ++k)
                    if (k < K) {
                        const float pv = live ? prevl[n * K + k] : 0.f;
                        F[c * kMlpFeat + k] = z[k];
                        F[c * kMlpFeat + K + k] = pr[k];
                        F[c * kMlpFeat + 2 * K + k] = pr[k] - pv;
                    }
                for (int t = 3 * K; t < kMlpFeat; ++t) F[c * kMlpFeat + t] = 0.f;
            }
            __syncthreads();
            const float u = mlp_mfma_16<true>(F, pl, lane, 0, p.H >> 4);
            if (q == 0 && live) {
                bool poisoned = false;
#pragma unroll
                for (int k = 0; k < KC; ++k)
                    if (k < K && z[k] != z[k]) poisoned = true;
                float sc = sigmoidf(b2 + u);
                if (poisoned) sc = quiet_nan();
                const int ex = (sc > p.threshold) ? 1 : 0;
                p.scores[gn] = sc;
                p.exit_flags[gn] = ex;
                exit_lds[n] = ex;
#pragma unroll
                for (int k = 0; k < KC; ++k)
                    if (k < K) {
                        p.logits[gn * K + k] = z[k];
                        p.probs[gn * K + k] = pr[k];
                    }
            }
            __syncthreads();  // F is rewritten in the next round
        }
    } else
    for (int n = n_begin + wave; n < n_end; n += kWaves) {
        const size_t gn = (size_t)g * N + n;
        float z[KC], prev[KC];
        if (WHOLE) {
            const float r = 1.0f / sqrtf(zsum[n * (K + 1) + K] / (float)p.d + p.eps);
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                z[k] = (k < K) ? zsum[n * (K + 1) + k] * r : 0.f;
                prev[k] = (k < K) ? prevl[n * K + k] : 0.f;
            }
        } else {
            // this node's ids, columns and previous probabilities were requested a round ago
            const int id = id_next;
            int col = col_next;
#pragma unroll
            for (int k = 0; k < KC; ++k) prev[k] = (k < K) ? prev_next[k] : 0.f;
            // lanes 0..K-1: one logit each; lane K: the sum of squares
            float a = 0.f;
            bool bad = M > p.Mcap;
            if (lane < K) {
                if (id < 0 || id >= p.V) bad = true;
                col = (col >= 0 && col < p.Mpad) ? col : 0;
                a = sum_slices(p.partial + ((size_t)g * S * p.Npad + n) * p.Mpad + col, pstride, S);
            } else if (lane == K) {
                a = sum_slices(p.ssq_part + (size_t)g * S * p.Npad + n, (size_t)p.Npad, S);
            }
            bad = __any(bad);
            const float r = 1.0f / sqrtf(__shfl(a, K, kWave) / (float)p.d + p.eps);
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                float v = __shfl(a, k < K ? k : 0, kWave);
                z[k] = (k < K) ? (bad ? quiet_nan() : v * r) : 0.f;
            }
        }
        if (!WHOLE && n + kWaves < n_end) request_node(n + kWaves);
        const int ex = finish_score_node<KC>(fr, p, gn, z, prev, lane);
        if (WHOLE && lane == kWave - 1) exit_lds[n] = ex;
    }
    if (WHOLE && p.path_exit) {  // whole tree in this workgroup: the path rule from LDS
        __syncthreads();
        finish_paths(exit_lds, p.parent + (size_t)g * N, N, tid, THREADS, p.path_exit + (size_t)g * N);
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

__global__ void zero_i32_kernel(int32_t *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// A fill kernel rather than a memset node: it behaves the same eagerly and under graph capture.
hipError_t launch_zero_i32(int32_t *p, int n, hipStream_t st) {
    hipLaunchKernelGGL(zero_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, n);
    return hipGetLastError();
}

hipError_t launch_merge(const int32_t *ids, int n, int G, int Mcap, int32_t *merged, int32_t *M_out, int32_t *cols,
                        hipStream_t st) {
    size_t lds = (size_t)merge_lds_ints(n) * sizeof(int32_t);
    hipLaunchKernelGGL(merge_kernel, dim3(G), dim3(kMergeThreads), lds, st, ids, n, Mcap, merged, M_out, cols);
    return hipGetLastError();
}

template <int KC>
static hipError_t launch_finish_kc(const TreeFinishParams &p, int G, hipStream_t st) {
    // Enough trees to fill the GPU with one workgroup each: every partial sum of a tree is gathered in
    // one sweep, the predictor runs on the matrix cores (or, for other shapes, with its rows held in
    // registers across nodes) and the path rule needs no second kernel.  With few trees the serial
    // instruction stream of one workgroup per tree is the bottleneck (measured: ~17 us for a 60-node
    // tree against ~5 us when every node has its own wavefront), so those take the shape below.
    const bool mfma = KC <= 8 && mlp_mfma_ok(p.K, p.H);
    size_t whole_lds = ((size_t)p.N * (p.K + 1) + (size_t)p.N * p.K + p.N) * sizeof(float) +
                       8 * 16 * kMlpFeat * sizeof(float);
    if (mfma) whole_lds = ((whole_lds + 15) & ~(size_t)15) + (size_t)mlp_lds_halves(p.K, p.H) * sizeof(half_t);
    if (G >= 32 && whole_lds <= 60 * 1024) {
        hipLaunchKernelGGL((tree_finish_kernel<KC, true>), dim3(1, G), dim3(512), whole_lds, st, p, p.N);
        return hipGetLastError();
    }
    const int per_wg = 4;  // one node per wavefront
    hipLaunchKernelGGL((tree_finish_kernel<KC, false>), dim3((p.N + per_wg - 1) / per_wg, G), dim3(256), 0, st, p,
                       per_wg);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !p.path_exit) return e;
    const int total = p.N * G;
    hipLaunchKernelGGL(path_kernel, dim3((total + 255) / 256), dim3(256), 0, st, p.exit_flags, p.parent, p.N, total,
                       p.path_exit);
    return hipGetLastError();
}

hipError_t launch_tree_finish(const TreeFinishParams &p, int G, hipStream_t st) {
    if (p.K <= 4) return launch_finish_kc<4>(p, G, st);
    if (p.K <= 8) return launch_finish_kc<8>(p, G, st);
    return launch_finish_kc<16>(p, G, st);
}

}  // namespace specee
