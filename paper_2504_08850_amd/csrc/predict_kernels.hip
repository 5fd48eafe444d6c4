// Fused per-layer predictor kernel (paper Sec. 4.3.1 features + Sec. 4.3.2
// judgment): one workgroup scores one (layer, token) pair.
//
// Why one workgroup per token: a call moves (K+2) rows of d halves plus ~13 KB
// of predictor weights -- far below the bandwidth-delay product of the memory
// system -- so what matters is the number of dependent memory round trips, not
// bytes per second.  Everything that does not depend on the speculative ids
// (hidden state, RMSNorm weight, the thread's MLP row) is requested first, the
// K LM-head rows follow as soon as the ids arrive, and because the RMSNorm
// scale is a scalar factor of every logit, sum(h^2) and the K dot products run
// in the same pass: the kernel makes exactly two dependent trips to memory.
// All loads are 16 bytes per lane; reductions are DPP within a wavefront and a
// fixed-order LDS exchange across the eight wavefronts.
#include "device_utils.h"
#include "kernels.h"
#include "predictor_tail.h"

namespace specee {

constexpr int kPredictThreads = 512;

// KC: speculative rows held in flight (K <= KC).  VPT: 16-byte vectors per
// thread per row (d/8 <= VPT * 512 * tiles).  SWEEP: the previous layer's local
// probabilities are recomputed from that layer's hidden state instead of read,
// which makes every (layer, token) workgroup independent.
// EXACT: K == KC is known at compile time (the common K = 4 and K = 8): every `k < K` predicate and
// the generic MLP path fold away, which shortens the serial instruction stream of this latency-bound
// kernel.
// T: threads per workgroup.  512 gives the shortest single call (one vector of a 4096-wide row and one
// hidden unit per thread).  With thousands of tokens per launch 256 is faster: twice as many
// workgroups fit on a CU, so more independent chains of the two memory trips are in flight, and the
// redundant feature arithmetic and the barriers halve; a thread then owns MU = 2 hidden units, both
// requested up front.
template <int KC, int VPT, bool SWEEP, bool EXACT, int T = kPredictThreads, int MU = 1>
__global__ __launch_bounds__(T) void predict_kernel(PredictParams p) {
    constexpr int kWaves = T / kWave;
    // throughput shape: hidden states pass through once, so they are read with the non-temporal hint; the
    // LM-head rows are not -- tokens of a batch share rows, and the hint costs those re-reads their cache
    // hits (16384 tokens with repeating ids: 91 -> 104 us with it, though 8000 tokens with distinct ids
    // gain 10 %)
    constexpr bool kStream = T != kPredictThreads;
    __shared__ float red[kWaves][2 * KC + 2];
    __shared__ float red_u[kWaves];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6;
    const int b = blockIdx.x;
    const int l = blockIdx.y;
    const int K = EXACT ? KC : p.K, H = p.H, d = p.d;
    const int nv = d >> 3;
    const size_t tok = (size_t)l * p.B + b;

    // ---- which layer supplies the previous probabilities (sweep only)
    int lprev = -1;
    if (SWEEP) {
        if (p.active && p.active[l] == 0) {
            if (tid < K) {
                p.logits[tok * K + tid] = 0.f;
                p.probs[tok * K + tid] = 0.f;
            }
            if (tid == 0) {
                p.scores[tok] = 0.f;
                p.exit_flags[tok] = 0;
            }
            return;
        }
        for (int q = l - 1; q >= 0; --q)
            if (!p.active || p.active[q] != 0) {
                lprev = q;
                break;
            }
    }

    // ---- the ids (and the token's done flag) are requested before anything else: the LM-head rows, the
    // longest chain of the kernel, hang on them
    // (single layer only: in the sweep the compiler would wait for them before requesting anything else)
    int idv[KC];
    if (!SWEEP) {
#pragma unroll
        for (int k = 0; k < KC; ++k) idv[k] = (k < K) ? p.ids[(size_t)tok * K + k] : 0;
    }

    // ---- requests that do not depend on the ids
    const half_t *W1 = p.W1 + (size_t)l * H * 3 * K;
    const half_t *w2 = p.w2 + (size_t)l * H;
    const half_t *b1 = p.b1 ? p.b1 + (size_t)l * H : nullptr;
    MlpRow<KC> rowm[MU];
#pragma unroll
    for (int m = 0; m < MU; ++m) mlp_row_load<KC>(rowm[m], W1, b1, w2, K, H, tid + m * T);

    const half_t *hrow = p.hidden + tok * d;
    const half_t *hprow = (SWEEP && lprev >= 0) ? p.hidden + ((size_t)lprev * p.B + b) * d : nullptr;
    half8 hv[VPT], gv[VPT], hp[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        int v = tid + u * T;
        bool in = v < nv;
        hv[u] = in ? (kStream ? load_half8_stream(hrow + v * 8) : load_half8(hrow + v * 8)) : zero_half8();
        gv[u] = in ? load_half8(p.gamma + v * 8) : zero_half8();
        hp[u] = (SWEEP && in && hprow) ? load_half8(hprow + v * 8) : zero_half8();
    }
    float prev[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) prev[k] = 0.f;
    const float *prev_src = SWEEP ? (lprev < 0 ? p.prev : nullptr) : p.prev;
    if (prev_src) {
#pragma unroll
        for (int k = 0; k < KC; ++k)
            if (k < K) prev[k] = prev_src[(size_t)b * K + k];
    }

    // ---- the K speculative LM-head rows
    // The token's done flag travels with the ids, so looking at it costs the live tokens nothing; a
    // token that already left the model stops here, before the rows are read.
    const int dn = (!SWEEP && p.done) ? p.done[b] : 0;
    const half_t *rows[KC];
    bool bad_id = false;
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        int id = SWEEP ? ((k < K) ? p.ids[(size_t)b * K + k] : 0) : idv[k];
        bool ok = id >= 0 && id < p.V;
        if (k < K && !ok) bad_id = true;
        rows[k] = p.lm_head + (size_t)(ok ? id : 0) * d;
    }
    if (!SWEEP && dn != 0) {  // uniform over the workgroup
        if (tid < K) {
            p.logits[tok * K + tid] = 0.f;
            p.probs[tok * K + tid] = p.prev[(size_t)b * K + tid];
        }
        if (tid == 0) {
            p.scores[tok] = 0.f;
            p.exit_flags[tok] = 0;
        }
        return;
    }
    half8 wv[KC][VPT];
#pragma unroll
    for (int k = 0; k < KC; ++k)
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            int v = tid + u * T;
            wv[k][u] = (k < K && v < nv) ? load_half8(rows[k] + v * 8) : zero_half8();
        }

    // ---- one pass: sum of squares and the K dot products (and the previous layer's)
    float ssq = 0.f, ssq_p = 0.f, acc[KC], acc_p[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) acc[k] = acc_p[k] = 0.f;
#pragma unroll
    for (int u = 0; u < VPT; ++u)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float g = (float)gv[u][e];
            float hf = (float)hv[u][e];
            float x = hf * g;
            ssq += hf * hf;
            float xp = 0.f;
            if (SWEEP) {
                float hpf = (float)hp[u][e];
                xp = hpf * g;
                ssq_p += hpf * hpf;
            }
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                float w = (float)wv[k][u][e];
                acc[k] += x * w;
                if (SWEEP) acc_p[k] += xp * w;
            }
        }
    // d larger than VPT * 512 vectors: remaining tiles, same arithmetic
    for (int v = tid + VPT * T; v < nv; v += T) {
        half8 h8 = load_half8(hrow + v * 8), g8 = load_half8(p.gamma + v * 8);
        half8 hp8 = (SWEEP && hprow) ? load_half8(hprow + v * 8) : zero_half8();
        half8 w8[KC];
#pragma unroll
        for (int k = 0; k < KC; ++k) w8[k] = (k < K) ? load_half8(rows[k] + v * 8) : zero_half8();
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float g = (float)g8[e], hf = (float)h8[e], hpf = (float)hp8[e];
            float x = hf * g, xp = hpf * g;
            ssq += hf * hf;
            ssq_p += hpf * hpf;
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                float w = (float)w8[k][e];
                acc[k] += x * w;
                acc_p[k] += xp * w;
            }
        }
    }

    // ---- wavefront reduction, then fixed-order combination of the eight wave partials
    ssq = wave_sum_to_last_row(ssq);
#pragma unroll
    for (int k = 0; k < KC; ++k) acc[k] = wave_sum_to_last_row(acc[k]);
    if (SWEEP) {
        ssq_p = wave_sum_to_last_row(ssq_p);
#pragma unroll
        for (int k = 0; k < KC; ++k) acc_p[k] = wave_sum_to_last_row(acc_p[k]);
    }
    if (lane == kWave - 1) {
        red[wave][0] = ssq;
        red[wave][1] = ssq_p;
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            red[wave][2 + k] = acc[k];
            red[wave][2 + KC + k] = acc_p[k];
        }
    }
    __syncthreads();
    ssq = ssq_p = 0.f;
#pragma unroll
    for (int k = 0; k < KC; ++k) acc[k] = acc_p[k] = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        ssq += red[w][0];
        if (SWEEP) ssq_p += red[w][1];
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            acc[k] += red[w][2 + k];
            if (SWEEP) acc_p[k] += red[w][2 + KC + k];
        }
    }

    // ---- features (every thread computes them redundantly: no second exchange)
    const float inv_d = 1.0f / (float)d;
    float z[KC], pr[KC];
    {
        float r = 1.0f / sqrtf(ssq * inv_d + p.eps);
#pragma unroll
        for (int k = 0; k < KC; ++k) z[k] = bad_id ? quiet_nan() : acc[k] * r;
        local_softmax<KC>(z, K, pr);
    }
    if (SWEEP && lprev >= 0) {
        float zp[KC];
        float rp = 1.0f / sqrtf(ssq_p * inv_d + p.eps);
#pragma unroll
        for (int k = 0; k < KC; ++k) zp[k] = bad_id ? quiet_nan() : acc_p[k] * rp;
        local_softmax<KC>(zp, K, prev);
    }

    // ---- MLP: thread j owns hidden unit j (+512, ...); f = [z | p | p - prev]
    float part = mlp_partial<KC, T, MU>(rowm, W1, b1, w2, K, H, tid, z, pr, prev);
    part = wave_sum_to_last_row(part);
    if (lane == kWave - 1) red_u[wave] = part;
    __syncthreads();

    if (tid == 0) {
        float u = p.b2 ? (float)p.b2[l] : 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) u += red_u[w];
        float s = sigmoidf(u);
        p.scores[tok] = s;
        p.exit_flags[tok] = (s > p.threshold) ? 1 : 0;
#pragma unroll
        for (int k = 0; k < KC; ++k)
            if (k < K) {
                p.logits[tok * K + k] = z[k];
                p.probs[tok * K + k] = pr[k];
            }
    }
}

// Shared tail of the quantised-row kernels: wavefront and workgroup sums (fixed order), RMSNorm scale,
// features, MLP, sigmoid, threshold, outputs.  All threads of the workgroup must call.
template <int KC, int T, int MU>
__device__ __forceinline__ void q4_tail(const PredictParams &p, int b, int K, float ssq, float (&acc)[KC], bool bad_id,
                                        const MlpRow<KC> (&rowm)[MU], const float (&prev)[KC],
                                        float (*red)[KC + 1], float *red_u) {
    constexpr int kWaves = T / kWave;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int H = p.H, d = p.d;
    // ---- wavefront reduction, then fixed-order combination of the eight wave partials
    ssq = wave_sum_to_last_row(ssq);
#pragma unroll
    for (int k = 0; k < KC; ++k) acc[k] = wave_sum_to_last_row(acc[k]);
    if (lane == kWave - 1) {
        red[wave][0] = ssq;
#pragma unroll
        for (int k = 0; k < KC; ++k) red[wave][1 + k] = acc[k];
    }
    __syncthreads();
    ssq = 0.f;
#pragma unroll
    for (int k = 0; k < KC; ++k) acc[k] = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        ssq += red[w][0];
#pragma unroll
        for (int k = 0; k < KC; ++k) acc[k] += red[w][1 + k];
    }
    float z[KC], pr[KC];
    const float r = 1.0f / sqrtf(ssq * (1.0f / (float)d) + p.eps);
#pragma unroll
    for (int k = 0; k < KC; ++k) z[k] = bad_id ? quiet_nan() : acc[k] * r;
    local_softmax<KC>(z, K, pr);
    float part = mlp_partial<KC, T, MU>(rowm, p.W1, p.b1, p.w2, K, H, tid, z, pr, prev);
    part = wave_sum_to_last_row(part);
    if (lane == kWave - 1) red_u[wave] = part;
    __syncthreads();
    if (tid == 0) {
        float u = p.b2 ? (float)p.b2[0] : 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) u += red_u[w];
        const float sc = sigmoidf(u);
        p.scores[b] = sc;
        p.exit_flags[b] = (sc > p.threshold) ? 1 : 0;
#pragma unroll
        for (int k = 0; k < KC; ++k)
            if (k < K) {
                p.logits[(size_t)b * K + k] = z[k];
                p.probs[(size_t)b * K + k] = pr[k];
            }
    }
}

// The predictor on a 4-bit group-quantised LM head (the quantised setting of the paper's cloud
// evaluation, Sec. 7.1 / 7.3; the storage format is this library's reading): element i of a row is a
// code c in 0..15 in bits 4*(i%8).. of 32-bit word i/8 and stands for scale[g] * (c - zero[g]),
// g = i / group.  A speculative row is then d/2 bytes instead of 2d, and the dequantisation never
// materialises: a thread owns eight consecutive elements (one word per row, all in one group), forms
//     sum_e x_e * c_e   and   sum_e x_e          (x = h * gamma, fp32)
// and adds scale * (first - zero * second) to the row's dot product -- one multiply-add per element
// plus three per word.  Same two dependent trips to memory and the same reductions and tail as
// predict_kernel; one workgroup per token.
// EXACT: K == KC at compile time (see predict_kernel).  Every load is unconditional on a clamped, valid
// address -- a load under a branch would make the compiler wait for all outstanding loads at the join
// and turn the K rows into K serial trips to memory; unused data is zeroed by selects instead.
template <int KC, int VPT, bool EXACT, int T = kPredictThreads, int MU = 1>
__global__ __launch_bounds__(T) void predict_q4_kernel(PredictParams p) {
    constexpr int kWaves = T / kWave;
    __shared__ float red[kWaves][KC + 1];
    __shared__ float red_u[kWaves];
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int K = EXACT ? KC : p.K, H = p.H, d = p.d;
    const int nv = d >> 3, ng = d / p.group;

    // ---- requests that do not depend on the ids
    MlpRow<KC> rowm[MU];
#pragma unroll
    for (int m = 0; m < MU; ++m) mlp_row_load<KC>(rowm[m], p.W1, p.b1, p.w2, K, H, tid + m * T);
    const half_t *hrow = p.hidden + (size_t)b * d;
    half8 hv[VPT], gv[VPT];
    int vc[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int v = tid + u * T;
        vc[u] = min(v, nv - 1);
        const half8 h8 = load_half8(hrow + vc[u] * 8), g8 = load_half8(p.gamma + vc[u] * 8);
        hv[u] = v < nv ? h8 : zero_half8();  // a zero hidden state silences the clamped duplicate
        gv[u] = g8;
    }
    float prev[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        const float pv = p.prev[(size_t)b * K + min(k, K - 1)];
        prev[k] = (k < K) ? pv : 0.f;
    }
    const int32_t *donep = p.done ? p.done + b : p.ids;  // always a valid address
    const int dn_raw = *donep;
    const int dn = p.done ? dn_raw : 0;

    // ---- the K speculative rows: one word of codes per row and vector, with its group's scale and zero-point
    int rowi[KC];
    bool bad_id = false;
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        const int id = p.ids[(size_t)b * K + min(k, K - 1)];
        const bool ok = id >= 0 && id < p.V;
        if (k < K && !ok) bad_id = true;
        rowi[k] = ok ? id : 0;
    }
    if (dn != 0) {  // uniform over the workgroup: the token already left the model
        if (tid < K) {
            p.logits[(size_t)b * K + tid] = 0.f;
            p.probs[(size_t)b * K + tid] = p.prev[(size_t)b * K + tid];
        }
        if (tid == 0) {
            p.scores[b] = 0.f;
            p.exit_flags[b] = 0;
        }
        return;
    }
    uint32_t qw[KC][VPT];
    half_t qs[KC][VPT], qz[KC][VPT];
#pragma unroll
    for (int k = 0; k < KC; ++k)
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            const size_t gi = (size_t)rowi[k] * ng + (vc[u] * 8) / p.group;
            qw[k][u] = p.qweight[(size_t)rowi[k] * nv + vc[u]];
            qs[k][u] = p.qscales[gi];
            qz[k][u] = p.qzeros[gi];
        }

    float ssq = 0.f, acc[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) acc[k] = 0.f;
    auto dot8 = [&](const half8 &h8, const half8 &g8, const uint32_t (&w)[KC], const half_t (&sc)[KC],
                    const half_t (&zp)[KC]) {
        float x[8], xs = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float hf = (float)h8[e];
            x[e] = hf * (float)g8[e];
            ssq += hf * hf;
            xs += x[e];
        }
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            const uint32_t even = w[k] & 0x0f0f0f0fu, odd = (w[k] >> 4) & 0x0f0f0f0fu;  // elements 0,2,4,6 / 1,3,5,7
            float pd = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                pd += x[2 * j] * (float)((even >> (8 * j)) & 0xffu);
                pd += x[2 * j + 1] * (float)((odd >> (8 * j)) & 0xffu);
            }
            acc[k] += (float)sc[k] * (pd - (float)zp[k] * xs);
        }
    };
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        uint32_t w[KC];
        half_t sc[KC], zp[KC];
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            w[k] = qw[k][u];
            sc[k] = qs[k][u];
            zp[k] = qz[k][u];
        }
        dot8(hv[u], gv[u], w, sc, zp);
    }
    // d larger than VPT * 512 vectors: remaining tiles, same arithmetic
    for (int v = tid + VPT * T; v < nv; v += T) {
        const half8 h8 = load_half8(hrow + v * 8), g8 = load_half8(p.gamma + v * 8);
        uint32_t w[KC];
        half_t sc[KC], zp[KC];
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            const size_t gi = (size_t)rowi[k] * ng + (v * 8) / p.group;
            w[k] = p.qweight[(size_t)rowi[k] * nv + v];
            sc[k] = p.qscales[gi];
            zp[k] = p.qzeros[gi];
        }
        dot8(h8, g8, w, sc, zp);
    }

    q4_tail<KC, T, MU>(p, b, K, ssq, acc, bad_id, rowm, prev, red, red_u);
}

// Throughput shape of predict_q4_kernel (thousands of tokens per launch).  A thread owns chunks of 32
// consecutive elements = four consecutive words of codes: one 16-byte load per row brings its codes, and
// because a chunk lies inside one quantisation group (group % 32 == 0) one scale and one zero-point per
// row serve all 32 elements.  Per token that is a third of the load instructions of the word-per-thread
// layout (the small scale / zero-point loads dominate there), and the vector memory path, not HBM, is
// what a CU runs out of first with rows this short.  CPT: chunks per thread (d <= 32 * T * CPT).
template <int KC, int T, int CPT, int MU>
__global__ __launch_bounds__(T) void predict_q4_wide_kernel(PredictParams p) {
    constexpr int kWaves = T / kWave;
    constexpr int K = KC;
    __shared__ float red[kWaves][KC + 1];
    __shared__ float red_u[kWaves];
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int H = p.H, d = p.d;
    const int nc = d >> 5, nv = d >> 3, ng = d / p.group;

    // ---- requests that do not depend on the ids
    MlpRow<KC> rowm[MU];
#pragma unroll
    for (int m = 0; m < MU; ++m) mlp_row_load<KC>(rowm[m], p.W1, p.b1, p.w2, K, H, tid + m * T);
    const half_t *hrow = p.hidden + (size_t)b * d;
    half8 hv[CPT][4], gv[CPT][4];
    int cc[CPT], gofs[CPT];
#pragma unroll
    for (int u = 0; u < CPT; ++u) {
        const int c = tid + u * T;
        cc[u] = min(c, nc - 1);
        gofs[u] = (cc[u] * 32) / p.group;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const half8 h8 = load_half8(hrow + cc[u] * 32 + i * 8);
            hv[u][i] = c < nc ? h8 : zero_half8();  // a zero hidden state silences the clamped duplicate
            gv[u][i] = load_half8(p.gamma + cc[u] * 32 + i * 8);
        }
    }
    float prev[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) prev[k] = p.prev[(size_t)b * K + k];
    const int32_t *donep = p.done ? p.done + b : p.ids;  // always a valid address
    const int dn_raw = *donep;
    const int dn = p.done ? dn_raw : 0;

    // ---- the K speculative rows
    int rowi[KC];
    bool bad_id = false;
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        const int id = p.ids[(size_t)b * K + k];
        const bool ok = id >= 0 && id < p.V;
        if (!ok) bad_id = true;
        rowi[k] = ok ? id : 0;
    }
    if (dn != 0) {  // uniform over the workgroup: the token already left the model
        if (tid < K) {
            p.logits[(size_t)b * K + tid] = 0.f;
            p.probs[(size_t)b * K + tid] = p.prev[(size_t)b * K + tid];
        }
        if (tid == 0) {
            p.scores[b] = 0.f;
            p.exit_flags[b] = 0;
        }
        return;
    }
    uintx4 qw[KC][CPT];
    half_t qs[KC][CPT], qz[KC][CPT];
#pragma unroll
    for (int k = 0; k < KC; ++k)
#pragma unroll
        for (int u = 0; u < CPT; ++u) {
            const size_t gi = (size_t)rowi[k] * ng + gofs[u];
            qw[k][u] = *reinterpret_cast<const uintx4 *>(p.qweight + (size_t)rowi[k] * nv + cc[u] * 4);
            qs[k][u] = p.qscales[gi];
            qz[k][u] = p.qzeros[gi];
        }

    float ssq = 0.f, acc[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) acc[k] = 0.f;
    // Byte j of a word holds elements 2j (low nibble) and 2j+1 (high nibble).  With a = x[2j] - x[2j+1]/16
    // and bq = x[2j+1]/16 (computed once, shared by the K rows),
    //     x[2j]*lo + x[2j+1]*hi = a*lo + bq*(lo + 16*hi) = a*lo + bq*byte,
    // so a row costs one mask per word and one byte-to-float conversion plus one FMA per nibble; the
    // high nibbles are never extracted.  This arithmetic, not memory, bounds the kernel.
#pragma unroll
    for (int u = 0; u < CPT; ++u) {
        float xs = 0.f, pd[KC];
#pragma unroll
        for (int k = 0; k < KC; ++k) pd[k] = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float a[4], bq[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const half2_t hh = {hv[u][i][2 * j], hv[u][i][2 * j + 1]};
                ssq = __builtin_amdgcn_fdot2(hh, hh, ssq, false);
                const float x0 = (float)hh[0] * (float)gv[u][i][2 * j];
                const float x1 = (float)hh[1] * (float)gv[u][i][2 * j + 1];
                xs += x0 + x1;
                bq[j] = x1 * 0.0625f;
                a[j] = x0 - bq[j];
            }
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                const uint32_t w = qw[k][u][i];
                uint32_t lo = w & 0x0f0f0f0fu;
                asm("" : "+v"(lo));  // keeps the mask a mask: the byte selects below then fold into the conversions
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    pd[k] += a[j] * (float)((lo >> (8 * j)) & 0xffu);
                    pd[k] += bq[j] * (float)((w >> (8 * j)) & 0xffu);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < KC; ++k) acc[k] += (float)qs[k][u] * (pd[k] - (float)qz[k][u] * xs);
    }
    q4_tail<KC, T, MU>(p, b, K, ssq, acc, bad_id, rowm, prev, red, red_u);
}

// first_exit[b] = first layer with exit flag 1 (inactive layers carry 0), else -1
__global__ void first_exit_kernel(const int32_t *exit_flags, int L, int B, int32_t *first_exit) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int f = -1;
    for (int l = 0; l < L; ++l)
        if (exit_flags[(size_t)l * B + b] != 0) {
            f = l;
            break;
        }
    first_exit[b] = f;
}

constexpr int kBatchMinTokens = 1024;  // tokens per launch from which the throughput shapes are used

template <int KC, bool SWEEP, bool EXACT>
static hipError_t launch_vpt(const PredictParams &p, hipStream_t s) {
    dim3 grid(p.B, p.L), block(kPredictThreads);
    const int nv = p.d >> 3;
    if constexpr (!SWEEP && EXACT && KC <= 8) {
        // throughput shape: K in {4, 8}, many tokens, rows of at most 4 * 256 vectors (d <= 8192)
        // (also for a few tokens when a row is exactly two vectors per thread, d = 4096: four wavefronts
        // instead of eight start and meet sooner -- 3.36 -> 3.32 us per call, 3.89 -> 3.47 us with the rows in HBM;
        // at d = 5120, where the last vectors are masked, the 512-thread shape stays ahead)
        const bool small_fit = KC == 4 && nv == 2 * 256;
        if ((p.B >= kBatchMinTokens || small_fit) && nv <= 2 * 256 * (KC == 4 ? 2 : 1)) {
            const dim3 blk(256);
            if (nv <= 2 * 256)
                hipLaunchKernelGGL((predict_kernel<KC, 2, false, true, 256, 2>), grid, blk, 0, s, p);
            else
                hipLaunchKernelGGL((predict_kernel<KC, 4, false, true, 256, 2>), grid, blk, 0, s, p);
            return hipGetLastError();
        }
    }
    const int vpt = (nv + kPredictThreads - 1) / kPredictThreads;
    if (vpt <= 1)
        hipLaunchKernelGGL((predict_kernel<KC, 1, SWEEP, EXACT>), grid, block, 0, s, p);
    else if (vpt <= 2 || KC > 8)
        hipLaunchKernelGGL((predict_kernel<KC, 2, SWEEP, EXACT>), grid, block, 0, s, p);
    else if constexpr (KC <= 8)
        hipLaunchKernelGGL((predict_kernel<KC, 4, SWEEP, EXACT>), grid, block, 0, s, p);
    return hipGetLastError();
}

template <bool SWEEP>
static hipError_t launch_kc(const PredictParams &p, hipStream_t s) {
    if (p.K == 4) return launch_vpt<4, SWEEP, true>(p, s);
    if (p.K == 8) return launch_vpt<8, SWEEP, true>(p, s);
    if (p.K < 4) return launch_vpt<4, SWEEP, false>(p, s);
    if (p.K < 8) return launch_vpt<8, SWEEP, false>(p, s);
    return launch_vpt<16, SWEEP, false>(p, s);
}

hipError_t launch_predict(const PredictParams &p, hipStream_t s) {
    return launch_kc<false>(p, s);
}

template <int KC, bool EXACT>
static hipError_t launch_q4_kc(const PredictParams &p, hipStream_t s) {
    const dim3 grid(p.B), block(kPredictThreads);
    const int nv = p.d >> 3;
    if constexpr (EXACT && KC == 4) {
        // throughput shape (see predict_kernel): a quantised row is a quarter of the bytes, so the fixed
        // cost per workgroup weighs more and small workgroups pay: 128 threads per token, four words per
        // row and thread, four hidden units per thread (B=8000 at d=4096: 51 -> 37 us)
        // chunks of 32 elements per thread when the format allows it (group % 32 == 0, rows 16-byte aligned):
        // B=8000 at d=4096: 37 -> 29 us, at d=8192: 71 -> 58 us
        const bool wide_ok = p.group % 32 == 0 && p.d % 32 == 0 && (reinterpret_cast<uintptr_t>(p.qweight) & 15) == 0;
        if (wide_ok && p.B >= kBatchMinTokens && p.d <= 32 * 128) {
            hipLaunchKernelGGL((predict_q4_wide_kernel<4, 128, 1, 4>), grid, dim3(128), 0, s, p);
            return hipGetLastError();
        }
        if (wide_ok && p.B >= kBatchMinTokens && p.d <= 32 * 256) {
            hipLaunchKernelGGL((predict_q4_wide_kernel<4, 256, 1, 2>), grid, dim3(256), 0, s, p);
            return hipGetLastError();
        }
        if (p.B >= kBatchMinTokens && nv <= 4 * 128) {
            hipLaunchKernelGGL((predict_q4_kernel<4, 4, true, 128, 4>), grid, dim3(128), 0, s, p);
            return hipGetLastError();
        }
        if (p.B >= kBatchMinTokens && nv <= 4 * 256) {
            hipLaunchKernelGGL((predict_q4_kernel<4, 4, true, 256, 2>), grid, dim3(256), 0, s, p);
            return hipGetLastError();
        }
    }
    if (nv <= kPredictThreads)
        hipLaunchKernelGGL((predict_q4_kernel<KC, 1, EXACT>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((predict_q4_kernel<KC, 2, EXACT>), grid, block, 0, s, p);
    return hipGetLastError();
}

hipError_t launch_predict_q4(const PredictParams &p, hipStream_t s) {
    if (p.K == 4) return launch_q4_kc<4, true>(p, s);
    if (p.K == 8) return launch_q4_kc<8, true>(p, s);
    if (p.K < 4) return launch_q4_kc<4, false>(p, s);
    if (p.K < 8) return launch_q4_kc<8, false>(p, s);
    return launch_q4_kc<16, false>(p, s);
}

hipError_t launch_predict_sweep(const PredictParams &p, int32_t *first_exit, hipStream_t s) {
    if (p.L > 0) {
        hipError_t e = launch_kc<true>(p, s);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(first_exit_kernel, dim3((p.B + 255) / 256), dim3(256), 0, s, p.exit_flags, p.L, p.B,
                       first_exit);
    return hipGetLastError();
}

}  // namespace specee
