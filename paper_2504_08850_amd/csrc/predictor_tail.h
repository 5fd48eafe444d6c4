// Feature construction and predictor MLP shared by the single-token and the
// token-tree kernels (paper Sec. 4.3.1 features (2),(3) and Sec. 4.3.2):
// local softmax over the K speculative logits, probability variation against
// the previous layer, then thread j evaluates hidden unit j of the 3K -> H MLP.
// A thread's first MLP row can be requested long before the logits exist, so
// its latency hides behind the LM-head row traffic.
#pragma once
#include "device_utils.h"

namespace specee {

// softmax over K values held in registers (K <= KC); NaN logits poison the row
template <int KC>
__device__ __forceinline__ void local_softmax(const float (&z)[KC], int K, float (&p)[KC]) {
    float m = z[0];
#pragma unroll
    for (int k = 1; k < KC; ++k)
        if (k < K) m = fmaxf(m, z[k]);
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        p[k] = (k < K) ? __expf(z[k] - m) : 0.f;
        s += p[k];
    }
    float inv = __frcp_rn(s);
#pragma unroll
    for (int k = 0; k < KC; ++k) p[k] *= inv;
    bool bad = false;  // fmaxf drops NaN, so propagate it by hand
#pragma unroll
    for (int k = 0; k < KC; ++k)
        if (k < K && z[k] != z[k]) bad = true;
    if (bad) {
#pragma unroll
        for (int k = 0; k < KC; ++k) p[k] = quiet_nan();
    }
}

template <int KC>
struct MlpRow {
    uint2 w1[(3 * KC + 3) / 4];  // 3*KC halves of W1[j][:], valid when K == KC
    half_t w2, b1;               // as loaded; widened where they are used, so that requesting a row never waits
    bool has_b1;
};

// Request hidden unit `j`'s weights.  Vector loads need K == KC (row length
// 3*KC halves is then a multiple of 8 bytes and feature indices are static).
template <int KC>
__device__ __forceinline__ void mlp_row_load(MlpRow<KC> &r, const half_t *W1, const half_t *b1, const half_t *w2,
                                             int K, int H, int j) {
    // Nothing here consumes what it loads and no load sits under a per-lane branch: the index is
    // clamped (callers ignore units j >= H) and an absent bias reads w2 instead, masked at use.
    const int jj = min(j, H - 1);
    if (K == KC) {
        const uint2 *src = reinterpret_cast<const uint2 *>(W1 + (size_t)jj * 3 * KC);
#pragma unroll
        for (int q = 0; q < (3 * KC) / 4; ++q) r.w1[q] = src[q];
    }
    r.w2 = w2[jj];
    r.b1 = (b1 ? b1 : w2)[jj];
    r.has_b1 = b1 != nullptr;
}

// w2[j] * relu(b1[j] + W1[j] . [z | p | p - prev]) for one hidden unit
template <int KC>
__device__ __forceinline__ float mlp_unit(const MlpRow<KC> &r, const half_t *W1, int K, int j, const float (&z)[KC],
                                          const float (&pr)[KC], const float (&prev)[KC]) {
    float a = r.has_b1 ? (float)r.b1 : 0.f;
    if (K == KC) {
        float f[3 * KC];
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            f[k] = z[k];
            f[KC + k] = pr[k];
            f[2 * KC + k] = pr[k] - prev[k];
        }
#pragma unroll
        for (int q = 0; q < (3 * KC) / 4; ++q) {
            half4 w4 = __builtin_bit_cast(half4, r.w1[q]);
#pragma unroll
            for (int e = 0; e < 4; ++e) a += (float)w4[e] * f[q * 4 + e];
        }
    } else {
        const half_t *src = W1 + (size_t)j * 3 * K;
#pragma unroll
        for (int k = 0; k < KC; ++k)
            if (k < K) a += (float)src[k] * z[k];
#pragma unroll
        for (int k = 0; k < KC; ++k)
            if (k < K) a += (float)src[K + k] * pr[k];
#pragma unroll
        for (int k = 0; k < KC; ++k)
            if (k < K) a += (float)src[2 * K + k] * (pr[k] - prev[k]);
    }
    float v = (float)r.w2 * fmaxf(a, 0.f);
    return (a != a) ? quiet_nan() : v;  // fmaxf drops NaN; keep invalid ids visible
}

// This thread's share of the output pre-activation: units tid, tid+T, ...
// `first[0..MU)` hold the prefetched rows of units tid, tid+T, ..., tid+(MU-1)*T; further units (H
// larger than MU*T) are fetched here.
template <int KC, int T, int MU>
__device__ __forceinline__ float mlp_partial(const MlpRow<KC> (&first)[MU], const half_t *W1, const half_t *b1,
                                             const half_t *w2, int K, int H, int tid, const float (&z)[KC],
                                             const float (&pr)[KC], const float (&prev)[KC]) {
    float part = 0.f;
#pragma unroll
    for (int m = 0; m < MU; ++m)
        if (tid + m * T < H) part += mlp_unit<KC>(first[m], W1, K, tid + m * T, z, pr, prev);
    for (int j = tid + MU * T; j < H; j += T) {
        MlpRow<KC> r;
        mlp_row_load<KC>(r, W1, b1, w2, K, H, j);
        part += mlp_unit<KC>(r, W1, K, j, z, pr, prev);
    }
    return part;
}

__device__ __forceinline__ float sigmoidf(float u) {
    return __frcp_rn(1.0f + __expf(-u));
}

}  // namespace specee
