// Full-vocabulary LM head on a 4-bit group-quantised head, with the final RMSNorm fused in: the
// search space and the verification step (paper Sec. 4.1, Sec. 4.3.3) in the weight-quantised setting
// of the cloud evaluation (Sec. 7.1 "Quantization", Sec. 7.3).  Format as for the quantised-rows
// predictor: element i of row v is a code c in 0..15 in bits 4*(i%8).. of 32-bit word i/8 and stands for
// scale[v][i/group] * (c - zero[v][i/group]).
//
// A row is d/2 bytes of codes plus 4*d/group bytes of scales and zero-points: a 32000 x 4096 head is
// 70 MB instead of 262 MB, so a pass is bound by HBM for a quarter of the time -- and by the arithmetic of
// unpacking, which is of the same order.  Per row
//     logit = r * sum_g scale_g * ( sum_{i in g} x_i c_i  -  zero_g * sum_{i in g} x_i ),   x = h * gamma,
// so the dequantised weights never exist: x sits in LDS as two float4 planes (as in the fp16 head), the
// per-group sums of x are formed once per workgroup, a lane takes 32 consecutive elements (one 16-byte
// load of codes, one scale) and forms its share of the first sum with one conversion and one FMA per
// nibble; the zero-point term costs one FMA per group and row.
#include "device_utils.h"
#include "kernels.h"
#include "q4_head_stream.h"

namespace specee {

constexpr int kQ4HeadThreads = 512;
constexpr int kQ4HeadWaves = kQ4HeadThreads / kWave;

// WIDE: group % 32 == 0 and rows of codes 16-byte aligned (d % 32 == 0): a lane owns chunks of 32 elements.
// Otherwise a lane owns single words (8 elements, always inside one group since group % 8 == 0).
// ARGMAX: one arg-max candidate per workgroup and hidden state instead of the V logits.
template <bool ARGMAX, bool WIDE>
__global__ __launch_bounds__(kQ4HeadThreads, 4) void lm_head_q4_kernel(int d, int V, float eps, const half_t *hidden,
                                                                    const half_t *gamma, const uint32_t *qweight,
                                                                    const half_t *scales, const half_t *zeros,
                                                                    int group, float *out, int rows_per_wg,
                                                                    float *best_val, int32_t *best_idx,
                                                                    const int32_t *gate, const int32_t *done) {
    extern __shared__ float4 q4_lds[];  // [2][nv] planes of x, then [ng] per-group sums of x
    __shared__ float red[kQ4HeadWaves];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int nv = d >> 3, ng = d / group;
    const int n = blockIdx.y;
    if (ARGMAX && ((gate && gate[n] == 0) || (done && done[n] != 0))) return;  // uniform: not verified
    floatx4 *xa = reinterpret_cast<floatx4 *>(q4_lds);
    floatx4 *xb = xa + nv;
    float *xs = reinterpret_cast<float *>(xb + nv);

    const half_t *h = hidden + (size_t)n * d;
    float ssq = 0.f;
    for (int v = tid; v < nv; v += kQ4HeadThreads) {
        const half8 h8 = load_half8(h + v * 8), g8 = load_half8(gamma + v * 8);
        floatx4 a, b;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float h0 = (float)h8[e], h1 = (float)h8[4 + e];
            a[e] = h0 * (float)g8[e];
            b[e] = h1 * (float)g8[4 + e];
            ssq += h0 * h0;
            ssq += h1 * h1;
        }
        xa[v] = a;
        xb[v] = b;
    }
    ssq = wave_sum(ssq);
    if (lane == 0) red[wave] = ssq;
    __syncthreads();
    ssq = 0.f;
#pragma unroll
    for (int w = 0; w < kQ4HeadWaves; ++w) ssq += red[w];
    const float r = 1.0f / sqrtf(ssq / (float)d + eps);
    q4_prepare_planes<kQ4HeadThreads, WIDE>(xa, xb, xs, nv, ng, group, tid);

    const int row_begin = blockIdx.x * rows_per_wg;
    const int row_end = min(V, row_begin + rows_per_wg);
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    q4_head_rows<WIDE>(qweight, scales, zeros, d, group, row_begin, row_end, wave, kQ4HeadWaves, lane, xa, xb, xs, r,
                       [&](int row, float v) {
                           if (ARGMAX) {
                               if (v > bv) {
                                   bv = v;
                                   bi = row;
                               }
                           } else if (lane == 0) {
                               out[(size_t)n * V + row] = v;
                           }
                       });
    if (ARGMAX) {
        // rows ascend within a wave, so strict '>' already kept the lowest row; combine the waves in LDS
        __shared__ float wv[kQ4HeadWaves];
        __shared__ int wi[kQ4HeadWaves];
        if (lane == 0) {
            wv[wave] = bv;
            wi[wave] = bi;
        }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < kQ4HeadWaves; ++w)
                if (wv[w] > bv || (wv[w] == bv && wi[w] < bi)) {
                    bv = wv[w];
                    bi = wi[w];
                }
            best_val[(size_t)n * gridDim.x + blockIdx.x] = bv;
            best_idx[(size_t)n * gridDim.x + blockIdx.x] = bi;
        }
    }
}

static int q4_rows_per_wg(int V) {
    const int wgs = 512;  // two resident workgroups per CU
    const int quantum = kQ4HeadWaves * kQ4HeadRows;
    return (((V + wgs - 1) / wgs + quantum - 1) / quantum) * quantum;
}

int lm_head_q4_workgroups(int V) {
    const int rows_per_wg = q4_rows_per_wg(V);
    return (V + rows_per_wg - 1) / rows_per_wg;
}

template <bool ARGMAX>
static hipError_t launch_q4_head(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                                 const uint32_t *qweight, const half_t *scales, const half_t *zeros, int group,
                                 float *out, float *best_val, int32_t *best_idx, const int32_t *gate,
                                 const int32_t *done, hipStream_t s) {
    const int rows_per_wg = q4_rows_per_wg(V);
    const int wgs = (V + rows_per_wg - 1) / rows_per_wg;
    const size_t lds = (size_t)d * sizeof(float) + (size_t)(d / group) * sizeof(float);
    const bool wide = group % 32 == 0 && d % 32 == 0 && (reinterpret_cast<uintptr_t>(qweight) & 15) == 0;
    auto kern = wide ? lm_head_q4_kernel<ARGMAX, true> : lm_head_q4_kernel<ARGMAX, false>;
    if (lds > 48 * 1024)  // per launch: the library keeps no state; a refusal shows as the launch error
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds);
    hipLaunchKernelGGL(kern, dim3(wgs, N), dim3(kQ4HeadThreads), lds, s, d, V, eps, hidden, gamma, qweight, scales,
                       zeros, group, out, rows_per_wg, best_val, best_idx, gate, done);
    return hipGetLastError();
}

hipError_t launch_lm_head_q4(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                             const uint32_t *qweight, const half_t *scales, const half_t *zeros, int group,
                             float *out, hipStream_t s) {
    return launch_q4_head<false>(d, V, eps, N, hidden, gamma, qweight, scales, zeros, group, out, nullptr, nullptr,
                                 nullptr, nullptr, s);
}

hipError_t launch_lm_head_q4_argmax(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                                    const uint32_t *qweight, const half_t *scales, const half_t *zeros, int group,
                                    float *best_val, int32_t *best_idx, const int32_t *gate, const int32_t *done,
                                    hipStream_t s) {
    return launch_q4_head<true>(d, V, eps, N, hidden, gamma, qweight, scales, zeros, group, nullptr, best_val,
                                best_idx, gate, done, s);
}

}  // namespace specee
