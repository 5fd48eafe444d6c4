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

namespace specee {

constexpr int kQ4HeadThreads = 512;
constexpr int kQ4HeadWaves = kQ4HeadThreads / kWave;
constexpr int kQ4HeadRows = 4;    // rows in flight per wavefront
constexpr int kQ4HeadChunks = 1;  // 16-byte chunks of each of them

// sum over the 32 elements of one 16-byte chunk of codes of x_i * c_i.
// Byte j of word i holds elements 8i+2j (low nibble) and 8i+2j+1 (high): with a = x0 - x1/16 and
// b = x1/16, x0*lo + x1*hi = a*lo + b*byte, so the high nibbles are never extracted.  The LDS planes hold
// a and b already (pairs (a, b) in element order: the workgroup transforms x once, after the group sums), so a
// lane spends two instructions per weight pair-half and holds no derived values: the registers that would keep
// x, a and b of a chunk alive across the rows in flight were what limited the kernel to two wavefronts per SIMD.
__device__ __forceinline__ float q4_chunk_dot(const uintx4 w, const floatx4 *xa, const floatx4 *xb, int v0) {
    float pd = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const floatx4 lo4 = xa[v0 + i], hi4 = xb[v0 + i];  // (a, b) of element pairs 0,1 and 2,3 of vector v0 + i
        const float ab[8] = {lo4[0], lo4[1], lo4[2], lo4[3], hi4[0], hi4[1], hi4[2], hi4[3]};
        const uint32_t word = w[i];
        uint32_t lo = word & 0x0f0f0f0fu;
        asm("" : "+v"(lo));  // keeps the mask a mask: the byte selects below then fold into the conversions
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            pd += ab[2 * j] * (float)((lo >> (8 * j)) & 0xffu);
            pd += ab[2 * j + 1] * (float)((word >> (8 * j)) & 0xffu);
        }
    }
    return pd;
}

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
    // per-group sums of x (fixed order: ascending elements)
    const int vpg = group >> 3;
    for (int g = tid; g < ng; g += kQ4HeadThreads) {
        float s = 0.f;
        for (int v = g * vpg; v < (g + 1) * vpg; ++v) {
            const floatx4 a = xa[v], b = xb[v];
            s += ((a[0] + a[1]) + (a[2] + a[3])) + ((b[0] + b[1]) + (b[2] + b[3]));
        }
        xs[g] = s;
    }
    __syncthreads();
    if (WIDE) {
        // x -> (a, b) in place, every thread on the vectors it wrote above
        for (int v = tid; v < nv; v += kQ4HeadThreads) {
            floatx4 a = xa[v], b = xb[v];
#pragma unroll
            for (int e = 0; e < 4; e += 2) {
                const float b0 = a[e + 1] * 0.0625f, b1 = b[e + 1] * 0.0625f;
                a[e] -= b0;
                a[e + 1] = b0;
                b[e] -= b1;
                b[e + 1] = b1;
            }
            xa[v] = a;
            xb[v] = b;
        }
        __syncthreads();
    }

    const int row_begin = blockIdx.x * rows_per_wg;
    const int row_end = min(V, row_begin + rows_per_wg);
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    constexpr int R = kQ4HeadRows;
    const int gz = min(lane, ng - 1);  // this lane's group in the zero-point term
    for (int row = row_begin + wave * R; row < row_end; row += kQ4HeadWaves * R) {
        size_t rr[R];
        half_t zs[R], zz[R];
#pragma unroll
        for (int q = 0; q < R; ++q) {
            rr[q] = (size_t)min(row + q, row_end - 1);  // clamped: rows past the end repeat the last one, unused
            zs[q] = scales[rr[q] * ng + gz];            // requested with the codes, used after them
            zz[q] = zeros[rr[q] * ng + gz];
        }
        float acc[R];
#pragma unroll
        for (int q = 0; q < R; ++q) acc[q] = 0.f;
        if (WIDE) {
            const int nc = d >> 5;
            constexpr int U = kQ4HeadChunks;  // chunks per row in flight, clamped and masked
            for (int c0 = lane; c0 < nc; c0 += U * kWave) {
                uintx4 w[R][U];
                half_t sc[R][U];
                int cc[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    cc[u] = min(c0 + u * kWave, nc - 1);
                    const int gi = (cc[u] * 32) / group;
#pragma unroll
                    for (int q = 0; q < R; ++q) {
                        w[q][u] = *reinterpret_cast<const uintx4 *>(qweight + rr[q] * nv + cc[u] * 4);
                        sc[q][u] = scales[rr[q] * ng + gi];
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const bool in = c0 + u * kWave < nc;
#pragma unroll
                    for (int q = 0; q < R; ++q) {
                        const float pd = q4_chunk_dot(w[q][u], xa, xb, cc[u] * 4);
                        acc[q] += in ? (float)sc[q][u] * pd : 0.f;
                    }
                }
            }
        } else {
            for (int v = lane; v < nv; v += kWave) {
                const int gi = (v * 8) / group;
                uint32_t w[R];
                half_t sc[R];
#pragma unroll
                for (int q = 0; q < R; ++q) {
                    w[q] = qweight[rr[q] * nv + v];
                    sc[q] = scales[rr[q] * ng + gi];
                }
                const floatx4 lo4 = xa[v], hi4 = xb[v];
                const float x[8] = {lo4[0], lo4[1], lo4[2], lo4[3], hi4[0], hi4[1], hi4[2], hi4[3]};
#pragma unroll
                for (int q = 0; q < R; ++q) {
                    float pd = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) pd += x[e] * (float)((w[q] >> (4 * e)) & 15u);
                    acc[q] += (float)sc[q] * pd;
                }
            }
        }
        // zero-point term: - sum_g scale_g * zero_g * xs_g (lane g; further groups, if any, in a loop)
        {
            const float t = lane < ng ? xs[gz] : 0.f;
#pragma unroll
            for (int q = 0; q < R; ++q) acc[q] -= (float)zs[q] * (float)zz[q] * t;
            for (int g = lane + kWave; g < ng; g += kWave) {
                const float tg = xs[g];
#pragma unroll
                for (int q = 0; q < R; ++q) acc[q] -= (float)scales[rr[q] * ng + g] * (float)zeros[rr[q] * ng + g] * tg;
            }
        }
#pragma unroll
        for (int q = 0; q < R; ++q) {
            const float v = wave_sum(acc[q]) * r;
            if (row + q < row_end) {  // uniform over the wavefront
                if (ARGMAX) {
                    if (v > bv) {
                        bv = v;
                        bi = row + q;
                    }
                } else if (lane == 0) {
                    out[(size_t)n * V + row + q] = v;
                }
            }
        }
    }
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
