// Full-vocabulary LM head with the final RMSNorm fused in (paper Sec. 4.1: the
// search space the speculative predictor avoids; Sec. 4.3.3: global logits for
// verification).  This is a pure HBM stream of V*d halves: the kernel exists to
// run at memory bandwidth.
//
// GEMV form (one hidden state per grid.y): the normalised-and-weighted hidden
// state x = h * gamma is built once per workgroup in LDS as fp32 (two planes of
// float4 so that every ds_read_b128 is bank-conflict free), then each wavefront
// streams whole LM-head rows with 16-byte-per-lane loads, two rows and four
// loads per row in flight, and reduces with DPP.  The RMSNorm scale multiplies
// the finished dot product.
#include "device_utils.h"
#include "kernels.h"

namespace specee {

constexpr int kGemvThreads = 512;
constexpr int kGemvWaves = kGemvThreads / kWave;
constexpr int kGemvUnroll = 4;   // 16-byte loads in flight per row per wavefront
constexpr int kGemvRows = 2;     // rows in flight per wavefront

__device__ __forceinline__ float dot8(half8 w, floatx4 xa, floatx4 xb, float acc) {
    acc += (float)w[0] * xa[0];
    acc += (float)w[1] * xa[1];
    acc += (float)w[2] * xa[2];
    acc += (float)w[3] * xa[3];
    acc += (float)w[4] * xb[0];
    acc += (float)w[5] * xb[1];
    acc += (float)w[6] * xb[2];
    acc += (float)w[7] * xb[3];
    return acc;
}

__global__ __launch_bounds__(kGemvThreads) void lm_head_gemv_kernel(int d, int V, float eps, const half_t *hidden,
                                                                    const half_t *gamma, const half_t *lm_head,
                                                                    float *out, int rows_per_wg) {
    extern __shared__ float4 lds_x[];  // [2][nv]: plane 0 = elements 0..3 of each vector, plane 1 = 4..7
    __shared__ float red[kGemvWaves];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int nv = d >> 3;
    const int n = blockIdx.y;
    floatx4 *xa = reinterpret_cast<floatx4 *>(lds_x);
    floatx4 *xb = xa + nv;

    const half_t *h = hidden + (size_t)n * d;
    float ssq = 0.f;
    for (int v = tid; v < nv; v += kGemvThreads) {
        half8 h8 = load_half8(h + v * 8), g8 = load_half8(gamma + v * 8);
        floatx4 a, b;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float h0 = (float)h8[e], h1 = (float)h8[4 + e];
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
    for (int w = 0; w < kGemvWaves; ++w) ssq += red[w];
    const float r = 1.0f / sqrtf(ssq / (float)d + eps);

    const int row_begin = blockIdx.x * rows_per_wg;
    const int row_end = min(V, row_begin + rows_per_wg);
    float *o = out + (size_t)n * V;
    for (int row = row_begin + wave * kGemvRows; row < row_end; row += kGemvWaves * kGemvRows) {
        const bool two = row + 1 < row_end;
        const half_t *w0 = lm_head + (size_t)row * d;
        const half_t *w1 = lm_head + (size_t)(two ? row + 1 : row) * d;
        float acc0 = 0.f, acc1 = 0.f;
        for (int v0 = lane; v0 < nv; v0 += kWave * kGemvUnroll) {
            half8 a[kGemvUnroll], b[kGemvUnroll];
#pragma unroll
            for (int u = 0; u < kGemvUnroll; ++u) {
                int v = v0 + u * kWave;
                bool in = v < nv;
                a[u] = in ? load_half8(w0 + v * 8) : zero_half8();
                b[u] = in ? load_half8(w1 + v * 8) : zero_half8();
            }
#pragma unroll
            for (int u = 0; u < kGemvUnroll; ++u) {
                int v = v0 + u * kWave;
                if (v < nv) {
                    floatx4 pa = xa[v], pb = xb[v];
                    acc0 = dot8(a[u], pa, pb, acc0);
                    acc1 = dot8(b[u], pa, pb, acc1);
                }
            }
        }
        acc0 = wave_sum(acc0);
        acc1 = wave_sum(acc1);
        if (lane == 0) {
            o[row] = acc0 * r;
            if (two) o[row + 1] = acc1 * r;
        }
    }
}

hipError_t launch_lm_head_gemv(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                               const half_t *lm_head, float *out, hipStream_t s) {
    // two resident workgroups per CU on 256 CUs; each takes a contiguous block of rows
    int wgs = 512;
    int rows_per_wg = (V + wgs - 1) / wgs;
    const int quantum = kGemvWaves * kGemvRows;
    rows_per_wg = ((rows_per_wg + quantum - 1) / quantum) * quantum;
    wgs = (V + rows_per_wg - 1) / rows_per_wg;
    size_t lds = (size_t)d * sizeof(float);
    hipLaunchKernelGGL(lm_head_gemv_kernel, dim3(wgs, N), dim3(kGemvThreads), lds, s, d, V, eps, hidden, gamma,
                       lm_head, out, rows_per_wg);
    return hipGetLastError();
}

}  // namespace specee
