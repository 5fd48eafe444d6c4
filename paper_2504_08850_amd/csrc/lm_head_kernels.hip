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
#include "head_stream.h"
#include "kernels.h"

namespace specee {

constexpr int kGemvThreads = 512;
constexpr int kGemvWaves = kGemvThreads / kWave;
constexpr int kGemvRows = kHeadRows;  // rows in flight per wavefront

// ARGMAX: instead of storing the V logits, keep the best (value, row) of this
// workgroup's rows (lowest row on ties) and store one candidate per workgroup:
// best_val / best_idx [N][gridDim.x].
// STREAM: the head is larger than the last-level cache, so its rows are read with the non-temporal hint
// (350 -> 310 us at 128256 x 8192); a head that fits is read normally and partly served by that cache from
// one call to the next (262 MB at 32000 x 4096: 39.7 us against 41.1 us with the hint).
template <bool ARGMAX, bool STREAM>
__global__ __launch_bounds__(kGemvThreads) void lm_head_gemv_kernel(int d, int V, float eps, const half_t *hidden,
                                                                    const half_t *gamma, const half_t *lm_head,
                                                                    float *out, int rows_per_wg, float *best_val,
                                                                    int32_t *best_idx, const int32_t *gate,
                                                                    const int32_t *done) {
    extern __shared__ float4 lds_x[];  // [2][nv]: plane 0 = elements 0..3 of each vector, plane 1 = 4..7
    __shared__ float red[kGemvWaves];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int nv = d >> 3;
    const int n = blockIdx.y;
    // uniform over the workgroup: this hidden state is not being verified
    if (ARGMAX && ((gate && gate[n] == 0) || (done && done[n] != 0))) return;
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
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    if (ARGMAX) {
        head_argmax_rows<STREAM>(lm_head, d, row_begin, row_end, wave, kGemvWaves, lane, xa, xb, r, bv, bi);
    } else {
        for (int row = row_begin + wave * kGemvRows; row < row_end; row += kGemvWaves * kGemvRows) {
            const bool two = row + 1 < row_end;
            const half_t *w0 = lm_head + (size_t)row * d;
            const half_t *w1 = lm_head + (size_t)(two ? row + 1 : row) * d;
            float acc0 = 0.f, acc1 = 0.f;
            head_two_rows<STREAM>(w0, w1, nv, lane, xa, xb, acc0, acc1);
            acc0 = wave_sum_to_last_row(acc0);  // DPP only; the total lands in the last 16 lanes
            acc1 = wave_sum_to_last_row(acc1);
            if (lane == kWave - 1) {
                o[row] = acc0 * r;
                if (two) o[row + 1] = acc1 * r;
            }
        }
    }
    if (ARGMAX) {
        // rows ascend within a wave, so strict '>' already kept the lowest row; combine the waves in LDS
        __shared__ float wv[kGemvWaves];
        __shared__ int wi[kGemvWaves];
        if (lane == 0) {
            wv[wave] = bv;
            wi[wave] = bi;
        }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < kGemvWaves; ++w)
                if (wv[w] > bv || (wv[w] == bv && wi[w] < bi)) {
                    bv = wv[w];
                    bi = wi[w];
                }
            best_val[(size_t)n * gridDim.x + blockIdx.x] = bv;
            best_idx[(size_t)n * gridDim.x + blockIdx.x] = bi;
        }
    }
}

// Verification tail (paper Sec. 4.3.3): combine P candidates per hidden state
// into the arg-max token (lowest id on ties) and test membership in the K ids.
__global__ __launch_bounds__(256) void verify_finish_kernel(const float *best_val, const int32_t *best_idx, int P,
                                                            const int32_t *ids, int K, const int32_t *gate,
                                                            int32_t *done, int32_t *token, float *max_logit,
                                                            int32_t *hit) {
    __shared__ float wv[4];
    __shared__ int wi[4];
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if ((gate && gate[n] == 0) || (done && done[n] != 0)) {  // not verified: no candidates were written
        if (tid == 0) {
            token[n] = -1;
            max_logit[n] = 0.f;
            hit[n] = 0;
        }
        return;
    }
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = tid; i < P; i += 256) {
        float v = best_val[(size_t)n * P + i];
        int ix = best_idx[(size_t)n * P + i];
        if (v > bv || (v == bv && ix < bi)) {
            bv = v;
            bi = ix;
        }
    }
    wave_argmax(bv, bi);
    if (lane == 0) {
        wv[wave] = bv;
        wi[wave] = bi;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w)
            if (wv[w] > bv || (wv[w] == bv && wi[w] < bi)) {
                bv = wv[w];
                bi = wi[w];
            }
        int h = 0;
        for (int k = 0; k < K; ++k)
            if (ids[(size_t)n * K + k] == bi) h = 1;
        token[n] = bi;
        max_logit[n] = bv;
        hit[n] = h;
        if (done && h) done[n] = 1;  // the token leaves the model at this layer
    }
}

// Rows per workgroup: two resident workgroups per CU on 256 CUs, each with a contiguous block of rows
// that is a whole number of rounds of its wavefronts.
// About three workgroups per CU (six wavefronts per SIMD at 64 registers): measured on 32000 x 4096 against two
// (40.7 -> 38.5 us) and four (44.7 us).
static int gemv_rows_per_wg(int V) {
    const int wgs = 768;
    const int quantum = kGemvWaves * kGemvRows;
    return (((V + wgs - 1) / wgs + quantum - 1) / quantum) * quantum;
}

int lm_head_gemv_workgroups(int V) {
    const int rows_per_wg = gemv_rows_per_wg(V);
    return (V + rows_per_wg - 1) / rows_per_wg;
}

// One launch of the head kernel.  x = h * gamma takes 4*d bytes of dynamic LDS; from d = 12288 on that is
// more than a kernel may use without asking, so the limit is raised (per launch: the library keeps no
// state; a refusal shows as the launch error).
template <bool ARGMAX, bool STREAM>
static void launch_gemv_one(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                            const half_t *lm_head, float *out, float *best_val, int32_t *best_idx,
                            const int32_t *gate, const int32_t *done, hipStream_t s) {
    const int rows_per_wg = gemv_rows_per_wg(V);
    const int wgs = (V + rows_per_wg - 1) / rows_per_wg;
    const size_t lds = (size_t)d * sizeof(float);
    auto kern = lm_head_gemv_kernel<ARGMAX, STREAM>;
    if (lds > 48 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds);
    hipLaunchKernelGGL(kern, dim3(wgs, N), dim3(kGemvThreads), lds, s, d, V, eps, hidden, gamma, lm_head, out,
                       rows_per_wg, best_val, best_idx, gate, done);
}

hipError_t launch_lm_head_gemv(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                               const half_t *lm_head, float *out, hipStream_t s) {
    if (head_streams(d, V))
        launch_gemv_one<false, true>(d, V, eps, N, hidden, gamma, lm_head, out, nullptr, nullptr, nullptr, nullptr, s);
    else
        launch_gemv_one<false, false>(d, V, eps, N, hidden, gamma, lm_head, out, nullptr, nullptr, nullptr, nullptr, s);
    return hipGetLastError();
}

hipError_t launch_lm_head_argmax_gemv(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                                      const half_t *lm_head, float *best_val, int32_t *best_idx, const int32_t *gate,
                                      const int32_t *done, hipStream_t s) {
    if (head_streams(d, V))
        launch_gemv_one<true, true>(d, V, eps, N, hidden, gamma, lm_head, nullptr, best_val, best_idx, gate, done, s);
    else
        launch_gemv_one<true, false>(d, V, eps, N, hidden, gamma, lm_head, nullptr, best_val, best_idx, gate, done, s);
    return hipGetLastError();
}

hipError_t launch_verify_finish(const float *best_val, const int32_t *best_idx, int P, int N, const int32_t *ids,
                                int K, const int32_t *gate, int32_t *done, int32_t *token, float *max_logit,
                                int32_t *hit, hipStream_t s) {
    hipLaunchKernelGGL(verify_finish_kernel, dim3(N), dim3(256), 0, s, best_val, best_idx, P, ids, K, gate, done,
                       token, max_logit, hit);
    return hipGetLastError();
}

}  // namespace specee
