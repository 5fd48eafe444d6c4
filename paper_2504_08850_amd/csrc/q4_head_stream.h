// Streaming of a 4-bit group-quantised LM head against one normalised hidden state held in LDS: the inner loop of
// the quantised full-vocabulary head (paper Sec. 4.1, Sec. 4.3.3 in the weight-quantised setting of Sec. 7.1 /
// 7.3), shared by the stand-alone kernels and by the verification pass of the persistent layer loop.
#pragma once
#include "device_utils.h"

namespace specee {

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

// The workgroup has written x = h * gamma into the planes xa / xb (elements 0..3 and 4..7 of every eight) and
// met at a barrier.  Forms the per-group sums of x (xs [ng], fixed order: ascending elements) and, for the wide
// path, turns the planes into the coefficients (a, b) in place.  Ends with a barrier.
template <int THREADS, bool WIDE>
__device__ __forceinline__ void q4_prepare_planes(floatx4 *xa, floatx4 *xb, float *xs, int nv, int ng, int group,
                                                  int tid) {
    const int vpg = group >> 3;
    for (int g = tid; g < ng; g += THREADS) {
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
        for (int v = tid; v < nv; v += THREADS) {
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

}

// Rows [row_begin, row_end) of the head: wavefront `wave` of `nwaves` takes groups of kQ4HeadRows rows in turn and
// calls emit(row, r * <x, W[row]>) for each, uniformly over the wavefront, rows ascending.
// WIDE: group % 32 == 0 and rows of codes 16-byte aligned (d % 32 == 0): a lane owns chunks of 32 elements.
// Otherwise a lane owns single words (8 elements, always inside one group since group % 8 == 0).
template <bool WIDE, class Emit>
__device__ __forceinline__ void q4_head_rows(const uint32_t *qweight, const half_t *scales, const half_t *zeros, int d,
                                             int group, int row_begin, int row_end, int wave, int nwaves, int lane,
                                             const floatx4 *xa, const floatx4 *xb, const float *xs, float r,
                                             Emit emit) {
    const int nv = d >> 3, ng = d / group;
    constexpr int R = kQ4HeadRows;
    const int gz = min(lane, ng - 1);  // this lane's group in the zero-point term
    for (int row = row_begin + wave * R; row < row_end; row += nwaves * R) {
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
            if (row + q < row_end) emit(row + q, v);  // uniform over the wavefront; rows ascend
        }
    }
}

}  // namespace specee
