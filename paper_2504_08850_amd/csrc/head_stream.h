// Streaming of full LM-head rows against one normalised hidden state held in LDS: the inner loop of
// the full-vocabulary head (paper Sec. 4.1, Sec. 4.3.3), shared by the stand-alone head kernels and by
// the verification pass of the persistent layer loop.
#pragma once
#include "device_utils.h"

namespace specee {

constexpr int kHeadUnroll = 4;   // 16-byte loads in flight per row per wavefront
constexpr int kHeadRows = 2;     // rows in flight per wavefront

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

// One wavefront's partial dot products of two LM-head rows (w0, w1: nv 16-byte vectors each) with
// x = h * gamma, which sits in LDS as two planes of float4 (xa: elements 0..3 of every vector,
// xb: 4..7; every 16-byte LDS read is then free of bank conflicts).  Lane l takes vectors l, l+64, ...
// The loads are unconditional (vector index clamped, contribution selected afterwards) so that the
// compiler keeps them all in flight instead of draining the memory pipeline at a branch join.
// STREAM: rows are read with the non-temporal hint (heads that no cache can keep).
template <bool STREAM>
__device__ __forceinline__ void head_two_rows(const half_t *w0, const half_t *w1, int nv, int lane, const floatx4 *xa,
                                              const floatx4 *xb, float &acc0, float &acc1) {
    for (int v0 = lane; v0 < nv; v0 += kWave * kHeadUnroll) {
        half8 a[kHeadUnroll], b[kHeadUnroll];
#pragma unroll
        for (int u = 0; u < kHeadUnroll; ++u) {
            const int v = min(v0 + u * kWave, nv - 1);
            a[u] = STREAM ? load_half8_stream(w0 + v * 8) : load_half8(w0 + v * 8);
            b[u] = STREAM ? load_half8_stream(w1 + v * 8) : load_half8(w1 + v * 8);
        }
#pragma unroll
        for (int u = 0; u < kHeadUnroll; ++u) {
            const bool in = v0 + u * kWave < nv;
            const int v = min(v0 + u * kWave, nv - 1);
            const floatx4 pa = xa[v], pb = xb[v];
            const float t0 = dot8(a[u], pa, pb, 0.f), t1 = dot8(b[u], pa, pb, 0.f);
            acc0 += in ? t0 : 0.f;
            acc1 += in ? t1 : 0.f;
        }
    }
}

// Arg-max (lowest row on ties) of r * <x, W[row]> over this wavefront's share of rows
// [row_begin, row_end): wavefront `wave` of `nwaves` takes pairs of rows in turn.  Every lane returns
// the wavefront's candidate; rows ascend, so the strict comparison keeps the lowest row.
template <bool STREAM>
__device__ __forceinline__ void head_argmax_rows(const half_t *lm_head, int d, int row_begin, int row_end, int wave,
                                                 int nwaves, int lane, const floatx4 *xa, const floatx4 *xb, float r,
                                                 float &bv, int &bi) {
    const int nv = d >> 3;
    for (int row = row_begin + wave * kHeadRows; row < row_end; row += nwaves * kHeadRows) {
        const bool two = row + 1 < row_end;
        const half_t *w0 = lm_head + (size_t)row * d;
        const half_t *w1 = lm_head + (size_t)(two ? row + 1 : row) * d;
        float acc0 = 0.f, acc1 = 0.f;
        head_two_rows<STREAM>(w0, w1, nv, lane, xa, xb, acc0, acc1);
        acc0 = wave_sum(acc0);
        acc1 = wave_sum(acc1);
        const float v0 = acc0 * r, v1 = acc1 * r;
        if (v0 > bv) {
            bv = v0;
            bi = row;
        }
        if (two && v1 > bv) {
            bv = v1;
            bi = row + 1;
        }
    }
}

// A head beyond this size cannot stay in the 256 MB last-level cache between passes: stream it.
inline bool head_streams(int d, int V) {
    return (size_t)V * d * sizeof(half_t) > ((size_t)288 << 20);
}

}  // namespace specee
