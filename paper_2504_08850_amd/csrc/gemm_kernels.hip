// Full-vocabulary LM head for several hidden states on the matrix cores (paper Sec. 4.1:
// the search space of earlier early-exit predictors; Sec. 4.3.3: global logits for
// verification):  Y[n][v] = r_n * sum_i (h[n][i] * gamma[i]) * W[v][i],  n < N <= 64 per
// workgroup column, all V rows.  The work is one pass over the V*d halves of the head, so
// the kernel is built to stream: one workgroup owns 64*TPW consecutive rows over all of d.
//
// Mapping onto v_mfma_f32_16x16x32_f16 (64 lanes; lane = 16*q + c):
//   A operand = LM-head rows: lane holds 8 consecutive halves of row (m0 + c) at a k-offset
//               chosen by q -- exactly one 16-byte global load, so streamed rows feed the
//               matrix core with no LDS hop;
//   B operand = x = h*gamma for hidden state (n0 + c), same k-offsets, shared by the four
//               wavefronts through double-buffered LDS;
//   D         = lane holds Y[m0 + 4q .. 4q+3][n0 + c]  -> one 16-byte store.
// Any assignment of k-slots to (q, element) is valid as long as A and B use the same one;
// it is chosen so that the four q-groups of a row read 128 contiguous bytes per
// 64-element stage (q*32 bytes + 16*j).
//
// x is not representable in fp16 (it is a product of two fp16 numbers), and rounding it
// would cost ~4e-4 of a logit's standard deviation.  It is split exactly instead:
// hi = round(h*gamma), lo = round(fma(h, gamma, -hi)) in packed fp16 arithmetic, and both
// halves are multiplied; the matrix cores have the headroom because the pass is bound by
// memory.
//
// MODE 1: normalised logits are stored.  MODE 2: they are reduced to one arg-max candidate
// per hidden state and workgroup (verification never needs the [N][V] array).
#include "device_utils.h"
#include "kernels.h"

namespace specee {

constexpr int kGemmThreads = 256;
constexpr int kGemmWaves = 4;
constexpr int kKC = 64;           // k elements per LDS stage (128 bytes of every row)
constexpr int kNB = 64;           // hidden states per workgroup (4 n-tiles of 16)
constexpr int kLdsRow = kKC + 8;  // halves per LDS row: 144 bytes, keeps 16-byte reads spread over banks

// PD: stages of global loads kept in flight per wavefront.  The stage loop is free of
// branches (loads past the end are issued on clamped addresses and contribute zeros): a load
// under a branch makes the compiler drain every outstanding load at the join.
template <int TPW, int MODE, int PD>
// (two wavefronts per SIMD asked for: unbounded, the 256-row shape took 272 registers, i.e. one workgroup per CU)
__global__ __launch_bounds__(kGemmThreads, 2) void full_head_gemm_kernel(GemmParams p) {
    __shared__ __attribute__((aligned(16))) half_t lds_hi[2][kNB][kLdsRow];
    __shared__ __attribute__((aligned(16))) half_t lds_lo[2][kNB][kLdsRow];
    __shared__ float lds_ssq[kNB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, q = lane >> 4;
    const int n0 = blockIdx.z * kNB;
    const int d = p.d, M = p.V;
    if (MODE == 2 && (p.gate || p.done)) {
        // verification is gated by the predictor's exit flags: when none of this block's hidden states
        // is to be verified the pass over the LM head is skipped (the tail kernel fills in the outputs)
        int any = 0;
        if (tid < kNB && n0 + tid < p.N)
            any = (!p.gate || p.gate[n0 + tid] != 0) && (!p.done || p.done[n0 + tid] == 0);
        if (__syncthreads_or(any) == 0) return;
    }
    const int nchunks = (d + kKC - 1) / kKC;
    const int m0 = blockIdx.x * (16 * TPW * kGemmWaves);

    // ---- A side: this lane's rows (clamped: rows past the end are loaded but never stored)
    const half_t *rowptr[TPW];
#pragma unroll
    for (int tp = 0; tp < TPW; ++tp) {
        const int m = min(m0 + (wave * TPW + tp) * 16 + c, M - 1);
        rowptr[tp] = p.lm_head + (size_t)m * d;
    }
    // ---- B side: this thread stages vector column vc of hidden states r0 and r0+32
    const int vc = tid & 7, r0 = tid >> 3;
    const half_t *hptr[2];
    bool hok[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int n = n0 + r0 + 32 * i;
        hok[i] = n < p.N;
        hptr[i] = p.hidden + (size_t)(hok[i] ? n : 0) * d;
    }

    half8 a_buf[PD][TPW][2], h_buf[PD][2], g_buf[PD];
    auto issue = [&](int kc, int slot) {
        const int k0 = kc * kKC;
#pragma unroll
        for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
            for (int j = 0; j < 2; ++j) a_buf[slot][tp][j] = load_half8(rowptr[tp] + min(k0 + q * 16 + j * 8, d - 8));
        const int ko = min(k0 + vc * 8, d - 8);
        g_buf[slot] = load_half8(p.gamma + ko);
#pragma unroll
        for (int i = 0; i < 2; ++i) h_buf[slot][i] = load_half8(hptr[i] + ko);
    };
#pragma unroll
    for (int u = 0; u < PD; ++u) issue(u, u);

    floatx4 acc[TPW][4];
#pragma unroll
    for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[tp][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
    float ssq[2] = {0.f, 0.f};

    const int nstages = ((nchunks + PD - 1) / PD) * PD;
    int buf = 0;
    for (int kc0 = 0; kc0 < nstages; kc0 += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const int kc = kc0 + u;
            const bool b_in = kc * kKC + vc * 8 < d;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const half8 hsel = (b_in && hok[i]) ? h_buf[u][i] : zero_half8();
                half8 hi, lo;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const half2_t hh = {hsel[2 * e], hsel[2 * e + 1]};
                    const half2_t gg = {g_buf[u][2 * e], g_buf[u][2 * e + 1]};
                    const half2_t x = hh * gg;
                    const half2_t rres = __builtin_elementwise_fma(hh, gg, -x);
                    ssq[i] = __builtin_amdgcn_fdot2(hh, hh, ssq[i], false);
                    hi[2 * e] = x[0];
                    hi[2 * e + 1] = x[1];
                    lo[2 * e] = rres[0];
                    lo[2 * e + 1] = rres[1];
                }
                const int r = r0 + 32 * i;
                *reinterpret_cast<half8 *>(&lds_hi[buf][r][vc * 8]) = hi;
                *reinterpret_cast<half8 *>(&lds_lo[buf][r][vc * 8]) = lo;
            }
            half8 a_cur[TPW][2];
#pragma unroll
            for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    a_cur[tp][j] = (kc * kKC + q * 16 + j * 8 < d) ? a_buf[u][tp][j] : zero_half8();
            __syncthreads();
            issue(kc + PD, u);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                half8 bh[4], bl[4];
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    bh[nt] = *reinterpret_cast<const half8 *>(&lds_hi[buf][nt * 16 + c][q * 16 + j * 8]);
                    bl[nt] = *reinterpret_cast<const half8 *>(&lds_lo[buf][nt * 16 + c][q * 16 + j * 8]);
                }
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                    for (int tp = 0; tp < TPW; ++tp)
                        acc[tp][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_cur[tp][j], bh[nt], acc[tp][nt], 0, 0, 0);
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                    for (int tp = 0; tp < TPW; ++tp)
                        acc[tp][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_cur[tp][j], bl[nt], acc[tp][nt], 0, 0, 0);
            }
            buf ^= 1;
        }
    }

    // ---- sum of squares of each hidden state: 8 consecutive lanes share a row
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        float v = ssq[i];
        v += dpp_f32<kDppXor1>(v);
        v += dpp_f32<kDppXor2>(v);
        v += dpp_f32<kDppHalfMirror>(v);
        ssq[i] = v;
    }
    if (vc == 0) {
        lds_ssq[r0] = ssq[0];
        lds_ssq[r0 + 32] = ssq[1];
    }
    __syncthreads();

    // ---- epilogue: lane holds Y[mt + 4q .. +3][n0 + nt*16 + c]
    if (MODE == 2) {
        __shared__ float cand_v[kGemmWaves][kNB];
        __shared__ int cand_i[kGemmWaves][kNB];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const float scale = 1.0f / sqrtf(lds_ssq[nt * 16 + c] / (float)d + p.eps);
            float bv = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int tp = 0; tp < TPW; ++tp) {
                const int m = m0 + (wave * TPW + tp) * 16 + q * 4;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float v = acc[tp][nt][r] * scale;
                    if (m + r < M && v > bv) {  // rows ascend: strict '>' keeps the lowest row on ties
                        bv = v;
                        bi = m + r;
                    }
                }
            }
#pragma unroll
            for (int off = 16; off <= 32; off <<= 1) {  // the four q-groups of column c
                const float ov = __shfl_xor(bv, off, kWave);
                const int oi = __shfl_xor(bi, off, kWave);
                if (ov > bv || (ov == bv && oi < bi)) {
                    bv = ov;
                    bi = oi;
                }
            }
            if (q == 0) {
                cand_v[wave][nt * 16 + c] = bv;
                cand_i[wave][nt * 16 + c] = bi;
            }
        }
        __syncthreads();
        if (tid < kNB && n0 + tid < p.N) {
            float bv = cand_v[0][tid];
            int bi = cand_i[0][tid];
            for (int w = 1; w < kGemmWaves; ++w)
                if (cand_v[w][tid] > bv || (cand_v[w][tid] == bv && cand_i[w][tid] < bi)) {
                    bv = cand_v[w][tid];
                    bi = cand_i[w][tid];
                }
            p.best_val[(size_t)(n0 + tid) * gridDim.x + blockIdx.x] = bv;
            p.best_idx[(size_t)(n0 + tid) * gridDim.x + blockIdx.x] = bi;
        }
        return;
    }
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        const int n = n0 + nt * 16 + c;
        if (n >= p.N) continue;
        const float scale = 1.0f / sqrtf(lds_ssq[nt * 16 + c] / (float)d + p.eps);
#pragma unroll
        for (int tp = 0; tp < TPW; ++tp) {
            const int m = m0 + (wave * TPW + tp) * 16 + q * 4;
            if (m >= M) continue;
            const floatx4 v = acc[tp][nt] * scale;
            float *dst = p.out + (size_t)n * p.V + m;
            if ((p.V & 3) == 0 && m + 3 < M) {
                *reinterpret_cast<floatx4 *>(dst) = v;
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (m + r < M) dst[r] = v[r];
            }
        }
    }
}

template <int MODE, int TPW, int PD>
static void launch_one(const GemmParams &p, hipStream_t st) {
    const int rows_per_wg = 16 * TPW * kGemmWaves;
    dim3 grid((p.V + rows_per_wg - 1) / rows_per_wg, 1, (p.N + kNB - 1) / kNB);
    hipLaunchKernelGGL((full_head_gemm_kernel<TPW, MODE, PD>), grid, dim3(kGemmThreads), 0, st, p);
}

// 256 rows per workgroup when that still gives >= 400 workgroups, otherwise 128
static int lm_head_tpw(int V) {
    return (V + 255) / 256 >= 400 ? 4 : 2;
}

// Measured on MI355X (N = 16..64): 256-row tiles with two stages in flight for large vocabularies
// (4.9 TB/s at 128256 x 8192), 128-row tiles with four stages for 32000-row heads (4.3-4.4 TB/s).
template <int MODE>
static hipError_t launch_stream(const GemmParams &p, hipStream_t st) {
    if (lm_head_tpw(p.V) == 4)
        launch_one<MODE, 4, 2>(p, st);
    else
        launch_one<MODE, 2, 4>(p, st);
    return hipGetLastError();
}

int lm_head_gemm_workgroups(int V) {
    const int rows = 64 * lm_head_tpw(V);
    return (V + rows - 1) / rows;
}

static GemmParams full_head_params(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                                   const half_t *lm_head) {
    GemmParams p{};
    p.d = d; p.V = V; p.N = N; p.eps = eps;
    p.hidden = hidden; p.gamma = gamma; p.lm_head = lm_head;
    return p;
}

hipError_t launch_lm_head_gemm(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                               const half_t *lm_head, float *out, hipStream_t st) {
    GemmParams p = full_head_params(d, V, eps, N, hidden, gamma, lm_head);
    p.out = out;
    return launch_stream<1>(p, st);
}

hipError_t launch_lm_head_argmax_gemm(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                                      const half_t *lm_head, float *best_val, int32_t *best_idx, const int32_t *gate,
                                      const int32_t *done, hipStream_t st) {
    GemmParams p = full_head_params(d, V, eps, N, hidden, gamma, lm_head);
    p.best_val = best_val;
    p.best_idx = best_idx;
    p.gate = gate;
    p.done = done;
    return launch_stream<2>(p, st);
}

}  // namespace specee
