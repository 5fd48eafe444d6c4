// MFMA gather-contraction: Z[n][m] = sum_i (h[n][i] * gamma[i]) * W[row(m)][i]
// for a block of hidden states against a list of LM-head rows.  Two users:
//   - the merged tree mapping (paper Sec. 6.2): rows are the merged speculative
//     tokens of a tree, the contraction is split along d over many workgroups
//     and partial sums go to a workspace (fixed-order reduction afterwards);
//   - the full-vocabulary head for several hidden states (Sec. 4.1 / 4.3.3):
//     rows are the whole vocabulary, one workgroup owns 64*TPW rows over all of
//     d and writes normalised logits.
// These are the only places in the library where the work is a dense
// contraction, so these are the only users of the matrix cores.
//
// Mapping onto v_mfma_f32_16x16x32_f16 (64 lanes; lane = 16*q + c):
//   A operand = LM-head rows: lane holds 8 consecutive halves of row (m0 + c)
//               at k-offset chosen by q -- exactly one 16-byte global load, so
//               streamed/gathered rows feed the matrix core with no LDS hop;
//   B operand = x = h*gamma for hidden state (n0 + c), same k-offsets;
//   D         = lane holds Z[m0 + 4q .. 4q+3][n0 + c]  -> one 16-byte store.
// Any assignment of k-slots to (q, element) is valid as long as A and B use the
// same one; we pick it so that the four q-groups of a row read 128 contiguous
// bytes per 64-element step (q*32 bytes + 16*j).
//
// x is not representable in fp16 (it is a product of two fp16 numbers), and
// rounding it would cost ~4e-4 of a logit's standard deviation.  It is split
// into hi + lo halves instead, hi = fp16(x), lo = fp16(x - hi), and both are
// multiplied: the matrix cores are idle most of the time anyway because the
// contraction is bound by memory, and the split makes the products exact to
// ~2^-22.  The split is computed once per workgroup and shared through LDS
// (double buffered, one barrier per 64-element step).
#include "device_utils.h"
#include "kernels.h"

namespace specee {

constexpr int kGemmThreads = 256;
constexpr int kGemmWaves = 4;
constexpr int kKC = 64;           // k elements per LDS stage (128 bytes of every row)
constexpr int kNB = 64;           // hidden states per workgroup (4 n-tiles of 16)
constexpr int kLdsRow = kKC + 8;  // halves per LDS row: 144 bytes, keeps 16-byte reads spread over banks

template <int TPW, bool FINAL>
__global__ __launch_bounds__(kGemmThreads) void gather_gemm_kernel(GemmParams p) {
    __shared__ __attribute__((aligned(16))) half_t lds_hi[2][kNB][kLdsRow];
    __shared__ __attribute__((aligned(16))) half_t lds_lo[2][kNB][kLdsRow];
    __shared__ float lds_ssq[kNB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, q = lane >> 4;
    const int NBn = (p.N + kNB - 1) / kNB;
    const int g = blockIdx.z / NBn, nb = blockIdx.z - g * NBn;
    const int n0 = nb * kNB;
    const int s = blockIdx.y;
    const int d = p.d;

    int M = p.Mptr ? p.Mptr[g] : p.Mcap;
    if (M > p.Mcap) M = p.Mcap;
    const int m0 = blockIdx.x * (16 * TPW * kGemmWaves);
    if (m0 >= M) return;  // uniform over the workgroup

    const int k_begin = s * p.dslice;
    const int k_end = min(d, k_begin + p.dslice);
    const int nchunks = (k_end - k_begin + kKC - 1) / kKC;

    // ---- A side: this lane's rows
    const half_t *rowptr[TPW];
    bool rowok[TPW];
#pragma unroll
    for (int tp = 0; tp < TPW; ++tp) {
        int m = m0 + (wave * TPW + tp) * 16 + c;
        rowok[tp] = m < M;
        int row = 0;
        if (rowok[tp]) {
            row = p.rowlist ? p.rowlist[(size_t)g * p.Mcap + m] : m;
            if (row < 0 || row >= p.V) row = 0;  // invalid id: finish kernel reports NaN, never read out of bounds
        }
        rowptr[tp] = p.lm_head + (size_t)row * d;
    }
    // ---- B side: this thread stages vector column vc of hidden states r0, r0+16, r0+32, r0+48
    const int vc = tid & 7, r0 = tid >> 3;  // 8 vectors per 64-element stage, 32 rows per pass, 2 passes
    const half_t *hbase = p.hidden + ((size_t)g * p.N + n0) * d;

    half8 a_next[TPW][2], h_next[2], g_next;
    auto issue_loads = [&](int kc) {
        const int k0 = k_begin + kc * kKC;
#pragma unroll
        for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                int ko = k0 + q * 16 + j * 8;
                a_next[tp][j] = (rowok[tp] && ko < k_end) ? load_half8(rowptr[tp] + ko) : zero_half8();
            }
        int ko = k0 + vc * 8;
        bool in = ko < k_end;
        g_next = in ? load_half8(p.gamma + ko) : zero_half8();
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int r = r0 + 32 * i;
            h_next[i] = (in && n0 + r < p.N) ? load_half8(hbase + (size_t)r * d + ko) : zero_half8();
        }
    };

    floatx4 acc[TPW][4];
#pragma unroll
    for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[tp][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
    float ssq[2] = {0.f, 0.f};

    issue_loads(0);
    int buf = 0;
    for (int kc = 0; kc < nchunks; ++kc) {
        // split x = h*gamma into hi + lo and publish this stage
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            half8 hi, lo;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float hf = (float)h_next[i][e];
                float x = hf * (float)g_next[e];
                half_t xh = (half_t)x;
                hi[e] = xh;
                lo[e] = (half_t)(x - (float)xh);
                ssq[i] += hf * hf;
            }
            int r = r0 + 32 * i;
            *reinterpret_cast<half8 *>(&lds_hi[buf][r][vc * 8]) = hi;
            *reinterpret_cast<half8 *>(&lds_lo[buf][r][vc * 8]) = lo;
        }
        half8 a_cur[TPW][2];
#pragma unroll
        for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
            for (int j = 0; j < 2; ++j) a_cur[tp][j] = a_next[tp][j];
        __syncthreads();
        if (kc + 1 < nchunks) issue_loads(kc + 1);
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                half8 bh = *reinterpret_cast<const half8 *>(&lds_hi[buf][nt * 16 + c][q * 16 + j * 8]);
                half8 bl = *reinterpret_cast<const half8 *>(&lds_lo[buf][nt * 16 + c][q * 16 + j * 8]);
#pragma unroll
                for (int tp = 0; tp < TPW; ++tp) {
                    acc[tp][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_cur[tp][j], bh, acc[tp][nt], 0, 0, 0);
                    acc[tp][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_cur[tp][j], bl, acc[tp][nt], 0, 0, 0);
                }
            }
        buf ^= 1;
    }

    // ---- sum of squares of each hidden state over this k-range: 8 consecutive lanes share a row
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        float v = ssq[i];
        v += dpp_f32<kDppXor1>(v);
        v += dpp_f32<kDppXor2>(v);
        v += dpp_f32<kDppHalfMirror>(v);
        ssq[i] = v;
    }
    if (FINAL) {
        if (vc == 0) {
            lds_ssq[r0] = ssq[0];
            lds_ssq[r0 + 32] = ssq[1];
        }
        __syncthreads();
    } else if (blockIdx.x == 0 && vc == 0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int n = n0 + r0 + 32 * i;
            if (n < p.N) p.ssq_part[((size_t)g * p.S + s) * p.Npad + n] = ssq[i];
        }
    }

    // ---- epilogue: lane holds Z[m0t + 4q .. +3][n0 + nt*16 + c]
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        const int n = n0 + nt * 16 + c;
        if (n >= p.N) continue;
        float scale = 1.f;
        if (FINAL) scale = 1.0f / sqrtf(lds_ssq[nt * 16 + c] / (float)d + p.eps);
#pragma unroll
        for (int tp = 0; tp < TPW; ++tp) {
            const int mt = m0 + (wave * TPW + tp) * 16;
            if (mt >= M) continue;
            const int m = mt + q * 4;
            floatx4 v = acc[tp][nt] * scale;
            if (FINAL) {
                float *dst = p.out + ((size_t)g * p.N + n) * p.V + m;
                if ((p.V & 3) == 0 && m + 3 < M) {
                    *reinterpret_cast<floatx4 *>(dst) = v;
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (m + r < M) dst[r] = v[r];
                }
            } else {
                float *dst = p.out + (((size_t)g * p.S + s) * p.Npad + n) * p.Mpad + m;
                *reinterpret_cast<floatx4 *>(dst) = v;  // Mpad is a multiple of 16: always in bounds and aligned
            }
        }
    }
}

template <bool FINAL>
static hipError_t launch_tpw(const GemmParams &p, int tpw, int G, hipStream_t st) {
    const int rows_per_wg = 16 * tpw * kGemmWaves;
    dim3 grid((p.Mcap + rows_per_wg - 1) / rows_per_wg, p.S, G * ((p.N + kNB - 1) / kNB));
    dim3 block(kGemmThreads);
    switch (tpw) {
        case 1: hipLaunchKernelGGL((gather_gemm_kernel<1, FINAL>), grid, block, 0, st, p); break;
        case 2: hipLaunchKernelGGL((gather_gemm_kernel<2, FINAL>), grid, block, 0, st, p); break;
        default: hipLaunchKernelGGL((gather_gemm_kernel<4, FINAL>), grid, block, 0, st, p); break;
    }
    return hipGetLastError();
}

hipError_t launch_tree_gemm(const GemmParams &p, int G, hipStream_t st) {
    return launch_tpw<false>(p, 1, G, st);
}

hipError_t launch_lm_head_gemm(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                               const half_t *lm_head, float *out, hipStream_t st) {
    GemmParams p{};
    p.d = d; p.V = V; p.N = N; p.eps = eps;
    p.hidden = hidden; p.gamma = gamma; p.lm_head = lm_head;
    p.rowlist = nullptr; p.Mptr = nullptr; p.Mcap = V;
    p.dslice = ((d + kKC - 1) / kKC) * kKC; p.S = 1;
    p.out = out; p.ssq_part = nullptr; p.Mpad = 0; p.Npad = 0;
    // enough workgroups to cover 256 CUs about twice, otherwise the widest tile (most reuse of the staged x)
    int tpw = 4;
    while (tpw > 1 && (V + 64 * tpw - 1) / (64 * tpw) < 400) tpw >>= 1;
    return launch_tpw<true>(p, tpw, 1, st);
}

}  // namespace specee
