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
#include "merge_block.h"
#include "tree_finish.h"

namespace specee {

constexpr int kGemmThreads = 256;
constexpr int kGemmWaves = 4;
constexpr int kKC = 64;           // k elements per LDS stage (128 bytes of every row)
constexpr int kNB = 64;           // hidden states per workgroup (4 n-tiles of 16)
constexpr int kLdsRow = kKC + 8;  // halves per LDS row: 144 bytes, keeps 16-byte reads spread over banks

// MODE 0: un-normalised partial sums per d-slice (tree); 1: normalised logits stored (full head);
// 2: normalised logits reduced to one arg-max candidate per hidden state and workgroup (verification);
// 3: whole tree in one workgroup (needs FUSED, one d-slice, N <= 64, Mcap <= 64*TPW): the logits stay
//    in LDS and the same workgroup scores every node and applies the path rule -- nothing but the
//    inputs is read from memory and nothing but the outputs is written.
// FUSED (tree only, N*K <= 1024): every workgroup merges the tree's ids itself in LDS before the
// contraction, which removes a kernel launch and a dependent round trip from the latency path;
// workgroup (0,0) of each tree publishes merged ids, their count and the columns.
constexpr int kGemmFusedMax = kMergePerThread * kGemmThreads;
constexpr int kStageHalves = 2 * kNB * kLdsRow;  // one operand (hi or lo), both buffers

// PD: prefetch distance in 64-element stages.  Streaming use keeps PD stages of global loads in
// flight per wavefront; the latency-bound tree use picks PD >= the number of stages of a d-slice, so
// every load of the workgroup is issued before the first one is consumed.
template <int TPW, int MODE, bool FUSED, int PD, int KC = 4>
__global__ __launch_bounds__(kGemmThreads) void gather_gemm_kernel(GemmParams p, TreeFinishParams f) {
    __shared__ __attribute__((aligned(16))) half_t smem[2 * kStageHalves];
    __shared__ float lds_ssq[kNB];
    __shared__ int32_t cols_lds[MODE == 3 ? kGemmFusedMax : 1];
    __shared__ float prev_lds[MODE == 3 ? kGemmFusedMax : 1];
    __shared__ int32_t exit_lds[MODE == 3 ? kNB : 1];
    static_assert(MODE != 3 || FUSED, "the whole-tree mode merges in its prologue");
    static_assert(sizeof(half_t) * 2 * kStageHalves >= sizeof(float) * kNB * 64 * (MODE == 3 ? TPW : 1),
                  "the logits of a whole tree must fit in the staging buffers");
    static_assert(sizeof(half_t) * 2 * kStageHalves >= sizeof(int32_t) * merge_lds_ints(kGemmFusedMax),
                  "merge scratch must fit in the staging buffers");
    typedef half_t (*stage_t)[kNB][kLdsRow];
    stage_t lds_hi = reinterpret_cast<stage_t>(smem);
    stage_t lds_lo = reinterpret_cast<stage_t>(smem + kStageHalves);
    constexpr bool FINAL = MODE != 0;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, q = lane >> 4;
    const int NBn = (p.N + kNB - 1) / kNB;
    const int g = blockIdx.z / NBn, nb = blockIdx.z - g * NBn;
    const int n0 = nb * kNB;
    const int s = blockIdx.y;
    const int d = p.d;
    const int k_begin = s * p.dslice;
    const int k_end = min(d, k_begin + p.dslice);
    const int nchunks = (k_end - k_begin + kKC - 1) / kKC;

    // ---- B side: this thread stages vector column vc of hidden states r0 and r0+32
    const int vc = tid & 7, r0 = tid >> 3;  // 8 vectors per 64-element stage, 32 rows per pass, 2 passes
    const half_t *hbase = p.hidden + ((size_t)g * p.N + n0) * d;
    half8 h_buf[PD][2], g_buf[PD];
    auto issue_b = [&](int kc, int slot) {
        const int ko = k_begin + kc * kKC + vc * 8;
        const bool in = kc < nchunks && ko < k_end;
        g_buf[slot] = in ? load_half8(p.gamma + ko) : zero_half8();
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = r0 + 32 * i;
            h_buf[slot][i] = (in && n0 + r < p.N) ? load_half8(hbase + (size_t)r * d + ko) : zero_half8();
        }
    };
    // the hidden states do not depend on the merged set: request them before merging
#pragma unroll
    for (int u = 0; u < PD; ++u) issue_b(u, u);
    if (MODE == 3) {
        for (int i = tid; i < p.N * p.K; i += kGemmThreads) prev_lds[i] = f.prev[(size_t)g * p.N * p.K + i];
    }

    int M;
    int32_t *uniq = nullptr;
    if (FUSED) {
        const int n_ids = p.N * p.K;
        int col_of[kMergePerThread];
        const int Mtrue = merge_block<kGemmThreads>(p.ids + (size_t)g * n_ids, n_ids, reinterpret_cast<int32_t *>(smem), uniq,
                                      col_of);
        if (blockIdx.x == 0 && blockIdx.y == 0 && nb == 0) {
            if (tid == 0) p.M_out[g] = Mtrue;
            for (int m = tid; m < p.Mcap; m += kGemmThreads)
                p.merged_out[(size_t)g * p.Mcap + m] = m < Mtrue ? uniq[m] : -1;
#pragma unroll
            for (int e = 0; e < kMergePerThread; ++e) {
                int i = tid + e * kGemmThreads;
                if (i < n_ids) p.cols_out[(size_t)g * n_ids + i] = col_of[e];
            }
        }
        if (MODE == 3) {
#pragma unroll
            for (int e = 0; e < kMergePerThread; ++e) {
                int i = tid + e * kGemmThreads;
                if (i < n_ids) cols_lds[i] = col_of[e];
            }
        }
        M = Mtrue;
    } else {
        M = p.Mptr ? p.Mptr[g] : p.Mcap;
    }
    const bool overflow = M > p.Mcap;
    if (overflow) M = p.Mcap;
    const int m0 = blockIdx.x * (16 * TPW * kGemmWaves);
    if (MODE != 3 && m0 >= M) return;  // uniform over the workgroup

    // ---- A side: this lane's rows
    const half_t *rowptr[TPW];
    bool rowok[TPW];
#pragma unroll
    for (int tp = 0; tp < TPW; ++tp) {
        int m = m0 + (wave * TPW + tp) * 16 + c;
        rowok[tp] = m < M;
        int row = 0;
        if (rowok[tp]) {
            row = FUSED ? uniq[m] : (p.rowlist ? p.rowlist[(size_t)g * p.Mcap + m] : m);
            if (row < 0 || row >= p.V) row = 0;  // invalid id: finish kernel reports NaN, never read out of bounds
        }
        rowptr[tp] = p.lm_head + (size_t)row * d;
    }
    if (FUSED) __syncthreads();  // the merge scratch becomes the staging buffers

    half8 a_buf[PD][TPW][2];
    auto issue_a = [&](int kc, int slot) {
        const int k0 = k_begin + kc * kKC;
#pragma unroll
        for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int ko = k0 + q * 16 + j * 8;
                a_buf[slot][tp][j] =
                    (kc < nchunks && rowok[tp] && ko < k_end) ? load_half8(rowptr[tp] + ko) : zero_half8();
            }
    };
#pragma unroll
    for (int u = 0; u < PD; ++u) issue_a(u, u);

    floatx4 acc[TPW][4];
#pragma unroll
    for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[tp][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
    float ssq[2] = {0.f, 0.f};

    int buf = 0;
    for (int kc0 = 0; kc0 < nchunks; kc0 += PD) {
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const int kc = kc0 + u;
            if (kc < nchunks) {  // uniform over the workgroup
                // split x = h*gamma into hi + lo and publish this stage.  Packed fp16 arithmetic does it
                // exactly: hi = round(h*gamma) and lo = round(fma(h, gamma, -hi)), whose argument is the
                // exact residual; the sum of squares accumulates in fp32 through the 2-way dot product.
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    half8 hi, lo;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const half2_t hh = {h_buf[u][i][2 * e], h_buf[u][i][2 * e + 1]};
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
                    for (int j = 0; j < 2; ++j) a_cur[tp][j] = a_buf[u][tp][j];
                __syncthreads();
                if (kc + PD < nchunks) {
                    issue_a(kc + PD, u);
                    issue_b(kc + PD, u);
                }
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) {
                        half8 bh = *reinterpret_cast<const half8 *>(&lds_hi[buf][nt * 16 + c][q * 16 + j * 8]);
                        half8 bl = *reinterpret_cast<const half8 *>(&lds_lo[buf][nt * 16 + c][q * 16 + j * 8]);
#pragma unroll
                        for (int tp = 0; tp < TPW; ++tp) {
                            acc[tp][nt] =
                                __builtin_amdgcn_mfma_f32_16x16x32_f16(a_cur[tp][j], bh, acc[tp][nt], 0, 0, 0);
                            acc[tp][nt] =
                                __builtin_amdgcn_mfma_f32_16x16x32_f16(a_cur[tp][j], bl, acc[tp][nt], 0, 0, 0);
                        }
                    }
                buf ^= 1;
            }
        }
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

    // ---- epilogue: lane holds Z[mt + 4q .. +3][n0 + nt*16 + c]
    if (MODE == 3) {
        // un-normalised logits of the whole tree into LDS (the staging buffers are dead: every wave
        // passed the barrier above after its last matrix instruction)
        // the predictor rows are requested only now: holding them across the contraction would halve
        // the number of resident workgroups
        FinishRows<KC> fr;
        finish_load_rows<KC>(fr, f, lane);
        float *Zl = reinterpret_cast<float *>(smem);
        const int Mpad = 64 * TPW;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int tp = 0; tp < TPW; ++tp) {
                const int m = (wave * TPW + tp) * 16 + q * 4;
                *reinterpret_cast<floatx4 *>(&Zl[(nt * 16 + c) * Mpad + m]) = acc[tp][nt];
            }
        __syncthreads();
        const int K = p.K, N = p.N;
        for (int n = wave; n < N; n += kGemmWaves) {
            const size_t gn = (size_t)g * N + n;
            float a = 0.f;
            bool bad = overflow;
            if (lane < K) {
                const int id = p.ids[gn * K + lane];
                if (id < 0 || id >= p.V) bad = true;
                int col = cols_lds[n * K + lane];
                col = (col >= 0 && col < Mpad) ? col : 0;
                a = Zl[n * Mpad + col];
            }
            bad = __any(bad);
            const float r = 1.0f / sqrtf(lds_ssq[n] / (float)d + p.eps);
            float z[KC], prev[KC];
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                float v = __shfl(a, k < K ? k : 0, kWave);
                z[k] = (k < K) ? (bad ? quiet_nan() : v * r) : 0.f;
                prev[k] = (k < K) ? prev_lds[n * K + k] : 0.f;
            }
            const int ex = finish_score_node<KC>(fr, f, gn, z, prev, lane);
            if (lane == 0) exit_lds[n] = ex;
        }
        if (f.path_exit) {
            __syncthreads();
            finish_paths(exit_lds, f.parent + (size_t)g * N, N, tid, kGemmThreads, f.path_exit + (size_t)g * N);
        }
        return;
    }
    if (MODE == 2) {
        __shared__ float cand_v[kGemmWaves][kNB];
        __shared__ int cand_i[kGemmWaves][kNB];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            float scale = 1.0f / sqrtf(lds_ssq[nt * 16 + c] / (float)d + p.eps);
            float bv = -INFINITY;
            int bi = 0x7fffffff;
#pragma unroll
            for (int tp = 0; tp < TPW; ++tp) {
                const int m = m0 + (wave * TPW + tp) * 16 + q * 4;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float v = acc[tp][nt][r] * scale;
                    if (m + r < M && v > bv) {  // rows ascend: strict '>' keeps the lowest row on ties
                        bv = v;
                        bi = m + r;
                    }
                }
            }
#pragma unroll
            for (int off = 16; off <= 32; off <<= 1) {  // the four q-groups of column c
                float ov = __shfl_xor(bv, off, kWave);
                int oi = __shfl_xor(bi, off, kWave);
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

constexpr int kTreePD = 4;    // a 256-element d-slice is requested in one go

template <int MODE, int TPW, int PD>
static void launch_one(const GemmParams &p, int G, hipStream_t st) {
    const int rows_per_wg = 16 * TPW * kGemmWaves;
    dim3 grid((p.Mcap + rows_per_wg - 1) / rows_per_wg, p.S, G * ((p.N + kNB - 1) / kNB));
    hipLaunchKernelGGL((gather_gemm_kernel<TPW, MODE, false, PD>), grid, dim3(kGemmThreads), 0, st, p,
                       TreeFinishParams{});
}

// Streaming configurations measured on MI355X (fp16 head, N = 16..64 hidden states):
//   256 rows per workgroup, one stage ahead   -- best when that still gives >= 400 workgroups
//   128 rows per workgroup, four stages ahead -- best for smaller vocabularies
template <int MODE>
static hipError_t launch_stream(const GemmParams &p, int tpw, hipStream_t st) {
    if (tpw == 4)
        launch_one<MODE, 4, 1>(p, 1, st);
    else
        launch_one<MODE, 2, 4>(p, 1, st);
    return hipGetLastError();
}

bool tree_gemm_can_fuse_merge(int n_ids) {
    return n_ids <= kGemmFusedMax;
}

hipError_t launch_tree_gemm(const GemmParams &p, int G, hipStream_t st) {
    const int rows_per_wg = 16 * kGemmWaves;
    dim3 grid((p.Mcap + rows_per_wg - 1) / rows_per_wg, p.S, G * ((p.N + kNB - 1) / kNB));
    if (p.ids)
        hipLaunchKernelGGL((gather_gemm_kernel<1, 0, true, kTreePD>), grid, dim3(kGemmThreads), 0, st, p,
                           TreeFinishParams{});
    else
        hipLaunchKernelGGL((gather_gemm_kernel<1, 0, false, kTreePD>), grid, dim3(kGemmThreads), 0, st, p,
                           TreeFinishParams{});
    return hipGetLastError();
}

// Whole tree per workgroup: one launch does merge, contraction, scoring and the path rule.
bool tree_whole_supported(int N, int K, int Mcap) {
    return N <= kNB && N * K <= kGemmFusedMax && Mcap <= 128;
}

template <int TPW, int KC>
static void launch_whole(const GemmParams &p, const TreeFinishParams &f, int G, hipStream_t st) {
    hipLaunchKernelGGL((gather_gemm_kernel<TPW, 3, true, kTreePD, KC>), dim3(1, 1, G), dim3(kGemmThreads), 0, st, p,
                       f);
}

hipError_t launch_tree_whole(const GemmParams &p, const TreeFinishParams &f, int G, hipStream_t st) {
    const bool wide = p.Mcap > 64;
    if (f.K <= 4) {
        if (wide) launch_whole<2, 4>(p, f, G, st); else launch_whole<1, 4>(p, f, G, st);
    } else if (f.K <= 8) {
        if (wide) launch_whole<2, 8>(p, f, G, st); else launch_whole<1, 8>(p, f, G, st);
    } else {
        if (wide) launch_whole<2, 16>(p, f, G, st); else launch_whole<1, 16>(p, f, G, st);
    }
    return hipGetLastError();
}

static int lm_head_tpw(int V) {
    return (V + 255) / 256 >= 400 ? 4 : 2;
}

int lm_head_gemm_workgroups(int V) {
    int rows = 64 * lm_head_tpw(V);
    return (V + rows - 1) / rows;
}

static GemmParams full_head_params(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                                   const half_t *lm_head) {
    GemmParams p{};
    p.d = d; p.V = V; p.N = N; p.eps = eps;
    p.hidden = hidden; p.gamma = gamma; p.lm_head = lm_head;
    p.rowlist = nullptr; p.Mptr = nullptr; p.Mcap = V;
    p.dslice = ((d + kKC - 1) / kKC) * kKC; p.S = 1;
    return p;
}

hipError_t launch_lm_head_gemm(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                               const half_t *lm_head, float *out, hipStream_t st) {
    GemmParams p = full_head_params(d, V, eps, N, hidden, gamma, lm_head);
    p.out = out;
    return launch_stream<1>(p, lm_head_tpw(V), st);
}

hipError_t launch_lm_head_argmax_gemm(int d, int V, float eps, int N, const half_t *hidden, const half_t *gamma,
                                      const half_t *lm_head, float *best_val, int32_t *best_idx, hipStream_t st) {
    GemmParams p = full_head_params(d, V, eps, N, hidden, gamma, lm_head);
    p.best_val = best_val;
    p.best_idx = best_idx;
    return launch_stream<2>(p, lm_head_tpw(V), st);
}

}  // namespace specee
