// Token trees under the merged mapping (paper Sec. 6.2) on a 4-bit group-quantised LM head (the
// weight-quantised setting of Sec. 7.1 / 7.3; format as for the quantised-rows predictor): one workgroup
// per tree does the merge, the N x M x d contraction on the matrix cores, the per-node features, MLP and
// judgment, and the path rule.
//
// The contraction never forms a dequantised weight.  With x = h * gamma split exactly into hi + lo (fp16),
//     Z[n][m] = sum_g scale[m][g] * ( sum_{i in g} x[n][i] * code[m][i]  -  zero[m][g] * sum_{i in g} x[n][i] ):
// the inner sum runs on v_mfma_f32_16x16x32_f16 with the CODES as the A operand -- integers 0..15, exact
// in fp16 -- into a per-group accumulator; at the end of a group every lane folds its four rows' sums into
// the running logits with that group's scale and zero-point (two FMAs per row) and starts over.  The
// group sums of x come from the same registers the B operand is built from.  A merged row is d/2 bytes of
// codes, so a tree reads its hidden states (N * 2d bytes) and an eighth as many row bytes as on the fp16
// head; the rows' scales and zero-points (4 * d / group bytes each) are staged in LDS once.
//
// Layout per stage of KCH elements: the row tile [16 * MT rows][KCH] is expanded from codes to fp16 in
// registers (0x6400 | c is the half 1024 + c) and written to double-buffered LDS; k-step j of a stage
// covers elements 32j .. 32j+31 (lane group q takes 8 consecutive ones), so a quantisation group --
// a multiple of 32 elements -- ends on a k-step boundary.  Within a k-step the eight elements of a lane
// sit in the order (0,4,1,5,2,6,3,7) on both operands (any order is valid if A and B agree), which is
// the order the nibble pairs come out of a 32-bit word.
#include <type_traits>

#include "device_utils.h"
#include "kernels.h"
#include "merge_block.h"
#include "tree_finish.h"

namespace specee {

// 512 threads: wavefronts w and w + 4 share node tile w and take half of the k-steps of every stage each (the
// fold is linear, so each folds its own share of a group); their logits are added through LDS at the end.
// One wavefront per node tile doing all of a stage was twice as slow: the per-stage instruction stream of a
// wavefront, not memory, bounds a workgroup that streams a whole tree.
constexpr int kTq4Threads = 512;
constexpr int kTq4Waves = kTq4Threads / kWave;
constexpr int kTq4Kh = kTq4Threads / 256;           // wavefronts per node tile
// Elements per stage: 256 with four row tiles, 128 with eight (the double-buffered row tiles of 256 would not
// leave room for the scales).  A stage costs about 0.3 us of barrier and LDS turn-around on top of its
// streaming, so the longer stage is worth a tenth of the loop.
constexpr size_t kTq4LdsBudget = 150 * 1024;
static size_t tq4_lds_bytes(int d, int rows, int group, int kch) {
    return sizeof(half_t) * ((size_t)2 * rows * (kch + 8) + (size_t)2 * (d / group) * rows + (size_t)d);
}
static int tq4_kch(int d, int rows, int group) {
    return rows <= 64 && tq4_lds_bytes(d, rows, group, 256) <= kTq4LdsBudget ? 256 : 128;
}
constexpr int kTq4MaxIds = 1024;                    // ids per tree (N * K)

// eight codes of a word as halves, in the order (0,4,1,5,2,6,3,7)
__device__ __forceinline__ half8 codes_to_half8(uint32_t w) {
    half8 out;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t bits = ((w >> (4 * p)) & 0x000f000fu) | 0x64006400u;  // nibbles p and p + 4
        const half2_t v = __builtin_bit_cast(half2_t, bits) - half2_t{(half_t)1024.f, (half_t)1024.f};
        out[2 * p] = v[0];
        out[2 * p + 1] = v[1];
    }
    return out;
}

// MT: row tiles of 16 merged rows (Mcap <= 16 * MT).  KC: as in the other predictor kernels.  KCH: elements per stage.
template <int MT, int KC, int KCH>
__global__ __launch_bounds__(kTq4Threads) void tree_q4_kernel(TreeQ4Params p, TreeFinishParams f) {
    constexpr int ROWS = 16 * MT;
    constexpr int kTq4Kch = KCH;
    constexpr int kTq4Row = kTq4Kch + 8;  // halves per LDS row
    constexpr int JN = kTq4Kch / 32 / kTq4Kh;             // k-steps per stage and wavefront
    constexpr int CPT = ROWS * (kTq4Kch / 16) / kTq4Threads;  // 8-byte code chunks (16 elements) per thread per stage
    extern __shared__ __attribute__((aligned(16))) half_t q4_smem[];
    // dynamic LDS: row tiles [2][ROWS][kTq4Row] halves | scales [ng][ROWS] | zero-points [ng][ROWS] | gamma [d]
    typedef half_t (*tile_t)[ROWS][kTq4Row];
    tile_t a_lds = reinterpret_cast<tile_t>(q4_smem);
    const int ng = p.d / p.group;
    half_t *sc_lds = q4_smem + 2 * ROWS * kTq4Row;
    half_t *zp_lds = sc_lds + (size_t)ng * ROWS;
    half_t *gam_lds = zp_lds + (size_t)ng * ROWS;  // the RMSNorm weight, staged once ([d]; 16-byte aligned: ROWS % 8 == 0)
    __shared__ int32_t cols_lds[kTq4MaxIds];
    __shared__ float prev_lds[kTq4MaxIds];
    __shared__ float ssq_lds[64];
    __shared__ int32_t bad_lds[64];
    __shared__ int32_t exit_lds[64];
    __shared__ int32_t par_lds[64];
    static_assert(sizeof(half_t) * 2 * ROWS * kTq4Row >= sizeof(int32_t) * merge_lds_ints(kTq4MaxIds),
                  "merge scratch must fit in the row tile buffers");
    static_assert(sizeof(half_t) * 2 * ROWS * kTq4Row >= sizeof(float) * 64 * ROWS, "the logits must fit");
    static_assert(CPT >= 1, "at least one chunk per thread");

    const int tid = threadIdx.x, lane = tid & 63;
    // in a scalar register: the group bookkeeping below branches on values derived from it, and the compiler
    // would otherwise run those branches as divergent vector code
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, q = lane >> 4;
    const int g = blockIdx.x;
    const int d = p.d, N = p.N, K = p.K, n_ids = N * K;
    const int nchunks = (d + kTq4Kch - 1) / kTq4Kch;

    // ---- the ids first; then what does not depend on them
    int ids_r[kMergePerThread];
    merge_load_ids<kTq4Threads>(p.ids + (size_t)g * n_ids, n_ids, ids_r);
    const int kh = wave >> 2, nt_w = wave & 3;  // k-share and node tile of this wavefront
    const int node = nt_w * 16 + c;
    const bool node_ok = node < N;
    const half_t *hrow = p.hidden + ((size_t)g * N + (node_ok ? node : 0)) * d;
    float prev_r[kMergePerThread];
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e)
        prev_r[e] = f.prev[(size_t)g * n_ids + min(tid + e * kTq4Threads, n_ids - 1)];
    const int32_t *pp = f.path_exit ? f.parent + (size_t)g * N + min(tid, N - 1) : p.ids;
    const int par_r = *pp;
    const half_t b2_r = *(f.b2 ? f.b2 : p.gamma);  // output bias (widened where it is used; masked when absent)
    if (tid < 64) bad_lds[tid] = 0;
    // the RMSNorm weight goes to LDS once (read again by every lane at every stage otherwise: cache hits, but
    // they take slots of the vector memory path that the streaming needs)
    // every eight of it in the order (0,4,1,5,2,6,3,7), the one the B operand is built in
    for (int v = tid; v < (d >> 3); v += kTq4Threads) {
        const half8 gv = load_half8(p.gamma + v * 8);
        half8 gp;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            gp[2 * e] = gv[e];
            gp[2 * e + 1] = gv[e + 4];
        }
        *reinterpret_cast<half8 *>(&gam_lds[v * 8]) = gp;
    }

    // ---- the first stages of hidden states go out once the ids (and the other prologue loads) have come back --
    // not before: every workgroup's burst of them ahead of its ids delays the ids -- and before the merge, so that
    // they stream in while it computes
    const int kq = 32 * kh * JN + 8 * q;  // this lane's first element within a stage
    constexpr int PD = 2;                 // stages in flight
    static_assert(PD % 2 == 0, "the LDS buffer of a stage is its slot's parity");
    half8 h_buf[PD][JN];
    // TAIL: the stage may reach past the end of the rows: loads are clamped into the row (and masked when
    // consumed); a full stage needs neither
    auto issue_hidden = [&](auto tail_c, int kc, int slot) {
        constexpr bool TAIL = decltype(tail_c)::value;
#pragma unroll
        for (int j = 0; j < JN; ++j) {
            const int ko = TAIL ? min(kc * kTq4Kch + kq + 32 * j, d - 8) : kc * kTq4Kch + kq + 32 * j;
            h_buf[slot][j] = load_half8(hrow + ko);
        }
    };
    const int nfull = d / kTq4Kch;  // stages that lie wholly inside the rows
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
    asm volatile("" ::: "memory");
#pragma unroll
    for (int u = 0; u < PD; ++u) {
        if (u < nfull) issue_hidden(std::false_type{}, u, u);
        else issue_hidden(std::true_type{}, u, u);
    }

    // ---- merge
    int32_t *uniq = nullptr;
    int col_of[kMergePerThread], own_id[kMergePerThread];
    const bool bitmap = p.V <= 65536 && (size_t)merge_bitmap_ints(p.V, n_ids) * sizeof(int32_t) <=
                                            sizeof(half_t) * 2 * ROWS * kTq4Row;
    const int Mtrue = bitmap ? merge_bitmap<kTq4Threads>(ids_r, n_ids, p.V, reinterpret_cast<int32_t *>(q4_smem), uniq,
                                                         col_of, own_id)
                             : merge_block<kTq4Threads>(ids_r, n_ids, reinterpret_cast<int32_t *>(q4_smem), uniq,
                                                        col_of, own_id);
    const bool overflow = Mtrue > p.Mcap;
    const int M = overflow ? p.Mcap : Mtrue;

    // ---- the rows' codes are requested the moment the rows are known: chunk (row, v) = tid + 512 * i.
    // Rows beyond the merged set and nodes beyond the tree read row 0 / node 0: their logits are never looked at.
    const uint32_t *crow[CPT];
    int c_r[CPT], c_v[CPT];
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        const int ci = tid + kTq4Threads * i;
        c_r[i] = ci / (kTq4Kch / 16);
        c_v[i] = ci % (kTq4Kch / 16);
        int row = c_r[i] < M ? uniq[c_r[i]] : 0;
        if (row < 0 || row >= p.V) row = 0;  // invalid id: the node is reported NaN, nothing is read out of bounds
        crow[i] = p.qweight + (size_t)row * (d >> 3);
    }
    uint2 a_buf[PD][CPT];
    auto issue_codes = [&](auto tail_c, int kc, int slot) {
        constexpr bool TAIL = decltype(tail_c)::value;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const int ko = TAIL ? min(kc * kTq4Kch + c_v[i] * 16, d - 16) : kc * kTq4Kch + c_v[i] * 16;
            a_buf[slot][i] = *reinterpret_cast<const uint2 *>(crow[i] + (ko >> 3));
        }
    };
    auto issue = [&](auto tail_c, int kc, int slot) {
        issue_codes(tail_c, kc, slot);
        issue_hidden(tail_c, kc, slot);
    };
#pragma unroll
    for (int u = 0; u < PD; ++u) {  // (the hidden states of these stages went out before the merge)
        if (u < nfull) issue_codes(std::false_type{}, u, u);
        else issue_codes(std::true_type{}, u, u);
    }

    // ---- publish the merge, park what the scoring phase needs, stage the rows' scales and zero-points
    if (tid == 0) p.M_out[g] = Mtrue;
    for (int m = tid; m < p.Mcap; m += kTq4Threads) p.merged_out[(size_t)g * p.Mcap + m] = m < Mtrue ? uniq[m] : -1;
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        const int i = tid + e * kTq4Threads;
        if (i < n_ids) {
            p.cols_out[(size_t)g * n_ids + i] = col_of[e];
            cols_lds[i] = col_of[e];
            prev_lds[i] = prev_r[e];
            if (own_id[e] < 0 || own_id[e] >= p.V) bad_lds[i / K] = 1;  // benign race: all writers store 1
        }
    }
    if (f.path_exit && tid < N) par_lds[tid] = par_r;
    if ((ng & 7) == 0 && (((uintptr_t)p.qscales | (uintptr_t)p.qzeros) & 15) == 0) {
        // eight groups of a row per 16-byte load; all of a thread's loads go out before the first is used
        // (a loop of load -> store would make one trip to memory per round)
        const int nvec = ROWS * (ng >> 3);
        constexpr int kRounds = 4;
        for (int i0 = tid; i0 < nvec; i0 += kTq4Threads * kRounds) {
            half8 sv[kRounds], zv[kRounds];
            int mm[kRounds], g0[kRounds];
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int i = min(i0 + r * kTq4Threads, nvec - 1);
                mm[r] = i / (ng >> 3);
                g0[r] = (i - mm[r] * (ng >> 3)) * 8;
                int row = mm[r] < M ? uniq[mm[r]] : 0;
                if (row < 0 || row >= p.V) row = 0;
                sv[r] = load_half8(p.qscales + (size_t)row * ng + g0[r]);
                zv[r] = load_half8(p.qzeros + (size_t)row * ng + g0[r]);
            }
#pragma unroll
            for (int r = 0; r < kRounds; ++r)
                if (i0 + r * kTq4Threads < nvec) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        sc_lds[(size_t)(g0[r] + e) * ROWS + mm[r]] = mm[r] < M ? sv[r][e] : (half_t)0.f;
                        zp_lds[(size_t)(g0[r] + e) * ROWS + mm[r]] = mm[r] < M ? zv[r][e] : (half_t)0.f;
                    }
                }
        }
    } else {
        for (int i = tid; i < ROWS * ng; i += kTq4Threads) {
            const int m = i / ng, gi = i - m * ng;
            int row = m < M ? uniq[m] : 0;
            if (row < 0 || row >= p.V) row = 0;
            sc_lds[(size_t)gi * ROWS + m] = m < M ? p.qscales[(size_t)row * ng + gi] : (half_t)0.f;
            zp_lds[(size_t)gi * ROWS + m] = m < M ? p.qzeros[(size_t)row * ng + gi] : (half_t)0.f;
        }
    }
    __syncthreads();  // the merge scratch becomes the row tile buffers; scales and zero-points are in place

    floatx4 acc[MT], tmp[MT], tsum = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = tmp[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
    float ssq = 0.f;
    half8 ones8;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones8[e] = (half_t)1.f;

    // the row tile of stage kc from the prefetched codes: 16 elements per chunk, two 16-byte LDS writes
    auto tile_to_lds = [&](auto tail_c, int kc, int slot, int b) {
        constexpr bool TAIL = decltype(tail_c)::value;
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            const bool in = !TAIL || kc * kTq4Kch + c_v[i] * 16 < d;
            const half8 lo = codes_to_half8(a_buf[slot][i].x), hi = codes_to_half8(a_buf[slot][i].y);
            *reinterpret_cast<half8 *>(&a_lds[b][c_r[i]][c_v[i] * 16]) = in ? lo : zero_half8();
            *reinterpret_cast<half8 *>(&a_lds[b][c_r[i]][c_v[i] * 16 + 8]) = in ? hi : zero_half8();
        }
    };
    // x = h * gamma of this lane's node, k-step j of stage kc, split exactly into hi + lo, elements in the
    // order (0,4,1,5,2,6,3,7) (the weight sits in LDS in that order already); also the lane's share of the
    // sum of squares
    auto build_b = [&](auto tail_c, int kc, int slot, int j, half8 &hi, half8 &lo) {
        constexpr bool TAIL = decltype(tail_c)::value;
        const int ko = kc * kTq4Kch + kq + 32 * j;
        const half8 hsel = (!TAIL || ko < d) ? h_buf[slot][j] : zero_half8();
        // (k-steps past the end read the tail of the weight: in bounds, and hsel is zero there)
        const half8 gvec = *reinterpret_cast<const half8 *>(&gam_lds[TAIL ? min(ko, d - 8) : ko]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const half2_t hh = {hsel[e], hsel[e + 4]};
            const half2_t gg = {gvec[2 * e], gvec[2 * e + 1]};
            const half2_t x = hh * gg;
            const half2_t rres = __builtin_elementwise_fma(hh, gg, -x);
            ssq = __builtin_amdgcn_fdot2(hh, hh, ssq, false);
            hi[2 * e] = x[0];
            hi[2 * e + 1] = x[1];
            lo[2 * e] = rres[0];
            lo[2 * e + 1] = rres[1];
        }
    };
    // end of a quantisation group: acc += scale * (tmp - zero * sum of x over the group), row by row.  The sum
    // of x comes off the matrix cores too: a row tile of ones beside the codes leaves it, for the lane's node,
    // in every register of tsum.
    auto fold = [&](int gi) {
        const float t = tsum[0];
        const half_t *scp = sc_lds + (size_t)gi * ROWS + 4 * q;
        const half_t *zpp = zp_lds + (size_t)gi * ROWS + 4 * q;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const half4 s4 = *reinterpret_cast<const half4 *>(scp + 16 * mt);
            const half4 z4 = *reinterpret_cast<const half4 *>(zpp + 16 * mt);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[mt][r] += (float)s4[r] * (tmp[mt][r] - (float)z4[r] * t);
            tmp[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
        }
        tsum = floatx4{0.f, 0.f, 0.f, 0.f};
    };

    // A wavefront's k-steps ascend, and a k-step lies inside one group (groups are multiples of 32 elements):
    // it folds whenever the next k-step it multiplies starts at or past the end of the group it has open.
    int gi = 0, gend = p.group;
    bool dirty = false;
    auto round = [&](auto tail_c, int kc0) {
        constexpr bool TAIL = decltype(tail_c)::value;
#pragma unroll
        for (int u = 0; u < PD; ++u) {
            const int kc = kc0 + u;
            constexpr int kBufOf[2] = {0, 1};
            const int buf = kBufOf[u & 1];
            half8 bhi[JN], blo[JN];
            tile_to_lds(tail_c, kc, u, buf);
#pragma unroll
            for (int j = 0; j < JN; ++j) build_b(tail_c, kc, u, j, bhi[j], blo[j]);
            __syncthreads();
            issue(tail_c, kc + PD, u);
#pragma unroll
            for (int j = 0; j < JN; ++j) {
                const int k0 = kc * kTq4Kch + 32 * (kh * JN + j);  // first element of this k-step
                if (!TAIL || k0 < d) {  // uniform over the wavefront: k-steps past the end belong to no group
                    if (k0 >= gend) {
                        if (dirty) fold(gi);
                        dirty = false;
                        do {
                            ++gi;
                            gend += p.group;
                        } while (k0 >= gend);
                    }
                    half8 a[MT];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        a[mt] = *reinterpret_cast<const half8 *>(&a_lds[buf][mt * 16 + c][32 * (kh * JN + j) + 8 * q]);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        tmp[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], bhi[j], tmp[mt], 0, 0, 0);
                    tsum = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones8, bhi[j], tsum, 0, 0, 0);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        tmp[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], blo[j], tmp[mt], 0, 0, 0);
                    tsum = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones8, blo[j], tsum, 0, 0, 0);
                    dirty = true;
                }
            }
        }
    };
    const int nstages = ((nchunks + PD - 1) / PD) * PD;
    for (int kc0 = 0; kc0 < nstages; kc0 += PD) {
        // a round is plain when its stages and the ones it prefetches all lie wholly inside the rows
        if (kc0 + 2 * PD <= nfull) round(std::false_type{}, kc0);
        else round(std::true_type{}, kc0);
    }
    if (dirty) fold(gi);
    ssq += __shfl_xor(ssq, 16, kWave);
    ssq += __shfl_xor(ssq, 32, kWave);

    // ---- score the tree: the two k-shares of a node tile are added in a fixed order through the logit array
    // itself
    __syncthreads();
    float *Zl = reinterpret_cast<float *>(q4_smem);  // [64 nodes][ROWS], the quads of a node's row rotated by the node
    // (lane c holds node c: with plain rows, a multiple of the 64 banks long, the sixteen nodes of a 16-byte access
    // would all fall on the same four banks)
    auto zq = [&](int n, int quad) __attribute__((always_inline)) { return n * ROWS + ((quad + n) & (ROWS / 4 - 1)) * 4; };
    auto zcell = [&](int n, int col) __attribute__((always_inline)) { return zq(n, col >> 2) + (col & 3); };
    if (kh == kTq4Kh - 1) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            *reinterpret_cast<floatx4 *>(&Zl[zq(nt_w * 16 + c, mt * 4 + q)]) = acc[mt];
        if (q == 0) ssq_lds[nt_w * 16 + c] = ssq;
    }
    __syncthreads();
    if (kTq4Kh == 2 && kh == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            floatx4 *cell = reinterpret_cast<floatx4 *>(&Zl[zq(nt_w * 16 + c, mt * 4 + q)]);
            *cell = acc[mt] + *cell;
        }
        if (q == 0) ssq_lds[nt_w * 16 + c] += ssq;
    }
    __syncthreads();
    if (KC <= 8 && mlp_mfma_ok(K, f.H)) {
        // The predictor MLP of the 16 nodes of a node tile on the matrix cores.  Lanes q == 0 of the first
        // wavefront of the tile build the features of node c; the tile's wavefronts then share the hidden units.
        static_assert(sizeof(half_t) * 2 * ROWS * kTq4Row >= sizeof(float) * (64 * ROWS + 4 * 16 * kMlpFeat),
                      "the features must fit behind the logits");
        float *F = Zl + 64 * ROWS + nt_w * 16 * kMlpFeat;
        const int n = nt_w * 16 + c;  // node within the tree
        const size_t gn = (size_t)g * N + n;
        bool poisoned = false;
        float z[KC], pr[KC];
        if (q == 0 && kh == 0) {
            const float r = 1.0f / sqrtf(ssq_lds[n] / (float)d + p.eps);
            const bool bad = overflow || (n < N && bad_lds[n] != 0);
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                float v = 0.f;
                if (k < K && n < N) {
                    int col = cols_lds[n * K + k];
                    col = (col >= 0 && col < ROWS) ? col : 0;
                    v = bad ? quiet_nan() : Zl[zcell(n, col)] * r;
                }
                z[k] = v;
            }
            local_softmax<KC>(z, K, pr);
            poisoned = bad;
#pragma unroll
            for (int k = 0; k < KC; ++k)
                if (k < K) {
                    const float pv = n < N ? prev_lds[n * K + k] : 0.f;
                    F[c * kMlpFeat + k] = z[k];
                    F[c * kMlpFeat + K + k] = pr[k];
                    F[c * kMlpFeat + 2 * K + k] = pr[k] - pv;
                }
            for (int t = 3 * K; t < kMlpFeat; ++t) F[c * kMlpFeat + t] = 0.f;
        }
        __syncthreads();
        const int htiles = f.H >> 4;
        const bool split = kTq4Kh == 2 && (htiles & 7) == 0;  // uniform over the workgroup
        const int per = split ? htiles >> 1 : htiles;
        float u = 0.f;
        if (kh == 0 || split) u = mlp_mfma_16<false>(F, f, lane, split ? kh * per : 0, per);
        if (split) {
            if (kh == 1 && q == 0) ssq_lds[n] = u;  // (the sums of squares were consumed before the barrier above)
            __syncthreads();
            if (kh == 0) u += ssq_lds[n];
        }
        if (q == 0 && kh == 0 && n < N) {
            float sc = sigmoidf((f.b2 ? (float)b2_r : 0.f) + u);
            if (poisoned) sc = quiet_nan();
            const int ex = (sc > f.threshold) ? 1 : 0;
            f.scores[gn] = sc;
            f.exit_flags[gn] = ex;
            exit_lds[n] = ex;
#pragma unroll
            for (int k = 0; k < KC; ++k)
                if (k < K) {
                    f.logits[gn * K + k] = z[k];
                    f.probs[gn * K + k] = pr[k];
                }
        }
    } else {
        FinishRows<KC> fr;
        finish_load_rows<KC>(fr, f, lane);
        for (int n = wave; n < N; n += kTq4Waves) {
            const size_t gn = (size_t)g * N + n;
            float a = 0.f;
            if (lane < K) {
                int col = cols_lds[n * K + lane];
                col = (col >= 0 && col < ROWS) ? col : 0;
                a = Zl[zcell(n, col)];
            }
            const bool bad = overflow || bad_lds[n] != 0;
            const float r = 1.0f / sqrtf(ssq_lds[n] / (float)d + p.eps);
            float z[KC], prev[KC];
    #pragma unroll
            for (int k = 0; k < KC; ++k) {
                const float v = __shfl(a, k < K ? k : 0, kWave);
                z[k] = (k < K) ? (bad ? quiet_nan() : v * r) : 0.f;
                prev[k] = (k < K) ? prev_lds[n * K + k] : 0.f;
            }
            const int ex = finish_score_node<KC>(fr, f, gn, z, prev, lane);
            if (lane == kWave - 1) exit_lds[n] = ex;
        }
    }
    if (f.path_exit) {
        __syncthreads();
        finish_paths(exit_lds, par_lds, N, tid, kTq4Threads, f.path_exit + (size_t)g * N);
    }
}

bool tree_q4_supported(int d, int N, int K, int Mcap, int group) {
    if (N > 64 || N * K > kTq4MaxIds || Mcap > 128 || group % 32 != 0 || d % group != 0) return false;
    return tree_q4_lds_bytes(d, Mcap, group) <= kTq4LdsBudget;
}

size_t tree_q4_lds_bytes(int d, int Mcap, int group) {
    const int rows = Mcap <= 64 ? 64 : 128;
    return tq4_lds_bytes(d, rows, group, tq4_kch(d, rows, group));
}

template <int MT, int KC, int KCH>
static hipError_t launch_tq4(const TreeQ4Params &p, const TreeFinishParams &f, int G, hipStream_t st) {
    const size_t lds = tq4_lds_bytes(p.d, 16 * MT, p.group, KCH);
    auto kern = tree_q4_kernel<MT, KC, KCH>;
    if (lds > 48 * 1024)  // per launch: the library keeps no state; a refusal shows as the launch error
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds);
    hipLaunchKernelGGL(kern, dim3(G), dim3(kTq4Threads), lds, st, p, f);
    return hipGetLastError();
}

template <int KC>
static hipError_t launch_tq4_kc(const TreeQ4Params &p, const TreeFinishParams &f, int G, hipStream_t st) {
    if (p.Mcap > 64) return launch_tq4<8, KC, 128>(p, f, G, st);
    return tq4_kch(p.d, 64, p.group) == 256 ? launch_tq4<4, KC, 256>(p, f, G, st) : launch_tq4<4, KC, 128>(p, f, G, st);
}

hipError_t launch_tree_q4(const TreeQ4Params &p, const TreeFinishParams &f, int G, hipStream_t st) {
    if (f.K <= 4) return launch_tq4_kc<4>(p, f, G, st);
    if (f.K <= 8) return launch_tq4_kc<8>(p, f, G, st);
    return launch_tq4_kc<16>(p, f, G, st);
}

}  // namespace specee
