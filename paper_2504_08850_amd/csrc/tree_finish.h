// Per-node tail of the token-tree predictor, shared by the stand-alone finish
// kernels and by the whole-tree contraction kernel: given a node's K logits it
// runs the feature/MLP/judgment tail (paper Sec. 4.3.1-4.3.2) on one wavefront
// and writes the node's outputs.  Eight hidden units per lane stay in registers
// across nodes when the predictor has the common shape (K in {4, 8}, H <= 512).
#pragma once
#include "device_utils.h"
#include "kernels.h"
#include "predictor_tail.h"

namespace specee {

constexpr int kFinishUnits = 8;  // hidden units per lane held in registers (H <= 512)
constexpr int kMlpFeat = 32;     // feature slots per node in the matrix-core MLP (3K <= 32)

// Shapes the matrix-core MLP handles; everything else takes the vector-ALU path.
__host__ __device__ inline bool mlp_mfma_ok(int K, int H) {
    return (K == 4 || K == 8) && (H & 63) == 0;
}

template <int KC>
struct FinishRows {
    MlpRow<KC> rows[KC <= 8 ? kFinishUnits : 1];
    bool regs;
    half_t b2;  // as loaded (widened at use, so that requesting it never waits); 0 when has_b2 is false
    bool has_b2;
};

template <int KC>
__device__ __forceinline__ void finish_load_rows(FinishRows<KC> &fr, const TreeFinishParams &p, int lane) {
    fr.regs = (p.K == KC) && (p.H <= kFinishUnits * kWave) && KC <= 8;
    if (fr.regs) {
#pragma unroll
        for (int u = 0; u < kFinishUnits; ++u)
            mlp_row_load<KC>(fr.rows[u], p.W1, p.b1, p.w2, p.K, p.H, lane + u * kWave);
    }
    fr.b2 = (p.b2 ? p.b2 : p.w2)[0];  // always a valid address; masked at use
    fr.has_b2 = p.b2 != nullptr;
}

// One wavefront scores node gn from its normalised logits z (NaN = invalid) and previous
// probabilities; writes logits, probs, score and exit flag; returns the exit flag, valid in the
// last lane (kWave - 1) only.
template <int KC>
__device__ __forceinline__ int finish_score_node(FinishRows<KC> &fr, const TreeFinishParams &p, size_t gn,
                                                 const float (&z)[KC], const float (&prev)[KC], int lane) {
    const int K = p.K, H = p.H;
    float pr[KC];
    local_softmax<KC>(z, K, pr);
    bool poisoned = false;  // a NaN logit (invalid id / overflowing merged set) poisons the whole node
#pragma unroll
    for (int k = 0; k < KC; ++k)
        if (k < K && z[k] != z[k]) poisoned = true;

    float part = 0.f;
    if (fr.regs) {
        // keep the rows packed as fp16 across nodes: without this the compiler widens all of them to
        // fp32 outside the node loop and runs out of registers
#pragma unroll
        for (int u = 0; u < kFinishUnits; ++u)
#pragma unroll
            for (int q = 0; q < (3 * KC) / 4; ++q)
                asm volatile("" : "+v"(fr.rows[u].w1[q].x), "+v"(fr.rows[u].w1[q].y));
#pragma unroll
        for (int u = 0; u < kFinishUnits; ++u)
            if (lane + u * kWave < H) part += mlp_unit<KC>(fr.rows[u], p.W1, K, lane + u * kWave, z, pr, prev);
    } else {
        for (int j = lane; j < H; j += kWave) {
            MlpRow<KC> row;
            mlp_row_load<KC>(row, p.W1, p.b1, p.w2, K, H, j);
            part += mlp_unit<KC>(row, p.W1, K, j, z, pr, prev);
        }
    }
    part = wave_sum_to_last_row(part);
    const float sc = sigmoidf((fr.has_b2 ? (float)fr.b2 : 0.f) + part);
    const int ex = (sc > p.threshold) ? 1 : 0;
    if (lane == kWave - 1) {
        p.scores[gn] = sc;
        p.exit_flags[gn] = ex;
    }
    if (lane < K) {
        float zl = 0.f, pl = 0.f;
#pragma unroll
        for (int k = 0; k < KC; ++k)
            if (k == lane) {
                zl = z[k];
                pl = pr[k];
            }
        p.logits[gn * K + lane] = poisoned ? quiet_nan() : zl;
        p.probs[gn * K + lane] = pl;
    }
    return ex;
}

// Predictor MLP for the 16 nodes of a wavefront on the matrix cores (needs K in {4, 8} and H a
// multiple of 64).  F: this wavefront's [16][kMlpFeat] fp32 features in LDS (zero beyond 3K).
// Covers the ht_count tiles of 16 hidden units from tile ht_begin (ht_count a multiple of 4) and
// returns their share of the output pre-activation (without b2) of node c = lane & 15 in every lane.
// The loop over tiles of 16 hidden units is free of branches -- every load is in bounds and
// unconditional, invalid k-slots are zeroed by selects -- so that it can be unrolled with the
// weight loads of several tiles in flight.
// LDS = true: the predictor pointers in f address a copy in LDS.  They are generic pointers, which
// the compiler would read with flat loads (a trip through the vector memory path before the request
// reaches LDS); the explicit address space turns them into plain LDS reads.
template <bool LDS>
__device__ __forceinline__ half4 mlp_load8(const half_t *p) {
#if defined(__HIP_DEVICE_COMPILE__)
    if constexpr (LDS) return *(const __attribute__((address_space(3))) half4 *)p;
#endif
    return *reinterpret_cast<const half4 *>(p);
}
template <bool LDS>
__device__ __forceinline__ float mlp_mfma_16(const float *F, const TreeFinishParams &f, int lane, int ht_begin,
                                             int ht_count) {
    const int c = lane & 15, q = lane >> 4;
    const int K3 = 3 * f.K, H = f.H;
    half8 bhi, blo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float v = F[c * kMlpFeat + q * 8 + e];
        const half_t h = (half_t)v;
        bhi[e] = h;
        blo[e] = (half_t)(v - (float)h);
    }
    const bool lo_ok = q * 8 < K3;       // first four k-slots of this lane group hold features
    const bool hi_ok = q * 8 + 4 < K3;   // so do the last four
    const half_t *wbase = f.W1 + (lo_ok ? q * 8 : 0);
    const half_t *b1p = f.b1 ? f.b1 : f.w2;  // always a valid address; masked below
    const float b1m = f.b1 ? 1.f : 0.f;
    float acc_u = 0.f;
    (void)H;
    for (int ht0 = ht_begin; ht0 < ht_begin + ht_count; ht0 += 4)
#pragma unroll
    for (int hi_ = 0; hi_ < 4; ++hi_) {
        const int ht = ht0 + hi_;
        const half_t *src = wbase + (size_t)(ht * 16 + c) * K3;
        const half4 lo4 = mlp_load8<LDS>(src);
        const half4 hi4 = mlp_load8<LDS>(src + (hi_ok ? 4 : 0));
        half8 a;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[e] = lo_ok ? lo4[e] : (half_t)0.f;
            a[4 + e] = hi_ok ? hi4[e] : (half_t)0.f;
        }
        const int u0 = ht * 16 + 4 * q;  // this lane's four hidden units of the tile
        const half4 w2v = mlp_load8<LDS>(f.w2 + u0);
        const half4 b1v = mlp_load8<LDS>(b1p + u0);
        floatx4 dacc = {0.f, 0.f, 0.f, 0.f};
        dacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bhi, dacc, 0, 0, 0);
        dacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, blo, dacc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) acc_u += (float)w2v[r] * fmaxf(dacc[r] + b1m * (float)b1v[r], 0.f);
    }
    acc_u += __shfl_xor(acc_u, 16, kWave);
    acc_u += __shfl_xor(acc_u, 32, kWave);
    return acc_u;
}

// Copy the predictor (W1 [H][3K] | w2 [H] | b1 [H], b1 zero-filled when absent) into LDS with
// 16-byte vectors, and return parameters that point at the copy.  The matrix-core MLP walks the
// weights tile by tile; from global memory that is a chain of cache-latency round trips, from LDS it
// is not.  Needs mlp_mfma_ok(K, H); dst must be 16-byte aligned with room for mlp_lds_halves(K, H).
__host__ __device__ inline int mlp_lds_halves(int K, int H) {
    return H * 3 * K + 2 * H;
}
// 16-byte vector i of that image, read from global memory; i is clamped into the image, so the load
// is always in bounds and needs no branch.
__device__ __forceinline__ half8 mlp_vector(const TreeFinishParams &f, int i) {
    const int nW8 = f.H * 3 * f.K / 8, H8 = f.H / 8;
    i = min(i, nW8 + 2 * H8 - 1);
    const half_t *src = f.W1 + (size_t)i * 8;
    if (i >= nW8) src = f.w2 + (size_t)(i - nW8) * 8;
    const bool bias = i >= nW8 + H8;
    if (bias) src = (f.b1 ? f.b1 : f.w2) + (size_t)(i - nW8 - H8) * 8;
    const half8 v = load_half8(src);
    return (bias && !f.b1) ? zero_half8() : v;
}
__device__ __forceinline__ TreeFinishParams mlp_params_at(half_t *dst, const TreeFinishParams &f) {
    const int nW = f.H * 3 * f.K;
    TreeFinishParams g = f;
    g.W1 = dst;
    g.w2 = dst + nW;
    g.b1 = dst + nW + f.H;
    return g;
}
__device__ __forceinline__ TreeFinishParams stage_mlp_to_lds(half_t *dst, const TreeFinishParams &f, int tid,
                                                            int threads) {
    const int nvec = mlp_lds_halves(f.K, f.H) / 8;
    for (int i = tid; i < nvec; i += threads) reinterpret_cast<half8 *>(dst)[i] = mlp_vector(f, i);
    return mlp_params_at(dst, f);
}

// Padded LDS image of the predictor for K <= 5 (3K + 1 <= 16): W1 rows padded to 16 halves with
// b1 in column 3K (the features carry a constant 1 there) and zeros after it, then w2 [H], then 16
// zero bytes.  A row is then one aligned 16-byte LDS read per k-slot group with nothing to mask, and
// the bias costs no instruction.  16 * H / 8 vectors of W1 rows, H / 8 of w2.
constexpr int kMlpPad = 16;
__host__ __device__ inline int mlp_padded_halves(int H) {
    return H * kMlpPad + H + 8;
}
__host__ __device__ inline bool mlp_padded_ok(int K, int H) {
    return 3 * K + 1 <= kMlpPad && (K & 3) == 0 && (H & 63) == 0;
}
// Vector i (two per row) of the padded W1 rows, from global memory.  Free of branches, so that it
// can be issued among other outstanding loads: i is clamped into the image, and with on == false
// (the image is not going to be used) every load goes to `safe`, any valid 16 bytes.
__device__ __forceinline__ half8 mlp_padded_vector(const TreeFinishParams &f, int i, bool on, const half_t *safe) {
    const int K3 = on ? 3 * f.K : 4;
    i = min(i, 2 * f.H - 1);
    const int j = i >> 1, part = i & 1;
    const half_t *row = on ? f.W1 + (size_t)j * K3 : safe;
    const half_t bias_raw = *((on && f.b1) ? f.b1 + j : safe);
    const half_t bias = f.b1 ? bias_raw : (half_t)0.f;
    half8 v;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int col0 = part * 8 + 4 * h;
        const half4 w = *reinterpret_cast<const half4 *>(row + min(col0, K3 - 4));
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            half_t x = (half_t)0.f;
            if (col0 + 4 <= K3) x = w[e];
            else if (col0 + e == K3) x = bias;
            v[4 * h + e] = x;
        }
    }
    return v;
}
// Same contract as mlp_mfma_16, on the padded image at img (LDS); F must hold 1.0 in slot 3K.
__device__ __forceinline__ float mlp_mfma_16_padded(const float *F, const half_t *img, int H, int lane, int ht_begin,
                                                    int ht_count) {
#if defined(__HIP_DEVICE_COMPILE__)
    typedef const __attribute__((address_space(3))) half8 *lds_half8_ptr;
    typedef const __attribute__((address_space(3))) half4 *lds_half4_ptr;
    const int c = lane & 15, q = lane >> 4;
    half8 bhi, blo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float v = F[c * kMlpFeat + q * 8 + e];
        const half_t h = (half_t)v;
        bhi[e] = h;
        blo[e] = (half_t)(v - (float)h);
    }
    // lane groups q >= 2 hold k-slots 16..31, which the padded rows do not have: they read the zero block
    const bool live = q * 8 < kMlpPad;
    const half_t *ap = live ? img + (size_t)(ht_begin * 16 + c) * kMlpPad + q * 8 : img + (size_t)H * kMlpPad + H;
    const int astep = live ? 16 * kMlpPad : 0;
    const half_t *wp = img + (size_t)H * kMlpPad + ht_begin * 16 + 4 * q;
    float acc0 = 0.f, acc1 = 0.f;
    for (int t0 = 0; t0 < ht_count; t0 += 4) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const half8 a = *(lds_half8_ptr)(ap + (size_t)(t0 + t) * astep);
            const half4 w2v = *(lds_half4_ptr)(wp + (t0 + t) * 16);
            floatx4 dacc = {0.f, 0.f, 0.f, 0.f};
            dacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bhi, dacc, 0, 0, 0);
            dacc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, blo, dacc, 0, 0, 0);
            float &acc = (t & 1) ? acc1 : acc0;
#pragma unroll
            for (int r = 0; r < 4; ++r) acc += (float)w2v[r] * fmaxf(dacc[r], 0.f);
        }
    }
    float acc_u = acc0 + acc1;
    acc_u += __shfl_xor(acc_u, 16, kWave);
    acc_u += __shfl_xor(acc_u, 32, kWave);
    return acc_u;
#else
    (void)F; (void)img; (void)H; (void)lane; (void)ht_begin; (void)ht_count;
    return 0.f;
#endif
}

// Path rule from exit flags in LDS (paper Sec. 6.2): a token path exits only if every token on it
// exits.  Parents precede children, so at most N steps; a malformed parent refuses the path.
__device__ __forceinline__ void finish_paths(const int32_t *exit_lds, const int32_t *par, int N, int tid,
                                             int threads, int32_t *path_out) {
    for (int n = tid; n < N; n += threads) {
        int cur = n, ok = 1;
        for (int step = 0; step < N && cur >= 0; ++step) {
            ok &= exit_lds[cur];
            int up = par[cur];
            if (up >= cur) {
                ok = 0;
                break;
            }
            cur = up;
        }
        path_out[n] = ok;
    }
}

}  // namespace specee
