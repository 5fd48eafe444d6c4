// The early-exit decode loop of a token down the layer stack in ONE launch (paper Sec. 4.3.3 dataflow
// -- predict, verify after a positive prediction, leave the model at the first accepted verification --
// with the active-predictor set of the scheduler, Sec. 5.3).
//
// A launch of one kernel per step costs about two microseconds on this system even when the kernel is
// empty, which is as much as the predictor itself; and a static sequence of launches cannot stop at the
// exit.  Here a group of Pg workgroups stays resident for a token and walks the layers:
//   * the predictor of a layer is evaluated redundantly by every workgroup of the group (its reads hit
//     in L2 after the first workgroup): all of them reach the same exit decision with no communication,
//     so a layer that does not fire costs no synchronisation.  Such a layer measures 2.1 us at d = 4096:
//     about 600 instructions of one wavefront's stream (hidden state to float, sum of squares, K dot
//     products, two workgroup-wide reductions, softmax and MLP), not memory, which is prefetched one
//     active layer ahead;
//   * the K speculative LM-head rows and the RMSNorm weight do not change from layer to layer: they are
//     loaded once and stay in registers, so a layer reads only its hidden state and its predictor;
//   * when the predictor fires, the group streams the whole LM head once (workgroup w takes a block
//     of rows), every workgroup leaves its arg-max candidate in the workspace, the group meets at an
//     arrival counter, and every workgroup combines all candidates itself -- again the same decision
//     everywhere.  One group-wide meeting per verification, none otherwise;
//   * after the exit the loop ends: the remaining layers cost nothing.
// The meeting needs every workgroup of a group to be resident: the host sizes the grid from the
// occupancy the runtime reports, and every wait is bounded (spin limit), so a group that cannot meet
// (another kernel holds the CUs) ends with status 1 instead of hanging.
#include "device_utils.h"
#include "head_stream.h"
#include "q4_head_stream.h"
#include "kernels.h"
#include "predictor_tail.h"

namespace specee {

constexpr int kLoopThreads = 512;
constexpr int kLoopWaves = kLoopThreads / kWave;
struct LoopRare {
    float *logits, *probs, *scores;
    int32_t *exit_flags, *ver_token, *hit, *exit_layer, *token, *status;
    float *cand_val;
    int32_t *cand_idx, *arrive, *abort;
    long long spin_limit;
};
constexpr int kLoopMaskLds = 1024;  // layers of the active mask kept in LDS (deeper stacks read the rest in place)

// KC / EXACT / VPT as in predict_kernel.  KEEP: the K rows stay in registers across layers (up to 64
// registers of them; wider shapes read their rows again at every layer, from L2).
// HEAD: 0 = fp16 LM head, 1 = 4-bit group-quantised head read in 16-byte chunks (group % 32 == 0, aligned rows),
// 2 = quantised head read word by word.  On a quantised head the token's K rows are dequantised once, into
// the float registers that hold them anyway (with the RMSNorm weight folded in), so the predictor of a layer is
// the same code; the verification streams the codes (q4_head_rows).  Needs KEEP (K <= 8).
template <int KC, int VPT, bool EXACT, bool STREAM, int HEAD = 0>
__global__ __launch_bounds__(kLoopThreads) void layer_loop_kernel(LoopParams p) {
    constexpr bool KEEP = KC * VPT <= 16 && KC <= 8;
    constexpr bool Q4 = HEAD != 0;
    static_assert(!Q4 || KEEP, "the quantised head needs the rows kept in registers");
    extern __shared__ float4 loop_lds_x[];  // verification: x = h * gamma as two float4 planes, [2][d/8]
                                            // (quantised head: then [d/group] per-group sums of x)
    __shared__ __attribute__((aligned(16))) float red[KC + 1][kLoopWaves];  // [value][wavefront]: a value's partial
    __shared__ __attribute__((aligned(16))) float red_u[kLoopWaves];        // sums are two 16-byte reads
    static_assert(kLoopWaves == 8, "the cross-wavefront sums below read two float4 per value");
    __shared__ float cv[kLoopWaves];
    __shared__ int ci[kLoopWaves];
    __shared__ int met_lds;
    // Parameters that only the thread that writes outputs or meets the group needs: parked in LDS, because as kernel
    // arguments they stay in scalar registers for the whole loop, and with two dozen of them the compiler spills
    // scalars into vector lanes and reloads them in every layer.
    __shared__ LoopRare rare;
    __shared__ unsigned char act_lds[kLoopMaskLds];

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int w = blockIdx.x, b = blockIdx.y, Pg = gridDim.x, B = p.B;
    const int K = EXACT ? KC : p.K, H = p.H, d = p.d, L = p.L;
    const int nv = d >> 3;
    const bool writer = w == 0;  // the workgroup of the group that writes the token's outputs
    floatx4 *xa = reinterpret_cast<floatx4 *>(loop_lds_x);
    floatx4 *xb = xa + nv;

    // ---- once per token: ids, rows, RMSNorm weight, carried probabilities
    int idv[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) idv[k] = p.ids[(size_t)b * K + min(k, K - 1)];
    half8 gv[VPT];
#pragma unroll
    for (int u = 0; u < VPT; ++u) gv[u] = load_half8(p.gamma + min(tid + u * kLoopThreads, nv - 1) * 8);
    float prev[KC];
#pragma unroll
    for (int k = 0; k < KC; ++k) prev[k] = 0.f;
    if (p.prev0) {
#pragma unroll
        for (int k = 0; k < KC; ++k)
            if (k < K) prev[k] = p.prev0[(size_t)b * K + k];
    }
    const half_t *rows[KC];
    size_t rowi[KC];
    bool bad_id = false;
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        const bool ok = idv[k] >= 0 && idv[k] < p.V;
        if (k < K && !ok) bad_id = true;
        rowi[k] = (size_t)(ok ? idv[k] : 0);
        rows[k] = Q4 ? nullptr : p.lm_head + rowi[k] * d;
    }
    half8 wv[KC][VPT];
    auto load_rows = [&]() {
#pragma unroll
        for (int k = 0; k < KC; ++k)
#pragma unroll
            for (int u = 0; u < VPT; ++u) {
                const int v = tid + u * kLoopThreads;
                const half8 x = load_half8(rows[k] + min(v, nv - 1) * 8);
                wv[k][u] = (k < K && v < nv) ? x : zero_half8();
            }
    };
    if (KEEP && !Q4) load_rows();
    // KEEP: the rows stay for the whole call, so they are kept as floats with the RMSNorm weight folded in
    // (the product of two halves is exact in fp32): a layer then costs one conversion of its hidden state
    // and K + 1 FMAs per element instead of twice as many instructions.
    float wg[KEEP ? KC : 1][KEEP ? VPT : 1][8];
    if (KEEP && !Q4) {
#pragma unroll
        for (int k = 0; k < KC; ++k)
#pragma unroll
            for (int u = 0; u < VPT; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) wg[KEEP ? k : 0][KEEP ? u : 0][e] = (float)wv[k][u][e] * (float)gv[u][e];
    }
    if (Q4) {
        // element e of vector v is the code in bits 4e of word v of the row; its group is (8v) / group
        const int ng = d / p.group;
#pragma unroll
        for (int k = 0; k < KC; ++k)
#pragma unroll
            for (int u = 0; u < VPT; ++u) {
                const int v = tid + u * kLoopThreads;
                const int vc = min(v, nv - 1);
                const uint32_t word = p.qweight[rowi[k] * nv + vc];
                const int gi = (vc * 8) / p.group;
                const float sc = (float)p.qscales[rowi[k] * ng + gi], zp = (float)p.qzeros[rowi[k] * ng + gi];
                const bool live = k < K && v < nv;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float wq = sc * ((float)((word >> (4 * e)) & 15u) - zp);
                    wg[KEEP ? k : 0][KEEP ? u : 0][e] = live ? wq * (float)gv[u][e] : 0.f;
                }
            }
    }

    const int row_begin = min(p.V, w * p.rows_per_wg);
    const int row_end = min(p.V, row_begin + p.rows_per_wg);
    int meetings = 0;       // verifications so far: the arrival counter stands at meetings * Pg afterwards
    int exit_layer = -1, exit_token = -1;
    int status = 0;
    // The mask is read once.  Up to 128 layers it becomes two 64-bit words in scalar registers (one ballot each), and
    // the next active layer is a shift and a count of trailing zeros; deeper stacks keep the first kLoopMaskLds
    // layers of it in LDS.  Scanning it in global memory costs a dependent round trip per inactive layer -- half a
    // microsecond each, a third of a layer's evaluation.
    if (threadIdx.x == 0) {
        rare.logits = p.logits; rare.probs = p.probs; rare.scores = p.scores; rare.exit_flags = p.exit_flags;
        rare.ver_token = p.ver_token; rare.hit = p.hit; rare.exit_layer = p.exit_layer; rare.token = p.token;
        rare.status = p.status; rare.cand_val = p.cand_val; rare.cand_idx = p.cand_idx; rare.arrive = p.arrive;
        rare.abort = p.abort; rare.spin_limit = p.spin_limit;
    }
    unsigned long long m0 = ~0ull, m1 = ~0ull;
    const bool mask_bits = L <= 128;
    if (p.active) {
        if (mask_bits) {
            const int a0 = lane < L ? p.active[lane] : 0, a1 = lane + 64 < L ? p.active[lane + 64] : 0;
            m0 = __ballot(a0 != 0);
            m1 = __ballot(a1 != 0);
        } else {
            for (int i = tid; i < min(L, kLoopMaskLds); i += kLoopThreads) act_lds[i] = p.active[i] != 0 ? 1 : 0;
        }
    }
    __syncthreads();
    auto is_active = [&](int q) {
        if (!p.active) return true;
        if (mask_bits) return (((q < 64 ? m0 : m1) >> (q & 63)) & 1ull) != 0;
        // (in a scalar register: a value read from LDS counts as divergent, and the layer index, with every address
        // derived from it, would move to the vector units)
        const int a = q < kLoopMaskLds ? (int)act_lds[q] : (int)(p.active[q] != 0);
        return __builtin_amdgcn_readfirstlane(a) != 0;
    };
    // first layer from l0 on whose predictor is active (L if none); uniform over the grid
    auto next_active = [&](int l0) {
        int q = l0;
        if (!p.active || q >= L) return min(q, L);  // (no mask: the compiler keeps a copy of the loop that steps by one)
        if (mask_bits) {
            if (q < 64) {
                const unsigned long long r = m0 >> q;
                if (r) return min(L, q + (int)__builtin_ctzll(r));
                q = 64;
            }
            const unsigned long long r = q < 128 ? m1 >> (q - 64) : 0ull;
            return r ? min(L, q + (int)__builtin_ctzll(r)) : L;
        }
        while (q < L && !is_active(q)) ++q;
        return q;
    };
    // A layer's inputs -- its hidden state, this thread's predictor row and the output bias -- are requested
    // one active layer ahead (every layer's hidden state exists before the call), so that a layer that does
    // not fire costs arithmetic and two barriers, not a trip to memory.
    half8 hv_pf[VPT];
    MlpRow<KC> row_pf;
    half_t b2_pf;
    auto prefetch = [&](int q) {
        const half_t *hrow = p.hidden + ((size_t)q * B + b) * d;
#pragma unroll
        for (int u = 0; u < VPT; ++u) hv_pf[u] = load_half8(hrow + min(tid + u * kLoopThreads, nv - 1) * 8);
        mlp_row_load<KC>(row_pf, p.W1 + (size_t)q * H * 3 * K, p.b1 ? p.b1 + (size_t)q * H : nullptr,
                         p.w2 + (size_t)q * H, K, H, tid);
        b2_pf = (p.b2 ? p.b2 : p.gamma)[p.b2 ? q : 0];  // always a valid address; masked at use
    };
    int l = next_active(0);
    int lnext = l < L ? next_active(l + 1) : L;  // known one layer ahead, so that the scan of the mask is never
                                                 // between a layer's start and the request of the next one's inputs
    int evaluated_upto = -1;  // last layer whose outputs below are final
    if (l < L) prefetch(l);
    while (l < L) {
        const size_t tok = (size_t)l * B + b;
        // the layer after the next: looked up before this layer's requests go out -- an LDS read behind them would
        // wait for the scalar load among them too (LDS and scalar memory share a counter), a trip to memory per layer
        const int lnext2 = lnext < L ? next_active(lnext + 1) : L;
        const half_t *W1 = p.W1 + (size_t)l * H * 3 * K;
        const half_t *w2 = p.w2 + (size_t)l * H;
        const half_t *b1 = p.b1 ? p.b1 + (size_t)l * H : nullptr;
        MlpRow<KC> rowm[1];
        rowm[0] = row_pf;
        const half_t b2raw = b2_pf;
        half8 hv[VPT];
#pragma unroll
        for (int u = 0; u < VPT; ++u) hv[u] = tid + u * kLoopThreads < nv ? hv_pf[u] : zero_half8();
        prefetch(min(lnext, L - 1));  // unconditional (a load under a branch would make the compiler drain the others)
        if (!KEEP) load_rows();

        float ssq = 0.f, acc[KC];
#pragma unroll
        for (int k = 0; k < KC; ++k) acc[k] = 0.f;
#pragma unroll
        for (int u = 0; u < VPT; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float hf = (float)hv[u][e];
                ssq += hf * hf;
                if (KEEP) {
#pragma unroll
                    for (int k = 0; k < KC; ++k) acc[k] += hf * wg[KEEP ? k : 0][KEEP ? u : 0][e];
                } else {
                    const float x = hf * (float)gv[u][e];
#pragma unroll
                    for (int k = 0; k < KC; ++k) acc[k] += x * (float)wv[k][u][e];
                }
            }
        ssq = wave_sum_to_last_row(ssq);
#pragma unroll
        for (int k = 0; k < KC; ++k) acc[k] = wave_sum_to_last_row(acc[k]);
        if (lane == kWave - 1) {
            red[0][wave] = ssq;
#pragma unroll
            for (int k = 0; k < KC; ++k) red[1 + k][wave] = acc[k];
        }
        __syncthreads();
        auto sum8 = [&](const float *v) {  // wavefront order, as before: ((((((v0 + v1) + v2) + ...
            const floatx4 a = *reinterpret_cast<const floatx4 *>(v), c4 = *reinterpret_cast<const floatx4 *>(v + 4);
            return ((((((a[0] + a[1]) + a[2]) + a[3]) + c4[0]) + c4[1]) + c4[2]) + c4[3];
        };
        ssq = sum8(red[0]);
#pragma unroll
        for (int k = 0; k < KC; ++k) acc[k] = sum8(red[1 + k]);
        const float r = 1.0f / sqrtf(ssq * (1.0f / (float)d) + p.eps);
        float z[KC], pr[KC];
#pragma unroll
        for (int k = 0; k < KC; ++k) z[k] = bad_id ? quiet_nan() : acc[k] * r;
        local_softmax<KC>(z, K, pr);
        float part = mlp_partial<KC, kLoopThreads, 1>(rowm, W1, b1, w2, K, H, tid, z, pr, prev);
        part = wave_sum_to_last_row(part);
        if (lane == kWave - 1) red_u[wave] = part;
        __syncthreads();
        float uo = p.b2 ? (float)b2raw : 0.f;
        {
            const floatx4 a = *reinterpret_cast<const floatx4 *>(red_u), c4 = *reinterpret_cast<const floatx4 *>(red_u + 4);
#pragma unroll
            for (int q = 0; q < 4; ++q) uo += a[q];
#pragma unroll
            for (int q = 0; q < 4; ++q) uo += c4[q];
        }
        const float sc = sigmoidf(uo);
        const bool fire = sc > p.threshold;  // the same bits in every thread of every workgroup of the group
        if (writer && tid == 0) {
            rare.scores[tok] = sc;
            rare.exit_flags[tok] = fire ? 1 : 0;
#pragma unroll
            for (int k = 0; k < KC; ++k)
                if (k < K) {
                    rare.logits[tok * K + k] = z[k];
                    rare.probs[tok * K + k] = pr[k];
                }
            if (!fire) {
                rare.ver_token[tok] = -1;
                rare.hit[tok] = 0;
            }
        }
#pragma unroll
        for (int k = 0; k < KC; ++k) prev[k] = pr[k];
        if (!fire) {
            evaluated_upto = l;
            l = lnext;
            lnext = lnext2;
            continue;
        }

        // ---- verification: this workgroup's block of LM-head rows against x = h * gamma
#pragma unroll
        for (int u = 0; u < VPT; ++u) {
            const int v = tid + u * kLoopThreads;
            if (v < nv) {
                floatx4 a4, b4;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    a4[e] = (float)hv[u][e] * (float)gv[u][e];
                    b4[e] = (float)hv[u][4 + e] * (float)gv[u][4 + e];
                }
                xa[v] = a4;
                xb[v] = b4;
            }
        }
        __syncthreads();
        float bv = -INFINITY;
        int bi = 0x7fffffff;
        if (Q4) {
            float *xs = reinterpret_cast<float *>(xb + nv);
            q4_prepare_planes<kLoopThreads, HEAD == 1>(xa, xb, xs, nv, d / p.group, p.group, tid);
            q4_head_rows<HEAD == 1>(p.qweight, p.qscales, p.qzeros, d, p.group, row_begin, row_end, wave, kLoopWaves, lane,
                                    xa, xb, xs, r, [&](int row, float v) {
                                        if (v > bv) {  // rows ascend: the strict comparison keeps the lowest row
                                            bv = v;
                                            bi = row;
                                        }
                                    });
        } else {
            head_argmax_rows<STREAM>(p.lm_head, d, row_begin, row_end, wave, kLoopWaves, lane, xa, xb, r, bv, bi);
        }
        if (lane == 0) {
            cv[wave] = bv;
            ci[wave] = bi;
        }
        __syncthreads();
        // candidates of successive verifications alternate between two buffers: a workgroup that runs ahead
        // into the next verification writes the other buffer while a slower one still reads this one, and
        // it cannot get two verifications ahead, because the next meeting needs everybody
        const size_t cbase = ((size_t)(meetings & 1) * B + b) * Pg;
        if (tid == 0) {
            for (int q = 1; q < kLoopWaves; ++q)
                if (cv[q] > bv || (cv[q] == bv && ci[q] < bi)) {
                    bv = cv[q];
                    bi = ci[q];
                }
            __hip_atomic_store(rare.cand_val + cbase + w, bv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(rare.cand_idx + cbase + w, bi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);  // the candidate has landed where every XCD reads it
            __hip_atomic_fetch_add(rare.arrive + b, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int target = (meetings + 1) * Pg;
            int met = 0;
            for (long long it = 0; it < rare.spin_limit; ++it) {
                if (__hip_atomic_load(rare.arrive + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) {
                    met = 1;
                    break;
                }
                if (__hip_atomic_load(rare.abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
                __builtin_amdgcn_s_sleep(8);
            }
            if (!met) __hip_atomic_store(rare.abort, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            met_lds = met;
        }
        __syncthreads();
        if (!met_lds) {  // uniform: the group could not meet within the spin limit
            status = 1;
            break;
        }
        ++meetings;
        // every workgroup combines the group's candidates itself (lowest row on ties)
        bv = -INFINITY;
        bi = 0x7fffffff;
        for (int i = tid; i < Pg; i += kLoopThreads) {
            const float v = __hip_atomic_load(rare.cand_val + cbase + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int ix = __hip_atomic_load(rare.cand_idx + cbase + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (v > bv || (v == bv && ix < bi)) {
                bv = v;
                bi = ix;
            }
        }
        wave_argmax(bv, bi);
        __syncthreads();  // cv / ci were read by thread 0 before the meeting; met_lds by everybody
        if (lane == 0) {
            cv[wave] = bv;
            ci[wave] = bi;
        }
        __syncthreads();
        bv = cv[0];
        bi = ci[0];
#pragma unroll
        for (int q = 1; q < kLoopWaves; ++q)
            if (cv[q] > bv || (cv[q] == bv && ci[q] < bi)) {
                bv = cv[q];
                bi = ci[q];
            }
        bool hit = false;
#pragma unroll
        for (int k = 0; k < KC; ++k)
            if (k < K && idv[k] == bi) hit = true;
        if (writer && tid == 0) {
            rare.ver_token[tok] = bi;
            rare.hit[tok] = hit ? 1 : 0;
        }
        evaluated_upto = l;
        if (hit) {  // the token leaves the model at this layer
            exit_layer = l;
            exit_token = bi;
            break;
        }
        __syncthreads();  // cv / ci are rewritten by the next verification
        l = lnext;
        lnext = lnext2;
    }

    // ---- layers that were not evaluated (inactive, after the exit, or from a failed meeting on): defined outputs
    if (writer) {
        for (int ll = 0; ll < L; ++ll) {
            if (ll <= evaluated_upto && is_active(ll)) continue;
            const size_t tok = (size_t)ll * B + b;
            if (tid < K) {
                rare.logits[tok * K + tid] = 0.f;
                rare.probs[tok * K + tid] = 0.f;
            }
            if (tid == 0) {
                rare.scores[tok] = 0.f;
                rare.exit_flags[tok] = 0;
                rare.ver_token[tok] = -1;
                rare.hit[tok] = 0;
            }
        }
        if (tid == 0) {
            rare.exit_layer[b] = exit_layer;
            rare.token[b] = exit_token;
            rare.status[b] = status;
        }
    }
}

// An empty layer stack: every token runs "the whole stack" without an exit.  No input is touched.
__global__ void layer_loop_empty_kernel(int32_t *exit_layer, int32_t *token, int32_t *status, int B) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) {
        exit_layer[b] = -1;
        token[b] = -1;
        status[b] = 0;
    }
}

template <int KC, int VPT, bool EXACT>
static hipError_t launch_loop_one(LoopParams p, int max_wgs, hipStream_t s) {
    const bool stream = head_streams(p.d, p.V);
    constexpr bool kCanQ4 = KC * VPT <= 16 && KC <= 8;
    void (*kern)(LoopParams) = stream ? layer_loop_kernel<KC, VPT, EXACT, true> : layer_loop_kernel<KC, VPT, EXACT, false>;
    size_t lds = (size_t)p.d * sizeof(float);
    int quantum = kLoopWaves * kHeadRows;
    if (p.qweight) {
        if constexpr (kCanQ4) {
            const bool wide = p.group % 32 == 0 && p.d % 32 == 0 && (reinterpret_cast<uintptr_t>(p.qweight) & 15) == 0;
            kern = wide ? layer_loop_kernel<KC, VPT, EXACT, false, 1> : layer_loop_kernel<KC, VPT, EXACT, false, 2>;
            lds += (size_t)(p.d / p.group) * sizeof(float);
            quantum = kLoopWaves * kQ4HeadRows;
        } else {
            return hipErrorInvalidValue;
        }
    }
    if (lds > 48 * 1024)  // per launch: the library keeps no state; a refusal shows as the launch error
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds);
    // every workgroup of a group must be resident while the group meets: size the grid from what the
    // runtime says fits on the device
    int dev = 0, cus = 0, per_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess)
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(kern), kLoopThreads, lds);
    if (e != hipSuccess) return e;
    long long fit = (long long)cus * (per_cu > 2 ? 2 : per_cu);
    if (fit > max_wgs) fit = max_wgs;
    const int Pg = (int)(fit / p.B);
    if (Pg < 1) return hipErrorInvalidConfiguration;
    p.rows_per_wg = (((p.V + Pg - 1) / Pg + quantum - 1) / quantum) * quantum;
    hipLaunchKernelGGL(kern, dim3(Pg, p.B), dim3(kLoopThreads), lds, s, p);
    return hipGetLastError();
}

template <int KC, bool EXACT>
static hipError_t launch_loop_vpt(const LoopParams &p, int max_wgs, hipStream_t s) {
    if ((p.d >> 3) <= kLoopThreads) return launch_loop_one<KC, 1, EXACT>(p, max_wgs, s);
    return launch_loop_one<KC, 2, EXACT>(p, max_wgs, s);
}

// d <= 8192 (two 16-byte vectors per thread and row).  max_wgs bounds the grid (the workspace holds two
// candidates per workgroup).
hipError_t launch_layer_loop(const LoopParams &p, int max_wgs, hipStream_t s) {
    if (p.L == 0) {
        hipLaunchKernelGGL(layer_loop_empty_kernel, dim3(1), dim3(64), 0, s, p.exit_layer, p.token, p.status, p.B);
        return hipGetLastError();
    }
    if (p.K == 4) return launch_loop_vpt<4, true>(p, max_wgs, s);
    if (p.K == 8) return launch_loop_vpt<8, true>(p, max_wgs, s);
    if (p.K < 4) return launch_loop_vpt<4, false>(p, max_wgs, s);
    if (p.K < 8) return launch_loop_vpt<8, false>(p, max_wgs, s);
    return launch_loop_vpt<16, false>(p, max_wgs, s);
}

}  // namespace specee
