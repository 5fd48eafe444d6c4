// Token-tree contraction (paper Sec. 6.2, merged mapping): Z[n][m] = x_n . W[merged_m]
// for the N <= 64 nodes of a tree against its M merged LM-head rows, on the matrix cores.
//
// A tree has few rows (M is tens to a couple of hundred) and up to 64 nodes, so the
// operand that every wavefront needs in full is the small tile of LM-head rows, and the
// operand that can stay private is a wavefront's own 16 nodes:
//   * wavefront w owns node tile w.  Its B operand -- x = h*gamma of its 16 nodes, split
//     exactly into hi + lo halves -- is built in registers from two 16-byte loads per
//     lane and never touches LDS;
//   * the A operand -- 16*MT gathered LM-head rows, 128 bytes of each per stage -- is
//     loaded once per workgroup (16 bytes per lane, coalesced per row) into a
//     double-buffered LDS tile and read by all four wavefronts.
// Per 64-element stage the workgroup moves 8 KB into LDS and reads it four times, half
// the LDS traffic of sharing x instead, and there is one barrier per stage.
// v_mfma_f32_16x16x32_f16: lane = 16*q + c holds A[row c][k-slots of q], B[k-slots of q][node c]
// and D[rows 4q..4q+3][node c].
//
// MODE 0: one d-slice per workgroup, un-normalised partial sums and partial sums of
//         squares go to the workspace (few trees: many CUs share one tree).
// MODE 3: one workgroup per tree over all of d.  The logits stay in LDS; the same
//         workgroup gathers every node's K columns, builds the features and evaluates the
//         predictor MLP -- for K in {4, 8} also on the matrix cores (W1 rows are the A
//         operand, the 16 nodes' hi/lo-split features the B operand) -- then applies the
//         path rule.  Only inputs are read and only outputs written.
// FUSED: the merge of the tree's ids runs in the prologue (N*K <= 1024).
#include <type_traits>

#include "device_utils.h"
#include "kernels.h"
#include "merge_block.h"
#include "tree_finish.h"

namespace specee {

constexpr int kTcFusedMax = kMergePerThread * 256;  // ids per tree when the merge is fused
constexpr int kWholeWideMaxWgs = 256;               // one 512-thread workgroup per CU
constexpr int kMergeBitmapMaxV = 65536;               // vocabularies up to here are merged through a bitmap
constexpr int kGammaLds = 4096;                     // elements of the RMSNorm weight a workgroup may stage in LDS
// shape of the sixteen-row-tile whole-tree variant: stages in flight, threads, k elements per stage
constexpr int kWide16Pd = 2, kWide16Threads = 512, kWide16Kch = 128;

// KCH: k elements per stage (64 or 128).  A stage is one barrier and one LDS write -> read -> matrix
// instruction dependency chain, so longer stages amortise that latency; 128 needs the row tile to
// fit twice in LDS (MT = 4).  k-slots of lane group q within a stage: 64*(j/2) + 16*q + 8*(j%2).
// THREADS: 256 (wavefront w owns node tile w) or 512 (wavefronts w and w+4 share node tile w and
// split the k-steps of every stage between them; their accumulators are added through LDS at the
// end).  Eight wavefronts halve the per-wavefront instruction stream of a stage, which is what bounds
// a workgroup that streams a whole tree on its own.
// GL: the RMSNorm weight of the workgroup's d-slice (at most kGammaLds elements) is staged in LDS
// once instead of being fetched again by every lane at every stage: those fetches are cache hits,
// but they take a third of the slots of the vector memory path, which is what a CU streaming a
// tree runs out of first.
template <int MT, int MODE, bool FUSED, int PD, int KC, int KCH, int THREADS = 256, bool GL = false>
__global__ __launch_bounds__(THREADS) void tree_contract_kernel(GemmParams p, TreeFinishParams f) {
    constexpr int kTcThreads = THREADS;
    constexpr int kTcWaves = THREADS / 64;
    constexpr int KH = THREADS / 256;        // wavefronts per node tile
    constexpr int kTcKC = KCH;
    constexpr int kTcRow = KCH + 8;          // halves per LDS row (pad keeps 16-byte reads spread over banks)
    constexpr int JN = KCH / 32 / KH;        // matrix-instruction k-steps per stage and wavefront
    constexpr int VPR = KCH / 8;             // 16-byte vectors per row per stage
    constexpr int ROWS = 16 * MT;            // LM-head rows per workgroup
    constexpr int APT = ROWS * VPR / kTcThreads;  // 16-byte A vectors per thread per stage
    constexpr int kALdsHalves = 2 * ROWS * kTcRow;
    // the row tile buffers: static up to 64 KB; sixteen row tiles need 72 KB, which only dynamic LDS offers
    // (the launcher raises the kernel's limit)
    constexpr bool kDynLds = MT == 16;
    extern __shared__ __attribute__((aligned(16))) half_t dyn_smem[];
    __shared__ __attribute__((aligned(16))) half_t static_smem[kDynLds ? 8 : kALdsHalves];
    half_t *smem = kDynLds ? dyn_smem : static_smem;
    __shared__ int32_t cols_lds[MODE == 3 ? kTcFusedMax : 1];
    __shared__ float prev_lds[MODE == 3 ? kTcFusedMax : 1];
    __shared__ float feat_lds[MODE == 3 ? 4 * 16 * kMlpFeat : 1];
    __shared__ float ssq_lds[MODE == 3 ? 64 : 1];
    __shared__ int32_t bad_lds[MODE == 3 ? 64 : 1];
    __shared__ int32_t exit_lds[MODE == 3 ? 64 : 1];
    __shared__ int32_t par_lds[MODE == 3 ? 64 : 1];
    __shared__ int32_t last_lds;
    __shared__ __attribute__((aligned(16))) half_t gam_lds[GL ? kGammaLds : 8];
    static_assert(MT == 4 || MT == 8 || MT == 16, "row tiles per workgroup");
    static_assert(sizeof(half_t) * kALdsHalves >= sizeof(int32_t) * merge_lds_ints(kTcFusedMax),
                  "merge scratch must fit in the row tile buffers");
    static_assert(sizeof(half_t) * kALdsHalves >= sizeof(float) * 64 * ROWS, "whole-tree logits must fit");
    static_assert(MODE != 3 || FUSED, "the whole-tree mode merges in its prologue");
    typedef half_t (*tile_t)[ROWS][kTcRow];
    tile_t a_lds = reinterpret_cast<tile_t>(smem);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, q = lane >> 4;
    const int kh = (tid >> 6) >> 2, nt_w = (tid >> 6) & 3;  // k-share and node tile of this wavefront
    auto koff = [&](int jj) {
        const int j = kh * JN + jj;
        return 64 * (j >> 1) + 16 * q + 8 * (j & 1);
    };
    const int NBn = (p.N + 63) / 64;
    const int g = blockIdx.z / NBn, nb = blockIdx.z - g * NBn;
    const int n0 = nb * 64;
    // d-slice in blockIdx.x, row group in blockIdx.y: workgroups are dealt to the eight XCDs round-robin
    // by linear id, so the row groups of one d-slice (which re-read the same hidden-state slice) land on
    // the same XCD and share its L2 when the number of slices is a multiple of eight
    const int s = blockIdx.x;
    const int d = p.d;
    const int k_begin = s * p.dslice;
    const int k_end = min(d, k_begin + p.dslice);
    const int nchunks = (k_end - k_begin + kTcKC - 1) / kTcKC;

    // ---- the tree's ids go out first of all: the rows, the longest chain of the kernel, hang on them, and
    // behind the hidden-state requests below they would arrive a microsecond or two later
    int ids_r[kMergePerThread];
    if (FUSED) merge_load_ids<kTcThreads>(p.ids + (size_t)g * p.N * p.K, p.N * p.K, ids_r);

    // ---- B side: this lane's node and k-slots
    const int node = n0 + nt_w * 16 + c;
    const bool node_ok = node < p.N;
    const half_t *hrow = p.hidden + ((size_t)g * p.N + (node_ok ? node : 0)) * d;
    half8 h_buf[PD][JN], g_buf[GL ? 1 : PD][JN];
    // Loads are unconditional (addresses clamped into the row, results zeroed by a select when they
    // are consumed): a load under a branch makes the compiler drain every outstanding load at the
    // join, which would serialise the prefetch stages.
    auto issue_b = [&](int kc, int slot) {
#pragma unroll
        for (int j = 0; j < JN; ++j) {
            const int ko = min(k_begin + kc * kTcKC + koff(j), k_end - 8);  // stages past the end re-read the slice's tail
            if (!GL) g_buf[slot][j] = load_half8(p.gamma + ko);
            h_buf[slot][j] = load_half8(hrow + ko);
        }
    };
    auto b_valid = [&](int kc, int j) {
        return node_ok && k_begin + kc * kTcKC + koff(j) < k_end;
    };
    // With the merge fused in, the first stages of hidden states are NOT requested here: every workgroup
    // of the launch would do so at once, and behind that burst the ids -- and with them the merge and the
    // rows, the chain that decides when the stage loop can start -- come back microseconds later.  They
    // follow the row requests below.
    constexpr int PD0 = FUSED ? 0 : PD;
#pragma unroll
    for (int u = 0; u < PD0; ++u) issue_b(u, u);
    // GL: this thread's share of the slice's RMSNorm weight, parked in LDS after the merge
    constexpr int kGamPt = GL ? kGammaLds / 8 / kTcThreads : 1;
    half8 gam_r[kGamPt];
    if (GL) {
#pragma unroll
        for (int e = 0; e < kGamPt; ++e)
            gam_r[e] = load_half8(p.gamma + min(k_begin + (tid + e * kTcThreads) * 8, k_end - 8));
    }
    // MODE 3: previous probabilities and parents are requested now and parked in LDS after the merge,
    // whose own wait for the ids then covers them (clamped addresses: no branch around a load)
    constexpr int kPrevPt = MODE == 3 ? kTcFusedMax / kTcThreads : 1;
    float prev_r[kPrevPt];
    int par_r = -1;
    half_t b2_r = (half_t)0.f;  // output bias, widened where it is used
    if (MODE == 3) {
        const int n_ids = p.N * p.K;
#pragma unroll
        for (int e = 0; e < kPrevPt; ++e) prev_r[e] = f.prev[(size_t)g * n_ids + min(tid + e * kTcThreads, n_ids - 1)];
        const int32_t *pp = f.path_exit ? f.parent + (size_t)g * p.N + min(tid, p.N - 1) : p.ids;
        par_r = *pp;
        b2_r = *(f.b2 ? f.b2 : p.gamma);
        if (tid < 64) bad_lds[tid] = 0;
    }

    // The first stages of hidden states go out once the ids (and the other prologue loads, requested with them)
    // have come back: not before -- every workgroup's hidden-state burst ahead of its ids delays the ids -- but
    // before the merge, so that they stream in while it computes and only the rows remain to be waited for after it.
    if (FUSED && MODE == 3) {
        __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
        asm volatile("" ::: "memory");
#pragma unroll
        for (int u = 0; u < PD; ++u) issue_b(u, u);
    }

    // ---- merged rows
    int M, Mtrue = 0;
    int32_t *uniq = nullptr;
    int col_of[kMergePerThread], own_id[kMergePerThread];
    if (FUSED) {
        const int n_ids = p.N * p.K;
        // through a bitmap of the vocabulary when it fits in the row tile buffers, else by hashing
        // (a bitmap of a larger vocabulary costs more to clear and to count than the hash table does: measured
        // equal at 32000 tokens, 3 % behind at 128256)
        const bool bitmap = p.V <= kMergeBitmapMaxV &&
                            (size_t)merge_bitmap_ints(p.V, n_ids) * sizeof(int32_t) <=
                                (kDynLds ? (size_t)2 * ROWS * kTcRow * sizeof(half_t) : sizeof(static_smem));
        Mtrue = bitmap ? merge_bitmap<kTcThreads>(ids_r, n_ids, p.V, reinterpret_cast<int32_t *>(smem), uniq, col_of,
                                                  own_id)
                       : merge_block<kTcThreads>(ids_r, n_ids, reinterpret_cast<int32_t *>(smem), uniq, col_of, own_id);
        M = Mtrue;
    } else {
        M = p.Mptr ? p.Mptr[g] : p.Mcap;
    }
    const bool overflow = M > p.Mcap;
    if (overflow) M = p.Mcap;
    const int m0 = blockIdx.y * ROWS;
    if (MODE != 3 && m0 >= M) return;  // uniform over the workgroup

    // ---- A side: this thread copies vectors (row, v) of the row tile: index = tid + 256*i.  The rows are
    // requested the moment they are known; everything else the merge produced is put away afterwards.
    const half_t *arow[APT];
    bool arow_ok[APT];
    int a_r[APT], a_v[APT];
#pragma unroll
    for (int i = 0; i < APT; ++i) {
        const int vi = tid + kTcThreads * i;
        a_r[i] = vi / VPR;
        a_v[i] = vi % VPR;
        const int m = m0 + a_r[i];
        arow_ok[i] = m < M;
        int row = 0;
        if (arow_ok[i]) {
            row = FUSED ? uniq[m] : (p.rowlist ? p.rowlist[(size_t)g * p.Mcap + m] : m);
            if (row < 0 || row >= p.V) row = 0;  // invalid id: the node is reported NaN, nothing is read out of bounds
        }
        arow[i] = p.lm_head + (size_t)row * d;
    }
    half8 a_buf[PD][APT];
    // LA (a compile-time constant wrapped in a type): slices of the row tile -- kTcThreads / VPR rows each --
    // that are loaded and written to LDS.  All of them, except in the sixteen-tile variant, whose stage loop
    // exists in a few versions for trees that fill less of the capacity (see below); within a version every
    // load is unconditional, so the compiler's count of outstanding loads stays exact.
    typedef std::integral_constant<int, APT> all_slices;
    auto issue_a = [&](int kc, int slot, auto la) {
#pragma unroll
        for (int i = 0; i < decltype(la)::value; ++i) {
            const int ko = min(k_begin + kc * kTcKC + a_v[i] * 8, k_end - 8);
            a_buf[slot][i] = load_half8(arow[i] + ko);
        }
    };
    auto a_valid = [&](int kc, int i) {
        return arow_ok[i] && k_begin + kc * kTcKC + a_v[i] * 8 < k_end;
    };
#pragma unroll
    for (int u = 0; u < PD; ++u) {  // in the order the stages need them
        if (u >= PD0 && !(FUSED && MODE == 3)) issue_b(u, u);
        issue_a(u, u, all_slices{});
    }

    if (FUSED) {
        const int n_ids = p.N * p.K;
        if (blockIdx.x == 0 && blockIdx.y == 0 && nb == 0) {
            if (tid == 0) p.M_out[g] = Mtrue;
            for (int m = tid; m < p.Mcap; m += kTcThreads)
                p.merged_out[(size_t)g * p.Mcap + m] = m < Mtrue ? uniq[m] : -1;
#pragma unroll
            for (int e = 0; e < kMergePerThread; ++e) {
                const int i = tid + e * kTcThreads;
                if (i < n_ids) p.cols_out[(size_t)g * n_ids + i] = col_of[e];
            }
        }
        if (MODE == 3) {
#pragma unroll
            for (int e = 0; e < kMergePerThread; ++e) {
                const int i = tid + e * kTcThreads;
                if (i < n_ids) {
                    cols_lds[i] = col_of[e];
                    if (own_id[e] < 0 || own_id[e] >= p.V) bad_lds[i / p.K] = 1;  // benign race: all writers store 1
                }
            }
#pragma unroll
            for (int e = 0; e < kPrevPt; ++e)
                if (tid + e * kTcThreads < n_ids) prev_lds[tid + e * kTcThreads] = prev_r[e];
            if (f.path_exit && tid < p.N) par_lds[tid] = par_r;
        }
    }
    if (GL) {
        static_assert(!GL || FUSED, "the barrier below publishes the staged weight");
#pragma unroll
        for (int e = 0; e < kGamPt; ++e) {
            const int idx = (tid + e * kTcThreads) * 8;
            if (idx < k_end - k_begin) *reinterpret_cast<half8 *>(&gam_lds[idx]) = gam_r[e];
        }
    }
    if (FUSED) __syncthreads();  // the merge scratch becomes the row tile buffers

    // MODE 3: for the matrix-core MLP the predictor goes to LDS after the contraction, as a padded
    // image in the part of the row-tile buffers that the logits leave free (when it fits).  Up to
    // kMlpPf vectors per thread are requested here and ride in registers through the stage loop, so
    // that the scoring phase does not start with a round trip to memory.
    constexpr int kMlpPf = 1024 / kTcThreads;
    constexpr size_t kMlpFree = sizeof(half_t) * kALdsHalves - sizeof(float) * 64 * ROWS;
    const bool mfma_mlp = MODE == 3 && KC <= 8 && mlp_mfma_ok(p.K, f.H);
    // only these instances carry the code (with eight row tiles the logits leave next to nothing free)
    constexpr bool kPadded = MODE == 3 && MT == 4 && 3 * KC + 1 <= kMlpPad;
    const bool mlp_in_lds = kPadded && mfma_mlp && mlp_padded_ok(p.K, f.H) &&
                            (size_t)mlp_padded_halves(f.H) * sizeof(half_t) <= kMlpFree;
    half8 mlp_pf[kPadded ? kMlpPf : 1], w2_pf;
    if (kPadded) {  // unconditional loads (a branch here would drain the stage prefetch at its join)
#pragma unroll
        for (int e = 0; e < kMlpPf; ++e)
            mlp_pf[e] = mlp_padded_vector(f, tid + e * kTcThreads, mlp_in_lds, p.gamma);
        w2_pf = load_half8(mlp_in_lds ? f.w2 + (size_t)min(tid, f.H / 8 - 1) * 8 : p.gamma);
    }

    floatx4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
    float ssq = 0.f;

    // The stage loop is free of branches (stages past the end are issued on clamped addresses and
    // contribute zeros) so that the compiler can keep PD stages of loads outstanding instead of
    // draining the memory pipeline at every control-flow join.
    //
    // It is software-pipelined by one stage: while the matrix cores work on stage kc (row tile in
    // a_lds[buf], B operand in bhi/blo), the vector units turn the prefetched registers of stage kc+1
    // into the next B operand and the next row tile (a_lds[buf ^ 1]), and that slot's registers are
    // re-used for the loads of stage kc+1+PD.  One barrier per stage publishes the next tile and
    // retires the reads of the current one.
    auto tile_to_lds = [&](int kc, int slot, int b, auto la) {
#pragma unroll
        for (int i = 0; i < decltype(la)::value; ++i)
            *reinterpret_cast<half8 *>(&a_lds[b][a_r[i]][a_v[i] * 8]) =
                a_valid(kc, i) ? a_buf[slot][i] : zero_half8();
    };
    // x = h*gamma split exactly into hi = round(h*gamma), lo = round(fma(h, gamma, -hi))
    auto build_b = [&](int kc, int slot, int j, half8 &hi, half8 &lo) {
        const half8 hsel = b_valid(kc, j) ? h_buf[slot][j] : zero_half8();
        half8 gvec;
        if (GL)  // stages past the end read the slice's tail: in bounds, and hsel is zero there
            gvec = *reinterpret_cast<const half8 *>(&gam_lds[min(kc * kTcKC + koff(j), k_end - k_begin - 8)]);
        else
            gvec = g_buf[slot][j];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const half2_t hh = {hsel[2 * e], hsel[2 * e + 1]};
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
    const int nstages = ((nchunks + PD - 1) / PD) * PD;
    if constexpr (MODE == 0) {
        // d-slices of a stage or two: nothing to pipeline, so stage by stage (operand build, barrier,
        // matrix instructions) without the extra trip of a pipelined loop
        int buf = 0;
        for (int kc0 = 0; kc0 < nstages; kc0 += PD) {
#pragma unroll
            for (int u = 0; u < PD; ++u) {
                const int kc = kc0 + u;
                half8 bhi[JN], blo[JN];
                tile_to_lds(kc, u, buf, all_slices{});
#pragma unroll
                for (int j = 0; j < JN; ++j) build_b(kc, u, j, bhi[j], blo[j]);
                __syncthreads();
                issue_a(kc + PD, u, all_slices{});
                issue_b(kc + PD, u);
#pragma unroll
                for (int j = 0; j < JN; ++j) {
                    half8 a[MT];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        a[mt] = *reinterpret_cast<const half8 *>(&a_lds[buf][mt * 16 + c][koff(j)]);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], bhi[j], acc[mt], 0, 0, 0);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
                        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], blo[j], acc[mt], 0, 0, 0);
                }
                buf ^= 1;
            }
        }
    } else {
        // The stage loop as a function of LA live slices of the row tile and LG live groups of four row
        // tiles (compile-time constants).  Rows between the two granularities hold stale LDS contents and
        // only feed logit columns that no node refers to.
        auto stage_loop = [&](auto la, auto lg) {
            half8 bhi[JN], blo[JN];
            tile_to_lds(0, 0, 0, la);
#pragma unroll
            for (int j = 0; j < JN; ++j) build_b(0, 0, j, bhi[j], blo[j]);
            issue_a(PD, 0, la);
            issue_b(PD, 0);
            __syncthreads();
            int buf = 0;
            for (int kc0 = 0; kc0 < nstages; kc0 += PD) {
#pragma unroll
                for (int u = 0; u < PD; ++u) {
                    const int kc = kc0 + u;
                    const int nslot = (u + 1) % PD;  // folds: u is an unrolled constant
                    half8 nhi[JN], nlo[JN];
                    tile_to_lds(kc + 1, nslot, buf ^ 1, la);
#pragma unroll
                    for (int j = 0; j < JN; ++j) {
                        if constexpr (MT == 16) {
                            // sixteen row tiles are a capacity: groups of four tiles beyond the merged rows of
                            // this version of the loop are not multiplied
                            build_b(kc + 1, nslot, j, nhi[j], nlo[j]);
#pragma unroll
                            for (int gq = 0; gq < MT; gq += 4) {
                                if (gq < 4 * decltype(lg)::value) {
                                    half8 a[4];
#pragma unroll
                                    for (int mt = 0; mt < 4; ++mt)
                                        a[mt] = *reinterpret_cast<const half8 *>(&a_lds[buf][(gq + mt) * 16 + c][koff(j)]);
#pragma unroll
                                    for (int mt = 0; mt < 4; ++mt)
                                        acc[gq + mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], bhi[j], acc[gq + mt], 0, 0, 0);
#pragma unroll
                                    for (int mt = 0; mt < 4; ++mt)
                                        acc[gq + mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], blo[j], acc[gq + mt], 0, 0, 0);
                                }
                            }
                        } else {
                            half8 a[MT];
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt)
                                a[mt] = *reinterpret_cast<const half8 *>(&a_lds[buf][mt * 16 + c][koff(j)]);
                            build_b(kc + 1, nslot, j, nhi[j], nlo[j]);
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt)
                                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], bhi[j], acc[mt], 0, 0, 0);
#pragma unroll
                            for (int mt = 0; mt < MT; ++mt)
                                acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[mt], blo[j], acc[mt], 0, 0, 0);
                        }
                    }
                    issue_a(kc + 1 + PD, nslot, la);
                    issue_b(kc + 1 + PD, nslot);
                    __syncthreads();
#pragma unroll
                    for (int j = 0; j < JN; ++j) {
                        bhi[j] = nhi[j];
                        blo[j] = nlo[j];
                    }
                    buf ^= 1;
                }
            }
        };
        if constexpr (MT == 16) {
            // sixteen row tiles are a capacity (129..256 merged rows): a tree that fills less of it takes a
            // version of the loop that leaves the empty slices alone
            constexpr int kSliceRows = kTcThreads / VPR;
            const int slices = __builtin_amdgcn_readfirstlane((M + kSliceRows - 1) / kSliceRows);
            static_assert(APT * kSliceRows == ROWS && ROWS == 256 && (APT == 8 || APT == 4), "slice arithmetic below");
            if (APT == 8 && slices <= 5)
                stage_loop(std::integral_constant<int, APT == 8 ? 5 : APT>{}, std::integral_constant<int, 3>{});
            else if (slices * kSliceRows <= 192)
                stage_loop(std::integral_constant<int, (3 * APT) / 4>{}, std::integral_constant<int, 3>{});
            else
                stage_loop(all_slices{}, std::integral_constant<int, 4>{});
        } else {
            stage_loop(all_slices{}, std::integral_constant<int, (MT + 3) / 4>{});
        }
    }
    // sum of squares of node c over this k-range: combine the four k-slot groups
    ssq += __shfl_xor(ssq, 16, kWave);
    ssq += __shfl_xor(ssq, 32, kWave);

    if (MODE == 0) {
        if (blockIdx.y == 0 && q == 0 && node_ok) p.ssq_part[((size_t)g * p.S + s) * p.Npad + node] = ssq;
        if (node_ok) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int mtile = m0 + mt * 16;
                if (mtile < M) {  // Mpad is a multiple of 16: the quad is in bounds and aligned
                    float *dst = p.out + (((size_t)g * p.S + s) * p.Npad + node) * p.Mpad + mtile + q * 4;
                    *reinterpret_cast<floatx4 *>(dst) = acc[mt];
                }
            }
        }
        return;
    }

    // ---- MODE 3: score the whole tree here
    __syncthreads();  // every wavefront is done with the row tiles: reuse them for the logits
    float *Zl = reinterpret_cast<float *>(smem);  // [64 nodes][ROWS], the quads of a node's row rotated by the node
    // (lane c of a wavefront holds node c: with plain rows, whose length is a multiple of the 64 banks, the sixteen
    // nodes of a 16-byte access would all fall on the same four banks)
    auto zq = [&](int n, int quad) { return n * ROWS + ((quad + n) & (ROWS / 4 - 1)) * 4; };
    auto zcell = [&](int n, int col) { return zq(n, col >> 2) + (col & 3); };
    if (KH == 2 && MT == 16) {
        // the two wavefronts of a node tile hold complementary k-shares: add them in a fixed order, through
        // the cells of the logit array that the sum goes to anyway (a separate staging area would not fit)
        if (kh == 1) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                *reinterpret_cast<floatx4 *>(&Zl[zq(nt_w * 16 + c, mt * 4 + q)]) = acc[mt];
            if (q == 0) ssq_lds[nt_w * 16 + c] = ssq;
        }
        __syncthreads();
        if (kh == 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt] += *reinterpret_cast<const floatx4 *>(&Zl[zq(nt_w * 16 + c, mt * 4 + q)]);
            ssq += ssq_lds[nt_w * 16 + c];
        }
        __syncthreads();
    } else if (KH == 2) {
        // the two wavefronts of a node tile hold complementary k-shares: add them in a fixed order
        float *tmp = Zl + 64 * ROWS;  // [4 tiles][MT quads][64 lanes]: a wavefront's 16-byte accesses are contiguous
        static_assert(KH == 1 || MT == 16 || sizeof(half_t) * kALdsHalves >= sizeof(float) * 2 * 64 * ROWS,
                      "room for the second wavefront's accumulators");
        if (kh == 1) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                *reinterpret_cast<floatx4 *>(&tmp[((nt_w * MT + mt) * 64 + lane) * 4]) = acc[mt];
            if (q == 0) ssq_lds[nt_w * 16 + c] = ssq;
        }
        __syncthreads();
        if (kh == 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                acc[mt] += *reinterpret_cast<const floatx4 *>(&tmp[((nt_w * MT + mt) * 64 + lane) * 4]);
            ssq += ssq_lds[nt_w * 16 + c];
        }
        __syncthreads();
    }
    if (p.S > 1) {
        // This workgroup covered one d-slice of the tree.  Every slice leaves its accumulators in the
        // workspace and draws a ticket; the holder of the last one adds the slices up in slice order
        // (so the result does not depend on which workgroup that is) and goes on to score the tree.
        // The accumulators travel as relaxed device-scope atomics: such stores are written through to
        // the level all XCDs share and such loads are served from there, so no cache has to be flushed
        // or invalidated around the ticket (a device-scope fence would walk this XCD's whole L2).
        // What orders them before the ticket: every storing thread waits until its own stores have
        // been acknowledged (the vector-memory counter reaches zero only when written-through stores
        // have arrived at that shared level), then the barrier, then thread 0 draws the ticket.  The
        // barrier alone would not do: its fences are workgroup scope and wait for no global store.
        // On the other side the winner's loads are issued after the ticket's value has come back
        // (it travels through LDS and a barrier), and they bypass the caches that are not coherent.
        const int t256 = tid & 255;  // kh == 0 wavefronts are threads 0..255
        // [G][S][row-tile quad element][256 threads]: a wavefront's accesses are contiguous
        float *part = p.out + (size_t)g * p.S * (256 * MT * 4) + t256;
        float *ssq_part = p.ssq_part + (size_t)g * p.S * 64 + nt_w * 16 + c;
        const size_t sstride = (size_t)256 * MT * 4;
        if (kh == 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    __hip_atomic_store(part + s * sstride + (mt * 4 + r) * 256, acc[mt][r], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
            if (q == 0)
                __hip_atomic_store(ssq_part + (size_t)s * 64, ssq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);  // this thread's stores have landed
        }
        __syncthreads();
        if (tid == 0)
            last_lds = __hip_atomic_fetch_add(&p.tickets[g], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == p.S - 1;
        __syncthreads();
        if (!last_lds) return;  // uniform over the workgroup
        if (kh == 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt] = floatx4{0.f, 0.f, 0.f, 0.f};
            ssq = 0.f;
            constexpr int MC = MT < 4 ? MT : 4;  // row tiles per batch of loads (bounds the registers held)
            for (int s0 = 0; s0 < p.S; s0 += 4) {
                float sq[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    sq[u] = __hip_atomic_load(ssq_part + (size_t)min(s0 + u, p.S - 1) * 64, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (int m0c = 0; m0c < MT; m0c += MC) {
                    floatx4 v[4][MC];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int ss = min(s0 + u, p.S - 1);  // clamped: always in bounds, masked below
#pragma unroll
                        for (int mt = 0; mt < MC; ++mt)
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                v[u][mt][r] = __hip_atomic_load(part + ss * sstride + ((m0c + mt) * 4 + r) * 256,
                                                                __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (s0 + u < p.S) {
#pragma unroll
                            for (int mt = 0; mt < MC; ++mt) acc[m0c + mt] += v[u][mt];
                        }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (s0 + u < p.S) ssq += sq[u];
            }
        }
    }
    if (kh == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            *reinterpret_cast<floatx4 *>(&Zl[zq(nt_w * 16 + c, mt * 4 + q)]) = acc[mt];
        if (q == 0) ssq_lds[nt_w * 16 + c] = ssq;
    }
    __syncthreads();

    const int K = p.K, N = p.N;
    if (mfma_mlp) {
        // the copy of the predictor is published by the barrier after the features are written
        half_t *img = reinterpret_cast<half_t *>(Zl + 64 * ROWS);
        if (kPadded && mlp_in_lds) {
            half8 *img8 = reinterpret_cast<half8 *>(img);
            const int nrowvec = 2 * f.H;
#pragma unroll
            for (int e = 0; e < kMlpPf; ++e)
                if (tid + e * kTcThreads < nrowvec) img8[tid + e * kTcThreads] = mlp_pf[e];
            for (int i = tid + kMlpPf * kTcThreads; i < nrowvec; i += kTcThreads) img8[i] = mlp_padded_vector(f, i, true, p.gamma);
            if (tid < f.H / 8) img8[nrowvec + tid] = w2_pf;
            if (tid == 0) img8[nrowvec + f.H / 8] = zero_half8();
        }
        // lanes q == 0 build the features of node c; all lanes then feed the matrix cores
        float *F = feat_lds + nt_w * 16 * kMlpFeat;
        const int n = nt_w * 16 + c;  // node within the tree (N <= 64: n0 == 0)
        const size_t gn = (size_t)g * N + n;
        bool poisoned = false;
        float z[KC], pr[KC];
        float zq = 0.f, pq = 0.f;  // KC <= 4: this lane's own slot k = q
        if (KC <= 4 && kh == 0) {
            // one slot per lane group: lane (c, q) handles slot k = q of node c, and the softmax over the
            // K slots runs across the four lanes c, c+16, c+32, c+48
            const int k = q;
            const bool slot = k < K;
            const float r = 1.0f / sqrtf(ssq_lds[n] / (float)d + p.eps);
            const bool bad = overflow || (n < N && bad_lds[n] != 0);
            float v = 0.f;
            if (slot && n < N) {
                int col = cols_lds[n * K + k];
                col = (col >= 0 && col < ROWS) ? col : 0;
                v = bad ? quiet_nan() : Zl[zcell(n, col)] * r;
            }
            float zm = slot ? v : -INFINITY;  // fmaxf drops NaN; the sums below carry it to every lane
            zm = fmaxf(zm, __shfl_xor(zm, 16, kWave));
            zm = fmaxf(zm, __shfl_xor(zm, 32, kWave));
            float e = slot ? __expf(v - zm) : 0.f;
            float es = e + __shfl_xor(e, 16, kWave);
            es += __shfl_xor(es, 32, kWave);
            zq = v;
            pq = e * __frcp_rn(es);
            poisoned = bad;
            if (slot) {
                const float pv = n < N ? prev_lds[n * K + k] : 0.f;
                F[c * kMlpFeat + k] = zq;
                F[c * kMlpFeat + K + k] = pq;
                F[c * kMlpFeat + 2 * K + k] = pq - pv;
            }
            for (int t = 3 * K + q; t < kMlpFeat; t += 4) F[c * kMlpFeat + t] = 0.f;
            if (kPadded && mlp_in_lds && q == 0) F[c * kMlpFeat + 3 * K] = 1.f;  // same lane as the zero fill of that slot
        } else if (q == 0 && kh == 0) {
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
            if (kPadded && mlp_in_lds) F[c * kMlpFeat + 3 * K] = 1.f;  // the bias column of the padded image
        }
        __syncthreads();
        // the two wavefronts of a node tile take half of the hidden units each
        const int htiles = f.H >> 4;
        const bool split = KH == 2 && (htiles & 7) == 0;
        const int per = split ? htiles >> 1 : htiles;
        float u = 0.f;
        if (kh == 0 || split)
            u = (kPadded && mlp_in_lds) ? mlp_mfma_16_padded(F, img, f.H, lane, split ? kh * per : 0, per)
                                        : mlp_mfma_16<false>(F, f, lane, split ? kh * per : 0, per);
        if (KH == 2 && split) {
            if (kh == 1 && q == 0) ssq_lds[n] = u;
            __syncthreads();
            if (kh == 0) u += ssq_lds[n];
        }
        if (KC <= 4 && kh == 0 && q < K && n < N) {
            f.logits[gn * K + q] = zq;
            f.probs[gn * K + q] = pq;
        }
        if (q == 0 && kh == 0 && n < N) {
            const float b2 = f.b2 ? (float)b2_r : 0.f;
            float sc = sigmoidf(b2 + u);
            if (poisoned) sc = quiet_nan();
            const int ex = (sc > f.threshold) ? 1 : 0;
            f.scores[gn] = sc;
            f.exit_flags[gn] = ex;
            exit_lds[n] = ex;
            if (KC > 4) {
#pragma unroll
                for (int k = 0; k < KC; ++k)
                    if (k < K) {
                        f.logits[gn * K + k] = z[k];
                        f.probs[gn * K + k] = pr[k];
                    }
            }
        }
    } else {
        FinishRows<KC> fr;
        finish_load_rows<KC>(fr, f, lane);
        for (int n = wave; n < N; n += kTcWaves) {
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
                float v = __shfl(a, k < K ? k : 0, kWave);
                z[k] = (k < K) ? (bad ? quiet_nan() : v * r) : 0.f;
                prev[k] = (k < K) ? prev_lds[n * K + k] : 0.f;
            }
            const int ex = finish_score_node<KC>(fr, f, gn, z, prev, lane);
            if (lane == kWave - 1) exit_lds[n] = ex;
        }
    }
    if (f.path_exit) {
        __syncthreads();
        finish_paths(exit_lds, par_lds, N, tid, kTcThreads, f.path_exit + (size_t)g * N);
    }
}

// 256 elements of every row in flight per wavefront: four 64-element stages, or two of 128

bool tree_gemm_can_fuse_merge(int n_ids) {
    return n_ids <= kTcFusedMax;
}

// d-slice partial sums: grid (d-slices, row groups of 64, trees x node blocks)
hipError_t launch_tree_gemm(const GemmParams &p, int G, hipStream_t st) {
    dim3 grid(p.S, (p.Mcap + 63) / 64, G * ((p.N + 63) / 64));
    if (p.ids)
        hipLaunchKernelGGL((tree_contract_kernel<4, 0, true, 2, 4, 128>), grid, dim3(256), 0, st, p,
                           TreeFinishParams{});
    else
        hipLaunchKernelGGL((tree_contract_kernel<4, 0, false, 2, 4, 128>), grid, dim3(256), 0, st, p,
                           TreeFinishParams{});
    return hipGetLastError();
}

// Row tiles of 16 merged rows that a whole-tree workgroup holds: 4, 8 or 16.
int tree_whole_row_tiles(int Mcap) {
    return Mcap <= 64 ? 4 : (Mcap <= 128 ? 8 : 16);
}

// Whole tree per workgroup: one launch does merge, contraction, scoring and the path rule.
bool tree_whole_supported(int N, int K, int Mcap) {
    return N <= 64 && N * K <= kTcFusedMax && Mcap <= 256;
}

// Variants of the whole-tree kernel.  Up to 64 merged rows: 512 threads (two wavefronts share a
// node tile) when each CU gets at most one workgroup, 256 threads when there are more workgroups
// than CUs, because two of those fit on a CU and one's prologue and scoring overlap the other's
// streaming.  65..128 merged rows: 256 threads, eight row tiles.
template <int MT, int KC, bool GL>
static void launch_whole(const GemmParams &p, const TreeFinishParams &f, int G, hipStream_t st) {
    const dim3 grid(p.S, 1, G);
    if constexpr (MT == 4) {
        if ((long long)G * p.S <= kWholeWideMaxWgs)
            hipLaunchKernelGGL((tree_contract_kernel<4, 3, true, 2, KC, 128, 512, GL>), grid, dim3(512), 0, st, p, f);
        else
            hipLaunchKernelGGL((tree_contract_kernel<4, 3, true, 4, KC, 64, 256, GL>), grid, dim3(256), 0, st, p, f);
    } else if constexpr (MT == 8) {
        hipLaunchKernelGGL((tree_contract_kernel<8, 3, true, 4, KC, 64, 256, GL>), grid, dim3(256), 0, st, p, f);
    } else {
        // 129..256 merged rows: sixteen row tiles in stages of 128 elements.  The two tile buffers (136 KB)
        // are dynamic LDS, so one workgroup per CU; the staged RMSNorm weight does not fit beside them.
        constexpr int kLds = 2 * 16 * MT * (kWide16Kch + 8) * (int)sizeof(half_t);
        auto kern = tree_contract_kernel<MT, 3, true, kWide16Pd, KC, kWide16Kch, kWide16Threads, GL && kWide16Kch == 64>;
        // the limit is a property of the loaded kernel, set again at every launch: the library keeps no state
        // (on failure the launch below fails too, and the caller sees that error)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
        hipLaunchKernelGGL(kern, grid, dim3(kWide16Threads), kLds, st, p, f);
    }
}

template <int MT, int KC>
static void launch_whole_gl(const GemmParams &p, const TreeFinishParams &f, int G, hipStream_t st) {
    if (p.dslice <= kGammaLds) launch_whole<MT, KC, true>(p, f, G, st);
    else launch_whole<MT, KC, false>(p, f, G, st);
}

hipError_t launch_tree_whole(const GemmParams &p, const TreeFinishParams &f, int G, hipStream_t st) {
    const int mt = tree_whole_row_tiles(p.Mcap);
    if (f.K <= 4) {
        if (mt == 16) launch_whole_gl<16, 4>(p, f, G, st);
        else if (mt == 8) launch_whole_gl<8, 4>(p, f, G, st);
        else launch_whole_gl<4, 4>(p, f, G, st);
    } else if (f.K <= 8) {
        if (mt == 16) launch_whole_gl<16, 8>(p, f, G, st);
        else if (mt == 8) launch_whole_gl<8, 8>(p, f, G, st);
        else launch_whole_gl<4, 8>(p, f, G, st);
    } else {
        if (mt == 16) launch_whole_gl<16, 16>(p, f, G, st);
        else if (mt == 8) launch_whole_gl<8, 16>(p, f, G, st);
        else launch_whole_gl<4, 16>(p, f, G, st);
    }
    return hipGetLastError();
}

}  // namespace specee
