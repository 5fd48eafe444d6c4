// Workgroup-level merge of a token tree's speculative ids (paper Sec. 6.2, the
// merged mapping): sorted distinct ids, their count, and the column of every
// (node, slot) in that set.  Pure integer work in LDS.
//
// The ids of a tree overlap heavily (that is the point of merging), so sorting
// all N*K of them is wasted work.  Instead:
//   1. de-duplicate through an open-addressing hash table in LDS (one LDS
//      compare-and-swap per element; the table stores element indices so every
//      int32 value is a legal key);
//   2. compact the M representatives with a ballot/popcount scan;
//   3. rank each distinct key among the M distinct keys by counting
//      (M^2 / threads comparisons, keys read four at a time as LDS broadcasts);
//   4. every element looks up the rank of its representative.
// Which duplicate wins the table slot is timing dependent, but every output is
// a function of the key values only, so results are deterministic.
#pragma once
#include "device_utils.h"

namespace specee {

constexpr int kMergePerThread = 4;  // elements a thread may own: n <= 4 * blockDim.x

// LDS the caller provides, in ints (n4 = n rounded up to a multiple of 4).
__host__ __device__ constexpr int merge_lds_ints(int n) {
    return 3 * ((n + 3) & ~3) + 72;
}

// All threads of the workgroup must call.  On return (after the final barrier
// inside) uniq[0..M) holds the sorted distinct ids and `col_of[e]` (for the
// e-th element owned by this thread: i = tid + e * blockDim.x) its column.
// Returns M.  `lds` is clobbered; uniq points into it.
// T = blockDim.x (compile time, so the short serial loops over per-wave totals unroll into
// independent LDS reads).
// own_ids[e] returns the thread's own ids (INT_MAX for slots beyond n) to callers that go on to
// validate them, which saves reading them a second time.
// This thread's ids of a tree, element i = tid + e * T: the merges below take them in registers, so that a
// caller can request them before anything else it loads.  Clamped address, no branch, nothing consumed:
// slots beyond n hold a copy of the last id and are masked (INT_MAX) by the merges.
template <int T>
__device__ __forceinline__ void merge_load_ids(const int32_t *ids, int n, int (&kreg)[kMergePerThread]) {
    const int E = (((n + 3) & ~3) + T - 1) / T;
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        kreg[e] = 0x7fffffff;
        if (e < E) {  // uniform over the workgroup
            const int i = threadIdx.x + e * T;
            kreg[e] = ids[min(i, n - 1)];  // raw: masking it here would make the caller wait for it
        }
    }
}

template <int T>
__device__ inline int merge_block(const int (&kin)[kMergePerThread], int n, int32_t *lds, int32_t *&uniq,
                                  int (&col_of)[kMergePerThread], int (&own_ids)[kMergePerThread]) {
    const int tid = threadIdx.x;
    constexpr int nwaves = T >> 6;
    constexpr int kTotals = kMergePerThread * nwaves;
    const int lane = tid & 63, wave = tid >> 6;
    const int n4 = (n + 3) & ~3;
    const unsigned TS = 2u * (unsigned)n4;  // table slots: load factor <= 1/2
    int32_t *key = lds;                     // [n4]  keys by element; later distinct keys, later their ranks
    int32_t *table = lds + n4;              // [2*n4] hash table of element indices
    int32_t *cidx = table;                  // [n4]  (after the table is dead) compact index of a representative
    int32_t *wtot = lds + 3 * n4;           // [<= 64] ballot totals
    uniq = table + n4;                      // [n4]  (after the table is dead) sorted distinct keys

    // element slots in use: a tree of at most T ids needs one per thread, and every loop below skips
    // the unused slots with a workgroup-uniform test (this code sits on the latency path of a tree call)
    const int E = (n4 + T - 1) / T;
    int kreg[kMergePerThread], rep[kMergePerThread];
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        const int i = tid + e * T;
        kreg[e] = (e < E && i < n) ? kin[e] : 0x7fffffff;
        if (e < E && i < n4) key[i] = kreg[e];
    }
    for (unsigned t = tid; t < TS; t += T) table[t] = -1;
    __syncthreads();

    // 1. insert: the first element to claim a slot represents its key
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        const int i = tid + e * T;
        rep[e] = -1;
        if (e < E && i < n) {
            const int k = kreg[e];
            unsigned h = (unsigned)(((unsigned long long)((unsigned)k * 2654435761u) * TS) >> 32);
            for (unsigned probe = 0; probe < TS; ++probe) {  // the table is larger than n: always ends early
                const int old = atomicCAS(&table[h], -1, i);
                if (old == -1) {
                    rep[e] = i;
                    break;
                }
                if (key[old] == k) {
                    rep[e] = old;
                    break;
                }
                h = h + 1 == TS ? 0 : h + 1;
            }
        }
    }
    __syncthreads();

    // 2. compact the representatives (order by element index)
    int incl[kMergePerThread];
    bool isrep[kMergePerThread];
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        const int i = tid + e * T;
        isrep[e] = i < n && rep[e] == i;
        incl[e] = 0;
        if (e < E) {
            const unsigned long long mask = __ballot(isrep[e]);
            incl[e] = __popcll(mask & (~0ull >> (63 - lane)));
            if (lane == 0) wtot[e * nwaves + wave] = __popcll(mask);
        } else if (lane == 0) {
            wtot[e * nwaves + wave] = 0;
        }
    }
    __syncthreads();
    int M = 0;
    int before[kMergePerThread];
    {
        int tot[kTotals];
#pragma unroll
        for (int w = 0; w < kTotals; w += 4) {
            const int4 t4 = *reinterpret_cast<const int4 *>(wtot + w);
            tot[w] = t4.x;
            tot[w + 1] = t4.y;
            tot[w + 2] = t4.z;
            tot[w + 3] = t4.w;
        }
#pragma unroll
        for (int e = 0; e < kMergePerThread; ++e) before[e] = 0;
#pragma unroll
        for (int w = 0; w < kTotals; ++w) {
#pragma unroll
            for (int e = 0; e < kMergePerThread; ++e)
                if (w < e * nwaves + wave) before[e] += tot[w];
            M += tot[w];
        }
    }
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        const int i = tid + e * T;
        if (isrep[e]) {
            const int ci = before[e] + incl[e] - 1;
            key[ci] = kreg[e];  // key[] is dead: every thread holds its keys in registers
            cidx[i] = ci;       // the table is dead after the barrier above
        }
    }
    const int M4 = (M + 3) & ~3;
    __syncthreads();
    for (int a = M + tid; a < M4; a += T) key[a] = 0x7fffffff;  // pad for the 4-wide reads
    __syncthreads();

    // 3. rank of every distinct key among the distinct keys
    int rnk[kMergePerThread], kd[kMergePerThread];
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        const int a = tid + e * T;
        rnk[e] = 0;
        kd[e] = 0;
        if (e < E && a < M) {
            const int k = key[a];
            int r0 = 0, r1 = 0, r2 = 0, r3 = 0;
#pragma unroll 4
            for (int b = 0; b < M4; b += 4) {
                const int4 kb = *reinterpret_cast<const int4 *>(key + b);
                r0 += kb.x < k;
                r1 += kb.y < k;
                r2 += kb.z < k;
                r3 += kb.w < k;
            }
            rnk[e] = (r0 + r1) + (r2 + r3);
            kd[e] = k;
        }
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        const int a = tid + e * T;
        if (a < M) {
            uniq[rnk[e]] = kd[e];
            key[a] = rnk[e];  // distinct keys are dead: reuse as rank by compact index
        }
    }
    __syncthreads();

    // 4. column of every element = rank of its representative's key
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        const int i = tid + e * T;
        col_of[e] = (i < n && rep[e] >= 0) ? key[cidx[rep[e]]] : 0;
        own_ids[e] = kreg[e];
    }
    __syncthreads();
    return M;
}

template <int T>
__device__ inline int merge_block(const int32_t *ids, int n, int32_t *lds, int32_t *&uniq,
                                  int (&col_of)[kMergePerThread]) {
    int kin[kMergePerThread], own_ids[kMergePerThread];
    merge_load_ids<T>(ids, n, kin);
    return merge_block<T>(kin, n, lds, uniq, col_of, own_ids);
}

// The same merge through a bitmap of the vocabulary, for trees whose ids all lie in [0, V) with a
// vocabulary that fits (V bits and one running count per 32-bit word in LDS): every id sets its bit
// (one LDS atomic, no probing), a prefix sum over the words' population counts ranks the words, and the
// column of an id is its word's prefix plus the set bits below it in the word.  Sorted order comes for
// free, there is no comparison loop, and four barriers do instead of eight -- this merge sits in the
// prologue of the one-launch tree kernel, where nothing else can run until the rows are known.
// A tree with an id outside [0, V) takes merge_block (any int32 is a legal key there); the choice is
// uniform over the workgroup.  Contract as merge_block: all threads call, kin from merge_load_ids, uniq /
// col_of / own_ids as there; lds needs merge_bitmap_ints(V, n) ints (and merge_lds_ints(n) for the fallback).
__host__ __device__ constexpr int merge_bitmap_words(int V) {
    return (V + 31) >> 5;
}
__host__ __device__ constexpr int merge_bitmap_ints(int V, int n) {
    return 2 * merge_bitmap_words(V) + ((n + 3) & ~3) + 16;
}
template <int T>
__device__ inline int merge_bitmap(const int (&kin)[kMergePerThread], int n, int V, int32_t *lds, int32_t *&uniq,
                                   int (&col_of)[kMergePerThread], int (&own_ids)[kMergePerThread]) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int nwaves = T >> 6;
    const int W = merge_bitmap_words(V);
    const int n4 = (n + 3) & ~3;
    uint32_t *bits = reinterpret_cast<uint32_t *>(lds);   // [W]
    int32_t *pre = lds + W;                                // [W] set bits in all lower words
    int32_t *out = lds + 2 * W;                            // [n4] sorted distinct ids
    int32_t *wtot = lds + 2 * W + n4;                      // [nwaves <= 16]
    const int E = (n4 + T - 1) / T;
    int kreg[kMergePerThread];
    bool bad = false;
    for (int w = tid; w < W; w += T) bits[w] = 0u;  // before the ids are looked at: they may still be on their way
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        const bool live = e < E && tid + e * T < n;
        kreg[e] = live ? kin[e] : 0x7fffffff;
        if (live) bad |= kreg[e] < 0 || kreg[e] >= V;
    }
    if (__syncthreads_or(bad)) return merge_block<T>(kin, n, lds, uniq, col_of, own_ids);  // uniform

    // 1. every id sets its bit
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e)
        if (e < E && tid + e * T < n) atomicOr(&bits[kreg[e] >> 5], 1u << (kreg[e] & 31));
    __syncthreads();

    // 2. thread t owns the words [t * wpt, (t + 1) * wpt): exclusive prefix of their population counts
    const int wpt = (W + T - 1) / T;
    const int w0 = tid * wpt;
    int cnt = 0;
    for (int j = 0; j < wpt; ++j)
        if (w0 + j < W) cnt += __popc(bits[w0 + j]);
    int incl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    if (lane == 63) wtot[wave] = incl;
    __syncthreads();
    int before = incl - cnt, M = 0;
#pragma unroll
    for (int q = 0; q < nwaves; ++q) {
        const int t = wtot[q];
        if (q < wave) before += t;
        M += t;
    }

    // 3. running count per word, and the sorted distinct ids: the set bits in order
    for (int j = 0; j < wpt; ++j) {
        const int w = w0 + j;
        if (w < W) {
            uint32_t x = bits[w];
            pre[w] = before;
            while (x) {
                const int b = __ffs((int)x) - 1;
                out[before++] = (w << 5) + b;
                x &= x - 1;
            }
        }
    }
    __syncthreads();

    // 4. column of an id: set bits in lower words plus set bits below it in its own word
#pragma unroll
    for (int e = 0; e < kMergePerThread; ++e) {
        col_of[e] = 0;
        if (e < E && tid + e * T < n) {
            const int k = kreg[e];
            col_of[e] = pre[k >> 5] + __popc(bits[k >> 5] & ((1u << (k & 31)) - 1u));
        }
        own_ids[e] = kreg[e];
    }
    uniq = out;
    return M;
}

}  // namespace specee
