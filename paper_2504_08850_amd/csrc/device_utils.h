// Device-side helpers shared by the gfx950 kernels: 16-byte fp16 vectors,
// wavefront (64-lane) reductions built from DPP lane permutes, and fixed-order
// block reductions through LDS.  Nothing here depends on launch shape beyond
// "blockDim.x is a multiple of 64".
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specee {

typedef _Float16 half_t;
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// DPP control words (CDNA ISA): quad_perm packs four 2-bit selectors.
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // reverse within 8 lanes
constexpr int kDppMirror = 0x140;     // reverse within 16 lanes

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    int i = __builtin_bit_cast(int, v);
    i = __builtin_amdgcn_update_dpp(0, i, CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(float, i);
}

// Sum over the 64 lanes of a wavefront; every lane returns the total.  The
// first four steps stay inside a 16-lane DPP row (no LDS traffic); the last two
// cross rows through the LDS crossbar.  The combination order is fixed, so the
// result is reproducible.
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f32<kDppXor1>(v);
    v += dpp_f32<kDppXor2>(v);
    v += dpp_f32<kDppHalfMirror>(v);
    v += dpp_f32<kDppMirror>(v);
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
    return v;
}

// Sum over the 64 lanes with DPP only (no LDS crossbar): after the four in-row steps every lane
// of a 16-lane row holds its row's sum; row_bcast15 adds row 0 into row 1 and row 2 into row 3,
// row_bcast31 adds rows 0+1 into rows 2 and 3.  The total is valid in lanes 48..63 ONLY.
constexpr int kDppRowBcast15 = 0x142;
constexpr int kDppRowBcast31 = 0x143;
__device__ __forceinline__ float wave_sum_to_last_row(float v) {
    v += dpp_f32<kDppXor1>(v);
    v += dpp_f32<kDppXor2>(v);
    v += dpp_f32<kDppHalfMirror>(v);
    v += dpp_f32<kDppMirror>(v);
    int i = __builtin_bit_cast(int, v);
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, i, kDppRowBcast15, 0xA, 0xF, false));
    i = __builtin_bit_cast(int, v);
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, i, kDppRowBcast31, 0xC, 0xF, false));
    return v;
}

template <int CTRL>
__device__ __forceinline__ void dpp_argmax_step(float &v, int &i) {
    float ov = dpp_f32<CTRL>(v);
    int oi = __builtin_amdgcn_update_dpp(0, i, CTRL, 0xF, 0xF, true);
    if (ov > v || (ov == v && oi < i)) {
        v = ov;
        i = oi;
    }
}

// Arg-max over a wavefront, lowest index on ties; every lane returns the winner.
__device__ __forceinline__ void wave_argmax(float &v, int &i) {
    dpp_argmax_step<kDppXor1>(v, i);
    dpp_argmax_step<kDppXor2>(v, i);
    dpp_argmax_step<kDppHalfMirror>(v, i);
    dpp_argmax_step<kDppMirror>(v, i);
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        float ov = __shfl_xor(v, off, kWave);
        int oi = __shfl_xor(i, off, kWave);
        if (ov > v || (ov == v && oi < i)) {
            v = ov;
            i = oi;
        }
    }
}

__device__ __forceinline__ half8 load_half8(const half_t *p) {
    return *reinterpret_cast<const half8 *>(p);
}

// Streaming variant for data that is read once (LM-head rows of a full pass): the non-temporal hint keeps
// the stream from displacing what the caches hold and measures ~17 % more bandwidth on plain streams.
__device__ __forceinline__ half8 load_half8_stream(const half_t *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const half8 *>(p));
}

__device__ __forceinline__ half8 zero_half8() {
    half8 z;
#pragma unroll
    for (int e = 0; e < 8; ++e) z[e] = (half_t)0.0f;
    return z;
}

// s_waitcnt operand (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8) that waits
// for every outstanding vector-memory operation of the wavefront, stores included, and for nothing else.
constexpr int kWaitVmcnt0 = 0x0F70;

__device__ __forceinline__ float quiet_nan() {
    return __builtin_bit_cast(float, 0x7fc00000);
}

}  // namespace specee
