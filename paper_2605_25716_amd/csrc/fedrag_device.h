// Device-side helpers shared by the gfx950 kernels: storage-type traits, MFMA wrappers, wave helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fedrag {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// 16-bit storage types.  vec8 is the 16-byte MFMA operand (8 contraction elements per lane).
struct BF16 {
    typedef __bf16 elem;
    typedef bf16x8_t vec8;
    typedef bf16x4_t vec4;
    // D(16x16) += A(16x32) . B(32x16); lane l: A row l%16, B column l%16, contraction elements (l/16)*8..+8;
    // D column l%16, rows (l/16)*4..+4.
    static __device__ __forceinline__ f32x4_t mfma16(vec8 a, vec8 b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    // D(32x32) += A(32x16) . B(16x32); lane l: A row l%32, B column l%32, contraction elements (l/32)*8..+8;
    // D column l%32, rows 8*(r/4) + 4*(l/32) + r%4 for r in 0..15.
    static __device__ __forceinline__ f32x16_t mfma32(vec8 a, vec8 b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ elem from_float(float x) { return static_cast<__bf16>(x); }
    static __device__ __forceinline__ float to_float(elem x) { return static_cast<float>(x); }
};

struct F16 {
    typedef _Float16 elem;
    typedef f16x8_t vec8;
    typedef f16x4_t vec4;
    static __device__ __forceinline__ f32x4_t mfma16(vec8 a, vec8 b, f32x4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ f32x16_t mfma32(vec8 a, vec8 b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ elem from_float(float x) { return static_cast<_Float16>(x); }
    static __device__ __forceinline__ float to_float(elem x) { return static_cast<float>(x); }
};

template <class V>
__device__ __forceinline__ V zero_vec() {
    V v;
#pragma unroll
    for (int i = 0; i < (int)(sizeof(V) / sizeof(v[0])); ++i) v[i] = 0;
    return v;
}

// Lanes of one wave exchange data through LDS: order this wave's LDS writes before its later LDS reads.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Max / sum over the lane pair (l, l ^ 32).
__device__ __forceinline__ float xor32_max(float x) { return fmaxf(x, __shfl_xor(x, 32)); }
__device__ __forceinline__ float xor32_sum(float x) { return x + __shfl_xor(x, 32); }

// min / max over aligned groups of N = 8 or 16 consecutive lanes, result in every lane of the group, with data-parallel
// primitives only (no LDS crossbar): exchange inside quads, then mirror the half row (lane k <-> 7 - k: the other
// quad, whose lanes already agree), then mirror the row of 16.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
template <int N, class Op>
__device__ __forceinline__ float group_reduce(float x, Op op) {
    static_assert(N == 8 || N == 16, "groups of 8 or 16 lanes");
    x = op(x, dpp_move<0xB1>(x));   // quad_perm [1,0,3,2]
    x = op(x, dpp_move<0x4E>(x));   // quad_perm [2,3,0,1]
    x = op(x, dpp_move<0x141>(x));  // row_half_mirror
    if (N == 16) x = op(x, dpp_move<0x140>(x));  // row_mirror
    return x;
}
template <int N>
__device__ __forceinline__ float group_min(float x) {
    return group_reduce<N>(x, [](float a, float b) { return fminf(a, b); });
}
template <int N>
__device__ __forceinline__ float group_max(float x) {
    return group_reduce<N>(x, [](float a, float b) { return fmaxf(a, b); });
}

// Keep a value's computation above this point: the compiler may otherwise sink pure register arithmetic towards
// its first use (past a barrier, into the next loop iteration), out of the scheduling region it was written for.
template <class V>
__device__ __forceinline__ void pin_here(V& v) {
    asm volatile("" : "+v"(v));
}

// exp2(a - b) with the convention that a == -inf gives 0 even when b == -inf.
__device__ __forceinline__ float exp2_diff(float a, float b) {
    return (a == -INFINITY) ? 0.0f : fast_exp2(a - b);
}

// 8x8 transpose of 16-bit elements held as 8 registers-of-8 (in[r][c] -> out[c][r]).
// Each 32-bit word holds two adjacent columns; v_perm_b32 picks halves of two words.
__device__ __forceinline__ void transpose8x8_b16(const u32x4_t in[8], u32x4_t out[8]) {
#pragma unroll
    for (int c2 = 0; c2 < 4; ++c2) {          // word index along the input row = column pair (2*c2, 2*c2+1)
#pragma unroll
        for (int r2 = 0; r2 < 4; ++r2) {      // input row pair (2*r2, 2*r2+1)
            const uint32_t a = in[2 * r2][c2];      // row 2r2   : cols 2c2 (lo), 2c2+1 (hi)
            const uint32_t b = in[2 * r2 + 1][c2];  // row 2r2+1 : same columns
            // out row (=in col) 2c2   : word r2 = { in[2r2][2c2]   (lo), in[2r2+1][2c2]   (hi) }
            // out row          2c2+1 : word r2 = { in[2r2][2c2+1] (lo), in[2r2+1][2c2+1] (hi) }
            out[2 * c2][r2] = __builtin_amdgcn_perm(b, a, 0x05040100u);
            out[2 * c2 + 1][r2] = __builtin_amdgcn_perm(b, a, 0x07060302u);
        }
    }
}

}  // namespace fedrag
