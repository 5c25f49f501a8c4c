// Transport codec (Section 7.5: affine min-max quantisation of the states that travel between nodes), per token row
// of D channels, to 8 or 4 bits:
//   lo = min x, hi = max x, levels = 2^bits - 1, scale = (hi - lo) / levels, steps = levels / (hi - lo),
//   code = clamp(floor(fma(x - lo, steps, 1/2)), 0, levels)   (0 for a constant row),   value = fma(code, scale, lo).
// Every operation is a single-precision IEEE operation (the codes are integers decided by floating point, so the
// precision is part of the definition).  params[row] = (scale, lo); 4-bit codes are packed two per byte, channel 2k
// in the low half.  HBM-bound streaming kernels: a row is held by D/8 lanes with 8 channels each (one 16-byte load
// for 16-bit storage), the row's range is reduced across those lanes with data-parallel lane moves, codes leave as 8 (or 4)
// contiguous bytes per lane.
#include "fedrag_device.h"
#include "fedrag_host.h"

namespace fedrag {

constexpr int kCodecThreads = 256;
constexpr int kCodecUnroll = 4;  // row groups in flight per wave

template <class T>
struct CodecIO;  // 8 channels of a row: load as fp32, store from fp32 (RNE)

template <>
struct CodecIO<float> {
    static __device__ __forceinline__ void load(const void* p, float (&x)[8]) {
        const f32x4_t a = __builtin_nontemporal_load((const f32x4_t*)p);
        const f32x4_t b = __builtin_nontemporal_load((const f32x4_t*)p + 1);
        for (int e = 0; e < 4; ++e) { x[e] = a[e]; x[4 + e] = b[e]; }
    }
    static __device__ __forceinline__ void store(void* p, const float (&x)[8]) {
        f32x4_t a, b;
        for (int e = 0; e < 4; ++e) { a[e] = x[e]; b[e] = x[4 + e]; }
        __builtin_nontemporal_store(a, (f32x4_t*)p);
        __builtin_nontemporal_store(b, (f32x4_t*)p + 1);
    }
    static constexpr int kBytes = 32;
};

template <class S>
struct CodecIO16 {
    typedef typename S::vec8 vec8;
    static __device__ __forceinline__ void load(const void* p, float (&x)[8]) {
        const vec8 v = __builtin_nontemporal_load((const vec8*)p);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = S::to_float(v[e]);
    }
    static __device__ __forceinline__ void store(void* p, const float (&x)[8]) {
        vec8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = S::from_float(x[e]);
        __builtin_nontemporal_store(v, (vec8*)p);
    }
    static constexpr int kBytes = 16;
};
template <> struct CodecIO<BF16> : CodecIO16<BF16> {};
template <> struct CodecIO<F16> : CodecIO16<F16> {};

template <class T, int D, int BITS>
__global__ __launch_bounds__(kCodecThreads) void quantize_rows_kernel(const char* __restrict__ X, int64_t n_rows,
                                                                      uint8_t* __restrict__ codes,
                                                                      float* __restrict__ params) {
    typedef CodecIO<T> IO;
    constexpr int LPR = D / 8;           // lanes per row
    constexpr int RPW = kWave / LPR;     // rows per wave-wide load
    constexpr int LEVELS = (1 << BITS) - 1;
    constexpr int CODE_ROWB = D * BITS / 8;
    const int lane = threadIdx.x % kWave;
    const int64_t wave = ((int64_t)blockIdx.x * kCodecThreads + threadIdx.x) / kWave;
    const int64_t n_waves = (int64_t)gridDim.x * (kCodecThreads / kWave);
    const int64_t n_groups = (n_rows + RPW - 1) / RPW;
    const int r_in = lane / LPR, c_in = lane % LPR;

    for (int64_t g0 = wave * kCodecUnroll; g0 < n_groups; g0 += n_waves * kCodecUnroll) {
        float x[kCodecUnroll][8];
        int64_t row[kCodecUnroll];
#pragma unroll
        for (int u = 0; u < kCodecUnroll; ++u) {
            row[u] = (g0 + u) * RPW + r_in;
            const int64_t r = row[u] < n_rows ? row[u] : n_rows - 1;  // clamped rows are computed, not stored
            IO::load(X + (r * LPR + c_in) * IO::kBytes, x[u]);
        }
#pragma unroll
        for (int u = 0; u < kCodecUnroll; ++u) {
            float lo = x[u][0], hi = x[u][0];
#pragma unroll
            for (int e = 1; e < 8; ++e) { lo = fminf(lo, x[u][e]); hi = fmaxf(hi, x[u][e]); }
            lo = group_min<LPR>(lo);
            hi = group_max<LPR>(hi);
            const float range = hi - lo;
            const float scale = range / (float)LEVELS;
            // x - lo >= 0, so the sum is >= 1/2: converting to unsigned truncates = floors, and only the upper clamp
            // can act; a constant row (range 0) gets steps 0, hence code 0
            const float steps = range > 0.0f ? (float)LEVELS / range : 0.0f;
            uint32_t q[8];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                q[e] = (uint32_t)fminf(__builtin_fmaf(x[u][e] - lo, steps, 0.5f), (float)LEVELS);
            if (row[u] < n_rows) {
                uint8_t* out = codes + row[u] * CODE_ROWB;
                if (BITS == 8) {
                    u32x2_t w;
                    w[0] = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
                    w[1] = q[4] | (q[5] << 8) | (q[6] << 16) | (q[7] << 24);
                    __builtin_nontemporal_store(w, (u32x2_t*)(out + c_in * 8));
                } else {
                    const uint32_t w = q[0] | (q[1] << 4) | (q[2] << 8) | (q[3] << 12) | (q[4] << 16) | (q[5] << 20) |
                                       (q[6] << 24) | (q[7] << 28);
                    __builtin_nontemporal_store(w, (uint32_t*)(out + c_in * 4));
                }
                if (c_in == 0) {
                    params[2 * row[u]] = scale;
                    params[2 * row[u] + 1] = lo;
                }
            }
        }
    }
}

template <class T, int D, int BITS>
__global__ __launch_bounds__(kCodecThreads) void dequantize_rows_kernel(const uint8_t* __restrict__ codes,
                                                                        const float* __restrict__ params,
                                                                        int64_t n_rows, char* __restrict__ X) {
    typedef CodecIO<T> IO;
    constexpr int LPR = D / 8;
    constexpr int RPW = kWave / LPR;
    constexpr int CODE_ROWB = D * BITS / 8;
    const int lane = threadIdx.x % kWave;
    const int64_t wave = ((int64_t)blockIdx.x * kCodecThreads + threadIdx.x) / kWave;
    const int64_t n_waves = (int64_t)gridDim.x * (kCodecThreads / kWave);
    const int64_t n_groups = (n_rows + RPW - 1) / RPW;
    const int r_in = lane / LPR, c_in = lane % LPR;

    for (int64_t g0 = wave * kCodecUnroll; g0 < n_groups; g0 += n_waves * kCodecUnroll) {
        uint32_t w[kCodecUnroll][2];
        float scale[kCodecUnroll], lo[kCodecUnroll];
        int64_t row[kCodecUnroll];
#pragma unroll
        for (int u = 0; u < kCodecUnroll; ++u) {
            row[u] = (g0 + u) * RPW + r_in;
            const int64_t r = row[u] < n_rows ? row[u] : n_rows - 1;
            const uint8_t* in = codes + r * CODE_ROWB;
            if (BITS == 8) {
                const u32x2_t v = __builtin_nontemporal_load((const u32x2_t*)(in + c_in * 8));
                w[u][0] = v[0]; w[u][1] = v[1];
            } else {
                w[u][0] = __builtin_nontemporal_load((const uint32_t*)(in + c_in * 4));
                w[u][1] = 0;
            }
            scale[u] = params[2 * r];
            lo[u] = params[2 * r + 1];
        }
#pragma unroll
        for (int u = 0; u < kCodecUnroll; ++u) {
            float x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t q = BITS == 8 ? (w[u][e / 4] >> (8 * (e % 4))) & 255u : (w[u][0] >> (4 * e)) & 15u;
                x[e] = __builtin_fmaf((float)q, scale[u], lo[u]);
                pin_here(x[e]);  // the value is defined as the fp32 result, narrowed afterwards: keep the compiler
                                 // from folding the two into one mixed-precision operation with a single rounding
            }
            if (row[u] < n_rows) IO::store(X + (row[u] * LPR + c_in) * IO::kBytes, x);
        }
    }
}

static unsigned codec_grid(int64_t n_rows, int rows_per_wave) {
    const int64_t groups = (n_rows + rows_per_wave - 1) / rows_per_wave;
    const int64_t waves = (groups + kCodecUnroll - 1) / kCodecUnroll;
    int64_t wgs = (waves + kCodecThreads / kWave - 1) / (kCodecThreads / kWave);
    if (wgs > 2048) wgs = 2048;  // grid-stride beyond: 8 workgroups per CU
    return (unsigned)(wgs < 1 ? 1 : wgs);
}

template <class T, int D>
static hipError_t launch_codec_t(const CodecJob& j, hipStream_t stream) {
    const dim3 grid(codec_grid(j.n_rows, kWave / (D / 8))), block(kCodecThreads);
    if (j.quantize) {
        if (j.bits == 8)
            hipLaunchKernelGGL((quantize_rows_kernel<T, D, 8>), grid, block, 0, stream, (const char*)j.X, j.n_rows,
                               j.codes, j.params);
        else
            hipLaunchKernelGGL((quantize_rows_kernel<T, D, 4>), grid, block, 0, stream, (const char*)j.X, j.n_rows,
                               j.codes, j.params);
    } else {
        if (j.bits == 8)
            hipLaunchKernelGGL((dequantize_rows_kernel<T, D, 8>), grid, block, 0, stream, j.codes, j.params, j.n_rows,
                               (char*)j.X);
        else
            hipLaunchKernelGGL((dequantize_rows_kernel<T, D, 4>), grid, block, 0, stream, j.codes, j.params, j.n_rows,
                               (char*)j.X);
    }
    return hipGetLastError();
}

hipError_t launch_codec(const CodecJob& j, hipStream_t stream) {
    if (j.n_rows == 0) return hipSuccess;
    switch (j.dtype) {
        case FEDRAG_F32: return j.D == 128 ? launch_codec_t<float, 128>(j, stream) : launch_codec_t<float, 64>(j, stream);
        case FEDRAG_BF16: return j.D == 128 ? launch_codec_t<BF16, 128>(j, stream) : launch_codec_t<BF16, 64>(j, stream);
        case FEDRAG_F16: return j.D == 128 ? launch_codec_t<F16, 128>(j, stream) : launch_codec_t<F16, 64>(j, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace fedrag
