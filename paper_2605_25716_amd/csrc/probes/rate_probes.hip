// Reference rates of the device the bench runs on, measured beside the library's kernels: what a plain streaming
// copy, a plain streaming read and a bare MFMA issue loop reach.  They are not part of the hot path and live in a
// library of their own (libfedrag_probes.so); bench.py reports them as "achievable" next to the published peaks.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kCopyThreads = 256;
constexpr int kCopyBlocks = 256;  // one workgroup per compute unit: more workgroups in flight measured slower (a
                                  // 1 GiB copy: 6.1 TB/s with 256 workgroups, 4.2-5.6 TB/s with 512 to 8192)

// dst[i] = src[i] over n 16-byte words, grid-stride, every load and store a full 1 KiB wave access, non-temporal
__global__ __launch_bounds__(kCopyThreads) void copy_kernel(u32x4_t* __restrict__ dst, const u32x4_t* __restrict__ src,
                                                            size_t n) {
    const size_t stride = (size_t)gridDim.x * kCopyThreads;
    size_t i = (size_t)blockIdx.x * kCopyThreads + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {  // four loads in flight per lane before the first store
        const u32x4_t a = __builtin_nontemporal_load(src + i);
        const u32x4_t b = __builtin_nontemporal_load(src + i + stride);
        const u32x4_t c = __builtin_nontemporal_load(src + i + 2 * stride);
        const u32x4_t d = __builtin_nontemporal_load(src + i + 3 * stride);
        __builtin_nontemporal_store(a, dst + i);
        __builtin_nontemporal_store(b, dst + i + stride);
        __builtin_nontemporal_store(c, dst + i + 2 * stride);
        __builtin_nontemporal_store(d, dst + i + 3 * stride);
    }
    for (; i < n; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// reads n 16-byte words; the xor of everything goes to sink only if it has an (impossible to predict) value, so the
// loads cannot be dropped and nothing is written in practice
__global__ __launch_bounds__(kCopyThreads) void read_kernel(const u32x4_t* __restrict__ src, size_t n,
                                                            uint32_t* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * kCopyThreads;
    u32x4_t acc = {0u, 0u, 0u, 0u};
    size_t i = (size_t)blockIdx.x * kCopyThreads + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const u32x4_t a = __builtin_nontemporal_load(src + i);
        const u32x4_t b = __builtin_nontemporal_load(src + i + stride);
        const u32x4_t c = __builtin_nontemporal_load(src + i + 2 * stride);
        const u32x4_t d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u) sink[0] = acc[0];
}

constexpr int kMfmaThreads = 512;  // two waves per SIMD
constexpr int kMfmaBlocks = 256;   // one workgroup per compute unit
constexpr int kMfmaAcc = 8;        // independent accumulators per wave

__device__ inline uint32_t mix32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// roughly normal value in (-2, 2) from 32 hashed bits: the centred sum of its four bytes
__device__ inline float bell(uint32_t h) {
    return ((float)(h & 255u) + (float)((h >> 8) & 255u) + (float)((h >> 16) & 255u) + (float)(h >> 24) - 510.f) * (1.f / 128.f);
}

// iters x kMfmaAcc dense bf16 32x32x16 MFMAs per wave on register operands: the matrix pipe's issue rate with nothing
// else going on.  RANDOM = false: every MFMA multiplies the same two smooth operands (few bits toggle from one
// instruction to the next).  RANDOM = true: every accumulator has operands of its own, filled with hashed
// bell-shaped values as activations are; the chip then runs at a lower clock under its power limit, and this is
// the rate a kernel working on real data can be compared with.
template <bool RANDOM>
__global__ __launch_bounds__(kMfmaThreads) void mfma_kernel(float* __restrict__ sink, int iters) {
    bf16x8_t a[kMfmaAcc], b[kMfmaAcc];
    for (int k = 0; k < kMfmaAcc; ++k)
        for (int j = 0; j < 8; ++j) {
            if (RANDOM) {
                const uint32_t h = mix32(threadIdx.x * 977u + blockIdx.x * 131u + k * 17u + j);
                a[k][j] = (__bf16)bell(h);
                b[k][j] = (__bf16)bell(mix32(h + 0x9e3779b9u));
            } else {
                a[k][j] = (__bf16)(0.001f * (float)(threadIdx.x % 64 + j));
                b[k][j] = (__bf16)(0.002f * (float)(j + 1));
            }
        }
    f32x16_t c[kMfmaAcc];
    for (int k = 0; k < kMfmaAcc; ++k)
        for (int j = 0; j < 16; ++j) c[k][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < kMfmaAcc; ++k) c[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[k], b[k], c[k], 0, 0, 0);
    }
    float s = 0.f;
    for (int k = 0; k < kMfmaAcc; ++k)
        for (int j = 0; j < 16; ++j) s += c[k][j];
    if (s == 12345.678f) sink[0] = s;
}

}  // namespace

extern "C" {

// Device-to-device copy of `bytes` bytes (a multiple of 16; both pointers 16-byte aligned) on `stream`.
// Returns 0, or a non-zero value for bad arguments or a failed launch.
int fedrag_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src || bytes == 0 || (bytes & 15u) || ((uintptr_t)dst & 15u) || ((uintptr_t)src & 15u)) return 1;
    hipLaunchKernelGGL(copy_kernel, dim3(kCopyBlocks), dim3(kCopyThreads), 0, (hipStream_t)stream, (u32x4_t*)dst,
                       (const u32x4_t*)src, bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// Streaming read of `bytes` bytes (a multiple of 16); sink: one device uint32 (left untouched in practice).
int fedrag_probe_read(const void* src, size_t bytes, uint32_t* sink, void* stream) {
    if (!src || !sink || bytes == 0 || (bytes & 15u) || ((uintptr_t)src & 15u)) return 1;
    hipLaunchKernelGGL(read_kernel, dim3(kCopyBlocks), dim3(kCopyThreads), 0, (hipStream_t)stream, (const u32x4_t*)src,
                       bytes / 16, sink);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// Floating-point operations of one fedrag_probe_mfma_bf16 launch with this `iters`.
double fedrag_probe_mfma_bf16_flop(int iters) {
    return (double)kMfmaBlocks * (kMfmaThreads / 64) * (double)iters * kMfmaAcc * (2.0 * 32 * 32 * 16);
}

// The bare MFMA loop on two smooth operands; sink: one device float (left untouched in practice).
// 1 <= iters <= 1 << 20.
int fedrag_probe_mfma_bf16(float* sink, int iters, void* stream) {
    if (!sink || iters < 1 || iters > (1 << 20)) return 1;
    hipLaunchKernelGGL(mfma_kernel<false>, dim3(kMfmaBlocks), dim3(kMfmaThreads), 0, (hipStream_t)stream, sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

// The same loop with hashed, bell-shaped operand values, different for every accumulator (same flop count).
int fedrag_probe_mfma_bf16_random(float* sink, int iters, void* stream) {
    if (!sink || iters < 1 || iters > (1 << 20)) return 1;
    hipLaunchKernelGGL(mfma_kernel<true>, dim3(kMfmaBlocks), dim3(kMfmaThreads), 0, (hipStream_t)stream, sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

}  // extern "C"
