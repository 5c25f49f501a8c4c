// Global aggregation of Section 4.1 in the log domain:
//   M = max_i lse_i, a_i = exp(lse_i - M), O = sum_i a_i O_i / sum_i a_i, lse = M + ln sum_i a_i
// which equals sum_i w_i (.) O_i / sum_i w_i with w_i = exp(lse_i).  Also used to fold the intra-shard KV
// splits of the decode kernel.  Pure streaming: one thread per (row, 4 output columns).
#include "fedrag_device.h"
#include "fedrag_host.h"

namespace fedrag {

template <int D>
__global__ __launch_bounds__(256) void lse_merge_kernel(const float* __restrict__ O_parts,
                                                        const float* __restrict__ lses, int S, int64_t rows,
                                                        float* __restrict__ O, float* __restrict__ lse,
                                                        const int32_t* __restrict__ q_lens, int64_t Lq,
                                                        int64_t rows_per_seq) {
    constexpr int TPR = D / 4;  // threads per row
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t r = gid / TPR;
    const int c4 = (int)(gid % TPR) * 4;
    if (r >= rows) return;
    // padded batch with per-sequence query counts: padding rows hold no partials and are not written
    if (q_lens && (r % Lq) >= q_lens[r / rows_per_seq]) return;
    float M = -INFINITY;
    for (int i = 0; i < S; ++i) M = fmaxf(M, lses[(int64_t)i * rows + r]);
    f32x4_t acc = zero_vec<f32x4_t>();
    float den = 0.f;
    if (M != -INFINITY) {
        for (int i = 0; i < S; ++i) {
            const float li = lses[(int64_t)i * rows + r];
            if (li == -INFINITY) continue;  // weight zero: its O is not read
            const float a = expf(li - M);
            den += a;
            const f32x4_t o = *(const f32x4_t*)(O_parts + ((int64_t)i * rows + r) * D + c4);
            acc[0] = __builtin_fmaf(a, o[0], acc[0]);
            acc[1] = __builtin_fmaf(a, o[1], acc[1]);
            acc[2] = __builtin_fmaf(a, o[2], acc[2]);
            acc[3] = __builtin_fmaf(a, o[3], acc[3]);
        }
        const float inv = 1.0f / den;
        acc[0] *= inv; acc[1] *= inv; acc[2] *= inv; acc[3] *= inv;
    }
    *(f32x4_t*)(O + r * D + c4) = acc;
    if (c4 == 0) lse[r] = (M == -INFINITY) ? -INFINITY : M + logf(den);
}

template <int D>
__global__ __launch_bounds__(256) void fill_empty_kernel(float* __restrict__ O, float* __restrict__ lse,
                                                         int64_t rows) {
    constexpr int TPR = D / 4;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t r = gid / TPR;
    const int c4 = (int)(gid % TPR) * 4;
    if (r >= rows) return;
    *(f32x4_t*)(O + r * D + c4) = zero_vec<f32x4_t>();
    if (c4 == 0) lse[r] = -INFINITY;
}

hipError_t launch_lse_merge(const float* O_parts, const float* lses, int S, int64_t rows, int D, float* O, float* lse,
                            hipStream_t stream, const int32_t* q_lens, int64_t Lq, int64_t rows_per_seq) {
    if (rows == 0) return hipSuccess;
    if (q_lens && (Lq < 1 || rows_per_seq < 1)) return hipErrorInvalidValue;
    const int64_t threads = rows * (D / 4);
    if (!grid_fits((threads + 255) / 256)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((threads + 255) / 256));
    if (D == 128)
        hipLaunchKernelGGL(lse_merge_kernel<128>, grid, dim3(256), 0, stream, O_parts, lses, S, rows, O, lse,
                           q_lens, Lq, rows_per_seq);
    else
        hipLaunchKernelGGL(lse_merge_kernel<64>, grid, dim3(256), 0, stream, O_parts, lses, S, rows, O, lse,
                           q_lens, Lq, rows_per_seq);
    return hipGetLastError();
}

hipError_t launch_fill_empty(float* O, float* lse, int64_t rows, int D, hipStream_t stream) {
    if (rows == 0) return hipSuccess;
    const int64_t threads = rows * (D / 4);
    if (!grid_fits((threads + 255) / 256)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((threads + 255) / 256));
    if (D == 128)
        hipLaunchKernelGGL(fill_empty_kernel<128>, grid, dim3(256), 0, stream, O, lse, rows);
    else
        hipLaunchKernelGGL(fill_empty_kernel<64>, grid, dim3(256), 0, stream, O, lse, rows);
    return hipGetLastError();
}

// out[bh, perm[i]] = in[bh, i]: the log-sum-exps of permuted query rows put back in the rows' own order (the
// token-permutation part of Dec, Section 4.2, for the per-row scalar that travels with the output).
__global__ void scatter_rows_f32_kernel(const float* __restrict__ in, const int32_t* __restrict__ perm, int64_t L,
                                        int64_t total, float* __restrict__ out) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    const int64_t bh = e / L, i = e % L;
    const int64_t dst = perm ? (int64_t)perm[i] : i;
    out[bh * L + dst] = in[e];
}

hipError_t launch_scatter_rows_f32(const float* in, const int32_t* perm, int64_t n_bh, int64_t L, float* out,
                                   hipStream_t stream) {
    const int64_t total = n_bh * L;
    if (total == 0) return hipSuccess;
    if (!grid_fits((total + 255) / 256)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(scatter_rows_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, in, perm,
                       L, total, out);
    return hipGetLastError();
}

}  // namespace fedrag
