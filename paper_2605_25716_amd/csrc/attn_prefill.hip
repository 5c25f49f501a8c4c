// Prefill-shaped partial attention (Section 4.1, per-node local computation) for 16-bit storage: many query rows
// per head against one KV shard, non-causal.  MFMA-bound: K'/V' tiles are staged in LDS and shared by the
// workgroup's waves; both products are computed transposed (S^T = K' Q'^T, O^T = V'^T P^T) so that the fp32 score
// tile already sits in the lane layout the second product wants for P^T.
#include "fedrag_device.h"
#include "fedrag_host.h"

namespace fedrag {

template <int NC>
__device__ __forceinline__ void transpose_keys_b16(const uint32_t (&in)[8][NC / 2], u32x4_t (&out)[NC]) {
#pragma unroll
    for (int c2 = 0; c2 < NC / 2; ++c2) {
#pragma unroll
        for (int r2 = 0; r2 < 4; ++r2) {
            const uint32_t a = in[2 * r2][c2];
            const uint32_t b = in[2 * r2 + 1][c2];
            out[2 * c2][r2] = __builtin_amdgcn_perm(b, a, 0x05040100u);      // {a.lo, b.lo}
            out[2 * c2 + 1][r2] = __builtin_amdgcn_perm(b, a, 0x07060302u);  // {a.hi, b.hi}
        }
    }
}

constexpr int kPreWaves = 4;
constexpr int kPreThreads = kPreWaves * kWave;
constexpr int kPreQ = 32;                    // query rows per wave (one 32-wide MFMA column tile)
constexpr int kPreQTile = kPreWaves * kPreQ; // query rows per workgroup
constexpr int kPreK = 64;                    // keys per LDS tile
constexpr int kPrePad = 8;

// One workgroup = 128 query rows of one (sequence, query head) against the whole shard.
// Lane l: li = l % 32, lh = l / 32.  32x32x16 MFMA:
//   S^T(64 keys x 32 q) = K'tile . Q'^T : two 32-key tiles x (d/16) steps; lane gets query li and, per tile, keys
//   8*(r/4) + 4*lh + r%4 (r = 0..15).  Registers r in [8kk', 8kk'+8) are this lane's contraction slice of the
//   16-key step kk = 2 mt + kk' of O^T(d x 32 q) += V'^T . P^T, whose d-rows are assigned d = DCH*i + mt'
//   (DCH = d/32) so lane (i = li) reads DCH contiguous elements of each of its 8 keys from the LDS tile and
//   transposes them in registers.
template <class T, int D>
__global__ __launch_bounds__(kPreThreads) void prefill_attn_kernel(const typename T::elem* __restrict__ Q,
                                                                   const typename T::elem* __restrict__ K,
                                                                   const typename T::elem* __restrict__ V, int Hq,
                                                                   int Hkv, int64_t Lq, int64_t L, int q_tiles,
                                                                   int n_units, float scale_log2,
                                                                   float* __restrict__ O, float* __restrict__ lse) {
    typedef typename T::elem elem;
    typedef typename T::vec8 vec8;
    constexpr int LDP = D + kPrePad;
    constexpr int KS = D / 16;   // contraction steps of S^T
    constexpr int DCH = D / 32;  // V' elements per lane per key = 32-row tiles of O^T
    constexpr int CH = D / 8;    // 16-byte chunks per row
    constexpr int LPT = (kPreK * CH) / kPreThreads;  // 16-byte loads per thread per tile (K or V)

    __shared__ __attribute__((aligned(16))) elem ks_[kPreK * LDP];
    __shared__ __attribute__((aligned(16))) elem vs_[kPreK * LDP];

    // XCD-aware placement: consecutive workgroup ids are dealt round-robin to the 8 XCDs (one L2 each);
    // give every XCD whole (sequence, KV head) units so that the workgroups sharing K'/V' share an L2.
    const int G = Hq / Hkv;
    const int per_unit = G * q_tiles;
    const int xcd = blockIdx.x % 8;
    const int slot = blockIdx.x / 8;
    const int unit = xcd + 8 * (slot / per_unit);
    if (unit >= n_units) return;
    const int w_in_unit = slot % per_unit;
    const int hg = w_in_unit / q_tiles;
    const int qt = w_in_unit % q_tiles;
    const int b = unit / Hkv;
    const int g = unit % Hkv;
    const int h = g * G + hg;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);  // wave-uniform
    const int lane = tid % kWave;
    const int li = lane % 32;
    const int lh = lane / 32;

    const elem* Qh = Q + ((int64_t)b * Hq + h) * Lq * D;
    const elem* Kg = K + ((int64_t)b * Hkv + g) * L * D;
    const elem* Vg = V + ((int64_t)b * Hkv + g) * L * D;
    float* Oh = O + ((int64_t)b * Hq + h) * Lq * D;
    float* Lh = lse + ((int64_t)b * Hq + h) * Lq;

    const int64_t q_row = (int64_t)qt * kPreQTile + wave * kPreQ + li;  // this lane's query row
    const int64_t q_ld = q_row < Lq ? q_row : Lq - 1;
    vec8 qop[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qop[ks] = *(const vec8*)(Qh + q_ld * D + ks * 16 + lh * 8);

    f32x16_t acc_o[DCH];
#pragma unroll
    for (int i = 0; i < DCH; ++i) acc_o[i] = zero_vec<f32x16_t>();
    float m_run = -INFINITY, l_run = 0.f;

    vec8 kreg[LPT], vreg[LPT];
    auto load_tile = [&](int64_t key0) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int c = i * kPreThreads + tid;
            int64_t key = key0 + c / CH;
            if (key >= L) key = L - 1;
            kreg[i] = *(const vec8*)(Kg + key * D + (c % CH) * 8);
            vreg[i] = *(const vec8*)(Vg + key * D + (c % CH) * 8);
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int c = i * kPreThreads + tid;
            *(vec8*)(&ks_[(c / CH) * LDP + (c % CH) * 8]) = kreg[i];
            *(vec8*)(&vs_[(c / CH) * LDP + (c % CH) * 8]) = vreg[i];
        }
    };

    if (L > 0) load_tile(0);
    for (int64_t key0 = 0; key0 < L; key0 += kPreK) {
        __syncthreads();  // everyone finished reading the previous tile
        store_tile();
        __syncthreads();
        if (key0 + kPreK < L) load_tile(key0 + kPreK);

        // S^T for this wave's 32 queries
        f32x16_t s[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            s[mt] = zero_vec<f32x16_t>();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const vec8 kop = *(const vec8*)(&ks_[(mt * 32 + li) * LDP + ks * 16 + lh * 8]);
                s[mt] = T::mfma32(kop, qop[ks], s[mt]);
            }
        }
        // online softmax over this lane's 32 keys and its partner lane's 32 keys
        const bool tail = key0 + kPreK > L;
        float mx = -INFINITY;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float v = s[mt][r] * scale_log2;
                if (tail) {
                    const int64_t key = key0 + mt * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
                    if (key >= L) v = -INFINITY;
                }
                s[mt][r] = v;
                mx = fmaxf(mx, v);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = exp2_diff(m_run, m_new);
        float psum = 0.f;
        vec8 pop[4];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pe = fast_exp2(s[mt][r] - m_new);
                psum += pe;
                pop[2 * mt + r / 8][r % 8] = T::from_float(pe);
            }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (alpha != 1.0f) {
#pragma unroll
            for (int i = 0; i < DCH; ++i) acc_o[i] *= alpha;
        }
        // O^T += V'^T P^T, 16 keys per step
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            uint32_t vin[8][DCH / 2];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int key = kk * 16 + 8 * (e / 4) + 4 * lh + (e % 4);
                const uint32_t* p = (const uint32_t*)(&vs_[key * LDP + li * DCH]);
                if constexpr (DCH == 4) {
                    const u32x2_t w = *(const u32x2_t*)p;
                    vin[e][0] = w[0]; vin[e][1] = w[1];
                } else {
                    vin[e][0] = *p;
                }
            }
            u32x4_t vt[DCH];
            transpose_keys_b16<DCH>(vin, vt);
#pragma unroll
            for (int i = 0; i < DCH; ++i)
                acc_o[i] = T::mfma32(__builtin_bit_cast(vec8, vt[i]), pop[kk], acc_o[i]);
        }
    }

    // epilogue: lane holds query li, rows d = DCH * (8*(r/4) + 4*lh + r%4) + i of O^T
    float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = (l_tot > 0.f) ? 1.0f / l_tot : 0.f;
    if (q_row < Lq) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 8 * (r / 4) + 4 * lh + (r % 4);
            if constexpr (DCH == 4) {
                f32x4_t o;
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = acc_o[i][r] * inv;
                *(f32x4_t*)(Oh + q_row * D + row * 4) = o;
            } else {
                Oh[q_row * D + row * 2 + 0] = acc_o[0][r] * inv;
                Oh[q_row * D + row * 2 + 1] = acc_o[1][r] * inv;
            }
        }
        if (lh == 0) Lh[q_row] = (l_tot > 0.f) ? (m_run + fast_log2(l_tot)) * kLn2 : -INFINITY;
    }
}


template <class T, int D>
static hipError_t launch_prefill_t(const AttnProblem& p, hipStream_t stream) {
    typedef typename T::elem elem;
    const float scale_log2 = p.scale * kLog2e;
    const int q_tiles = (int)((p.Lq + kPreQTile - 1) / kPreQTile);
    const int n_units = p.B * p.Hkv;
    const int per_unit = (p.Hq / p.Hkv) * q_tiles;
    const int64_t grid = (int64_t)8 * ((n_units + 7) / 8) * per_unit;
    hipLaunchKernelGGL((prefill_attn_kernel<T, D>), dim3((unsigned)grid), dim3(kPreThreads), 0, stream,
                       (const elem*)p.Q, (const elem*)p.K, (const elem*)p.V, p.Hq, p.Hkv, p.Lq, p.Lkv, q_tiles,
                       n_units, scale_log2, p.O, p.lse);
    return hipGetLastError();
}

hipError_t launch_prefill_attn(const AttnProblem& p, hipStream_t stream) {
    if (p.dtype == FEDRAG_BF16)
        return p.D == 128 ? launch_prefill_t<BF16, 128>(p, stream) : launch_prefill_t<BF16, 64>(p, stream);
    return p.D == 128 ? launch_prefill_t<F16, 128>(p, stream) : launch_prefill_t<F16, 64>(p, stream);
}

}  // namespace fedrag
