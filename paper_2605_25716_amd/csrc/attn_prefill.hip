// Prefill-shaped partial attention (Section 4.1, per-node local computation) for 16-bit storage: many query rows
// per head against one KV shard, non-causal.  MFMA-bound, with the softmax VALU work a close second, so the kernel
// is organised to let the two overlap:
//   * one workgroup = 8 waves (two per SIMD) x 32 query rows = 256 query rows of one (sequence, query head);
//   * K'/V' tiles of 64 keys are shared by the 8 waves through a double-buffered LDS stage (one barrier per
//     tile); the next tile's global loads fly during the current tile's arithmetic;
//   * both products are computed transposed, S^T = K' Q'^T and O^T = V'^T P^T (32x32x16 MFMA), so the fp32
//     score tile already sits in the lane layout the second product wants for P^T: probabilities never cross
//     lanes.  K' operands are plain 16-byte LDS reads; V'^T operands come from the row-major V' tile through
//     the transposing LDS read (ds_read_b64_tr_b16), so V' is never transposed in memory or in registers;
//   * workgroups that share a KV head are placed on the same XCD (shared L2).
#include "fedrag_device.h"
#include "fedrag_host.h"

namespace fedrag {

constexpr int kPreWaves = 8;
constexpr int kPreThreads = kPreWaves * kWave;
constexpr int kPreQ = 32;                     // query rows per wave (one 32-wide MFMA column tile)
constexpr int kPreQTile = kPreWaves * kPreQ;  // query rows per workgroup
constexpr int kPreK = 64;                     // keys per LDS tile
constexpr int kPreKPad = 16;                  // bytes of row padding, K' tile: 16-byte operand reads, 32 rows
constexpr int kPreVPad = 64;                  // bytes of row padding, V' tile: transposing reads, 4 rows x 64 bytes

typedef short s16x4_t __attribute__((ext_vector_type(4)));

// Transposing LDS read: within each group of 16 lanes, lane j receives element (j % 4) of the 8 bytes addressed
// by lane 4 e + j / 4, for e = 0..3.  With lane s of the group pointing at row (s / 4), columns 4 (s % 4)..+4 of
// a row-major 4 x 16 block, lane j gets column j of the block, rows 0..3.
__device__ __forceinline__ u32x2_t lds_read_tr16(const char* p) {
    const s16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)p);
    return __builtin_bit_cast(u32x2_t, v);
}

template <int D>
constexpr int prefill_lds_bytes() {
    return 2 * kPreK * (D * 2 + kPreKPad) + 2 * kPreK * (D * 2 + kPreVPad);
}

template <class T, int D>
__global__ __launch_bounds__(kPreThreads, 1) void prefill_attn_kernel(const typename T::elem* __restrict__ Q,
                                                                      const typename T::elem* __restrict__ K,
                                                                      const typename T::elem* __restrict__ V, int Hq,
                                                                      int Hkv, int64_t Lq, int64_t L, int q_tiles,
                                                                      int n_units, float scale_log2,
                                                                      float* __restrict__ O, float* __restrict__ lse) {
    typedef typename T::elem elem;
    typedef typename T::vec8 vec8;
    constexpr int KROW = D * 2 + kPreKPad;  // bytes per K' tile row in LDS
    constexpr int VROW = D * 2 + kPreVPad;  // bytes per V' tile row in LDS
    constexpr int KS = D / 16;              // contraction steps of S^T
    constexpr int MT = D / 32;              // 32-row tiles of O^T
    constexpr int CH = D / 8;               // 16-byte chunks per row
    constexpr int LPT = (kPreK * CH) / kPreThreads;  // 16-byte loads per thread per tile (K' and V' each)

    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* const ks_ = smem;                      // [2][64][KROW]
    char* const vs_ = smem + 2 * kPreK * KROW;   // [2][64][VROW]

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
    vec8 qop[KS];  // Q'^T operands: column li, contraction slice 16 ks + 8 lh
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qop[ks] = *(const vec8*)(Qh + q_ld * D + ks * 16 + lh * 8);

    f32x16_t acc_o[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc_o[i] = zero_vec<f32x16_t>();
    float m_run = -INFINITY, l_run = 0.f;

    // global -> registers -> LDS staging of the next tile
    vec8 kreg[LPT], vreg[LPT];
    auto load_tile = [&](int64_t key0) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int c = i * kPreThreads + tid;
            int key = (int)key0 + c / CH;  // L fits in 31 bits (checked by the caller)
            if (key >= (int)L) key = (int)L - 1;
            kreg[i] = *(const vec8*)(Kg + (int64_t)key * D + (c % CH) * 8);
            vreg[i] = *(const vec8*)(Vg + (int64_t)key * D + (c % CH) * 8);
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int c = i * kPreThreads + tid;
            *(vec8*)(ks_ + (buf * kPreK + c / CH) * KROW + (c % CH) * 16) = kreg[i];
            *(vec8*)(vs_ + (buf * kPreK + c / CH) * VROW + (c % CH) * 16) = vreg[i];
        }
    };

    // per-lane LDS offsets
    const int k_rd = li * KROW + lh * 16;  // K' operand: row 32 mt + li, bytes 32 ks + 16 lh
    // V'^T operand through the transposing read: 16-lane group gq covers d-rows 16 (gq % 2) .. +16 of the 32-row
    // tile; lane s of the group points at key row (4 lh + s / 4) (+8 for the second read), columns 4 (s % 4)..+4
    const int s16 = lane % 16;
    const int gq = lane / 16;
    const int v_rd = (4 * lh + s16 / 4) * VROW + ((gq % 2) * 16 + 4 * (s16 % 4)) * 2;

    if (L > 0) {
        load_tile(0);
        store_tile(0);
    }
    __syncthreads();
    const int n_tiles = (int)((L + kPreK - 1) / kPreK);
    for (int t = 0; t < n_tiles; ++t) {
        const int buf = t & 1;
        const int64_t key0 = (int64_t)t * kPreK;
        if (t + 1 < n_tiles) load_tile(key0 + kPreK);
        const char* kt = ks_ + buf * kPreK * KROW;
        const char* vt = vs_ + buf * kPreK * VROW;

        // S^T (64 keys x 32 queries) for this wave: lane gets query li and, per 32-key tile mt, keys
        // 8 (r / 4) + 4 lh + r % 4, r = 0..15.  All K' operands are requested before the first MFMA so that the
        // LDS latency is paid once; the two 32-key tiles form two independent accumulation chains.
        f32x16_t s[2];
        {
            vec8 kop[2][KS];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    kop[mt][ks] = *(const vec8*)(kt + mt * 32 * KROW + k_rd + ks * 32);
            __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the MFMAs
            s[0] = zero_vec<f32x16_t>();
            s[1] = zero_vec<f32x16_t>();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s[0] = T::mfma32(kop[0][ks], qop[ks], s[0]);
                s[1] = T::mfma32(kop[1][ks], qop[ks], s[1]);
            }
        }
        // V'^T operands of the first two 16-key steps: requested now, consumed after the softmax
        auto read_vop = [&](int kk, int i) -> vec8 {
            const char* p = vt + kk * 16 * VROW + v_rd + i * 64;
            const u32x2_t lo = lds_read_tr16(p);
            const u32x2_t hi = lds_read_tr16(p + 8 * VROW);
            u32x4_t w;
            w[0] = lo[0]; w[1] = lo[1]; w[2] = hi[0]; w[3] = hi[1];
            return __builtin_bit_cast(vec8, w);
        };
        vec8 vop_a[2][MT];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int i = 0; i < MT; ++i) vop_a[kk][i] = read_vop(kk, i);
        __builtin_amdgcn_sched_barrier(0);  // requested before the softmax starts

        // online softmax over this lane's 32 keys and its partner lane's 32 keys (base-2 domain)
        if (key0 + kPreK > L) {  // ragged last tile
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = (int)key0 + mt * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
                    if (key >= (int)L) s[mt][r] = -INFINITY;
                }
        }
        float mx = s[0][0];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[mt][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx * scale_log2);  // scale > 0: max commutes with the scaling
        const float alpha = exp2_diff(m_run, m_new);
        float psum = 0.f;
        vec8 pop[4];  // P^T operands: step kk = 2 mt + r / 8 holds registers r = 8 (kk % 2) .. +8
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pe = fast_exp2(__builtin_fmaf(s[mt][r], scale_log2, -m_new));
                psum += pe;
                pop[2 * mt + r / 8][r % 8] = T::from_float(pe);
            }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        // second half of the V'^T operands: in flight behind the first eight MFMAs
        vec8 vop_b[2][MT];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int i = 0; i < MT; ++i) vop_b[kk][i] = read_vop(2 + kk, i);
        __builtin_amdgcn_sched_barrier(0);
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {  // wave-uniform: skip when no row's maximum moved
#pragma unroll
            for (int i = 0; i < MT; ++i) acc_o[i] *= alpha;
        }
        // O^T += V'^T P^T, 16 keys per step: contraction element e <-> key 16 kk + 8 (e / 4) + 4 lh + e % 4
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int i = 0; i < MT; ++i) acc_o[i] = T::mfma32(vop_a[kk][i], pop[kk], acc_o[i]);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int i = 0; i < MT; ++i) acc_o[i] = T::mfma32(vop_b[kk][i], pop[2 + kk], acc_o[i]);
        if (t + 1 < n_tiles) store_tile(buf ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds query li and rows d = 32 i + 8 (r / 4) + 4 lh + r % 4 of O^T
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = (l_tot > 0.f) ? 1.0f / l_tot : 0.f;
    if (q_row < Lq) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                f32x4_t o;
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r] = acc_o[i][4 * r4 + r] * inv;
                *(f32x4_t*)(Oh + q_row * D + 32 * i + 8 * r4 + 4 * lh) = o;
            }
        if (lh == 0) Lh[q_row] = (l_tot > 0.f) ? (m_run + fast_log2(l_tot)) * kLn2 : -INFINITY;
    }
}

template <class T, int D>
static hipError_t launch_prefill_t(const AttnProblem& p, hipStream_t stream) {
    typedef typename T::elem elem;
    static bool configured = false;  // opt in to more than 64 KiB of LDS once per kernel instantiation
    if (!configured) {
        hipError_t e = hipFuncSetAttribute((const void*)prefill_attn_kernel<T, D>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, prefill_lds_bytes<D>());
        if (e != hipSuccess) return e;
        configured = true;
    }
    const float scale_log2 = p.scale * kLog2e;
    const int q_tiles = (int)((p.Lq + kPreQTile - 1) / kPreQTile);
    const int n_units = p.B * p.Hkv;
    const int per_unit = (p.Hq / p.Hkv) * q_tiles;
    const int64_t grid = (int64_t)8 * ((n_units + 7) / 8) * per_unit;
    hipLaunchKernelGGL((prefill_attn_kernel<T, D>), dim3((unsigned)grid), dim3(kPreThreads), prefill_lds_bytes<D>(),
                       stream, (const elem*)p.Q, (const elem*)p.K, (const elem*)p.V, p.Hq, p.Hkv, p.Lq, p.Lkv, q_tiles,
                       n_units, scale_log2, p.O, p.lse);
    return hipGetLastError();
}

hipError_t launch_prefill_attn(const AttnProblem& p, hipStream_t stream) {
    if (p.dtype == FEDRAG_BF16)
        return p.D == 128 ? launch_prefill_t<BF16, 128>(p, stream) : launch_prefill_t<BF16, 64>(p, stream);
    return p.D == 128 ? launch_prefill_t<F16, 128>(p, stream) : launch_prefill_t<F16, 64>(p, stream);
}

}  // namespace fedrag
