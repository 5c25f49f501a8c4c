// Prefill-shaped partial attention (Section 4.1, per-node local computation) for 16-bit storage: many query rows
// per head against one KV shard, non-causal.  MFMA-bound, with the softmax VALU work a close second.  On this
// chip vector instructions overlap matrix instructions only inside one wave (in the shadow of that wave's own
// MFMAs), so each wave software-pipelines across key tiles: in iteration t it computes S^T(t) = K'(t) Q'^T and then
// issues the MFMAs of O^T += V'(t-1)^T P(t-1)^T together with the online softmax of tile t.
//   * one workgroup = 8 waves x 32 query rows = 256 query rows of one (sequence, query head);
//   * K'/V' tiles of 64 keys are shared by the 8 waves through LDS (two slots each), filled by LDS-direct global
//     loads one iteration ahead (no staging registers), one workgroup barrier per iteration;
//   * LDS tiles are unpadded (LDS-direct loads write 64 consecutive 16-byte slots per wave); bank conflicts are
//     avoided by XOR-swizzling the 16-byte chunk index with the row;
//   * both products are computed transposed, S^T = K' Q'^T and O^T = V'^T P^T (32x32x16 MFMA), so the fp32 score
//     tile already sits in the lane layout the second product wants for P^T: probabilities never cross lanes.
//     K' operands are 16-byte LDS reads; V'^T operands come from the row-major V' tile through the transposing LDS
//     read (ds_read_b64_tr_b16), so V' is never transposed in memory or in registers;
//   * workgroups that share a KV head are placed on the same XCD (shared L2).
#include <type_traits>

#include "fedrag_device.h"
#include "fedrag_host.h"

namespace fedrag {

constexpr int kPreWaves = 8;
constexpr int kPreThreads = kPreWaves * kWave;
constexpr int kPreQ = 32;                     // query rows per wave (one 32-wide MFMA column tile)
constexpr int kPreQTile = kPreWaves * kPreQ;  // query rows per workgroup
constexpr int kPreK = 64;                     // keys per LDS tile

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
    return 4 * kPreK * D * 2;  // two K' slots + two V' slots
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
    constexpr int ROWB = D * 2;             // bytes per tile row in LDS (no padding)
    constexpr int SLOT = kPreK * ROWB;      // bytes per tile slot
    constexpr int KS = D / 16;              // contraction steps of S^T
    constexpr int MT = D / 32;              // 32-row tiles of O^T
    constexpr int CH = D / 8;               // 16-byte chunks per row
    constexpr int LPT = (kPreK * CH) / kPreThreads;  // LDS-direct loads per thread per tile

    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* const ks_ = smem;             // [2][64][ROWB]
    char* const vs_ = smem + 2 * SLOT;  // [2][64][ROWB]

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
    const char* Kg = (const char*)(K + ((int64_t)b * Hkv + g) * L * D);
    const char* Vg = (const char*)(V + ((int64_t)b * Hkv + g) * L * D);
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

    // ---- global -> LDS (direct).  One wave-wide load fills 64 consecutive 16-byte slots = 64 / CH tile rows.
    // LDS slot p of row r holds global chunk p ^ swz(r): K' swz(r) = r % CH, V' swz(r) = (4 (r % 4)) % CH.
    constexpr int RPW = kWave / CH;  // rows per wave-wide load
    const int ld_r = lane / CH;      // row within the load
    const int ld_p = lane % CH;      // slot within the row
    auto load_tile = [&](const char* G_, char* slot_base, int tile, bool is_k) {
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            const int r = (j * kPreWaves + wave) * RPW + ld_r;  // tile row
            const int swz = is_k ? (r % CH) : ((4 * (r % 4)) % CH);
            int key = tile * kPreK + r;  // L fits in 31 bits (checked by the caller)
            if (key >= (int)L) key = (int)L - 1;  // rows past the end re-read the last row; masked in the softmax
            const char* gp = G_ + (int64_t)key * ROWB + ((ld_p ^ swz) << 4);
            char* lp = slot_base + (j * kPreWaves + wave) * (RPW * ROWB);  // wave-uniform LDS base
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)gp,
                                             (void __attribute__((address_space(3)))*)lp, 16, 0, 0);
        }
    };

    // ---- per-lane LDS read offsets
    // K' operand (row 32 mt + li, elements 16 ks + 8 lh): chunk (2 ks + lh) ^ (li % CH)
    int k_off[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) k_off[ks] = li * ROWB + ((((2 * ks + lh) % CH) ^ (li % CH)) << 4);
    // V'^T operand through the transposing read: 16-lane group gq covers d-rows 16 (gq % 2) .. +16 of the 32-row
    // tile i; lane s of the group points at key row 4 lh + s / 4 (+8 for the second read), elements
    // 32 i + 16 (gq % 2) + 4 (s % 4) .. +4, i.e. chunk 4 i + 2 (gq % 2) + (s % 4) / 2, byte 8 ((s % 4) % 2) in it
    const int s16 = lane % 16;
    const int gq = lane / 16;
    int v_off[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const int chunk = 4 * i + 2 * (gq % 2) + (s16 % 4) / 2;
        const int swz = (4 * ((s16 / 4) % 4)) % CH;
        v_off[i] = (4 * lh + s16 / 4) * ROWB + (((chunk % CH) ^ swz) << 4) + 8 * ((s16 % 4) % 2);
    }

    const int n_tiles = (int)((L + kPreK - 1) / kPreK);
    f32x16_t S[2];   // S^T of the tile whose softmax runs in this iteration (two 32-key halves)
    vec8 P[2][4];    // P[t & 1]: P^T operands of tile t, one per 16-key step
    float alph[2];   // alph[t & 1]: rescale factor of the running output that goes with P(t)

    auto read_vop = [&](const char* vt, int kk, int i) -> vec8 {
        const char* p = vt + kk * 16 * ROWB + v_off[i];
        const u32x2_t lo = lds_read_tr16(p);
        const u32x2_t hi = lds_read_tr16(p + 8 * ROWB);
        u32x4_t w;
        w[0] = lo[0]; w[1] = lo[1]; w[2] = hi[0]; w[3] = hi[1];
        return __builtin_bit_cast(vec8, w);
    };

    // One pipeline iteration: A(t) = S^T(t) = K'(t) Q'^T, then C(t-1) = O^T += V'(t-1)^T P(t-1)^T issued together
    // with B(t) = online softmax of tile t.  `par` carries t % 2 as a compile-time constant so that the
    // double-buffered register sets are addressed statically.
    auto iteration = [&](int t, auto par, bool doC, bool doAB, bool ldK, bool may_mask) {
        constexpr int p = decltype(par)::value;  // t & 1
        constexpr int q = 1 - p;                 // (t - 1) & 1 == (t + 1) & 1
        if (ldK) load_tile(Kg, ks_ + q * SLOT, t + 1, true);    // K'(t+1) -> slot (t+1) & 1 (last read by A(t-1))
        if (doAB) load_tile(Vg, vs_ + p * SLOT, t, false);      // V'(t)   -> slot t & 1     (last read by C(t-2))

        if (doAB) {  // A(t): lane gets query li and, per 32-key half mt, keys 8 (r / 4) + 4 lh + r % 4, r = 0..15
            const char* kt = ks_ + p * SLOT;
            vec8 kop[2][KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                kop[0][ks] = *(const vec8*)(kt + k_off[ks]);
                kop[1][ks] = *(const vec8*)(kt + 32 * ROWB + k_off[ks]);
            }
            S[0] = zero_vec<f32x16_t>();
            S[1] = zero_vec<f32x16_t>();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                S[0] = T::mfma32(kop[0][ks], qop[ks], S[0]);
                S[1] = T::mfma32(kop[1][ks], qop[ks], S[1]);
            }
            // issue order: operands run four reads ahead of the MFMAs that consume them
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
            for (int j = 0; j < 2 * KS - 4; ++j) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        const char* vt = vs_ + q * SLOT;
        if (doC) {
            if (__builtin_amdgcn_ballot_w64(alph[q] != 1.0f) != 0) {  // wave-uniform: skip when no maximum moved
#pragma unroll
                for (int i = 0; i < MT; ++i) acc_o[i] *= alph[q];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // --- C(t-1) and B(t).  Contraction element e of step kk <-> key 16 kk + 8 (e / 4) + 4 lh + e % 4.
        if (doC && doAB && !may_mask) {
            // Steady state: the 4 MT MFMAs of C(t-1) and the online softmax of tile t are issued as 16 slices,
            // one MFMA each, with scheduling fences between slices: a slice holds the MFMA, its share of the
            // softmax (which runs in the MFMA's shadow) and the transposing reads of the operand four MFMAs
            // ahead.  Softmax shares: slices 0-1 the row maximum, slice 2 the new running maximum and the rescale
            // factor, slices 2-15 the 16 pairs of probabilities (exp2, sum, narrowing).
            constexpr int NM = 4 * MT;
            static_assert(NM == 16 || NM == 8, "slice plan assumes d = 128 or 64");
            constexpr int NP = 16;                 // probability pairs
            constexpr int FIRST = 2;               // first slice that produces probabilities
            vec8 vop[NM];
#pragma unroll
            for (int j = 0; j < 4; ++j) vop[j] = read_vop(vt, j / MT, j % MT);
            float mx = S[0][0];
            float m_new = 0.f, psum = 0.f;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < NM; ++j) {
                if (j + 4 < NM) vop[j + 4] = read_vop(vt, (j + 4) / MT, (j + 4) % MT);
                acc_o[j % MT] = T::mfma32(vop[j], P[q][j / MT], acc_o[j % MT]);
                if (j < 2) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[j][r]);
                }
                if (j == FIRST) {
                    mx = xor32_max(mx);
                    m_new = fmaxf(m_run, mx * scale_log2);  // scale > 0: max commutes with the scaling
                    alph[p] = exp2_diff(m_run, m_new);
                }
                if (j >= FIRST) {
                    // pairs handled by this slice: spread NP pairs over slices FIRST .. NM-1
                    constexpr int NS = NM - FIRST;
                    const int pr0 = ((j - FIRST) * NP) / NS, pr1 = ((j - FIRST + 1) * NP) / NS;
#pragma unroll
                    for (int pr = pr0; pr < pr1; ++pr) {
#pragma unroll
                        for (int u = 0; u < 2; ++u) {
                            const int f = 2 * pr + u;  // flattened score index: half f / 16, register f % 16
                            const float pe = fast_exp2(__builtin_fmaf(S[f / 16][f % 16], scale_log2, -m_new));
                            psum += pe;
                            P[p][f / 8][f % 8] = T::from_float(pe);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            l_run = l_run * alph[p] + psum;
            m_run = m_new;
        } else {
            if (doC) {
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                    for (int i = 0; i < MT; ++i) acc_o[i] = T::mfma32(read_vop(vt, kk, i), P[q][kk], acc_o[i]);
            }
            if (doAB) {  // online softmax of tile t over this lane's 32 keys and its partner lane's 32 keys
                const int key0 = t * kPreK;
                if (key0 + kPreK > (int)L) {  // ragged last tile
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int key = key0 + mt * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
                            if (key >= (int)L) S[mt][r] = -INFINITY;
                        }
                }
                float mx = S[0][0];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[mt][r]);
                mx = xor32_max(mx);
                const float m_new = fmaxf(m_run, mx * scale_log2);
                alph[p] = exp2_diff(m_run, m_new);
                float psum = 0.f;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {  // step kk = 2 mt + r / 8 holds registers r = 8 (kk % 2) .. +8
                        const float pe = fast_exp2(__builtin_fmaf(S[mt][r], scale_log2, -m_new));
                        psum += pe;
                        P[p][2 * mt + r / 8][r % 8] = T::from_float(pe);
                    }
                l_run = l_run * alph[p] + psum;
                m_run = m_new;
            }
        }
        // keep this iteration's results above the barrier that follows (they are consumed in the next iteration)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            u32x4_t w = __builtin_bit_cast(u32x4_t, P[p][kk]);
            pin_here(w);
            P[p][kk] = __builtin_bit_cast(vec8, w);
        }
        pin_here(l_run);
        __builtin_amdgcn_sched_barrier(0);
    };

    std::integral_constant<int, 0> even;
    std::integral_constant<int, 1> odd;

    // prologue: K'(0)
    load_tile(Kg, ks_, 0, true);
    alph[0] = alph[1] = 1.0f;
    __syncthreads();

    // iterations t = 0 .. n_tiles; the steady-state ones (1 <= t, t + 1 < n_tiles) run with every stage on
    iteration(0, even, false, true, n_tiles > 1, true);
    __syncthreads();
    int t = 1;
    for (; t + 2 < n_tiles; t += 2) {
        iteration(t, odd, true, true, true, false);
        __syncthreads();
        iteration(t + 1, even, true, true, true, false);
        __syncthreads();
    }
    for (; t <= n_tiles; ++t) {
        if (t & 1) iteration(t, odd, true, t < n_tiles, t + 1 < n_tiles, true);
        else iteration(t, even, true, t < n_tiles, t + 1 < n_tiles, true);
        __syncthreads();
    }

    // epilogue: lane holds query li and rows d = 32 i + 8 (r / 4) + 4 lh + r % 4 of O^T
    const float l_tot = xor32_sum(l_run);
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
    static bool configured = false;  // opt in to 64 KiB of dynamic LDS once per kernel instantiation
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
