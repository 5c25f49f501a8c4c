// The Compute Node's work on one KV shard (Section 4.1, per-node local computation):
//   O_i = softmax(Q' K_i'^T * scale) V_i'   and   lse_i = ln sum_t exp(Q' K_i'^T * scale)   (= ln w_i)
// evaluated with a running maximum so that outlier logits cannot overflow.  Three kernels:
//   attn_f32_kernel     fp32 storage, plain FMAs, one wave per query row (accuracy path)
//   decode_attn_kernel  16-bit storage, <= 16 query rows per KV head (GQA group packed): HBM-bound streaming
//                       of K'/V' with the shard's keys split across workgroups; splits are folded afterwards by
//                       the Section 4.1 aggregation (merge.hip)
//   prefill_attn_kernel 16-bit storage, many query rows: MFMA-bound tiled kernel, K'/V' tiles staged in LDS
// Both MFMA kernels compute the transposed products S^T = K' Q'^T and O^T = V'^T P^T: the fp32 score tile then
// already sits in the lane layout the second product wants for P^T, so probabilities never cross lanes.
#include "fedrag_device.h"
#include "fedrag_host.h"

namespace fedrag {

// ------------------------------------------------------------------------------------------------ fp32 path
template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(const float* __restrict__ Q, const float* __restrict__ K,
                                                       const float* __restrict__ V, int Hq, int Hkv, int64_t Lq,
                                                       int64_t L, int64_t total_rows, float scale,
                                                       float* __restrict__ O, float* __restrict__ lse) {
    constexpr int CPL = D / kWave;  // output columns per lane
    __shared__ float qs[4][D];
    const int wave = threadIdx.x / kWave;
    const int lane = threadIdx.x % kWave;
    const int64_t row = (int64_t)blockIdx.x * 4 + wave;
    if (row >= total_rows) return;  // no workgroup barrier below
    const int64_t bh = row / Lq;
    const int b = (int)(bh / Hq);
    const int h = (int)(bh % Hq);
    const int g = h / (Hq / Hkv);
    const float* q = Q + row * D;
    const float* Kg = K + ((int64_t)b * Hkv + g) * L * D;
    const float* Vg = V + ((int64_t)b * Hkv + g) * L * D;
    for (int c = lane; c < D; c += kWave) qs[wave][c] = q[c];
    wave_lds_fence();

    float m = -INFINITY, l = 0.f;
    float acc[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) acc[c] = 0.f;

    for (int64_t t0 = 0; t0 < L; t0 += kWave) {
        const int64_t t = t0 + lane;
        float s = -INFINITY;
        if (t < L) {
            const float* kr = Kg + t * D;
            float dot = 0.f;
#pragma unroll 8
            for (int c = 0; c < D; c += 4) {
                const f32x4_t kv = *(const f32x4_t*)(kr + c);
                const f32x4_t qv = *(const f32x4_t*)(&qs[wave][c]);
                dot = __builtin_fmaf(qv[0], kv[0], dot);
                dot = __builtin_fmaf(qv[1], kv[1], dot);
                dot = __builtin_fmaf(qv[2], kv[2], dot);
                dot = __builtin_fmaf(qv[3], kv[3], dot);
            }
            s = dot * scale;
        }
        float mx = s;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        const float m_new = fmaxf(m, mx);  // finite: lane 0 of this tile always has a key
        const float alpha = (m == -INFINITY) ? 0.f : expf(m - m_new);
        const float p = (t < L) ? expf(s - m_new) : 0.f;
        float ps = p;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) ps += __shfl_xor(ps, o);
        l = l * alpha + ps;
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] *= alpha;
        const int n = (L - t0 < kWave) ? (int)(L - t0) : kWave;
        for (int j = 0; j < n; ++j) {
            const float pj = __shfl(p, j);
            const float* vr = Vg + (t0 + j) * D;
#pragma unroll
            for (int c = 0; c < CPL; ++c) acc[c] = __builtin_fmaf(pj, vr[c * kWave + lane], acc[c]);
        }
        m = m_new;
    }
    const float inv = (l > 0.f) ? 1.0f / l : 0.f;
#pragma unroll
    for (int c = 0; c < CPL; ++c) O[row * D + c * kWave + lane] = acc[c] * inv;
    if (lane == 0) lse[row] = (l > 0.f) ? m + logf(l) : -INFINITY;
}

// ------------------------------------------------------------------------------------------------ decode path
constexpr int kDecWaves = 4;
constexpr int kDecThreads = kDecWaves * kWave;
constexpr int kDecTile = 32;                        // keys per wave step
constexpr int kDecStride = kDecWaves * kDecTile;    // keys per workgroup step

// Transpose NK(=8) rows of NC 16-bit elements: in[e] holds NC elements (NC/2 words), out[c] holds 8 (4 words).
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

// One workgroup = one (sequence, KV head) unit x one split of the shard's keys.
// R = G * L_q <= 16 query rows of the unit are contiguous in memory (heads of a group are adjacent).
// Lane l of a wave: lr = l % 16, lq = l / 16.
//   S^T tile (32 keys x 16 queries) = K'(32 x d) . Q'^T(d x 16): two 16-key MFMA tiles; this lane ends up with
//   query lr and keys {16 mt + 4 lq + r}.  The same eight keys are this lane's contraction slice of the second
//   product O^T(d x 16) += V'^T(d x 32) . P^T(32 x 16), whose d-rows are assigned as d = DCH * i + mt so that
//   lane (i = lr) needs exactly the DCH contiguous elements [DCH*lr, DCH*lr + DCH) of each of its eight keys:
//   full-row coalesced loads and an in-register 8 x DCH transpose, no LDS on the streaming path.
template <class T, int D>
__global__ __launch_bounds__(kDecThreads) void decode_attn_kernel(const typename T::elem* __restrict__ Q,
                                                                  const typename T::elem* __restrict__ K,
                                                                  const typename T::elem* __restrict__ V, int R,
                                                                  int64_t L, int n_splits, int64_t keys_per_split,
                                                                  float scale_log2, float* __restrict__ O,
                                                                  float* __restrict__ lse, int64_t total_rows) {
    typedef typename T::elem elem;
    typedef typename T::vec8 vec8;
    constexpr int KS = D / 32;   // contraction steps of the first product
    constexpr int DCH = D / 16;  // elements per lane per key of V' (= number of 16-row tiles of O^T)
    constexpr int NW = DCH / 2;  // 32-bit words of that

    __shared__ float sm_m[kDecWaves][16];
    __shared__ float sm_l[kDecWaves][16];
    __shared__ float sm_o[kDecWaves][16][D + 4];

    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const int lane = tid % kWave;
    const int lr = lane % 16;
    const int lq = lane / 16;
    const int64_t unit = blockIdx.x / n_splits;
    const int split = blockIdx.x % n_splits;
    const int64_t k_begin = (int64_t)split * keys_per_split;
    int64_t k_end = k_begin + keys_per_split;
    if (k_end > L) k_end = L;

    const elem* Qu = Q + unit * R * D;
    const elem* Ku = K + unit * L * D;
    const elem* Vu = V + unit * L * D;

    // Q'^T operands: column lr (query), contraction slice 32 ks + 8 lq; padding queries are zero
    vec8 qop[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        qop[ks] = (lr < R) ? *(const vec8*)(Qu + lr * D + ks * 32 + lq * 8) : zero_vec<vec8>();

    f32x4_t acc_o[DCH];
#pragma unroll
    for (int i = 0; i < DCH; ++i) acc_o[i] = zero_vec<f32x4_t>();
    float m_run = -INFINITY, l_run = 0.f;

    struct TileRegs {
        vec8 k[2][KS];
        uint32_t v[8][NW];
    };

    auto load_tile = [&](int64_t key0, TileRegs& t) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            int64_t key = key0 + mt * 16 + lr;
            if (key >= L) key = L - 1;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) t.k[mt][ks] = *(const vec8*)(Ku + key * D + ks * 32 + lq * 8);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int64_t key = key0 + (e / 4) * 16 + lq * 4 + (e % 4);
            if (key >= L) key = L - 1;
            const uint32_t* p = (const uint32_t*)(Vu + key * D + lr * DCH);
            if constexpr (NW == 4) {
                const u32x4_t w = *(const u32x4_t*)p;
                t.v[e][0] = w[0]; t.v[e][1] = w[1]; t.v[e][2] = w[2]; t.v[e][3] = w[3];
            } else {
                const u32x2_t w = *(const u32x2_t*)p;
                t.v[e][0] = w[0]; t.v[e][1] = w[1];
            }
        }
    };

    auto compute_tile = [&](int64_t key0, const TileRegs& t) {
        f32x4_t s[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            s[mt] = zero_vec<f32x4_t>();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) s[mt] = T::mfma16(t.k[mt][ks], qop[ks], s[mt]);
        }
        float p[8];
        float mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int64_t key = key0 + (e / 4) * 16 + lq * 4 + (e % 4);
            const float v = s[e / 4][e % 4] * scale_log2;
            p[e] = (key < k_end) ? v : -INFINITY;
            mx = fmaxf(mx, p[e]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);  // finite: key0 < k_end
        const float alpha = exp2_diff(m_run, m_new);
        float psum = 0.f;
        vec8 ph, pl;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float pe = fast_exp2(p[e] - m_new);
            psum += pe;
            ph[e] = T::from_float(pe);
            pl[e] = T::from_float(pe - T::to_float(ph[e]));
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        u32x4_t vt[DCH];
        transpose_keys_b16<DCH>(t.v, vt);
#pragma unroll
        for (int i = 0; i < DCH; ++i) {
            acc_o[i] *= alpha;
            const vec8 vop = __builtin_bit_cast(vec8, vt[i]);
            acc_o[i] = T::mfma16(vop, ph, acc_o[i]);
            acc_o[i] = T::mfma16(vop, pl, acc_o[i]);
        }
    };

    // wave w takes the 32-key tiles w, w+4, ... of the split; next tile's loads fly while this one is computed
    {
        TileRegs ta, tb;
        int64_t key0 = k_begin + (int64_t)wave * kDecTile;
        if (key0 < k_end) load_tile(key0, ta);
        while (key0 < k_end) {
            int64_t next = key0 + kDecStride;
            if (next < k_end) load_tile(next, tb);
            compute_tile(key0, ta);
            key0 = next;
            if (key0 >= k_end) break;
            next = key0 + kDecStride;
            if (next < k_end) load_tile(next, ta);
            compute_tile(key0, tb);
            key0 = next;
        }
    }

    // fold the four waves (Section 4.1 aggregation, in base 2)
    float l_tot = l_run + __shfl_xor(l_run, 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (lq == 0) {
        sm_m[wave][lr] = m_run;
        sm_l[wave][lr] = l_tot;
    }
    if (lr < R) {
#pragma unroll
        for (int i = 0; i < DCH; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) sm_o[wave][lr][DCH * (4 * lq + r) + i] = acc_o[i][r];
    }
    __syncthreads();
    float* Oout = O + ((int64_t)split * total_rows + unit * R) * D;
    float* Lout = lse + (int64_t)split * total_rows + unit * R;
    for (int idx = tid; idx < R * D; idx += kDecThreads) {
        const int n = idx / D;
        const int d = idx % D;
        float M = sm_m[0][n];
#pragma unroll
        for (int w = 1; w < kDecWaves; ++w) M = fmaxf(M, sm_m[w][n]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) {
            const float a = exp2_diff(sm_m[w][n], M);
            num = __builtin_fmaf(a, sm_o[w][n][d], num);
            den = __builtin_fmaf(a, sm_l[w][n], den);
        }
        const bool any = den > 0.f;
        Oout[n * D + d] = any ? num / den : 0.f;
        if (d == 0) Lout[n] = any ? (M + fast_log2(den)) * kLn2 : -INFINITY;
    }
}

// ------------------------------------------------------------------------------------------------ prefill path
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
    const int wave = tid / kWave;
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

// ------------------------------------------------------------------------------------------------ launchers
static bool use_decode_kernel(int Hq, int Hkv, int64_t Lq) { return (int64_t)(Hq / Hkv) * Lq <= 16; }

int attn_kv_splits(int B, int Hq, int Hkv, int D, int dtype, int64_t Lq, int64_t Lkv) {
    (void)D;
    if (dtype == FEDRAG_F32 || Lkv <= 0 || Lq <= 0 || !use_decode_kernel(Hq, Hkv, Lq)) return 1;
    const int64_t units = (int64_t)B * Hkv;
    if (units <= 0) return 1;
    // ~2 workgroups per CU over 256 CUs; a split is a whole number of 128-key workgroup steps
    int64_t want = (512 + units - 1) / units;
    if (want < 1) want = 1;
    int64_t per = (Lkv + want - 1) / want;
    per = ((per + kDecStride - 1) / kDecStride) * kDecStride;
    if (per < 4 * kDecStride) per = 4 * kDecStride;
    return (int)((Lkv + per - 1) / per);
}

static int64_t decode_keys_per_split(int64_t Lkv, int n_splits) {
    int64_t per = (Lkv + n_splits - 1) / n_splits;
    return ((per + kDecStride - 1) / kDecStride) * kDecStride;
}

size_t attn_workspace_bytes(int B, int Hq, int Hkv, int D, int dtype, int64_t Lq, int64_t Lkv) {
    const int s = attn_kv_splits(B, Hq, Hkv, D, dtype, Lq, Lkv);
    if (s <= 1) return 0;
    const size_t rows = (size_t)B * Hq * (size_t)Lq;
    return (size_t)s * rows * (size_t)(D + 1) * sizeof(float);
}

template <class T, int D>
static hipError_t launch_attn16(const AttnProblem& p, hipStream_t stream) {
    typedef typename T::elem elem;
    const float scale_log2 = p.scale * kLog2e;
    const int64_t rows = (int64_t)p.B * p.Hq * p.Lq;
    if (use_decode_kernel(p.Hq, p.Hkv, p.Lq)) {
        const int splits = attn_kv_splits(p.B, p.Hq, p.Hkv, D, p.dtype, p.Lq, p.Lkv);
        const int64_t per = decode_keys_per_split(p.Lkv, splits);
        const int R = (int)((p.Hq / p.Hkv) * p.Lq);
        const int64_t units = (int64_t)p.B * p.Hkv;
        float* Odst = p.O;
        float* Ldst = p.lse;
        if (splits > 1) {
            Odst = (float*)p.workspace;
            Ldst = Odst + (size_t)splits * rows * D;
        }
        hipLaunchKernelGGL((decode_attn_kernel<T, D>), dim3((unsigned)(units * splits)), dim3(kDecThreads), 0, stream,
                           (const elem*)p.Q, (const elem*)p.K, (const elem*)p.V, R, p.Lkv, splits, per, scale_log2,
                           Odst, Ldst, rows);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess || splits == 1) return e;
        return launch_lse_merge(Odst, Ldst, splits, rows, D, p.O, p.lse, stream);
    }
    const int q_tiles = (int)((p.Lq + kPreQTile - 1) / kPreQTile);
    const int n_units = p.B * p.Hkv;
    const int per_unit = (p.Hq / p.Hkv) * q_tiles;
    const int64_t grid = (int64_t)8 * ((n_units + 7) / 8) * per_unit;
    hipLaunchKernelGGL((prefill_attn_kernel<T, D>), dim3((unsigned)grid), dim3(kPreThreads), 0, stream,
                       (const elem*)p.Q, (const elem*)p.K, (const elem*)p.V, p.Hq, p.Hkv, p.Lq, p.Lkv, q_tiles,
                       n_units, scale_log2, p.O, p.lse);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_attn_f32(const AttnProblem& p, hipStream_t stream) {
    const int64_t rows = (int64_t)p.B * p.Hq * p.Lq;
    hipLaunchKernelGGL(attn_f32_kernel<D>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, (const float*)p.Q,
                       (const float*)p.K, (const float*)p.V, p.Hq, p.Hkv, p.Lq, p.Lkv, rows, p.scale, p.O, p.lse);
    return hipGetLastError();
}

hipError_t launch_partial_attn(const AttnProblem& p, hipStream_t stream) {
    const int64_t rows = (int64_t)p.B * p.Hq * p.Lq;
    if (rows == 0) return hipSuccess;
    if (p.Lkv == 0) return launch_fill_empty(p.O, p.lse, rows, p.D, stream);
    switch (p.dtype) {
        case FEDRAG_F32:
            return p.D == 128 ? launch_attn_f32<128>(p, stream) : launch_attn_f32<64>(p, stream);
        case FEDRAG_BF16:
            return p.D == 128 ? launch_attn16<BF16, 128>(p, stream) : launch_attn16<BF16, 64>(p, stream);
        case FEDRAG_F16:
            return p.D == 128 ? launch_attn16<F16, 128>(p, stream) : launch_attn16<F16, 64>(p, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace fedrag
