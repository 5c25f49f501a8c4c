// Decode-shaped partial attention (Section 4.1, per-node local computation) for 16-bit storage:
// at most 16 query rows per (sequence, KV head) unit, i.e. the GQA group packed into one MFMA column tile.
// HBM-bound: every K'/V' byte of the shard is read exactly once, nothing is reused, so the kernel is built
// around keeping many full-row loads in flight per wave and no LDS traffic on the streaming path.
//
// One workgroup = one unit x one split of the shard's keys; its four waves take 32-key tiles round-robin.
// Lane l of a wave: lr = l % 16, lq = l / 16.
//   S^T tile (32 keys x 16 queries) = K'(32 x d) . Q'^T(d x 16): two 16-key MFMA tiles; this lane ends up with
//   query lr and keys {16 mt + 4 lq + r}.  Those eight keys are also this lane's contraction slice of
//   O^T(d x 16) += V'^T(d x 32) . P^T(32 x 16), whose d-rows are assigned d = DCH * i + j (tile j, row i) so
//   that lane (i = lr) needs exactly the DCH contiguous elements [DCH*lr, DCH*lr + DCH) of each of its eight
//   keys: full-row coalesced loads and an in-register 8 x DCH transpose.
// P is split into two storage-type terms (hi + lo) so that the probabilities enter the second product with
// ~16 significant bits; the matrix pipe is idle most of the time anyway.
// Splits are normalised partials (O, lse) in the caller's workspace and are folded by the Section 4.1
// aggregation kernel (merge.hip).
#include "fedrag_device.h"
#include "fedrag_host.h"

namespace fedrag {

// Transpose 8 rows of NC 16-bit elements: in[e] holds NC elements (NC/2 words), out[c] holds 8 (4 words).
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

// One 32-key tile in registers.  QB = 0: K' rows as MFMA operands, V' rows as loaded.  QB = 8 or 4: the transport
// codec's codes of the same elements (Section 7.5) plus the (scale, lo) of the rows this lane touches.
template <class T, int D, int QB>
struct DecTile {
    typename T::vec8 k[2][D / 32];
    uint32_t v[8][D / 32];
};
template <class T, int D>
struct DecTile<T, D, 8> {
    u32x4_t kc[2][D / 64];  // 16 codes per (16-key tile, pair of contraction steps): one 16-byte load each
    u32x2_t vc[8];          // 8 codes per key (D = 128: DCH = 8 elements per lane and key)
    u32x2_t kp[2];          // (scale, lo) as bits, of key rows 16 mt + lr
    u32x2_t vp[8];          // of this lane's eight keys
};
template <class T, int D>
struct DecTile<T, D, 4> {
    u32x4_t kc[2];          // 32 codes per 16-key tile (all four contraction steps): one 16-byte load
    uint32_t vc[8];
    u32x2_t kp[2];
    u32x2_t vp[8];
};

// 8 codes -> 8 storage-type values, exactly as dequantize_rows_kernel produces them: fma(code, scale, lo) in fp32,
// narrowed once.  (The fp32 value is pinned so that the two roundings are not folded into one.)
template <class T>
__device__ __forceinline__ typename T::vec8 dequant_codes(const uint32_t (&q)[8], u32x2_t prm) {
    const uint32_t scale_bits = prm[0], lo_bits = prm[1];  // (bit-casting a vector element in place picks element 0)
    const float scale = __builtin_bit_cast(float, scale_bits), lo = __builtin_bit_cast(float, lo_bits);
    typename T::vec8 out;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float x = __builtin_fmaf((float)q[e], scale, lo);
        pin_here(x);
        out[e] = T::from_float(x);
    }
    return out;
}
template <class T>
__device__ __forceinline__ typename T::vec8 dequant8(u32x2_t w, u32x2_t prm) {  // 8-bit codes
    uint32_t q[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) q[e] = (w[e / 4] >> (8 * (e % 4))) & 255u;
    return dequant_codes<T>(q, prm);
}
template <class T>
__device__ __forceinline__ typename T::vec8 dequant8(uint32_t w, u32x2_t prm) {  // 4-bit codes
    // even and odd nibbles spread to bytes first (3 instructions for 8 codes), so that each code then converts with
    // one byte-to-float instruction
    const uint32_t ev = w & 0x0f0f0f0fu, od = (w >> 4) & 0x0f0f0f0fu;
    uint32_t q[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) q[e] = ((e % 2 ? od : ev) >> (8 * (e / 2))) & 255u;
    return dequant_codes<T>(q, prm);
}

// On codes the kernel is bound by its own instruction stream (rebuilding every element costs more than fetching
// it).  At 4 bits it runs with one register tile set per wave and kDecCodesOcc workgroups per compute unit instead
// of one workgroup with a ring of two: the other workgroup's waves fill the issue slots a wave leaves while it
// waits (measured 61 -> 56 us per shard of the decode workload; at 8 bits the ring of two stayed ahead, 60 vs 62).
#ifndef FEDRAG_DEC_NBUF_Q8
#define FEDRAG_DEC_NBUF_Q8 2
#endif
#ifndef FEDRAG_DEC_NBUF_Q4
#define FEDRAG_DEC_NBUF_Q4 1
#endif
#ifndef FEDRAG_DEC_NBUF
#define FEDRAG_DEC_NBUF 2   // register tile sets per wave
#endif
#ifndef FEDRAG_DEC_OCC
#define FEDRAG_DEC_OCC 1    // workgroups per CU the register budget is sized for
#endif
#ifndef FEDRAG_DEC_AUX
#define FEDRAG_DEC_AUX 2    // cache-policy bits of the streaming loads: non-temporal (K'/V' are read once)
#endif

template <class T, int D, int QB>
__global__ __launch_bounds__(kDecThreads, QB == 4 ? kDecCodesOcc : FEDRAG_DEC_OCC) void decode_attn_kernel(const typename T::elem* __restrict__ Q,
                                                                     const KeyRuns runs,
                                                                     const float* __restrict__ Kprm,
                                                                     const float* __restrict__ Vprm, int R,
                                                                     float scale_log2, float* __restrict__ O,
                                                                     float* __restrict__ lse, int64_t total_rows,
                                                                     const int32_t* __restrict__ kv_lens,
                                                                     const int32_t* __restrict__ q_lens, int Lq,
                                                                     int Hkv) {
    typedef typename T::elem elem;
    typedef typename T::vec8 vec8;
    typedef DecTile<T, D, QB> Tile;
    static_assert(QB == 0 || D == 128, "the quantised path is laid out for d = 128");
    constexpr int KS = D / 32;   // contraction steps of the first product
    constexpr int DCH = D / 16;  // elements per lane per key of V' (= number of 16-row tiles of O^T)
    constexpr int NW = DCH / 2;  // 32-bit words of that
    constexpr int ROWB = QB ? D * QB / 8 : D * 2;  // bytes per row of K' / V' as stored (values, or codes)
    constexpr int TILEB = kDecTile * ROWB;
    constexpr int NBUF = QB == 0 ? FEDRAG_DEC_NBUF : (QB == 8 ? FEDRAG_DEC_NBUF_Q8 : FEDRAG_DEC_NBUF_Q4);
    constexpr int AUX = FEDRAG_DEC_AUX;

    __shared__ float sm_m[kDecWaves][16];
    __shared__ float sm_l[kDecWaves][16];
    __shared__ float sm_o[kDecWaves][16][D + 4];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);  // wave-uniform: keeps the tile loop scalar
    const int lane = tid % kWave;
    const int lr = lane % 16;
    const int lq = lane / 16;
    const int64_t unit = blockIdx.x / runs.n_runs;
    const int run = blockIdx.x % runs.n_runs;  // index of this workgroup's partial
    // the shard this run belongs to (scalar compares against the table; first[] is INT_MAX past the last shard)
    const void* K = runs.K[0];
    const void* V = runs.V[0];
    int64_t L = runs.L[0];
    int64_t keys_per_split = runs.per[0];
    int split = run;
#pragma unroll
    for (int i = 1; i < kMaxShards; ++i) {
        if (run >= runs.first[i]) {
            K = runs.K[i];
            V = runs.V[i];
            L = runs.L[i];
            keys_per_split = runs.per[i];
            split = run - runs.first[i];
        }
    }
    const int64_t k_begin = (int64_t)split * keys_per_split;
    // keys of this unit's sequence: all L rows, or the first kv_lens[b] of them (padded batch of unequal sequences);
    // a split that starts past them is empty and returns O = 0, lse = -inf like an empty shard
    int64_t L_seq = L;
    if (kv_lens) {
        const int64_t v = kv_lens[unit / Hkv];
        L_seq = v < 0 ? 0 : (v < L ? v : L);
    }
    int64_t k_end = k_begin + keys_per_split;
    if (k_end > L_seq) k_end = L_seq;
    if (k_end < k_begin) k_end = k_begin;

    const elem* Qu = Q + unit * R * D;
    const char* Kb = (const char*)K + unit * L * ROWB;
    const char* Vb = (const char*)V + unit * L * ROWB;

    // Q'^T operands: column lr (query), contraction slice 32 ks + 8 lq; padding queries are zero
    // Which 8 channels lane group lq contracts in step ks is free as long as Q' and K' agree.  16-bit K': 32 ks + 8 lq
    // (a step's 32 channels are contiguous: 64 bytes per row and load).  Codes: every lane fetches 16 bytes of its
    // row at once - 16 codes = steps 2h, 2h+1 (8 bits) or 32 codes = all four steps (4 bits) - so that a load still
    // covers 64 contiguous bytes per row; with 8- or 4-byte loads the kernel was bound by the number of rows a load
    // instruction touches, not by bytes.
    auto chan0 = [&](int ks) -> int {
        return QB == 0 ? ks * 32 + lq * 8 : (QB == 8 ? 16 * lq + 64 * (ks / 2) + 8 * (ks % 2) : 32 * lq + 8 * ks);
    };
    vec8 qop[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        qop[ks] = (lr < R) ? *(const vec8*)(Qu + lr * D + chan0(ks)) : zero_vec<vec8>();

    f32x4_t acc_o[DCH];
#pragma unroll
    for (int i = 0; i < DCH; ++i) acc_o[i] = zero_vec<f32x4_t>();
    float m_run = -INFINITY, l_run = 0.f;

    // per-lane byte offsets inside a 32-key tile (the tile base is wave-uniform)
    constexpr int EB = QB ? QB : 16;  // bits per stored element
    const uint32_t koff = (uint32_t)(lr * ROWB + lq * EB);          // 8 elements per lane and contraction step
    const uint32_t kqoff = (uint32_t)(lr * ROWB + lq * 16);         // codes: 16 bytes per lane
    const uint32_t voff = (uint32_t)(lq * 4 * ROWB + lr * DCH * EB / 8);

    // Streaming loads go through buffer resources based at the split's first key: the address is
    // (scalar resource base) + (scalar tile offset) + (per-lane 32-bit offset), one VGPR per lane in total.
    const int64_t split_bytes = (k_end - k_begin) * ROWB;  // < 2^31, guaranteed by the split planner
    const __amdgpu_buffer_rsrc_t rk =
        __builtin_amdgcn_make_buffer_rsrc((void*)(Kb + k_begin * ROWB), 0, (int)split_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rv =
        __builtin_amdgcn_make_buffer_rsrc((void*)(Vb + k_begin * ROWB), 0, (int)split_bytes, 0x00020000);
    // quantised path: the (scale, lo) pairs of the split's rows, 8 bytes per key
    const int64_t n_split_keys = k_end - k_begin;
    const __amdgpu_buffer_rsrc_t rkp = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(QB ? Kprm + (unit * L + k_begin) * 2 : nullptr), 0, QB ? (int)(n_split_keys * 8) : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rvp = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(QB ? Vprm + (unit * L + k_begin) * 2 : nullptr), 0, QB ? (int)(n_split_keys * 8) : 0, 0x00020000);
    auto load_k = [&](int tile, Tile& t) {  // tile index inside the split; all 32 keys exist
        const int soff = tile * TILEB;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            if constexpr (QB == 0) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const int off = (int)koff + mt * 16 * ROWB + ks * 4 * EB;
                    t.k[mt][ks] = __builtin_bit_cast(vec8, __builtin_amdgcn_raw_buffer_load_b128(rk, off, soff, AUX));
                }
            } else if constexpr (QB == 8) {
#pragma unroll
                for (int h = 0; h < KS / 2; ++h)
                    t.kc[mt][h] = __builtin_amdgcn_raw_buffer_load_b128(rk, (int)kqoff + mt * 16 * ROWB + 64 * h, soff, AUX);
            } else {
                t.kc[mt] = __builtin_amdgcn_raw_buffer_load_b128(rk, (int)kqoff + mt * 16 * ROWB, soff, AUX);
            }
            if constexpr (QB != 0)
                t.kp[mt] = __builtin_amdgcn_raw_buffer_load_b64(rkp, (mt * 16 + lr) * 8, tile * kDecTile * 8, 0);
        }
    };
    auto load_v = [&](int tile, Tile& t) {
        const int soff = tile * TILEB;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int off = (int)voff + ((e / 4) * 16 + (e % 4)) * ROWB;
            if constexpr (QB != 0) {
                if constexpr (QB == 8) t.vc[e] = __builtin_amdgcn_raw_buffer_load_b64(rv, off, soff, AUX);
                else t.vc[e] = __builtin_amdgcn_raw_buffer_load_b32(rv, off, soff, AUX);
                t.vp[e] = __builtin_amdgcn_raw_buffer_load_b64(rvp, ((e / 4) * 16 + (e % 4) + lq * 4) * 8,
                                                               tile * kDecTile * 8, 0);
            } else if constexpr (NW == 4) {
                const u32x4_t w = __builtin_amdgcn_raw_buffer_load_b128(rv, off, soff, AUX);
                t.v[e][0] = w[0]; t.v[e][1] = w[1]; t.v[e][2] = w[2]; t.v[e][3] = w[3];
            } else {
                const u32x2_t w = __builtin_amdgcn_raw_buffer_load_b64(rv, off, soff, AUX);
                t.v[e][0] = w[0]; t.v[e][1] = w[1];
            }
        }
    };
    // ragged last tile: rows past the end of the run re-read its last key, k_end - 1 (the tail exists, so
    // k_end > k_begin).  Rows past k_end are never touched: with per-sequence key counts they are padding that may
    // hold anything, and a NaN there would survive the multiplication by a zero probability.
    auto load_clamped = [&](int64_t key0, Tile& t) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            int64_t key = key0 + mt * 16 + lr;
            if (key >= k_end) key = k_end - 1;
            if constexpr (QB == 0) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) t.k[mt][ks] = *(const vec8*)(Kb + key * ROWB + ks * 4 * EB + lq * EB);
            } else if constexpr (QB == 8) {
#pragma unroll
                for (int h = 0; h < KS / 2; ++h) t.kc[mt][h] = *(const u32x4_t*)(Kb + key * ROWB + lq * 16 + 64 * h);
            } else {
                t.kc[mt] = *(const u32x4_t*)(Kb + key * ROWB + lq * 16);
            }
            if constexpr (QB != 0) t.kp[mt] = *(const u32x2_t*)(Kprm + (unit * L + key) * 2);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int64_t key = key0 + (e / 4) * 16 + lq * 4 + (e % 4);
            if (key >= k_end) key = k_end - 1;
            const char* p = Vb + key * ROWB + lr * DCH * EB / 8;
            if constexpr (QB == 0) {
#pragma unroll
                for (int w = 0; w < NW; ++w) t.v[e][w] = ((const uint32_t*)p)[w];
            } else {
                if constexpr (QB == 8) t.vc[e] = *(const u32x2_t*)p;
                else t.vc[e] = *(const uint32_t*)p;
                t.vp[e] = *(const u32x2_t*)(Vprm + (unit * L + key) * 2);
            }
        }
    };

    // One 32-key tile.  `reload` refills the tile's registers for key `next0` as soon as each half has been
    // consumed (K' after the first product, V' after the in-register transpose), so the loads fly behind the
    // softmax, the second product and the other tile set's step.
    auto step = [&](Tile& t, int64_t key0, bool masked, bool reload, int next_tile) {
        f32x4_t s[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            s[mt] = zero_vec<f32x4_t>();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                vec8 kop;
                if constexpr (QB == 0) kop = t.k[mt][ks];
                else if constexpr (QB == 8) {
                    const u32x4_t w = t.kc[mt][ks / 2];
                    u32x2_t c;  // (vector elements are copied out one by one before use)
                    const uint32_t c0 = w[2 * (ks % 2)], c1 = w[2 * (ks % 2) + 1];
                    c[0] = c0;
                    c[1] = c1;
                    kop = dequant8<T>(c, t.kp[mt]);
                } else {
                    const uint32_t c = t.kc[mt][ks];
                    kop = dequant8<T>(c, t.kp[mt]);
                }
                s[mt] = T::mfma16(kop, qop[ks], s[mt]);
            }
        }
        if (reload) load_k(next_tile, t);
        float p[8];
        float mx = -INFINITY;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = s[e / 4][e % 4] * scale_log2;
            if (masked) {
                const int64_t key = key0 + (e / 4) * 16 + lq * 4 + (e % 4);
                if (key >= k_end) v = -INFINITY;
            }
            p[e] = v;
            mx = fmaxf(mx, v);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);  // finite: the tile's first key exists
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
        // second product in two halves of the d-rows to keep the transposed operands short-lived
        u32x4_t vt[DCH];
        if constexpr (QB == 0) {
            transpose_keys_b16<DCH>(t.v, vt);
        } else {
            uint32_t v16[8][DCH / 2];  // the eight keys' rows in the storage type, as the unquantised path loads them
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const u32x4_t w = __builtin_bit_cast(u32x4_t, dequant8<T>(t.vc[e], t.vp[e]));
#pragma unroll
                for (int c = 0; c < DCH / 2; ++c) v16[e][c] = w[c];
            }
            transpose_keys_b16<DCH>(v16, vt);
        }
        if (reload) load_v(next_tile, t);
#pragma unroll
        for (int i = 0; i < DCH; ++i) {
            acc_o[i] *= alpha;
            const vec8 vop = __builtin_bit_cast(vec8, vt[i]);
            acc_o[i] = T::mfma16(vop, ph, acc_o[i]);
            acc_o[i] = T::mfma16(vop, pl, acc_o[i]);
        }
    };

    // Wave w owns tiles w, w+4, ... of the split.  NBUF register tile sets form a ring: a set is refilled with
    // the tile NBUF steps ahead as soon as it has been consumed.  In the steady-state loop every refill is
    // unconditional, so the in-order load counter can be waited on precisely (oldest tile only).
    {
        const int64_t n_keys = k_end - k_begin;
        const int n_full_all = (int)(n_keys / kDecTile);  // full tiles in the split
        const int n_mine = (n_full_all > wave) ? (n_full_all - wave + kDecWaves - 1) / kDecWaves : 0;
        auto tile_of = [&](int i) { return wave + i * kDecWaves; };  // i-th tile of this wave
        auto tile_key = [&](int i) { return k_begin + (int64_t)tile_of(i) * kDecTile; };
        Tile t[NBUF];
#pragma unroll
        for (int j = 0; j < NBUF; ++j)
            if (j < n_mine) { load_k(tile_of(j), t[j]); load_v(tile_of(j), t[j]); }
        int i = 0;
        for (; i + 2 * NBUF <= n_mine; i += NBUF) {
#pragma unroll
            for (int j = 0; j < NBUF; ++j) step(t[j], tile_key(i + j), false, true, tile_of(i + j + NBUF));
        }
        // fewer than 2*NBUF tiles left: refills become conditional, then the ring drains
#pragma unroll
        for (int j = 0; j < NBUF; ++j) {
            if (i + j < n_mine) {
                if (i + j + NBUF < n_mine) step(t[j], tile_key(i + j), false, true, tile_of(i + j + NBUF));
                else step(t[j], tile_key(i + j), false, false, 0);
            }
        }
#pragma unroll
        for (int j = 0; j < NBUF; ++j)
            if (i + NBUF + j < n_mine) step(t[j], tile_key(i + NBUF + j), false, false, 0);
        // ragged tail of the split (fewer than 32 keys): the wave whose turn it is takes it
        const int rem = (int)(n_keys % kDecTile);
        if (rem > 0 && (n_full_all % kDecWaves) == wave) {
            const int64_t key0 = k_begin + (int64_t)n_full_all * kDecTile;
            load_clamped(key0, t[0]);
            step(t[0], key0, true, false, 0);
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
    float* Oout = O + ((int64_t)run * total_rows + unit * R) * D;
    float* Lout = lse + (int64_t)run * total_rows + unit * R;
    // padded batch with per-sequence query counts: row n of the unit is query n % Lq of its head; rows past the
    // sequence's count are padding and are not written
    int q_rows = Lq;
    if (q_lens) {
        const int v = q_lens[unit / Hkv];
        q_rows = v < 0 ? 0 : (v < Lq ? v : Lq);
    }
    for (int idx = tid; idx < R * D; idx += kDecThreads) {
        const int n = idx / D;
        const int d = idx % D;
        if (n % Lq >= q_rows) continue;
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

template <class T, int D, int QB>
static hipError_t launch_decode_t(const AttnProblem& p, hipStream_t stream) {
    typedef typename T::elem elem;
    const float scale_log2 = p.scale * kLog2e;
    const int64_t rows = (int64_t)p.B * p.Hq * p.Lq;
    const KeyRuns runs = attn_runs_of(p);
    const int splits = runs.n_runs;
    if (splits < 1) return hipErrorInvalidValue;
    if (QB != 0 && p.n_shards > 1) return hipErrorInvalidValue;
    for (int i = 0; i < kMaxShards; ++i)  // a run is addressed with 32-bit byte offsets
        if (runs.L[i] > 0 && runs.per[i] * (int64_t)(QB ? D * QB / 8 : D * 2) > 0x7fffffffLL) return hipErrorInvalidValue;
    const int R = (int)((p.Hq / p.Hkv) * p.Lq);
    const int64_t units = (int64_t)p.B * p.Hkv;
    float* Odst = p.O;
    float* Ldst = p.lse;
    if (splits > 1) {
        if (!p.workspace || p.workspace_bytes < (size_t)splits * rows * (D + 1) * sizeof(float)) return hipErrorInvalidValue;
        Odst = (float*)p.workspace;
        Ldst = Odst + (size_t)splits * rows * D;
    }
    if (!grid_fits(units * splits)) return hipErrorInvalidValue;
    hipLaunchKernelGGL((decode_attn_kernel<T, D, QB>), dim3((unsigned)(units * splits)), dim3(kDecThreads), 0, stream,
                       (const elem*)p.Q, runs, p.K_params, p.V_params, R, scale_log2, Odst, Ldst, rows, p.kv_lens,
                       p.q_lens, (int)p.Lq, p.Hkv);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || splits == 1) return e;
    return launch_lse_merge(Odst, Ldst, splits, rows, D, p.O, p.lse, stream, p.q_lens, p.Lq, (int64_t)p.Hq * p.Lq);
}

hipError_t launch_decode_attn(const AttnProblem& p, hipStream_t stream) {
    if (p.quant_bits != 0) {  // codes of the transport codec in place of K', V' (d = 128, checked by the caller)
        if (p.D != 128) return hipErrorInvalidValue;
        if (p.dtype == FEDRAG_BF16)
            return p.quant_bits == 8 ? launch_decode_t<BF16, 128, 8>(p, stream) : launch_decode_t<BF16, 128, 4>(p, stream);
        return p.quant_bits == 8 ? launch_decode_t<F16, 128, 8>(p, stream) : launch_decode_t<F16, 128, 4>(p, stream);
    }
    if (p.dtype == FEDRAG_BF16)
        return p.D == 128 ? launch_decode_t<BF16, 128, 0>(p, stream) : launch_decode_t<BF16, 64, 0>(p, stream);
    return p.D == 128 ? launch_decode_t<F16, 128, 0>(p, stream) : launch_decode_t<F16, 64, 0>(p, stream);
}

}  // namespace fedrag
