// Prefill-shaped partial attention (Section 4.1, per-node local computation) for 16-bit storage: many query rows
// per head against one KV shard.  Bound by the matrix pipe at the clock the chip sustains on real operand data plus
// the part of the softmax's vector work that does not overlap it.  Vector instructions overlap matrix instructions
// best inside one wave (in the shadow of that wave's own MFMAs), so each wave software-pipelines across key tiles:
// in iteration t it computes S^T(t) = K'(t) Q'^T and then issues the MFMAs of O^T += V'(t-1)^T P(t-1)^T together with
// the online softmax of tile t.
//   * one workgroup = 8 waves x 32 query rows = 256 query rows of one (sequence, query head);
//   * K'/V' tiles of 64 keys are shared by the 8 waves through LDS (two slots each), filled by LDS-direct global
//     loads one iteration ahead (no staging registers), one workgroup barrier per iteration;
//   * LDS tiles are unpadded (LDS-direct loads write 64 consecutive 16-byte slots per wave); bank conflicts are
//     avoided by XOR-swizzling the 16-byte chunk index with the row;
//   * both products are computed transposed, S^T = K' Q'^T and O^T = V'^T P^T (32x32x16 MFMA), so the fp32 score
//     tile already sits in the lane layout the second product wants for P^T: probabilities never cross lanes.
//     K' operands are 16-byte LDS reads; V'^T operands come from the row-major V' tile through the transposing LDS
//     read (ds_read_b64_tr_b16), so V' is never transposed in memory or in registers;
//   * workgroups that share a KV head are placed on the same XCD (shared L2);
//   * QB = 8 or 4: K', V' arrive as the transport codec's codes (Section 7.5).  The LDS-direct loads are replaced by
//     ordinary loads of the codes and of the rows' (scale, lo) one iteration ahead; each thread rebuilds its 8-element
//     chunk exactly as the dequantise call would (fp32 fma, one narrowing) and writes it to the same swizzled LDS slot,
//     so everything downstream is unchanged and consumes the same values as dequantise-then-attend.
#include <type_traits>

#include "fedrag_device.h"
#include "fedrag_host.h"

namespace fedrag {

constexpr int kPreThreads = kPreWaves * kWave;
#ifndef FEDRAG_PRE_PD
#define FEDRAG_PRE_PD 4
#endif
constexpr int kPrePD = FEDRAG_PRE_PD;         // MFMA operands are read from LDS this many MFMAs ahead

typedef short s16x4_t __attribute__((ext_vector_type(4)));

// Transposing LDS read: within each group of 16 lanes, lane j receives element (j % 4) of the 8 bytes addressed
// by lane 4 e + j / 4, for e = 0..3.  With lane s of the group pointing at row (s / 4), columns 4 (s % 4)..+4 of
// a row-major 4 x 16 block, lane j gets column j of the block, rows 0..3.
__device__ __forceinline__ u32x2_t lds_read_tr16(const char* p) {
    const s16x4_t v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)p);
    return __builtin_bit_cast(u32x2_t, v);
}

// CAUSAL: the queries are the last Lq of the L tokens whose K'/V' are given, and query i sees keys 0 .. i + (L - Lq)
// (Section 5.3: the Inquirer's own part of a decoder layer's attention).  That call works on plaintext V, whose
// outlier channels are not spread by a scrambling matrix (|v| of several tens), so a probability rounded once to the
// storage type (relative error 2^-9 in bf16) would move an output by more than the 16-bit output tolerance.  The
// CAUSAL instantiation therefore feeds the second product P = P_hi + P_lo, two storage-type terms (about 16
// significant bits), at the price of twice the MFMAs of that product.
template <class T, int D, bool CAUSAL, int QB>
__global__ __launch_bounds__(kPreThreads, 1) void prefill_attn_kernel(const typename T::elem* __restrict__ Q,
                                                                      const KeyRuns runs,
                                                                      const float* __restrict__ Kprm,
                                                                      const float* __restrict__ Vprm, int Hq, int Hkv,
                                                                      int64_t Lq,
                                                                      const int32_t* __restrict__ kv_lens,
                                                                      const int32_t* __restrict__ q_lens, int q_tiles,
                                                                      int n_units, float scale_log2,
                                                                      float* __restrict__ O, float* __restrict__ lse) {
    typedef typename T::elem elem;
    typedef typename T::vec8 vec8;
    constexpr int ROWB = D * 2;             // bytes per tile row in LDS (no padding)
    constexpr int SLOT = kPreK * ROWB;      // bytes per tile slot
    constexpr int KS = D / 16;              // contraction steps of S^T
    constexpr int MT = D / 32;              // 32-row tiles of O^T
    constexpr int CH = D / 8;               // 16-byte chunks per row
    constexpr int LPT = (kPreK * CH) / kPreThreads;  // LDS-direct loads (QB: 8-element chunks) per thread per tile
    static_assert(QB == 0 || QB == 8 || QB == 4, "16-bit values, or 8- / 4-bit codes");
    static_assert(QB == 0 || !CAUSAL, "codes are what travels to the Compute Node; the Inquirer's own K, V are plain");
    constexpr int CROWB = QB ? D * QB / 8 : ROWB;  // bytes per row of K' / V' as stored (values, or codes)

    // One array per tile slot: distinct objects let the compiler see that the LDS-direct load filling one slot
    // does not alias the LDS reads of another, so it does not make those reads wait for the load.
    __shared__ __attribute__((aligned(16))) char ks0[SLOT], ks1[SLOT], vs0[SLOT], vs1[SLOT];

    // XCD-aware placement: consecutive workgroup ids are dealt round-robin to the 8 XCDs (one L2 each);
    // give every XCD whole (sequence, KV head) units so that the workgroups sharing K'/V' share an L2.
    // With more than one run (several shards, or few query tiles and many keys; not CAUSAL) there is one workgroup
    // per (query tile, run) and O / lse are [n_runs][rows] partials that the Section 4.1 aggregation folds afterwards.
    const int G = Hq / Hkv;
    const int n_runs = runs.n_runs;
    const int per_unit = G * q_tiles * n_runs;
    const int xcd = blockIdx.x % 8;
    const int slot = blockIdx.x / 8;
    const int unit = xcd + 8 * (slot / per_unit);
    if (unit >= n_units) return;
    const int run = (slot % per_unit) % n_runs;
    const int w_in_unit = (slot % per_unit) / n_runs;
    // the shard this run belongs to (scalar compares against the table; first[] is INT_MAX past the last shard)
    const elem* K = (const elem*)runs.K[0];
    const elem* V = (const elem*)runs.V[0];
    int64_t L_stride = runs.L[0];
    int64_t keys_per_run = runs.per[0];
    int split = run;
#pragma unroll
    for (int i = 1; i < kMaxShards; ++i) {
        if (run >= runs.first[i]) {
            K = (const elem*)runs.K[i];
            V = (const elem*)runs.V[i];
            L_stride = runs.L[i];
            keys_per_run = runs.per[i];
            split = run - runs.first[i];
        }
    }
    // CAUSAL: later query tiles visit more keys.  Hand out the last tile of every head of the group first, then the
    // one before it, and so on: workgroups are started in index order as compute units free up, so every compute
    // unit ends up with a long tile followed by short ones and the launch does not wait on a late long tile.
    const int hg = CAUSAL ? w_in_unit % G : w_in_unit / q_tiles;
    const int qt = CAUSAL ? q_tiles - 1 - w_in_unit / G : w_in_unit % q_tiles;
    const int b = unit / Hkv;
    const int g = unit % Hkv;
    const int h = g * G + hg;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);  // wave-uniform
    const int lane = tid % kWave;
    const int li = lane % 32;
    const int lh = lane / 32;

    const elem* Qh = Q + ((int64_t)b * Hq + h) * Lq * D;
    const char* Kg = (const char*)K + ((int64_t)b * Hkv + g) * L_stride * CROWB;
    const char* Vg = (const char*)V + ((int64_t)b * Hkv + g) * L_stride * CROWB;
    const float* Kpg = QB ? Kprm + ((int64_t)b * Hkv + g) * L_stride * 2 : nullptr;  // (scale, lo) per key row
    const float* Vpg = QB ? Vprm + ((int64_t)b * Hkv + g) * L_stride * 2 : nullptr;
    // keys of this sequence: all L_stride rows, or the first kv_lens[b] of them (padded batch of unequal sequences)
    int64_t L = L_stride;
    if (kv_lens) {
        const int64_t v = kv_lens[b];
        L = v < 0 ? 0 : (v < L_stride ? v : L_stride);
    }
    // query rows of this sequence that exist (padded batch): rows past them are neither computed nor written
    int64_t Lq_rows = Lq;
    if (q_lens) {
        const int64_t v = q_lens[b];
        Lq_rows = v < 0 ? 0 : (v < Lq ? v : Lq);
    }
    if ((int64_t)qt * kPreQTile >= Lq_rows) return;  // workgroup-uniform, before any barrier
    const int64_t part_row0 = (int64_t)run * n_units * G * Lq;  // n_units * G * Lq = rows of one partial
    float* Oh = O + (part_row0 + ((int64_t)b * Hq + h) * Lq) * D;
    float* Lh = lse + part_row0 + ((int64_t)b * Hq + h) * Lq;
    if (!CAUSAL && n_runs > 1) {  // this workgroup's run of keys; a run past the end is empty
        const int64_t k_begin = (int64_t)split * keys_per_run;
        const int64_t k_end = k_begin + keys_per_run < L ? k_begin + keys_per_run : L;
        L = k_end > k_begin ? k_end - k_begin : 0;
        Kg += k_begin * CROWB;
        Vg += k_begin * CROWB;
        if (QB) {
            Kpg += k_begin * 2;
            Vpg += k_begin * 2;
        }
    }

    const int64_t q_row = (int64_t)qt * kPreQTile + wave * kPreQ + li;  // this lane's query row
    if (L == 0) {  // no keys (workgroup-uniform, before any barrier): O = 0, lse = -inf
        if (q_row < Lq_rows) {
            for (int c = lh * (D / 2); c < (lh + 1) * (D / 2); c += 4) *(f32x4_t*)(Oh + q_row * D + c) = zero_vec<f32x4_t>();
            if (lh == 0) Lh[q_row] = -INFINITY;
        }
        return;
    }
    const int64_t q_ld = q_row < Lq ? q_row : Lq - 1;
    vec8 qop[KS];  // Q'^T operands: column li, contraction slice 16 ks + 8 lh
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qop[ks] = *(const vec8*)(Qh + q_ld * D + ks * 16 + lh * 8);

    f32x16_t acc_o[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) acc_o[i] = zero_vec<f32x16_t>();
    float m_run = -INFINITY, l_run = 0.f;

    // ---- global -> LDS (direct buffer loads).  One wave-wide load fills 64 consecutive 16-byte slots = 64 / CH
    // tile rows.  LDS slot p of row r holds global chunk p ^ swz(r): K' swz(r) = r % CH, V' swz(r) = (4 (r % 4)) % CH;
    // both depend on r only through r % 16, which is the same for every load of a thread.  The buffer resource
    // starts at the tile and covers the rest of the shard, so rows past the end of the shard arrive as zeros.
    constexpr int RPW = kWave / CH;  // rows per wave-wide load
    const int ld_r = wave * RPW + lane / CH;  // row within a group of kPreWaves * RPW rows
    const int ld_p = lane % CH;               // slot within the row
    const int ld_voff_k = ld_r * ROWB + ((ld_p ^ (ld_r % CH)) << 4);
    const int ld_voff_v = ld_r * ROWB + ((ld_p ^ ((4 * (ld_r % 4)) % CH)) << 4);
    static_assert((kPreWaves * RPW) % 16 == 0, "swizzle must not depend on the load index");
    auto load_tile = [&](const char* G_, char* slot_base, int tile, bool is_k) {
        const int64_t byte0 = (int64_t)tile * SLOT;
        const int64_t left = L * ROWB - byte0;
        const int n_rec = (int)(left < 0x7fffffff ? left : 0x7fffffff);
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(G_ + byte0), 0, n_rec, 0x00020000);
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            char* lp = slot_base + (j * kPreWaves + wave) * (RPW * ROWB);  // wave-uniform LDS base
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (void __attribute__((address_space(3)))*)lp, 16,
                                                     is_k ? ld_voff_k : ld_voff_v, j * (kPreWaves * RPW * ROWB), 0, 0);
        }
    };

    // ---- QB: codes -> registers one iteration ahead, then -> LDS.  Chunk j of a thread is row (j * kPreThreads + tid)
    // / CH of the tile, 8 channels from 8 (tid % CH); reads past the end of the shard return zeros (code 0, scale 0,
    // lo 0: the row dequantises to zeros, as rows past the end arrive in the 16-bit path).
    struct CodeChunk {
        uint32_t c[QB == 8 ? 2 : 1];
        u32x2_t prm;
    };
    CodeChunk kst[QB ? LPT : 1], vst[QB ? LPT : 1];
    const int cq_row = tid / CH, cq_c = tid % CH;
    auto fetch_codes = [&](const char* G_, const float* Pg_, int tile, CodeChunk (&st)[QB ? LPT : 1]) {
        const int64_t row0 = (int64_t)tile * kPreK;
        const int64_t left_rows = L - row0 > 0 ? L - row0 : 0;
        const int64_t lc = left_rows * CROWB, lp = left_rows * 8;
        const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(G_ + row0 * CROWB), 0, (int)(lc < 0x7fffffff ? lc : 0x7fffffff), 0x00020000);
        const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(Pg_ + row0 * 2), 0, (int)(lp < 0x7fffffff ? lp : 0x7fffffff), 0x00020000);
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            const int r = j * (kPreThreads / CH) + cq_row;
            if constexpr (QB == 8) {
                const u32x2_t w = __builtin_amdgcn_raw_buffer_load_b64(rc, r * CROWB + cq_c * 8, 0, 0);
                st[j].c[0] = w[0];
                st[j].c[1] = w[1];
            } else {
                st[j].c[0] = __builtin_amdgcn_raw_buffer_load_b32(rc, r * CROWB + cq_c * 4, 0, 0);
            }
            st[j].prm = __builtin_amdgcn_raw_buffer_load_b64(rp, r * 8, 0, 0);
        }
    };
    auto store_codes = [&](char* slot_base, const CodeChunk (&st)[QB ? LPT : 1], bool is_k) {
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            const int r = j * (kPreThreads / CH) + cq_row;
            const uint32_t sb = st[j].prm[0], lb = st[j].prm[1];
            const float scale = __builtin_bit_cast(float, sb), lo = __builtin_bit_cast(float, lb);
            vec8 out;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t code = QB == 8 ? (st[j].c[e / 4] >> (8 * (e % 4))) & 255u : (st[j].c[0] >> (4 * e)) & 15u;
                float x = __builtin_fmaf((float)code, scale, lo);
                pin_here(x);  // the dequantised value is the fp32 result narrowed afterwards: two roundings, not one
                out[e] = T::from_float(x);
            }
            const int swz = is_k ? r % CH : (4 * (r % 4)) % CH;
            *(vec8*)(slot_base + r * ROWB + ((cq_c ^ swz) << 4)) = out;
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

    // keys this workgroup has to visit, and the first tile in which some key is hidden from some row of the
    // workgroup (past the end of the shard, or - CAUSAL - after the row's own position)
    const int64_t off = L - Lq;
    const int64_t q_first = (int64_t)qt * kPreQTile;
    const int64_t q_last = (q_first + kPreQTile < Lq ? q_first + kPreQTile : Lq) - 1;
    const int64_t wg_keys = CAUSAL ? (q_last + off + 1 < L ? q_last + off + 1 : L) : L;
    const int n_tiles = (int)((wg_keys + kPreK - 1) / kPreK);
    const int t_mask0 = (int)((CAUSAL ? (q_first + off + 1 < L ? q_first + off + 1 : L) : L) / kPreK);
    const int key_lim = (int)(CAUSAL ? (q_row + off + 1 < L ? q_row + off + 1 : L) : L);  // this lane's row sees keys < key_lim
    f32x16_t S0;      // S^T of the current tile, keys 0..31
    f32x16_t S1[2];   // S1[t & 1]: S^T of tile t, keys 32..63 (kept one iteration longer, see below)
    vec8 P[2][4];     // P[t & 1]: P^T operands of tile t, one per 16-key step
    constexpr bool SPLIT = CAUSAL;           // second storage-type term of every probability (see above)
    vec8 Plo[SPLIT ? 2 : 1][SPLIT ? 4 : 1];  // Plo[t & 1]: P - P as stored in P[t & 1], narrowed
    auto put_p = [&](int par, int kk, int e, float pe) {
        const elem hi = T::from_float(pe);
        P[par][kk][e] = hi;
        if constexpr (SPLIT) Plo[par][kk][e] = T::from_float(pe - T::to_float(hi));
    };
    float alph[2];    // alph[t & 1]: rescale factor of the running output that goes with P(t)

    auto read_vop = [&](const char* vt, int kk, int i) -> vec8 {
        const char* p = vt + kk * 16 * ROWB + v_off[i];
        const u32x2_t lo = lds_read_tr16(p);
        const u32x2_t hi = lds_read_tr16(p + 8 * ROWB);
        u32x4_t w;
        w[0] = lo[0]; w[1] = lo[1]; w[2] = hi[0]; w[3] = hi[1];
        return __builtin_bit_cast(vec8, w);
    };

    // One pipeline iteration t, in two MFMA phases with vector work in their shadow:
    //   A(t)   = S^T(t) = K'(t) Q'^T                     together with  B2(t-1) = probabilities of keys 32..63 of
    //                                                                   tile t-1 (its maximum is already known);
    //   C(t-1) = O^T += V'(t-1)^T P(t-1)^T               together with  B1(t) = row maximum of tile t, new running
    //                                                                   maximum, rescale factor, probabilities of
    //                                                                   keys 0..31 of tile t.
    // Splitting the softmax of a tile over two phases gives both MFMA phases about the same vector load.
    // `par` carries t % 2 as a compile-time constant so that the double-buffered register sets are addressed
    // statically.  m_run is the running maximum after tile t-1 until B1(t) replaces it.
    auto iteration = [&](int t, auto par, bool doC, bool doAB, bool ldK, bool may_mask) {
        constexpr int p = decltype(par)::value;  // t & 1
        constexpr int q = 1 - p;                 // (t - 1) & 1 == (t + 1) & 1
        constexpr int NM = 4 * MT;
        static_assert(NM == 16 || NM == 8, "slice plans assume d = 128 or 64");
        if constexpr (QB == 0) {
            if (ldK) load_tile(Kg, q ? ks1 : ks0, t + 1, true);    // K'(t+1) -> slot (t+1) & 1 (last read by A(t-1))
            if (doAB) load_tile(Vg, p ? vs1 : vs0, t, false);      // V'(t)   -> slot t & 1     (last read by C(t-2))
        } else {  // the codes of the same two tiles into registers; they reach their (free) slots between the phases
            if (ldK) fetch_codes(Kg, Kpg, t + 1, kst);
            if (doAB) fetch_codes(Vg, Vpg, t, vst);
        }
        const bool steady = doC && doAB && !may_mask;

        // --- A(t) and B2(t-1).  Lane gets query li and, per 32-key half, keys 8 (r / 4) + 4 lh + r % 4, r = 0..15.
        // Contraction element e of step kk of the second product <-> key 16 kk + 8 (e / 4) + 4 lh + e % 4, so
        // register r of half 1 goes to step 2 + r / 8, element r % 8.
        const char* kt = p ? ks1 : ks0;
        if (steady) {
            constexpr int NA = 2 * KS;  // MFMAs of A: slice j -> half j % 2, contraction step j / 2
            vec8 kop[NA];
#pragma unroll
            for (int j = 0; j < kPrePD; ++j) kop[j] = *(const vec8*)(kt + (j % 2) * 32 * ROWB + k_off[j / 2]);
            S0 = zero_vec<f32x16_t>();
            S1[p] = zero_vec<f32x16_t>();
            float psum = 0.f;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < NA; ++j) {
                if (j + kPrePD < NA) kop[j + kPrePD] = *(const vec8*)(kt + ((j + kPrePD) % 2) * 32 * ROWB + k_off[(j + kPrePD) / 2]);
                if (j % 2 == 0) S0 = T::mfma32(kop[j], qop[j / 2], S0);
                else S1[p] = T::mfma32(kop[j], qop[j / 2], S1[p]);
                const int r0 = (j * 16) / NA, r1 = ((j + 1) * 16) / NA;  // registers of half 1 handled here
#pragma unroll
                for (int r = r0; r < r1; ++r) {
                    const float pe = fast_exp2(__builtin_fmaf(S1[q][r], scale_log2, -m_run));
                    psum += pe;
                    put_p(q, 2 + r / 8, r % 8, pe);
                }
                pin_here(psum);  // the slice's vector work stays in the slice
                __builtin_amdgcn_sched_barrier(0);
            }
            l_run += psum;
        } else {
            if (doC) {  // B2(t-1)
                float psum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pe = fast_exp2(__builtin_fmaf(S1[q][r], scale_log2, -m_run));
                    psum += pe;
                    put_p(q, 2 + r / 8, r % 8, pe);
                }
                l_run += psum;
            }
            if (doAB) {
                S0 = zero_vec<f32x16_t>();
                S1[p] = zero_vec<f32x16_t>();
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    S0 = T::mfma32(*(const vec8*)(kt + k_off[ks]), qop[ks], S0);
                    S1[p] = T::mfma32(*(const vec8*)(kt + 32 * ROWB + k_off[ks]), qop[ks], S1[p]);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (QB != 0) {
            if (ldK) store_codes(q ? ks1 : ks0, kst, true);
            __builtin_amdgcn_sched_barrier(0);
        }
        const char* vt = q ? vs1 : vs0;
        if (doC) {
            if (__builtin_amdgcn_ballot_w64(alph[q] != 1.0f) != 0) {  // wave-uniform: skip when no maximum moved
#pragma unroll
                for (int i = 0; i < MT; ++i) acc_o[i] *= alph[q];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // --- C(t-1) and B1(t)
        if (steady) {
            // 4 MT slices of one MFMA each, with scheduling fences between slices: a slice holds the MFMA, its
            // share of B1 and the transposing reads of the operand four MFMAs ahead.  Shares: slices 0-1 the row
            // maximum, slice 2 the new running maximum and the rescale factor, slices 2.. the 16 probabilities.
            constexpr int FIRST = 2;  // first slice that produces probabilities
            vec8 vop[NM];
#pragma unroll
            for (int j = 0; j < kPrePD; ++j) vop[j] = read_vop(vt, j / MT, j % MT);
            float mx = S0[0];
            float m_new = 0.f, psum = 0.f;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < NM; ++j) {
                if (j + kPrePD < NM) vop[j + kPrePD] = read_vop(vt, (j + kPrePD) / MT, (j + kPrePD) % MT);
                acc_o[j % MT] = T::mfma32(vop[j], P[q][j / MT], acc_o[j % MT]);
                if constexpr (SPLIT) acc_o[j % MT] = T::mfma32(vop[j], Plo[q][j / MT], acc_o[j % MT]);
                if (j == 0) {
#pragma unroll
                    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, S0[r]);
                }
                if (j == 1) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S1[p][r]);
                }
                if (j == FIRST) {
                    mx = xor32_max(mx);
                    m_new = fmaxf(m_run, mx * scale_log2);  // scale > 0: max commutes with the scaling
                    alph[p] = exp2_diff(m_run, m_new);
                }
                if (j >= FIRST) {
                    constexpr int NS = NM - FIRST;
                    const int r0 = ((j - FIRST) * 16) / NS, r1 = ((j - FIRST + 1) * 16) / NS;
#pragma unroll
                    for (int r = r0; r < r1; ++r) {
                        const float pe = fast_exp2(__builtin_fmaf(S0[r], scale_log2, -m_new));
                        psum += pe;
                        put_p(p, r / 8, r % 8, pe);
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
                    for (int i = 0; i < MT; ++i) {
                        const vec8 vop = read_vop(vt, kk, i);
                        acc_o[i] = T::mfma32(vop, P[q][kk], acc_o[i]);
                        if constexpr (SPLIT) acc_o[i] = T::mfma32(vop, Plo[q][kk], acc_o[i]);
                    }
            }
            if (doAB) {  // B1(t); keys past the end of the shard get a score of -inf (also seen by B2(t) later)
                const int key0 = t * kPreK;
                if (t >= t_mask0) {  // ragged last tile, or tiles that reach past a row's own position
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = key0 + 8 * (r / 4) + 4 * lh + (r % 4);
                        if (key >= key_lim) S0[r] = -INFINITY;
                        if (key + 32 >= key_lim) S1[p][r] = -INFINITY;
                    }
                }
                float mx = S0[0];
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, fmaxf(S0[r], S1[p][r]));
                mx = xor32_max(mx);
                const float m_new = fmaxf(m_run, mx * scale_log2);
                alph[p] = exp2_diff(m_run, m_new);
                float psum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pe = fast_exp2(__builtin_fmaf(S0[r], scale_log2, -m_new));
                    psum += pe;
                    put_p(p, r / 8, r % 8, pe);
                }
                l_run = l_run * alph[p] + psum;
                m_run = m_new;
            }
        }
        if constexpr (QB != 0) {
            if (doAB) store_codes(p ? vs1 : vs0, vst, false);
        }
        // keep this iteration's results above the barrier that follows (they are consumed in the next iteration)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            u32x4_t w = __builtin_bit_cast(u32x4_t, P[p][kk]);
            pin_here(w);
            P[p][kk] = __builtin_bit_cast(vec8, w);
            if constexpr (SPLIT) {
                u32x4_t wl = __builtin_bit_cast(u32x4_t, Plo[p][kk]);
                pin_here(wl);
                Plo[p][kk] = __builtin_bit_cast(vec8, wl);
            }
        }
        pin_here(l_run);
        __builtin_amdgcn_sched_barrier(0);
    };

    std::integral_constant<int, 0> even;
    std::integral_constant<int, 1> odd;

    // prologue: K'(0)
    if constexpr (QB == 0) {
        load_tile(Kg, ks0, 0, true);
    } else {
        fetch_codes(Kg, Kpg, 0, kst);
        store_codes(ks0, kst, true);
    }
    alph[0] = alph[1] = 1.0f;
    __syncthreads();

    // iterations t = 0 .. n_tiles; the steady-state ones (1 <= t, t + 1 < n_tiles, no hidden keys) run with every
    // stage on and without the masking code
    iteration(0, even, false, true, n_tiles > 1, true);
    __syncthreads();
    int t = 1;
    for (; t + 2 < n_tiles && t + 1 < t_mask0; t += 2) {
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
    if (q_row < Lq_rows) {
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

template <class T, int D, bool CAUSAL, int QB = 0>
static hipError_t launch_prefill_t(const AttnProblem& p, hipStream_t stream) {
    typedef typename T::elem elem;
    const float scale_log2 = p.scale * kLog2e;
    // Without a mask or per-sequence query counts a row's position in its head means nothing, and the query heads of
    // a KV head are contiguous in Q, O and lse: the kernel then sees one head of G * Lq rows per KV head, so that
    // short segments fill their 256-row tiles (128 queries x 4 heads: 2 full tiles instead of 4 half-empty ones).
    const bool pack_group = !CAUSAL && !p.q_lens;
    const int Hq_k = pack_group ? p.Hkv : p.Hq;
    const int64_t Lq_k = pack_group ? (int64_t)(p.Hq / p.Hkv) * p.Lq : p.Lq;
    const int q_tiles = (int)((Lq_k + kPreQTile - 1) / kPreQTile);
    const int n_units = p.B * p.Hkv;
    // several runs: only the plain call (every key of every sequence, every query row, no mask) takes them
    KeyRuns runs = attn_runs_of(p);
    const bool one_run_only = CAUSAL || p.kv_lens || p.q_lens;
    if (one_run_only) {
        if (p.n_shards > 1) return hipErrorInvalidValue;
        runs.per[0] = runs.L[0] > 0 ? ((runs.L[0] + kPreK - 1) / kPreK) * kPreK : kPreK;
        runs.first[1] = 1;
        runs.n_runs = 1;
    }
    const int splits = runs.n_runs;
    if (splits < 1) return hipErrorInvalidValue;
    const int64_t rows = (int64_t)p.B * p.Hq * p.Lq;
    float* Odst = p.O;
    float* Ldst = p.lse;
    if (splits > 1) {
        if (!p.workspace || p.workspace_bytes < (size_t)splits * rows * (D + 1) * sizeof(float)) return hipErrorInvalidValue;
        Odst = (float*)p.workspace;
        Ldst = Odst + (size_t)splits * rows * D;
    }
    const int64_t per_unit = (int64_t)(Hq_k / p.Hkv) * q_tiles * splits;
    const int64_t grid = (int64_t)8 * ((n_units + 7) / 8) * per_unit;
    if (!grid_fits(grid)) return hipErrorInvalidValue;
    if (QB != 0 && (p.n_shards > 1 || !p.K_params || !p.V_params)) return hipErrorInvalidValue;
    hipLaunchKernelGGL((prefill_attn_kernel<T, D, CAUSAL, QB>), dim3((unsigned)grid), dim3(kPreThreads), 0, stream,
                       (const elem*)p.Q, runs, p.K_params, p.V_params, Hq_k, p.Hkv, Lq_k, p.kv_lens, p.q_lens,
                       q_tiles, n_units, scale_log2, Odst, Ldst);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess || splits == 1) return e;
    return launch_lse_merge(Odst, Ldst, splits, rows, D, p.O, p.lse, stream);
}

template <class T>
static hipError_t launch_prefill_d(const AttnProblem& p, hipStream_t stream) {
    if (p.quant_bits != 0) {  // K', V' as transport codes (never with the mask: the Inquirer's own K, V are plain)
        if (p.causal || (p.quant_bits != 8 && p.quant_bits != 4)) return hipErrorInvalidValue;
        if (p.quant_bits == 8)
            return p.D == 128 ? launch_prefill_t<T, 128, false, 8>(p, stream) : launch_prefill_t<T, 64, false, 8>(p, stream);
        return p.D == 128 ? launch_prefill_t<T, 128, false, 4>(p, stream) : launch_prefill_t<T, 64, false, 4>(p, stream);
    }
    if (p.causal)
        return p.D == 128 ? launch_prefill_t<T, 128, true>(p, stream) : launch_prefill_t<T, 64, true>(p, stream);
    return p.D == 128 ? launch_prefill_t<T, 128, false>(p, stream) : launch_prefill_t<T, 64, false>(p, stream);
}

hipError_t launch_prefill_attn(const AttnProblem& p, hipStream_t stream) {
    return p.dtype == FEDRAG_BF16 ? launch_prefill_d<BF16>(p, stream) : launch_prefill_d<F16>(p, stream);
}

}  // namespace fedrag
