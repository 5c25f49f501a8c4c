// Enc / Dec row transforms (Section 4.2, scrambled attention protocol, steps 1 and 3):
//   gather form   Y[j,:]       = X[perm[j],:] . Phi      (feature scramble + token permutation)
//   scatter form  Y[perm[i],:] = X[i,:] . Phi            (descramble + inverse permutation)
// One d x d matrix per KV head, shared by the G query heads of its group.
//
// 16-bit storage path: HBM-bound (each row is read once and written once, 2*d^2 flop per 4*d bytes), so the
// d x d product runs on MFMA only to stay far below the memory time.  A wave owns 16 rows at a time:
// rows are fetched with full-row coalesced 16-byte loads, staged through a wave-private LDS tile into the
// MFMA operand layout, multiplied against Phi^T held in registers for the whole kernel, and the fp32
// results are narrowed once (RNE), transposed back through the same LDS tile and stored as full rows.
#include "fedrag_device.h"
#include "fedrag_host.h"

namespace fedrag {

// Two shapes of the tiled kernel.  Plain rows (QB = 0): 4 waves per workgroup, one per SIMD, Phi^T in 128 registers
// per wave for the whole kernel - the wave does little besides moving rows, and memory time hides it.  Rows that
// leave through the transport codec (QB = 8, 4): the codec's ~110 vector instructions per 8-element chunk need a
// second wave per SIMD to hide behind the other wave's memory time, and two waves only fit when Phi^T stays in LDS
// and its operands are read per tile (32 KiB of LDS reads per 8 KiB of rows: a few per cent of the LDS rate).
constexpr int scr_waves(int qb) { return qb ? 8 : 4; }
constexpr int kScrPad = 8;    // elements of row padding in LDS (16 bytes: keeps 16-byte alignment, breaks bank stride)
constexpr int kScrRows = 32;  // rows per wave step (two 16-row MFMA column tiles)
#ifndef FEDRAG_SCR_NBUF
#define FEDRAG_SCR_NBUF 3     // register row-tile sets per wave (ring); the codec shape uses 2
#endif
#ifndef FEDRAG_SCR_WGS
#define FEDRAG_SCR_WGS 256    // workgroups to aim for over the whole launch (one per CU)
#endif

struct ScrambleJob {
    const void* X;
    const void* Phi;       // dense form: [Hkv, D, D]
    void* Y;
    // structured form (Section 4.2, Phi = S1 P1 H P2 S2), [Hkv, D] each; see structured_entry()
    const float* s_in;
    const int32_t* p_in;
    const int32_t* p_out;
    const float* s_out;
    // quantised output (transport codec of Section 7.5 applied to the narrowed rows): Y holds the codes, params the
    // per-row (scale, lo)
    float* params;
};

// Entry (k, n) of S1 P1 Hs P2 with the permutations as gathers and Hs the +-1 Sylvester matrix:
//   x S1 P1 Hs P2 = sum_k x[k] s_in[k] Hs[p_in^{-1}(k)][p_out[n]],   Hs[i][m] = (-1)^popcount(i & m).
// The 1/sqrt(d) of the normalised Hadamard matrix and S2 are applied to the fp32 sums afterwards, so that every
// product in the sums is x[k] times +-s_in[k] and nothing is rounded before the accumulation.
__device__ __forceinline__ float structured_entry(float s_in_k, int p_in_inv_k, int p_out_n) {
    return (__builtin_popcount(p_in_inv_k & p_out_n) & 1) ? -s_in_k : s_in_k;
}

// blockIdx.x = (head * members + member) * b_groups + bg; blockIdx.y selects the job (K or V).
// The `members` workgroups of one (job, head) share that head's Phi and sweep the sequences b = 0..B-1 together:
// every [L, d] slab is cut into 128-row groups dealt round-robin to the members, and the 4 waves of a member take
// the 32-row tiles of its group.  So at any moment the members of a (job, head) write one contiguous window that
// moves down the slab, the windows of all jobs and heads sit at the same offset inside their slabs (measured: a few
// per cent faster than one contiguous part per member, and than windows at staggered offsets), and Phi is staged
// once per workgroup for all sequences.  (When the slabs are too
// short to occupy the chip that way - decode queries - the sequences are dealt to b_groups workgroups instead.)
// A ring of NBUF register tile sets keeps NBUF-1 gathered tiles (8 KiB each) in flight per wave behind the LDS
// staging and the MFMAs (it runs straight through the slab boundaries); the gather indices of a tile are fetched
// one step before its rows.  Tiles that start past the end of a slab are computed on clamped rows and not stored.
// QB = 0: rows leave in the storage type.  QB = 8 or 4: each narrowed row goes through the transport codec instead
// (same arithmetic as quantize_rows_kernel on the stored row) and leaves as codes plus (scale, lo).
template <class T, int D, bool ST, int QB>
__global__ __launch_bounds__(scr_waves(QB) * kWave, 1) void scramble_rows_kernel(ScrambleJob job0, ScrambleJob job1,
                                                                       const int32_t* __restrict__ perm,
                                                                       int64_t perm_batch_stride,  // 0 or L
                                                                       int B, int H, int G, int64_t L, int members,
                                                                       int tiles_per_slab, int b_groups) {
    typedef typename T::elem elem;
    typedef typename T::vec8 vec8;
    typedef typename T::vec4 vec4;
    constexpr int LDP = D + kScrPad;
    constexpr int CH = D / 8;              // 16-byte chunks per row
    constexpr int RPI = kWave / CH;        // rows covered by one wave-wide 16-byte load
    constexpr int NI = kScrRows / RPI;     // wave-wide loads per 32-row tile
    constexpr int KS = D / 32;             // contraction steps
    constexpr int MT = D / 16;             // output-column tiles
    constexpr int kScrWaves = scr_waves(QB);
    constexpr int kScrThreads = kScrWaves * kWave;
    constexpr bool kScrPhiLds = QB != 0;
    constexpr int NBUF = QB ? 2 : FEDRAG_SCR_NBUF;
    constexpr int kPhiElems = D * LDP;
    constexpr int kTileElems = kScrWaves * kScrRows * LDP;
    constexpr int kLdsElems = kScrPhiLds ? kPhiElems + kTileElems : (kPhiElems > kTileElems ? kPhiElems : kTileElems);

    // Phi^T staging and the per-wave row tiles share one buffer when the operands are copied into registers (Phi^T
    // is then only needed until every wave has done so); with kScrPhiLds Phi^T stays and the row tiles follow it.
    __shared__ __attribute__((aligned(16))) elem lds[kLdsElems];

    const ScrambleJob job = blockIdx.y == 0 ? job0 : job1;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);  // wave-uniform
    const int lane = tid % kWave;
    const int h = blockIdx.x / (members * b_groups);
    const int member = (blockIdx.x / b_groups) % members;
    const int bg = blockIdx.x % b_groups;  // this workgroup takes sequences bg, bg + b_groups, ...

    // ---- stage Phi^T[n][k] = Phi[k][n] in LDS (once per workgroup) ----
    __shared__ int32_t p_in_inv[ST ? D : 1];
    if (ST) {
        // structured form: the matrix is S1 P1 Hs P2, generated here from the key (entries +-s_in[k], which the
        // storage type holds exactly by the caller's contract); indices are masked into range
        const int32_t* g1 = job.p_in + (int64_t)(h / G) * D;
        for (int k = tid; k < D; k += kScrThreads) p_in_inv[g1[k] & (D - 1)] = k;
        __syncthreads();
        const float* a = job.s_in + (int64_t)(h / G) * D;
        const int32_t* g2 = job.p_out + (int64_t)(h / G) * D;
        for (int c = tid; c < D * D; c += kScrThreads) {
            const int n = c / D;
            const int k = c % D;
            lds[n * LDP + k] = T::from_float(structured_entry(a[k], p_in_inv[k], g2[n] & (D - 1)));
        }
    } else {
        const elem* P = (const elem*)job.Phi + (int64_t)(h / G) * D * D;
        for (int c = tid; c < D * CH; c += kScrThreads) {
            const int k = c / CH;
            const int n0 = (c % CH) * 8;
            const vec8 v = *(const vec8*)(P + k * D + n0);
#pragma unroll
            for (int e = 0; e < 8; ++e) lds[(n0 + e) * LDP + k] = v[e];
        }
    }
    __syncthreads();

    // Phi^T operands for the whole kernel: phi[mt][ks] = Phi^T[16 mt + lane%16][32 ks + 8 (lane/16) .. +8]
    const int lr = lane % 16;
    const int lq = lane / 16;
    vec8 phi[kScrPhiLds ? 1 : MT][kScrPhiLds ? 1 : KS];
    if constexpr (!kScrPhiLds) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                phi[mt][ks] = *(const vec8*)(&lds[(mt * 16 + lr) * LDP + ks * 32 + lq * 8]);
        __syncthreads();  // Phi^T is dead from here on; the buffer becomes the row tiles
    }
    const elem* phi_lds = &lds[lr * LDP + lq * 8];  // kScrPhiLds: operand (mt, ks) at + mt * 16 * LDP + ks * 32
    // structured form: S2 and the Hadamard normalisation, for this lane's output columns 16 mt + 4 lq + r
    f32x4_t post[ST ? MT : 1];
    if (ST) {
        const float* b = job.s_out + (int64_t)(h / G) * D;
        const float norm = D == 128 ? 0.08838834764831845f : 0.125f;  // 1 / sqrt(D)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) post[mt][r] = b[mt * 16 + lq * 4 + r] * norm;
    }

    elem* my = lds + (kScrPhiLds ? kPhiElems : 0) + wave * (kScrRows * LDP);

    const int ld_row = lane / CH;        // row within one wave-wide load
    const int ld_col = (lane % CH) * 8;  // element offset of this lane's 16 bytes

    // tile i of this wave: sequence b = i / tiles_per_slab, k-th tile of the wave inside this member's part
    const int n_mine = ((B - bg + b_groups - 1) / b_groups) * tiles_per_slab;
    auto tile_b = [&](int i) { return bg + (i / tiles_per_slab) * b_groups; };
    auto tile_row0 = [&](int i) {
        const int k = i % tiles_per_slab;
        return ((int64_t)(k * members + member) * kScrWaves + wave) * kScrRows;
    };
    auto slab_off = [&](int i) { return ((int64_t)tile_b(i) * H + h) * L * D; };
    const elem* Xj = (const elem*)job.X;
    elem* Yj = (elem*)job.Y;

    // gather indices of a tile: lane l (< 32) holds the source row of tile row l; rows past the end re-read
    // row L-1 (computed, never stored)
    auto load_idx = [&](int i) -> int32_t {
        if (i >= n_mine) i = n_mine - 1;  // the index prefetch runs one tile past the end
        int64_t j = tile_row0(i) + (lane % kScrRows);
        if (j >= L) j = L - 1;
        return perm ? perm[(int64_t)tile_b(i) * perm_batch_stride + j] : (int32_t)j;
    };
    auto load_rows = [&](int i, int32_t idx, vec8 (&buf)[NI]) {
        const elem* X = Xj + slab_off(i);
#pragma unroll
        for (int k = 0; k < NI; ++k) {
            const int64_t src = __shfl(idx, k * RPI + ld_row);
            buf[k] = __builtin_nontemporal_load((const vec8*)(X + src * D + ld_col));
        }
    };

    auto step = [&](vec8 (&buf)[NI], int i, bool reload, int32_t& idx_next) {
        const int64_t row0 = tile_row0(i);
        elem* Y = Yj + slab_off(i);
        // rows -> LDS tile
#pragma unroll
        for (int k = 0; k < NI; ++k) *(vec8*)(&my[(k * RPI + ld_row) * LDP + ld_col]) = buf[k];
        wave_lds_fence();
        if (reload) {  // refill this register set with the tile NBUF steps ahead, then fetch the indices after it
            load_rows(i + NBUF, idx_next, buf);
            idx_next = load_idx(i + NBUF + 1);
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            // kScrPhiLds: an offset the compiler cannot see through (always 0), so that the Phi^T operand reads
            // stay with the MFMAs that use them instead of being hoisted into 128 registers again
            int phi_off = 0;
            if constexpr (kScrPhiLds) pin_here(phi_off);
            const elem* phi_t = phi_lds + phi_off;
            // X^T operands: column = row (16 half + lane%16) of the tile, contraction slice 32 ks + 8 (lane/16)
            vec8 xop[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                xop[ks] = *(const vec8*)(&my[(half * 16 + lr) * LDP + ks * 32 + lq * 8]);
            // Y^T tile (d x 16 rows) = Phi^T . X^T : lane holds tile row lane%16, output columns 16 mt + 4 lq + r
            f32x4_t acc[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc[mt] = zero_vec<f32x4_t>();
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    if constexpr (kScrPhiLds)
                        acc[mt] = T::mfma16(*(const vec8*)(phi_t + mt * 16 * LDP + ks * 32), xop[ks], acc[mt]);
                    else
                        acc[mt] = T::mfma16(phi[mt][ks], xop[ks], acc[mt]);
                }
            }
            // the 16 rows of this half are only read by the operand loads above (same wave, in order):
            // overwrite them with the narrowed results
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                vec4 o;
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r] = T::from_float(ST ? acc[mt][r] * post[mt][r] : acc[mt][r]);
                *(vec4*)(&my[(half * 16 + lr) * LDP + mt * 16 + lq * 4]) = o;
            }
        }
        wave_lds_fence();
        // full-row stores
#pragma unroll
        for (int k = 0; k < NI; ++k) {
            const int64_t j = row0 + k * RPI + ld_row;
            const vec8 v = *(const vec8*)(&my[(k * RPI + ld_row) * LDP + ld_col]);
            if (QB == 0) {
                if (j < L) __builtin_nontemporal_store(v, (vec8*)(Y + j * D + ld_col));
            } else {
                // the row is spread over CH consecutive lanes, 8 channels each
                constexpr int LEVELS = (1 << (QB ? QB : 1)) - 1;
                float x[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = T::to_float(v[e]);
                float lo = x[0], hi = x[0];
#pragma unroll
                for (int e = 1; e < 8; ++e) { lo = fminf(lo, x[e]); hi = fmaxf(hi, x[e]); }
                lo = group_min<CH>(lo);
                hi = group_max<CH>(hi);
                const float range = hi - lo;
                const float scale = range / (float)LEVELS;
                // x - lo >= 0, so the sum is >= 1/2: converting to unsigned truncates = floors, and only the upper
                // clamp can act; a constant row (range 0) gets steps 0, hence code 0
                const float steps = range > 0.0f ? (float)LEVELS / range : 0.0f;
                // 8 bits: floor, then the conversion to a byte, which saturates at 255 (the upper clamp of the
                // definition; the argument is >= 1/2, so there is no lower one) and packs the code into its place
                uint32_t q[8];
                u32x2_t w8;
                w8[0] = w8[1] = 0u;
                if (QB == 8) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint32_t old = e < 4 ? w8[0] : w8[1];
                        const uint32_t nw = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_floorf(__builtin_fmaf(x[e] - lo, steps, 0.5f)), e % 4, old);
                        if (e < 4) w8[0] = nw;
                        else w8[1] = nw;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        q[e] = (uint32_t)fminf(__builtin_fmaf(x[e] - lo, steps, 0.5f), (float)LEVELS);
                }
                if (j < L) {
                    const int64_t row = slab_off(i) / D + j;  // row index over the whole tensor
                    uint8_t* out = (uint8_t*)job.Y + row * (D * QB / 8);
                    if (QB == 8) {
                        __builtin_nontemporal_store(w8, (u32x2_t*)(out + (lane % CH) * 8));
                    } else {
                        const uint32_t w = q[0] | (q[1] << 4) | (q[2] << 8) | (q[3] << 12) | (q[4] << 16) |
                                           (q[5] << 20) | (q[6] << 24) | (q[7] << 28);
                        __builtin_nontemporal_store(w, (uint32_t*)(out + (lane % CH) * 4));
                    }
                    if (lane % CH == 0) {
                        job.params[2 * row] = scale;
                        job.params[2 * row + 1] = lo;
                    }
                }
            }
        }
        wave_lds_fence();  // reads of the output tile done before the next tile's rows land
    };

    vec8 buf[NBUF][NI];
    int32_t idx_next = 0;
#pragma unroll
    for (int j = 0; j < NBUF; ++j)
        if (j < n_mine) load_rows(j, load_idx(j), buf[j]);
    if (NBUF < n_mine) idx_next = load_idx(NBUF);
    int i = 0;
    // steady state: tiles i+NBUF .. exist for every set, index prefetch may run one tile past the end (clamped)
    for (; i + 2 * NBUF <= n_mine; i += NBUF) {
#pragma unroll
        for (int j = 0; j < NBUF; ++j) step(buf[j], i + j, true, idx_next);
    }
#pragma unroll
    for (int j = 0; j < NBUF; ++j) {
        if (i + j < n_mine) {
            if (i + j + NBUF < n_mine) step(buf[j], i + j, true, idx_next);
            else step(buf[j], i + j, false, idx_next);
        }
    }
#pragma unroll
    for (int j = 0; j < NBUF; ++j)
        if (i + NBUF + j < n_mine) step(buf[j], i + NBUF + j, false, idx_next);
}

// A handful of rows per head (the decoding step's queries): the tiled kernel above would stage a whole matrix per
// workgroup through LDS and registers for one or two rows.  Here a workgroup takes one (sequence, head) slab of at
// most kFewRows rows; thread (c, rg) owns output column c, reads column c of Phi straight from memory (coalesced
// over c, every load independent), takes the rows from LDS as fp32 broadcasts and narrows each fp32 sum once.
constexpr int kFewRows = 16;
constexpr int kF32Threads = 256;  // workgroup size of the plain-FMA kernels

template <class T, int D, bool ST>
__global__ __launch_bounds__(kF32Threads) void scramble_few_rows_kernel(ScrambleJob job0, ScrambleJob job1,
                                                                        const int32_t* __restrict__ perm,
                                                                        int64_t perm_batch_stride, int H, int G,
                                                                        int L) {
    typedef typename T::elem elem;
    constexpr int RG = kF32Threads / D;
    __shared__ float xs[kFewRows * D];
    __shared__ int32_t p_in_inv[ST ? D : 1];
    __shared__ float s_in[ST ? D : 1];
    const ScrambleJob job = blockIdx.y == 0 ? job0 : job1;
    const int tid = threadIdx.x;
    const int c = tid % D;
    const int rg = tid / D;
    const int bh = blockIdx.x;
    const int b = bh / H;
    const int h = bh % H;
    const elem* X = (const elem*)job.X + (int64_t)bh * L * D;
    elem* Y = (elem*)job.Y + (int64_t)bh * L * D;
    const int32_t* pm = perm ? perm + (int64_t)b * perm_batch_stride : nullptr;
    for (int e = tid; e < L * D; e += kF32Threads) {
        const int j = e / D;
        const int64_t src = pm ? (int64_t)pm[j] : j;
        xs[e] = T::to_float(X[src * D + e % D]);
    }
    float phi[D];
    float post = 1.0f;
    if (ST) {
        const int32_t* g1 = job.p_in + (int64_t)(h / G) * D;
        for (int k = tid; k < D; k += kF32Threads) {
            p_in_inv[g1[k] & (D - 1)] = k;
            // the matrix entries are +-scale_in narrowed to the storage type, as in the tiled kernel
            s_in[k] = T::to_float(T::from_float(job.s_in[(int64_t)(h / G) * D + k]));
        }
        __syncthreads();
        const int m = job.p_out[(int64_t)(h / G) * D + c] & (D - 1);
        post = job.s_out[(int64_t)(h / G) * D + c] * (D == 128 ? 0.08838834764831845f : 0.125f);
#pragma unroll
        for (int k = 0; k < D; ++k) phi[k] = structured_entry(s_in[k], p_in_inv[k], m);
    } else {
        const elem* P = (const elem*)job.Phi + (int64_t)(h / G) * D * D;
#pragma unroll
        for (int k = 0; k < D; ++k) phi[k] = T::to_float(P[k * D + c]);
    }
    __syncthreads();
    for (int r = rg; r < L; r += RG) {
        float acc = 0.f;
#pragma unroll
        for (int k4 = 0; k4 < D; k4 += 4) {
            const f32x4_t x = *(const f32x4_t*)(&xs[r * D + k4]);
            acc = __builtin_fmaf(x[0], phi[k4 + 0], acc);
            acc = __builtin_fmaf(x[1], phi[k4 + 1], acc);
            acc = __builtin_fmaf(x[2], phi[k4 + 2], acc);
            acc = __builtin_fmaf(x[3], phi[k4 + 3], acc);
        }
        Y[(int64_t)r * D + c] = T::from_float(ST ? acc * post : acc);
    }
}

// fp32 rows times fp32 matrix with plain FMAs (fp32 storage path of Enc, and Dec for every storage type).
// Thread (c, rg) owns output column c and holds column c of Phi in registers; rows are broadcast from LDS.
//   SCATTER == false: Y[j]       = X[perm[j]] . Phi   (perm NULL = identity)
//   SCATTER == true : Y[perm[i]] = X[i] . Phi
constexpr int kF32Rows = 32;

// mg.lse_in != NULL (scatter form only): the transformed row is one of two partials of Section 4.1 and is
// aggregated with the other one, which is already in destination order, before it is stored - the same arithmetic,
// in the same order, as lse_merge_kernel over (this row, the other partial).
template <int D, bool SCATTER, bool ST>
__global__ __launch_bounds__(kF32Threads) void rows_times_matrix_f32_kernel(ScrambleJob job0, ScrambleJob job1,
                                                                            const int32_t* __restrict__ perm,
                                                                            int64_t perm_batch_stride, int H, int G,
                                                                            int64_t L, int chunks, int tiles_per_wg,
                                                                            RowsMerge mg) {
    constexpr int RG = kF32Threads / D;  // row groups
    __shared__ __attribute__((aligned(16))) float xs[kF32Rows * D];
    const ScrambleJob job = blockIdx.y == 0 ? job0 : job1;
    const int tid = threadIdx.x;
    const int c = tid % D;
    const int rg = tid / D;
    const int bh = blockIdx.x / chunks;
    const int chunk = blockIdx.x % chunks;
    const int b = bh / H;
    const int h = bh % H;
    float phi[D];
    __shared__ int32_t p_in_inv[ST ? D : 1];
    __shared__ float s_in[ST ? D : 1];
    if (ST) {  // column c of S1 P1 H P2 S2, generated from the key
        const int32_t* g1 = job.p_in + (int64_t)(h / G) * D;
        for (int k = tid; k < D; k += kF32Threads) {
            p_in_inv[g1[k] & (D - 1)] = k;
            s_in[k] = job.s_in[(int64_t)(h / G) * D + k];
        }
        __syncthreads();
        const int m = job.p_out[(int64_t)(h / G) * D + c] & (D - 1);
        const float post = job.s_out[(int64_t)(h / G) * D + c] * (D == 128 ? 0.08838834764831845f : 0.125f);
#pragma unroll
        for (int k = 0; k < D; ++k) phi[k] = structured_entry(s_in[k], p_in_inv[k], m) * post;
    } else {
        const float* P = (const float*)job.Phi + (int64_t)(h / G) * D * D;
#pragma unroll
        for (int k = 0; k < D; ++k) phi[k] = P[k * D + c];
    }

    const float* X = (const float*)job.X + (int64_t)bh * L * D;
    float* Y = (float*)job.Y + (int64_t)bh * L * D;
    const int32_t* pm = perm ? perm + (int64_t)b * perm_batch_stride : nullptr;

    int64_t row0 = (int64_t)chunk * tiles_per_wg * kF32Rows;
    for (int t = 0; t < tiles_per_wg && row0 < L; ++t, row0 += kF32Rows) {
        __syncthreads();
        for (int e = tid; e < kF32Rows * (D / 4); e += kF32Threads) {
            const int r = e / (D / 4);
            const int c4 = (e % (D / 4)) * 4;
            int64_t j = row0 + r;
            if (j >= L) j = L - 1;
            const int64_t src = (!SCATTER && pm) ? (int64_t)pm[j] : j;
            *(f32x4_t*)(&xs[r * D + c4]) = *(const f32x4_t*)(X + src * D + c4);
        }
        __syncthreads();
        for (int r = rg; r < kF32Rows; r += RG) {
            const int64_t j = row0 + r;
            if (j >= L) break;
            float acc = 0.f;
#pragma unroll
            for (int k4 = 0; k4 < D; k4 += 4) {
                const f32x4_t x = *(const f32x4_t*)(&xs[r * D + k4]);
                acc = __builtin_fmaf(x[0], phi[k4 + 0], acc);
                acc = __builtin_fmaf(x[1], phi[k4 + 1], acc);
                acc = __builtin_fmaf(x[2], phi[k4 + 2], acc);
                acc = __builtin_fmaf(x[3], phi[k4 + 3], acc);
            }
            const int64_t dst = (SCATTER && pm) ? (int64_t)pm[j] : j;
            if (SCATTER && mg.lse_in) {
                const float la = mg.lse_in[(int64_t)bh * L + j];
                const float lb = mg.lse_other[(int64_t)bh * L + dst];
                const float M = fmaxf(fmaxf(-INFINITY, la), lb);
                float o = 0.f, den = 0.f;
                if (M != -INFINITY) {
                    if (la != -INFINITY) {
                        const float a = expf(la - M);
                        den += a;
                        o = __builtin_fmaf(a, acc, o);
                    }
                    if (lb != -INFINITY) {
                        const float a = expf(lb - M);
                        den += a;
                        o = __builtin_fmaf(a, mg.O_other[((int64_t)bh * L + dst) * D + c], o);
                    }
                    o *= 1.0f / den;
                }
                acc = o;
                if (c == 0) mg.lse_out[(int64_t)bh * L + dst] = (M == -INFINITY) ? -INFINITY : M + logf(den);
            }
            Y[dst * D + c] = acc;
        }
    }
}

// The same product on the fp32 matrix cores, for slabs of at least kMfMinRows rows (the plain kernel above spends
// its time on LDS broadcasts of the rows: 122 us for 65536 rows of 128, against 10 us of HBM time).
// v_mfma_f32_32x32x2_f32: A 32 x 2 (lane: row lane % 32, k = lane / 32), B 2 x 32 (lane: column lane % 32, k = lane / 32),
// C 32 x 32 (lane: column lane % 32, register r: row 8 (r / 4) + 4 (lane / 32) + r % 4).  Wave w of the 4 owns the
// 32-column slice w % (D / 32) of the output and keeps that slice of Phi in registers as B operands (D / 2 of them);
// the rows of a step (32 for D = 128, two tiles of 32 for D = 64) are staged once in LDS, coalesced, and every wave
// reads its tile's rows from there 16 bytes at a time: the 4 floats are the A operands of 4 steps, contraction index
// 8 j + 4 (lane / 32) + e for read j, element e.  The next step's rows are fetched into registers before the MFMAs
// of the current one and go to the other LDS buffer after them: one barrier per step.
constexpr int kMfMinRows = 64;
#ifndef FEDRAG_MF_WANT_WGS
#define FEDRAG_MF_WANT_WGS 512
#endif

template <int D, bool SCATTER, bool ST>
__global__ __launch_bounds__(kF32Threads) void rows_times_matrix_mfma_f32_kernel(ScrambleJob job0, ScrambleJob job1,
                                                                                 const int32_t* __restrict__ perm,
                                                                                 int64_t perm_batch_stride, int H,
                                                                                 int G, int64_t L, int chunks,
                                                                                 int steps_per_wg, RowsMerge mg) {
    constexpr int SL = D / 32;         // 32-column slices of the output
    constexpr int RT = 4 / SL;         // 32-row tiles per step
    constexpr int TR = 32 * RT;        // rows per step
    constexpr int LDP = D + 4;         // padded LDS row, floats: 16-byte reads of 8 rows cover all banks once
    constexpr int NJ = D / 8;          // 16-byte operand reads per row
    constexpr int CPR = D / 4;         // 16-byte chunks per row
    constexpr int CPT = TR * CPR / kF32Threads;  // chunks per thread per step
    static_assert(CPT * kF32Threads == TR * CPR, "a step's rows divide evenly over the threads");
    __shared__ __attribute__((aligned(16))) float xs[2][TR * LDP];
    __shared__ int32_t p_in_inv[ST ? D : 1];
    __shared__ float s_in[ST ? D : 1];

    const ScrambleJob job = blockIdx.y == 0 ? job0 : job1;
    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const int lane = tid % kWave;
    const int n = lane % 32;
    const int kk = lane / 32;
    const int slice = wave % SL;
    const int rt = wave / SL;
    const int bh = blockIdx.x / chunks;
    const int chunk = blockIdx.x % chunks;
    const int b = bh / H;
    const int h = bh % H;
    const int64_t first_row = (int64_t)chunk * steps_per_wg * TR;
    if (first_row >= L) return;  // workgroup-uniform, before any barrier
    int n_steps = (int)((L - first_row + TR - 1) / TR);
    if (n_steps > steps_per_wg) n_steps = steps_per_wg;

    const int col = 32 * slice + n;  // this lane's output column
    float phi[NJ][4];
    if (ST) {  // column `col` of S1 P1 H P2 S2, generated from the key
        const int32_t* g1 = job.p_in + (int64_t)(h / G) * D;
        for (int k = tid; k < D; k += kF32Threads) {
            p_in_inv[g1[k] & (D - 1)] = k;
            s_in[k] = job.s_in[(int64_t)(h / G) * D + k];
        }
        __syncthreads();
        const int m = job.p_out[(int64_t)(h / G) * D + col] & (D - 1);
        const float post = job.s_out[(int64_t)(h / G) * D + col] * (D == 128 ? 0.08838834764831845f : 0.125f);
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k = 8 * j + 4 * kk + e;
                phi[j][e] = structured_entry(s_in[k], p_in_inv[k], m) * post;
            }
    } else {
        const float* P = (const float*)job.Phi + (int64_t)(h / G) * D * D;
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) phi[j][e] = P[(8 * j + 4 * kk + e) * D + col];
    }

    const float* X = (const float*)job.X + (int64_t)bh * L * D;
    float* Y = (float*)job.Y + (int64_t)bh * L * D;
    const int32_t* pm = perm ? perm + (int64_t)b * perm_batch_stride : nullptr;

    auto fetch = [&](int64_t row0, f32x4_t (&buf)[CPT]) {
#pragma unroll
        for (int q = 0; q < CPT; ++q) {
            const int e = tid + q * kF32Threads;
            int64_t j = row0 + e / CPR;
            if (j >= L) j = L - 1;  // rows past the end: computed on a real row, never stored
            const int64_t src = (!SCATTER && pm) ? (int64_t)pm[j] : j;
            buf[q] = *(const f32x4_t*)(X + src * D + (e % CPR) * 4);
        }
    };
    auto stash = [&](int slot, const f32x4_t (&buf)[CPT]) {
#pragma unroll
        for (int q = 0; q < CPT; ++q) {
            const int e = tid + q * kF32Threads;
            *(f32x4_t*)(&xs[slot][(e / CPR) * LDP + (e % CPR) * 4]) = buf[q];
        }
    };

    f32x4_t buf[CPT];
    fetch(first_row, buf);
    stash(0, buf);
    __syncthreads();
    for (int s_ = 0; s_ < n_steps; ++s_) {
        const int64_t row0 = first_row + (int64_t)s_ * TR;
        const bool more = s_ + 1 < n_steps;
        if (more) fetch(row0 + TR, buf);
        const float* xr = &xs[s_ & 1][(32 * rt + n) * LDP + 4 * kk];
        f32x16_t acc = zero_vec<f32x16_t>();
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const f32x4_t a = *(const f32x4_t*)(xr + 8 * j);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], phi[j][e], acc, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t j = row0 + 32 * rt + 8 * (r / 4) + 4 * kk + (r % 4);
            if (j >= L) continue;
            const int64_t dst = (SCATTER && pm) ? (int64_t)pm[j] : j;
            float v = acc[r];
            if (SCATTER && mg.lse_in) {
                const float la = mg.lse_in[(int64_t)bh * L + j];
                const float lb = mg.lse_other[(int64_t)bh * L + dst];
                const float M = fmaxf(fmaxf(-INFINITY, la), lb);
                float o = 0.f, den = 0.f;
                if (M != -INFINITY) {
                    if (la != -INFINITY) {
                        const float a = expf(la - M);
                        den += a;
                        o = __builtin_fmaf(a, v, o);
                    }
                    if (lb != -INFINITY) {
                        const float a = expf(lb - M);
                        den += a;
                        o = __builtin_fmaf(a, mg.O_other[((int64_t)bh * L + dst) * D + col], o);
                    }
                    o *= 1.0f / den;
                }
                v = o;
                if (col == 0) mg.lse_out[(int64_t)bh * L + dst] = (M == -INFINITY) ? -INFINITY : M + logf(den);
            }
            Y[dst * D + col] = v;
        }
        if (more) stash((s_ + 1) & 1, buf);
        __syncthreads();
    }
}

__global__ void invert_perm_kernel(const int32_t* __restrict__ perm, int64_t L, int32_t* __restrict__ inv) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j < L) inv[perm[j]] = (int32_t)j;
}

// Debug aid: is every row of perm [n_perm, L] a permutation of 0..L-1?  marks [n_perm, L] counts the hits of every
// index; flag receives bit 0 for an index outside [0, L) and bit 1 for an index that occurs more than once (every
// index in range and none twice means all L occur).
__global__ void validate_perm_clear_kernel(int32_t* __restrict__ marks, int64_t total, int32_t* __restrict__ flag) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e < total) marks[e] = 0;
    if (e == 0) flag[0] = 0;
}
__global__ void validate_perm_kernel(const int32_t* __restrict__ perm, int64_t L, int64_t total,
                                     int32_t* __restrict__ marks, int32_t* __restrict__ flag) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    const int64_t row = e / L;
    const int32_t p = perm[e];
    if (p < 0 || p >= L) atomicOr(flag, 1);
    else if (atomicAdd(&marks[row * L + p], 1) != 0) atomicOr(flag, 2);
}

// ------------------------------------------------------------------------------------------------ launchers
static int ceil_div_i64(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

static ScrambleJob device_job(const RowsJob& j, int i) {
    return ScrambleJob{j.X[i], j.Phi[i], j.Y[i], j.s_in[i], j.p_in[i], j.p_out[i], j.s_out[i], j.params[i]};
}

template <class T, int D>
static hipError_t launch_scramble16(const RowsJob& j, hipStream_t stream) {
    if (j.L <= kFewRows && j.quant_bits == 0) {
        if (!grid_fits(j.BH)) return hipErrorInvalidValue;
        dim3 grid((unsigned)j.BH, (unsigned)j.n_jobs);
        const ScrambleJob a = device_job(j, 0), b = device_job(j, 1);
        if (j.structured)
            hipLaunchKernelGGL((scramble_few_rows_kernel<T, D, true>), grid, dim3(kF32Threads), 0, stream, a, b, j.perm,
                               j.perm_batch_stride, j.H, j.G, (int)j.L);
        else
            hipLaunchKernelGGL((scramble_few_rows_kernel<T, D, false>), grid, dim3(kF32Threads), 0, stream, a, b, j.perm,
                               j.perm_batch_stride, j.H, j.G, (int)j.L);
        return hipGetLastError();
    }
    const int waves = scr_waves(j.quant_bits);
    const int64_t rows_per_pass = (int64_t)waves * kScrRows;  // rows one workgroup covers per ring step
    const int64_t passes = (j.L + rows_per_pass - 1) / rows_per_pass;  // per [L, d] slab
    // about one workgroup per CU over the whole launch, split evenly over (job, head); never more members than a
    // slab has passes
    int members = FEDRAG_SCR_WGS / (j.H * j.n_jobs);
    if (members < 1) members = 1;
    if ((int64_t)members > passes) members = (int)passes;
    const int tiles_per_slab = ceil_div_i64(passes, members);
    const int B = (int)(j.BH / j.H);
    int b_groups = FEDRAG_SCR_WGS / (j.H * j.n_jobs * members);  // leftover parallelism goes to the sequences
    if (b_groups < 1) b_groups = 1;
    if (b_groups > B) b_groups = B;
    dim3 grid((unsigned)(j.H * members * b_groups), (unsigned)j.n_jobs);
    const ScrambleJob a = device_job(j, 0), b = device_job(j, 1);
#define FEDRAG_SCR_LAUNCH(ST_, QB_)                                                                              \
    hipLaunchKernelGGL((scramble_rows_kernel<T, D, ST_, QB_>), grid, dim3(waves * kWave), 0, stream, a, b, j.perm, \
                       j.perm_batch_stride, B, j.H, j.G, j.L, members, tiles_per_slab, b_groups)
    if (j.structured) {
        if (j.quant_bits == 8) FEDRAG_SCR_LAUNCH(true, 8);
        else if (j.quant_bits == 4) FEDRAG_SCR_LAUNCH(true, 4);
        else FEDRAG_SCR_LAUNCH(true, 0);
    } else {
        if (j.quant_bits == 8) FEDRAG_SCR_LAUNCH(false, 8);
        else if (j.quant_bits == 4) FEDRAG_SCR_LAUNCH(false, 4);
        else FEDRAG_SCR_LAUNCH(false, 0);
    }
#undef FEDRAG_SCR_LAUNCH
    return hipGetLastError();
}

template <int D, bool SCATTER>
static hipError_t launch_rows_mfma_f32(const RowsJob& j, hipStream_t stream) {
    constexpr int TR = 32 * (4 / (D / 32));  // rows per workgroup step
    const int64_t steps = (j.L + TR - 1) / TR;
    // about two workgroups per compute unit, at most 64 steps each (a workgroup loads its slice of Phi once)
    const int64_t want_wgs = FEDRAG_MF_WANT_WGS;
    const int64_t total = steps * j.BH * j.n_jobs;
    int spw = (int)(total / want_wgs);
    if (spw < 1) spw = 1;
    if (spw > 64) spw = 64;
    const int chunks = ceil_div_i64(steps, spw);
    if (!grid_fits(j.BH * chunks)) return hipErrorInvalidValue;
    dim3 grid((unsigned)(j.BH * chunks), (unsigned)j.n_jobs);
    const ScrambleJob a = device_job(j, 0), b = device_job(j, 1);
    if (j.structured)
        hipLaunchKernelGGL((rows_times_matrix_mfma_f32_kernel<D, SCATTER, true>), grid, dim3(kF32Threads), 0, stream, a,
                           b, j.perm, j.perm_batch_stride, j.H, j.G, j.L, chunks, spw, j.merge);
    else
        hipLaunchKernelGGL((rows_times_matrix_mfma_f32_kernel<D, SCATTER, false>), grid, dim3(kF32Threads), 0, stream,
                           a, b, j.perm, j.perm_batch_stride, j.H, j.G, j.L, chunks, spw, j.merge);
    return hipGetLastError();
}

template <int D, bool SCATTER>
static hipError_t launch_rows_f32(const RowsJob& j, hipStream_t stream) {
    if (j.L >= kMfMinRows) return launch_rows_mfma_f32<D, SCATTER>(j, stream);
    const int64_t tiles = (j.L + kF32Rows - 1) / kF32Rows;
    const int64_t want_wgs = 2048;
    const int64_t total = tiles * j.BH * j.n_jobs;
    int tpw = (int)((total + want_wgs - 1) / want_wgs);
    if (tpw < 1) tpw = 1;
    if (tpw > 64) tpw = 64;
    const int chunks = ceil_div_i64(tiles, tpw);
    if (!grid_fits(j.BH * chunks)) return hipErrorInvalidValue;
    dim3 grid((unsigned)(j.BH * chunks), (unsigned)j.n_jobs);
    const ScrambleJob a = device_job(j, 0), b = device_job(j, 1);
    if (j.structured)
        hipLaunchKernelGGL((rows_times_matrix_f32_kernel<D, SCATTER, true>), grid, dim3(kF32Threads), 0, stream, a, b,
                           j.perm, j.perm_batch_stride, j.H, j.G, j.L, chunks, tpw, j.merge);
    else
        hipLaunchKernelGGL((rows_times_matrix_f32_kernel<D, SCATTER, false>), grid, dim3(kF32Threads), 0, stream, a, b,
                           j.perm, j.perm_batch_stride, j.H, j.G, j.L, chunks, tpw, j.merge);
    return hipGetLastError();
}

hipError_t launch_rows_transform(const RowsJob& j, hipStream_t stream) {
    if (j.L == 0 || j.BH == 0) return hipSuccess;
    if (j.scatter) {  // Dec: always fp32
        return j.D == 128 ? launch_rows_f32<128, true>(j, stream) : launch_rows_f32<64, true>(j, stream);
    }
    switch (j.dtype) {
        case FEDRAG_F32:
            return j.D == 128 ? launch_rows_f32<128, false>(j, stream) : launch_rows_f32<64, false>(j, stream);
        case FEDRAG_BF16:
            return j.D == 128 ? launch_scramble16<BF16, 128>(j, stream) : launch_scramble16<BF16, 64>(j, stream);
        case FEDRAG_F16:
            return j.D == 128 ? launch_scramble16<F16, 128>(j, stream) : launch_scramble16<F16, 64>(j, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_invert_perm(const int32_t* perm, int64_t L, int32_t* inv, hipStream_t stream) {
    if (L == 0) return hipSuccess;
    hipLaunchKernelGGL(invert_perm_kernel, dim3((unsigned)((L + 255) / 256)), dim3(256), 0, stream, perm, L, inv);
    return hipGetLastError();
}

hipError_t launch_validate_perm(const int32_t* perm, int n_perm, int64_t L, int32_t* marks, int32_t* flag,
                                hipStream_t stream) {
    const int64_t total = (int64_t)n_perm * L;
    if (!grid_fits((total > 0 ? total + 255 : 256) / 256)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((total > 0 ? total + 255 : 256) / 256));
    hipLaunchKernelGGL(validate_perm_clear_kernel, grid, dim3(256), 0, stream, marks, total, flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || total == 0) return e;
    hipLaunchKernelGGL(validate_perm_kernel, grid, dim3(256), 0, stream, perm, L, total, marks, flag);
    return hipGetLastError();
}

}  // namespace fedrag
