// The Compute Node's work on one KV shard (Section 4.1, per-node local computation):
//   O_i = softmax(Q' K_i'^T * scale) V_i'   and   lse_i = ln sum_t exp(Q' K_i'^T * scale)   (= ln w_i)
// evaluated with a running maximum so that outlier logits cannot overflow.  Three kernels:
//   attn_f32_kernel     (here)             fp32 storage, plain FMAs, one wave per query row (accuracy path)
//   decode_attn_kernel  (attn_decode.hip)  16-bit storage, <= 16 query rows per KV head: HBM-bound streaming
//   prefill_attn_kernel (attn_prefill.hip) 16-bit storage, many query rows: MFMA-bound tiled kernel
// This file holds the fp32 kernel and the dispatch between the three.
#include "fedrag_device.h"
#include "fedrag_host.h"

#include <atomic>
#include <climits>
#include <cstdint>

namespace fedrag {

// ------------------------------------------------------------------------------------------------ fp32 path
template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(const float* __restrict__ Q, const float* __restrict__ K,
                                                       const float* __restrict__ V, int Hq, int Hkv, int64_t Lq,
                                                       int64_t Lkv, int causal, int64_t total_rows, float scale,
                                                       float* __restrict__ O, float* __restrict__ lse,
                                                       const int32_t* __restrict__ kv_lens,
                                                       const int32_t* __restrict__ q_lens) {
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
    if (q_lens && (row % Lq) >= q_lens[b]) return;  // padding query row of a shorter sequence: not computed
    const float* q = Q + row * D;
    const float* Kg = K + ((int64_t)b * Hkv + g) * Lkv * D;
    const float* Vg = V + ((int64_t)b * Hkv + g) * Lkv * D;
    // keys this row sees: all of them, or (causal) those up to its own position among the last Lq tokens
    int64_t L = causal ? (row % Lq) + (Lkv - Lq) + 1 : Lkv;
    if (kv_lens) {  // padded batch of unequal sequences: only the first kv_lens[b] keys exist
        const int64_t v = kv_lens[b];
        const int64_t cap = v < 0 ? 0 : (v < Lkv ? v : Lkv);
        if (L > cap) L = cap;
    }
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

// ------------------------------------------------------------------------------------------------ dispatch
// Decode workgroups to aim for over the whole launch: one per CU (the kernel is sized for one resident
// workgroup per CU; a single round of equal-sized workgroups measured fastest).  256 CUs on MI355X; the
// attribute query is host-only and falls back to that number when no device is present.
#ifndef FEDRAG_DEC_WGS
static int decode_target_wgs() {
    // the count belongs to the device that is current in the calling thread; it is cached per device ordinal in
    // atomics, so concurrent first calls only repeat the query
    constexpr int kMaxDev = 64;
    static std::atomic<int> cached[kMaxDev];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) {
        (void)hipGetLastError();
        return 256;
    }
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
            (void)hipGetLastError();
            return 256;
        }
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}
#define FEDRAG_DEC_WGS decode_target_wgs()
#endif
#ifndef FEDRAG_DEC_MIN_STEPS
#define FEDRAG_DEC_MIN_STEPS 4
#endif
static bool use_decode_kernel(int Hq, int Hkv, int64_t Lq) { return (int64_t)(Hq / Hkv) * Lq <= 16; }

// Decode kernel: about one workgroup per compute unit over the whole launch; a run is a whole number of 128-key
// workgroup steps, at least 4 of them, and stays below 2^31 bytes (32-bit buffer offsets).
// Prefill kernel: one workgroup per (sequence, query head, 256 query rows) walks a run, about 2 us per 64-key tile.
// When those workgroups cover less than half of the compute units, the keys are cut into runs of at least
// kPreMinTilesPerSplit tiles (so that a workgroup's fixed cost stays small beside its tiles) for one round of
// workgroups over the chip; otherwise every shard is one run.
KeyRuns attn_plan_runs(int B, int Hq, int Hkv, int dtype, int64_t Lq, int n, const int64_t* Ls, bool codes4) {
    KeyRuns r;
    for (int i = 0; i < kMaxShards; ++i) {
        r.K[i] = r.V[i] = nullptr;
        r.L[i] = 0;
        r.per[i] = 1;
        r.first[i] = INT_MAX;
    }
    r.first[kMaxShards] = INT_MAX;
    r.n_runs = 0;
    if (n < 1 || n > kMaxShards) return r;
    int64_t total = 0;
    for (int i = 0; i < n; ++i) total += Ls[i] > 0 ? Ls[i] : 0;
    const bool decode = use_decode_kernel(Hq, Hkv, Lq);
    const int64_t cus = (int64_t)FEDRAG_DEC_WGS * ((codes4 && decode) ? kDecCodesOcc : 1);
    int64_t per = INT64_MAX;  // keys per run before rebalancing inside a shard
    int64_t quantum = 1;
    if (dtype != FEDRAG_F32 && total > 0 && Lq > 0) {
        if (decode) {
            const int64_t units = (int64_t)B * Hkv;
            const int64_t want = units > 0 ? (cus + units - 1) / units : 1;
            quantum = kDecStride;
            per = (total + want - 1) / want;
            per = ((per + quantum - 1) / quantum) * quantum;
            if (per < FEDRAG_DEC_MIN_STEPS * quantum) per = FEDRAG_DEC_MIN_STEPS * quantum;
            if (per > (int64_t)1 << 22) per = (int64_t)1 << 22;
        } else {
            // the query heads of a KV head form one run of G * Lq rows (see launch_prefill_t)
            const int64_t wgs = (int64_t)B * Hkv * (((int64_t)(Hq / Hkv) * Lq + kPreQTile - 1) / kPreQTile);
            quantum = kPreK;
            if (wgs > 0 && wgs * 2 <= cus) {
                const int64_t want = cus / wgs;
                const int64_t tiles = (total + kPreK - 1) / kPreK;
                int64_t per_t = (tiles + want - 1) / want;
                if (per_t < kPreMinTilesPerSplit) per_t = kPreMinTilesPerSplit;
                per = per_t * kPreK;
            }
        }
    }
    int at = 0;
    for (int i = 0; i < n; ++i) {
        const int64_t L = Ls[i] > 0 ? Ls[i] : 0;
        r.L[i] = L;
        r.first[i] = at;
        if (L == 0) continue;  // no runs: first[i] == first[i + 1]
        const int64_t runs = per == INT64_MAX ? 1 : (L + per - 1) / per;
        int64_t mine = (L + runs - 1) / runs;  // rebalanced inside the shard
        mine = ((mine + quantum - 1) / quantum) * quantum;
        r.per[i] = mine;
        at += (int)((L + mine - 1) / mine);
    }
    for (int i = n; i <= kMaxShards; ++i) r.first[i] = i == n ? at : INT_MAX;
    r.n_runs = at;
    return r;
}

KeyRuns attn_runs_of(const AttnProblem& p) {
    if (p.n_shards <= 1) {
        KeyRuns r = attn_plan_runs(p.B, p.Hq, p.Hkv, p.dtype, p.Lq, 1, &p.Lkv, p.quant_bits == 4 && p.D == 128);
        r.K[0] = p.K;
        r.V[0] = p.V;
        if (p.single_run && r.n_runs > 1) {  // all keys of the shard in one run (a whole number of key tiles)
            const int64_t q = use_decode_kernel(p.Hq, p.Hkv, p.Lq) ? kDecStride : kPreK;
            r.per[0] = ((r.L[0] + q - 1) / q) * q;
            r.first[1] = 1;
            r.n_runs = 1;
        }
        return r;
    }
    KeyRuns r = attn_plan_runs(p.B, p.Hq, p.Hkv, p.dtype, p.Lq, p.n_shards, p.Ls);
    for (int i = 0; i < p.n_shards && i < kMaxShards; ++i) {
        r.K[i] = p.Ks[i];
        r.V[i] = p.Vs[i];
    }
    return r;
}

bool attn_uses_decode_kernel(int Hq, int Hkv, int64_t Lq) { return use_decode_kernel(Hq, Hkv, Lq); }

size_t attn_workspace_bytes(int B, int Hq, int Hkv, int D, int dtype, int64_t Lq, int n, const int64_t* Ls) {
    // one size serves a call on 16-bit values and the same call on 4-bit transport codes (more, shorter runs)
    int runs = attn_plan_runs(B, Hq, Hkv, dtype, Lq, n, Ls, false).n_runs;
    if (n == 1 && D == 128 && dtype != FEDRAG_F32) {
        const int on_codes = attn_plan_runs(B, Hq, Hkv, dtype, Lq, n, Ls, true).n_runs;
        if (on_codes > runs) runs = on_codes;
    }
    if (runs <= 1) return 0;
    const size_t rows = (size_t)B * Hq * (size_t)Lq;
    return (size_t)runs * rows * (size_t)(D + 1) * sizeof(float);
}

template <int D>
static hipError_t launch_attn_f32(const AttnProblem& p, hipStream_t stream) {
    const int64_t rows = (int64_t)p.B * p.Hq * p.Lq;
    if (!grid_fits((rows + 3) / 4)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_f32_kernel<D>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, (const float*)p.Q,
                       (const float*)p.K, (const float*)p.V, p.Hq, p.Hkv, p.Lq, p.Lkv, p.causal ? 1 : 0, rows, p.scale,
                       p.O, p.lse, p.kv_lens, p.q_lens);
    return hipGetLastError();
}

// Scratch for callers that cannot allocate: the key-run partials of a launch land in this file-scope device array
// instead of a caller's workspace.  Every GPU the library runs on holds its own copy (at its own address) until the
// process ends.  The name below is only the host's handle for the symbol: the device address is looked up once per
// device, with that device current, and only that pointer is ever handed to a kernel.
namespace {
__attribute__((used)) static __device__ __align__(256) unsigned char scratch[FEDRAG_STATIC_SCRATCH_BYTES];
}

hipError_t attn_static_scratch(void** ptr_out) {
    constexpr int kMaxDev = 64;
    static std::atomic<void*> ptrs[kMaxDev];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDev) return hipErrorInvalidDevice;
    void* p = ptrs[dev].load(std::memory_order_acquire);
    if (!p) {  // first call on this device (concurrent first calls look the same address up twice)
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptrs[dev].store(p, std::memory_order_release);
    }
    *ptr_out = p;
    return hipSuccess;
}

hipError_t launch_partial_attn(const AttnProblem& p_in, hipStream_t stream) {
    AttnProblem p = p_in;
    if (p.Lq == 1) p.causal = false;  // a single query at the last position sees every key
    const int64_t rows = (int64_t)p.B * p.Hq * p.Lq;
    if (rows == 0) return hipSuccess;
    if (p.n_shards > 1) {
        if (p.n_shards > kMaxShards || p.quant_bits != 0 || p.causal || p.kv_lens || p.q_lens) return hipErrorInvalidValue;
        int64_t total = 0;
        for (int i = 0; i < p.n_shards; ++i) total += p.Ls[i];
        if (total == 0) return launch_fill_empty(p.O, p.lse, rows, p.D, stream);
        const bool decode = use_decode_kernel(p.Hq, p.Hkv, p.Lq);
        bool one_launch_per_shard = p.dtype == FEDRAG_F32;  // the accuracy path has no run table
        if (!one_launch_per_shard && (!decode || (int64_t)p.B * p.Hkv >= decode_target_wgs())) {
            // The chip is already covered by one shard's workgroups (prefill: query tiles; decode: as many
            // (sequence, KV head) units as compute units) and every shard is one run: a launch per shard keeps the
            // workgroups of a launch on one shard's K', V' (prefill, 8 shards of 8192 keys, 4096 x 64 query rows:
            // 8.2 ms against 8.9 ms with all shards in one launch; decode, 8 shards of 8 GiB: 9.55 against 10.05 ms);
            // the partials and their aggregation are the same
            const KeyRuns plan = attn_runs_of(p);
            one_launch_per_shard = true;
            for (int i = 0; i < p.n_shards; ++i)
                if (plan.first[i + 1] - plan.first[i] > 1) one_launch_per_shard = false;
        }
        if (one_launch_per_shard) {
            // one launch per non-empty shard into the workspace ([n][rows][D] then [n][rows]), then the aggregation
            int idx[kMaxShards], n = 0;
            for (int i = 0; i < p.n_shards; ++i)
                if (p.Ls[i] > 0) idx[n++] = i;
            if (n > 1 && (!p.workspace || p.workspace_bytes < (size_t)n * rows * (p.D + 1) * sizeof(float)))
                return hipErrorInvalidValue;
            float* Ow = n > 1 ? (float*)p.workspace : p.O;
            float* Lw = n > 1 ? Ow + (size_t)n * rows * p.D : p.lse;
            for (int j = 0; j < n; ++j) {
                AttnProblem one = p;
                one.n_shards = 1;
                one.K = p.Ks[idx[j]];
                one.V = p.Vs[idx[j]];
                one.Lkv = p.Ls[idx[j]];
                one.single_run = true;  // the workspace holds the per-shard partials: no runs inside a shard
                one.workspace = nullptr;
                one.workspace_bytes = 0;
                one.O = Ow + (size_t)j * rows * p.D;
                one.lse = Lw + (size_t)j * rows;
                const hipError_t e = launch_partial_attn(one, stream);
                if (e != hipSuccess) return e;
            }
            return n > 1 ? launch_lse_merge(Ow, Lw, n, rows, p.D, p.O, p.lse, stream) : hipSuccess;
        }
        if (p.dtype != FEDRAG_BF16 && p.dtype != FEDRAG_F16) return hipErrorInvalidValue;
        return decode ? launch_decode_attn(p, stream) : launch_prefill_attn(p, stream);
    }
    if (p.Lkv == 0) return launch_fill_empty(p.O, p.lse, rows, p.D, stream);
    if (p.quant_bits != 0) {  // K', V' as transport codes: 16-bit storage, no mask
        if (p.dtype == FEDRAG_F32 || p.causal) return hipErrorInvalidValue;
        // the streaming kernel's code path is laid out for d = 128; everything else takes the tiled kernel
        return (use_decode_kernel(p.Hq, p.Hkv, p.Lq) && p.D == 128) ? launch_decode_attn(p, stream)
                                                                    : launch_prefill_attn(p, stream);
    }
    if (p.dtype == FEDRAG_F32) return p.D == 128 ? launch_attn_f32<128>(p, stream) : launch_attn_f32<64>(p, stream);
    if (p.dtype != FEDRAG_BF16 && p.dtype != FEDRAG_F16) return hipErrorInvalidValue;
    return (!p.causal && use_decode_kernel(p.Hq, p.Hkv, p.Lq)) ? launch_decode_attn(p, stream)
                                                               : launch_prefill_attn(p, stream);
}

}  // namespace fedrag
