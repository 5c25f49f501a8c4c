// Host-side internal interface between the C-ABI entry points (fedrag_api.hip) and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/fedrag.h"

namespace fedrag {

// A launch grid's x dimension: the launchers refuse (hipErrorInvalidValue) what would not fit instead of truncating.
inline bool grid_fits(int64_t n) { return n >= 1 && n <= 0x7fffffffLL; }

// Second partial for the scatter form (Dec followed by the Section 4.1 aggregation of two partials): row i of X has
// log-sum-exp lse_in[bh, i]; (O_other, lse_other) is the other partial, already in destination row order.
struct RowsMerge {
    const float* lse_in;     // [BH, L]; NULL = plain transform
    const float* O_other;    // [BH, L, D]
    const float* lse_other;  // [BH, L]
    float* lse_out;          // [BH, L]
};

// Rows-times-matrix job: up to two tensors (K and V) transformed in one launch.
struct RowsJob {
    int n_jobs;               // 1 or 2
    const void* X[2];
    const void* Phi[2];       // dense form: [Hkv, D, D]
    bool structured;          // true: the matrix is given as S1 P1 H P2 S2 by the four arrays below, [Hkv, D] each
    const float* s_in[2];
    const int32_t* p_in[2];
    const int32_t* p_out[2];
    const float* s_out[2];
    int quant_bits;           // 0, or 8 / 4: 16-bit gather form only - Y[i] receives the transport codes of the rows
    float* params[2];         //   and params[i] their (scale, lo), [BH * L, 2]
    void* Y[2];
    const int32_t* perm;      // NULL = identity
    int64_t perm_batch_stride;  // 0 (one permutation for all sequences) or L
    int64_t BH;               // batch * heads
    int H;                    // heads per sequence
    int G;                    // heads per scrambling matrix
    int64_t L;                // rows per (batch, head)
    int D;                    // 64 or 128
    int dtype;                // fedrag_dtype of X / Phi / Y (ignored when scatter: fp32)
    bool scatter;             // false: Y[j] = X[perm[j]].Phi ; true: Y[perm[i]] = X[i].Phi (fp32)
    RowsMerge merge;          // scatter, one job: aggregate every transformed row with a second partial (lse_in != NULL)
};
hipError_t launch_rows_transform(const RowsJob& job, hipStream_t stream);
hipError_t launch_invert_perm(const int32_t* perm, int64_t L, int32_t* inv, hipStream_t stream);
// flag[0] = 0 if every row of perm [n_perm, L] is a permutation of 0..L-1, else bit 0 (index out of range) and / or
// bit 1 (index repeated); marks [n_perm, L] is scratch.
hipError_t launch_validate_perm(const int32_t* perm, int n_perm, int64_t L, int32_t* marks, int32_t* flag,
                                hipStream_t stream);

// Partial attention problem: one KV shard (K, V, Lkv), or - n_shards > 1 - the shards a Compute Node holds for
// the same queries, (Ks[i], Vs[i], Ls[i]), whose partials are aggregated inside the call.
constexpr int kMaxShards = 16;
struct AttnProblem {
    int B, Hq, Hkv, D, dtype;
    int64_t Lq, Lkv;
    const void *Q, *K, *V;
    float scale;
    int quant_bits;          // 0, or 8 / 4: K, V hold the transport codec's codes and K_params, V_params their
    const float* K_params;   //   per-row (scale, lo), [B,Hkv,Lkv,2] (decode shapes, 16-bit dtype, D = 128 only)
    const float* V_params;
    int n_shards;            // 0 or 1: K, V, Lkv above; else Ks, Vs, Ls below (16-bit dtype, no codes, no lengths, no mask)
    const void* Ks[kMaxShards];
    const void* Vs[kMaxShards];
    int64_t Ls[kMaxShards];
    const int32_t* kv_lens;  // NULL, or [B] device array: sequence b has only its first kv_lens[b] keys (<= Lkv)
    const int32_t* q_lens;   // NULL, or [B] device array: only the first q_lens[b] query rows of sequence b are computed
                             //   and written (prefill and fp32 kernels; the decode kernel computes all its <= 16 rows)
    bool causal;  // the Lq queries are the last Lq of the Lkv tokens and see nothing after themselves
    bool single_run;  // one shard only: its keys are one run whatever the planner would choose, so the launch writes
                      //   (O, lse) directly and touches no workspace (the per-shard launches of a multi-shard call,
                      //   whose workspace already holds the per-shard partials)
    float* O;     // [B,Hq,Lq,D]
    float* lse;   // [B,Hq,Lq]
    void* workspace;
    size_t workspace_bytes;
};
// How a launch cuts the keys into runs, one workgroup per (unit of queries, run): what both attention kernels
// receive by value.  Shard i contributes runs first[i] .. first[i+1]-1 of per[i] keys each (the last one shorter);
// first[i] = INT_MAX past the last shard, so a kernel finds its shard with compares only.  With more than one run
// the kernels write one normalised partial per run into the workspace, [n_runs][rows][D] then [n_runs][rows], and
// the Section 4.1 aggregation folds them.
struct KeyRuns {
    const void* K[kMaxShards];
    const void* V[kMaxShards];
    int64_t L[kMaxShards];
    int64_t per[kMaxShards];
    int first[kMaxShards + 1];
    int n_runs;
};
// Plans the runs for n shards of lengths Ls (n >= 1); pointers are left unset.  codes4: the streaming kernel will
// read 4-bit transport codes (d = 128 decode shapes), where it wants kDecCodesOcc workgroups per compute unit.
KeyRuns attn_plan_runs(int B, int Hq, int Hkv, int dtype, int64_t Lq, int n, const int64_t* Ls, bool codes4 = false);
bool attn_uses_decode_kernel(int Hq, int Hkv, int64_t Lq);  // G * Lq <= 16: the HBM-bound streaming kernel
// bytes of workspace the plan needs (0 when there is a single run)
size_t attn_workspace_bytes(int B, int Hq, int Hkv, int D, int dtype, int64_t Lq, int n, const int64_t* Ls);
inline size_t attn_workspace_bytes(int B, int Hq, int Hkv, int D, int dtype, int64_t Lq, int64_t Lkv) {
    return attn_workspace_bytes(B, Hq, Hkv, D, dtype, Lq, 1, &Lkv);
}
// The plan of problem p with its pointers filled in.
KeyRuns attn_runs_of(const AttnProblem& p);
hipError_t launch_partial_attn(const AttnProblem& p, hipStream_t stream);
// Device address, on the current device, of the library's static scratch array of FEDRAG_STATIC_SCRATCH_BYTES bytes.
hipError_t attn_static_scratch(void** ptr_out);

// decode kernel geometry (shared by the split planner and the kernel)
constexpr int kDecWaves = 4;
constexpr int kDecThreads = kDecWaves * 64;
constexpr int kDecTile = 32;                      // keys per wave step
constexpr int kDecStride = kDecWaves * kDecTile;  // keys per workgroup step
#ifndef FEDRAG_DECQ_OCC
#define FEDRAG_DECQ_OCC 2
#endif
constexpr int kDecCodesOcc = FEDRAG_DECQ_OCC;     // workgroups per compute unit when the kernel reads 4-bit codes
// prefill kernel geometry (shared by the split planner and the kernel)
constexpr int kPreWaves = 8;
constexpr int kPreQ = 32;                     // query rows per wave (one 32-wide MFMA column tile)
constexpr int kPreQTile = kPreWaves * kPreQ;  // query rows per workgroup
constexpr int kPreK = 64;                     // keys per LDS tile
constexpr int kPreMinTilesPerSplit = 4;       // a KV split is at least this many tiles
hipError_t launch_decode_attn(const AttnProblem& p, hipStream_t stream);   // 16-bit storage, G * L_q <= 16
hipError_t launch_prefill_attn(const AttnProblem& p, hipStream_t stream);  // 16-bit storage, any L_q

// Aggregation of S partials: O_parts [S, rows, D], lses [S, rows] -> O [rows, D], lse [rows].
// q_lens (device, [B]) with Lq and rows_per_seq = Hq * Lq: row r is query r % Lq of sequence r / rows_per_seq, and rows
// at or past q_lens[sequence] are skipped (neither read nor written).
hipError_t launch_lse_merge(const float* O_parts, const float* lses, int S, int64_t rows, int D, float* O, float* lse,
                            hipStream_t stream, const int32_t* q_lens = nullptr, int64_t Lq = 1,
                            int64_t rows_per_seq = 1);
// O = 0, lse = -inf for `rows` rows (a shard with no keys).
hipError_t launch_fill_empty(float* O, float* lse, int64_t rows, int D, hipStream_t stream);
// out[bh, perm[i]] = in[bh, i] for n_bh rows of L values each (perm NULL = copy).
hipError_t launch_scatter_rows_f32(const float* in, const int32_t* perm, int64_t n_bh, int64_t L, float* out,
                                   hipStream_t stream);

// Transport codec job: quantize (X -> codes, params) or dequantize (codes, params -> X); X has n_rows rows of D values.
struct CodecJob {
    bool quantize;
    int64_t n_rows;
    int D;       // 64 or 128
    int dtype;   // fedrag_dtype of X
    int bits;    // 8 or 4
    void* X;
    uint8_t* codes;   // [n_rows, D * bits / 8]
    float* params;    // [n_rows, 2] = (scale, lo)
};
hipError_t launch_codec(const CodecJob& job, hipStream_t stream);

}  // namespace fedrag
