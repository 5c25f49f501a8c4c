/*
 * fedrag.h - C ABI of the MI355X (gfx950) hot path of FedRAG's Scrambled Distributed Attention:
 * one collaborating node's share of the protocol of Section 4 of the paper.
 *
 * General rules for every call
 * ----------------------------
 * - Every data pointer is DEVICE memory owned by the caller, 16-byte aligned, dense row-major.
 *   The library never allocates, frees or keeps a pointer after the call returns.  Two kinds of argument are HOST
 *   memory and say so where they are declared: the fedrag_structured_key structs (which hold device pointers) and
 *   the per-shard arrays of fedrag_partial_attn_shards; they are read during the call only.
 * - Tensors are laid out [batch, heads, tokens, d_head] ("[B,H,L,d]").  Query head h uses KV head
 *   h / (n_q_heads / n_kv_heads); scrambling matrices are per KV head, [n_kv_heads, d, d], row-major,
 *   and multiply ROW vectors from the right (x . Phi), the paper's convention (Section 2.1, footnote).
 * - `dtype` is the storage type of Q/K/V and of the scrambling matrices applied to them
 *   (FEDRAG_F32, FEDRAG_BF16 or FEDRAG_F16).  Partial outputs, log-sum-exps, merged and unscrambled
 *   outputs, and Phi_V^{-1}, are always fp32.
 * - Token permutations are int32 GATHER index arrays: out row j <- in row perm[j].  Being a
 *   bijection on [0, L) is the caller's responsibility and is not checked on the hot path.
 * - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue work;
 *   they never synchronise with the host and never copy between host and device.
 * - All argument checks happen on the host before anything is enqueued; on any error nothing is launched and
 *   no output is written.  Errors are return codes only.  FEDRAG_ERR_DEVICE reports a failed launch.
 * - Supported: d_head in {64, 128}; n_q_heads % n_kv_heads == 0; batch and token counts >= 0.  Zero is legal: a call
 *   whose output has no rows (no sequences, or no tokens) returns FEDRAG_OK at once (its tensor pointers may then be
 *   NULL), and attention over no keys writes O = 0, lse = -inf.
 * - The library draws no randomness: keys (Phi's, permutations) come from the key holders
 *   (Inquirer and Context Owner negotiate them per request, Section 5.1 / Section 6).
 *
 * Roles (Section 5.1), documented, not enforced: fedrag_scramble_kv is the Context Owner's call;
 * fedrag_scramble_q and fedrag_unscramble are the Inquirer's; fedrag_partial_attn is the Compute
 * Node's and takes no key material; fedrag_lse_merge may run on either side.
 */
#ifndef FEDRAG_H
#define FEDRAG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FEDRAG_OK = 0,
    FEDRAG_ERR_NULL = 1,        /* a required pointer is NULL */
    FEDRAG_ERR_SHAPE = 2,       /* negative size, heads not divisible, n_perm not in {1,B}, n_shards < 1 ... */
    FEDRAG_ERR_UNSUPPORTED = 3, /* d_head or dtype not supported */
    FEDRAG_ERR_WORKSPACE = 4,   /* workspace NULL or smaller than fedrag_partial_attn_workspace_bytes() */
    FEDRAG_ERR_ALIAS = 5,       /* an output overlaps an input of an out-of-place call, or misaligned pointer */
    FEDRAG_ERR_DEVICE = 6       /* the HIP runtime refused a launch */
} fedrag_status;

typedef enum { FEDRAG_F32 = 0, FEDRAG_BF16 = 1, FEDRAG_F16 = 2 } fedrag_dtype;

typedef struct {
    int32_t batch;      /* B: independent sequences */
    int32_t n_q_heads;  /* Hq */
    int32_t n_kv_heads; /* Hkv, divides Hq */
    int32_t d_head;     /* d: 64 or 128 */
    int32_t dtype;      /* fedrag_dtype of Q/K/V and of phi_q / phi_k / phi_v */
} fedrag_shape;

/*
 * Enc for the Context Owner's operands (Section 4.2, "Scrambled Attention Protocol", step 1;
 * token permutation paragraph):   K' = P_KV K Phi_KQ^{-T},   V' = P_KV V Phi_V,  i.e.
 *     K_out[b,g,j,:] = K[b,g,perm_kv[p,j],:] . phi_k[g]      V_out likewise with phi_v[g]
 * K, V, K_out, V_out : [B, Hkv, L_kv, d] in shape->dtype.  Out of place: outputs must not overlap
 *                      inputs (FEDRAG_ERR_ALIAS).
 * phi_k              : [Hkv, d, d] = Phi_KQ^{-T} (the caller inverts and transposes); phi_v = Phi_V.
 * perm_kv            : [n_perm, L_kv] int32 gather indices, n_perm == 1 (shared by every sequence) or
 *                      n_perm == B; NULL = identity.  One permutation serves all KV heads and both K and V.
 * Products are accumulated in fp32 and rounded once (RNE) to shape->dtype.
 */
fedrag_status fedrag_scramble_kv(const fedrag_shape* shape, int64_t L_kv,
                                 const void* K, const void* V,
                                 const void* phi_k, const void* phi_v,
                                 const int32_t* perm_kv, int32_t n_perm,
                                 void* K_out, void* V_out, void* stream);

/*
 * Enc for the Inquirer's operand (same passage):   Q' = P_Q Q Phi_KQ,
 *     Q_out[b,h,i,:] = Q[b,h,perm_q[i],:] . phi_q[h / G]
 * Q, Q_out : [B, Hq, L_q, d] in shape->dtype, out of place.  phi_q : [Hkv, d, d] = Phi_KQ.
 * perm_q   : [L_q] int32 gather indices or NULL (identity; decode has L_q == 1).
 */
fedrag_status fedrag_scramble_q(const fedrag_shape* shape, int64_t L_q, const void* Q,
                                const void* phi_q, const int32_t* perm_q,
                                void* Q_out, void* stream);

/*
 * The Compute Node's work on one KV shard (Section 4.1, "Per-Node Local Computation"):
 *     O_part[b,h,i,:] = softmax_t( <Qs[b,h,i], Ks[b,g,t]> * softmax_scale ) . Vs[b,g,:,:]
 *     lse[b,h,i]      = ln sum_t exp( <Qs[b,h,i], Ks[b,g,t]> * softmax_scale )  ( = ln [w_i]_l )
 * No mask: every query row sees every key of the shard.  The normalisation factor is carried as its
 * natural logarithm so that outlier logits cannot overflow; softmax_scale is applied in fp32 to the
 * accumulated dot product (pass 1/sqrt(d)); it must be finite and > 0 (FEDRAG_ERR_SHAPE otherwise).
 * Qs : [B,Hq,L_q,d], Ks/Vs : [B,Hkv,L_kv,d] in shape->dtype.  O_part : fp32 [B,Hq,L_q,d], lse : fp32 [B,Hq,L_q].
 * L_kv == 0 gives O_part = 0 and lse = -inf.
 * workspace : device scratch of at least fedrag_partial_attn_workspace_bytes(shape, L_q, L_kv) bytes
 *             (intra-shard KV splits land there and are merged with the Section 4.1 aggregation);
 *             contents are undefined afterwards.  May be NULL only when that size is 0.
 */
fedrag_status fedrag_partial_attn(const fedrag_shape* shape, int64_t L_q, int64_t L_kv,
                                  const void* Qs, const void* Ks, const void* Vs, float softmax_scale,
                                  float* O_part, float* lse,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace fedrag_partial_attn (and the calls that refer to it) needs for these sizes; 0 for arguments the
 * call would reject.  The key runs are planned for the compute-unit count of the device that is current in the
 * calling thread (256 when there is none), so ask with the device current on which the call will run. */
size_t fedrag_partial_attn_workspace_bytes(const fedrag_shape* shape, int64_t L_q, int64_t L_kv);

/*
 * fedrag_partial_attn for callers that cannot allocate device memory and so have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments (less the workspace), same
 * kernels, same results; the key-run partials land in a static device array of FEDRAG_STATIC_SCRATCH_BYTES bytes that
 * is part of the library's code object (each GPU the library runs on holds its copy until the process ends).  The
 * call allocates and frees nothing.  Sizes whose fedrag_partial_attn_workspace_bytes() exceeds
 * FEDRAG_STATIC_SCRATCH_BYTES are refused with FEDRAG_ERR_WORKSPACE and nothing is launched (every decode shape,
 * (n_q_heads / n_kv_heads) * L_q <= 16, needs at most about 4.3 MB).
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (different streams, or
 * graphs replayed concurrently) race on it and must be serialised by the caller; calls on one stream are safe.
 * Nothing has to be cleared between calls: every partial a launch reads, it has written itself.
 * The first call on a device looks the array's device address up (no allocation, but not a stream operation):
 * make it once outside any graph capture.  A failed lookup returns FEDRAG_ERR_DEVICE.
 */
#define FEDRAG_STATIC_SCRATCH_BYTES (16u << 20)
fedrag_status fedrag_partial_attn_static(const fedrag_shape* shape, int64_t L_q, int64_t L_kv,
                                         const void* Qs, const void* Ks, const void* Vs, float softmax_scale,
                                         float* O_part, float* lse, void* stream);

/*
 * Section 4.1 as a whole on a Compute Node that holds the shards of several Context Owners for the same queries:
 * the per-shard computation of fedrag_partial_attn on each of the n_shards shards and the aggregation of
 * fedrag_lse_merge over them, in one call.  Small problems take one attention launch over all shards' keys plus one
 * aggregation launch, instead of one of each per shard (what counts when a shard is a few thousand tokens and a
 * launch costs as much as its work); when a single shard's work already covers the chip the attention is launched
 * shard by shard and aggregated once.  The result equals attention over the concatenation of the shards' keys
 * (eq. (1)).
 * n_shards : 1 .. FEDRAG_MAX_SHARDS.  L_kv, Ks, Vs : HOST arrays of n_shards entries - shard lengths (>= 0; an empty
 * shard contributes nothing and its pointers may be NULL) and DEVICE pointers to [B,Hkv,L_kv[i],d] tensors in
 * shape->dtype (16-byte aligned).  The arrays are read during the call only.
 * Qs as in fedrag_partial_attn.  O : fp32 [B,Hq,L_q,d], lse : fp32 [B,Hq,L_q], aggregated over all shards; all
 * shards empty gives O = 0, lse = -inf.
 * workspace : at least fedrag_partial_attn_shards_workspace_bytes(shape, L_q, n_shards, L_kv) bytes of device
 * scratch (that function returns 0 for arguments this call would reject); may be NULL only when that is 0.
 * Errors as fedrag_partial_attn; n_shards out of range is FEDRAG_ERR_SHAPE.
 */
#define FEDRAG_MAX_SHARDS 16
fedrag_status fedrag_partial_attn_shards(const fedrag_shape* shape, int64_t L_q, int32_t n_shards,
                                         const int64_t* L_kv, const void* const* Ks, const void* const* Vs,
                                         const void* Qs, float softmax_scale, float* O, float* lse,
                                         void* workspace, size_t workspace_bytes, void* stream);

size_t fedrag_partial_attn_shards_workspace_bytes(const fedrag_shape* shape, int64_t L_q, int32_t n_shards,
                                                  const int64_t* L_kv);

/*
 * fedrag_partial_attn over a batch of sequences of unequal length stored padded to L_kv rows (Section 5.2: the
 * re-ranker scores several query-document pairs at once, each a sequence of its own): sequence b attends to its
 * first kv_lens[b] keys only; rows of Ks, Vs past that are never used in the result and may hold anything.
 * kv_lens : int32 [B], DEVICE memory, 0 <= kv_lens[b] <= L_kv (values outside are clamped into that range);
 * a sequence with 0 keys returns O_part = 0, lse = -inf.
 * q_lens  : NULL, or int32 [B], DEVICE memory: sequence b has q_lens[b] real query rows (clamped to [0, L_q]); the
 * rows after them are padding and are NOT written (O_part, lse keep what they held) and, when L_q is large, not
 * computed.  With NULL all L_q rows of every sequence are computed (padding rows give finite, meaningless rows).
 * Everything else, including the workspace size for (L_q, L_kv), as fedrag_partial_attn.
 */
fedrag_status fedrag_partial_attn_varlen(const fedrag_shape* shape, int64_t L_q, int64_t L_kv,
                                         const void* Qs, const void* Ks, const void* Vs,
                                         const int32_t* kv_lens, const int32_t* q_lens, float softmax_scale,
                                         float* O_part, float* lse,
                                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * The Inquirer's own part of a decoder layer's attention (Section 5.3, prefill and decoding phases): the queries
 * of the current input segment against the K, V the Inquirer holds itself, in plaintext, where a token attends
 * to itself and to the tokens before it.  The L_q queries are the LAST L_q of the L_kv local tokens:
 *     query i sees keys t <= i + (L_kv - L_q);  O_part, lse as in fedrag_partial_attn, over those keys.
 * The result is aggregated (fedrag_lse_merge) with the Compute Node's result after that has been descrambled
 * (fedrag_unscramble for the outputs, fedrag_unpermute_lse for their log-sum-exps).
 * Q : [B,Hq,L_q,d], K, V : [B,Hkv,L_kv,d], dtype storage; L_kv >= L_q (else FEDRAG_ERR_SHAPE).  Other arguments,
 * workspace rule (with the same sizes) and errors as fedrag_partial_attn.
 */
fedrag_status fedrag_local_attn(const fedrag_shape* shape, int64_t L_q, int64_t L_kv,
                                const void* Q, const void* K, const void* V, float softmax_scale,
                                float* O_part, float* lse,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * The token-permutation part of Dec (Section 4.2, protocol step 3) for the log-sum-exps that travel with the
 * outputs:  lse_out[b,h,perm_q[i]] = lse_scr[b,h,i]  (perm_q as given to fedrag_scramble_q; NULL copies).
 * fp32 [B,Hq,L_q] in and out, out of place.  shape->dtype is ignored.
 */
fedrag_status fedrag_unpermute_lse(const fedrag_shape* shape, int64_t L_q, const float* lse_scr,
                                   const int32_t* perm_q, float* lse_out, void* stream);

/*
 * Global aggregation (Section 4.1): sum_i w_i (.) O_i / sum_i w_i with w_i = exp(lse_i), evaluated as
 *     M = max_i lse_i, a_i = exp(lse_i - M), O = sum a_i O_i / sum a_i, lse = M + ln sum a_i.
 * O_parts : fp32 [S,B,Hq,L_q,d], lses : fp32 [S,B,Hq,L_q] -> O_out fp32 [B,Hq,L_q,d], lse_out fp32 [B,Hq,L_q].
 * A shard whose lse is -inf has weight 0; if all are -inf the row is O = 0, lse = -inf.  Never NaN for
 * finite O_parts.  Out of place: outputs must not overlap inputs.  shape->dtype is ignored.
 */
fedrag_status fedrag_lse_merge(const fedrag_shape* shape, int64_t L_q, int32_t n_shards,
                               const float* O_parts, const float* lses,
                               float* O_out, float* lse_out, void* stream);

/*
 * Dec (Section 4.2, protocol step 3):  P_Q^{-1} (.) Phi_V^{-1},
 *     O_out[b,h,perm_q[i],:] = O_scr[b,h,i,:] . phi_v_inv[h / G]
 * O_scr, O_out : fp32 [B,Hq,L_q,d], out of place.  phi_v_inv : fp32 [Hkv,d,d].
 * perm_q : the SAME gather array given to fedrag_scramble_q (the inverse is applied as a scatter), or NULL.
 * fp32 inputs are multiplied in fp32 (they are not narrowed to the storage type).  shape->dtype is ignored.
 */
fedrag_status fedrag_unscramble(const fedrag_shape* shape, int64_t L_q, const float* O_scr,
                                const float* phi_v_inv, const int32_t* perm_q,
                                float* O_out, void* stream);

/*
 * The Inquirer's last step of a decoder layer's attention in one call (Section 5.3): Dec of the Compute Node's
 * result (fedrag_unscramble on the outputs, fedrag_unpermute_lse on their log-sum-exps) followed by its
 * aggregation (fedrag_lse_merge over two partials, the descrambled one first) with the Inquirer's own partial from
 * fedrag_local_attn.  The values equal those of the three calls bit for bit.
 * O_scr : fp32 [B,Hq,L_q,d] and lse_scr : fp32 [B,Hq,L_q], as the Compute Node returned them (scrambled channels,
 * rows in the order fedrag_scramble_q gave them).  phi_v_inv, perm_q as in fedrag_unscramble.
 * O_local, lse_local : the Inquirer's own partial, rows in their own order.  O_out, lse_out : the aggregated result,
 * rows in their own order; they must not overlap any input (FEDRAG_ERR_ALIAS).  A row whose two log-sum-exps are both
 * -inf gives O = 0, lse = -inf.
 */
fedrag_status fedrag_unscramble_merge(const fedrag_shape* shape, int64_t L_q, const float* O_scr,
                                      const float* lse_scr, const float* phi_v_inv, const int32_t* perm_q,
                                      const float* O_local, const float* lse_local,
                                      float* O_out, float* lse_out, void* stream);

/*
 * The structured scrambling matrix of Section 4.2 ("Our construction"),  Phi = S1 P1 H P2 S2, given by its factors
 * instead of as a d x d matrix.  One key per transform; the struct itself is HOST memory holding four DEVICE
 * pointers, each to a [n_kv_heads, d] array (4-byte aligned), with both channel permutations as gathers:
 *     u[i] = x[i] * scale_in[i];  v[j] = u[perm_in[j]];  w = v . H;  y[j] = w[perm_out[j]] * scale_out[j]
 * where H[i][m] = (-1)^popcount(i & m) / sqrt(d) is Sylvester's Hadamard matrix, normalised.
 * From a key (a, g1, g2, b) of Phi the caller derives  Phi^{-T} = (1/a, g1, g2, 1/b)  and
 * Phi^{-1} = (1/b, g2^{-1}, g1^{-1}, 1/a)  (P and H are orthogonal, H is symmetric).
 * perm_in / perm_out must be permutations of 0..d-1 (not checked; indices are masked into range).
 * For 16-bit storage the kernels multiply the rows by the matrix S1 P1 Hs P2 (Hs = the +-1 matrix) on the matrix
 * cores, its entries +-scale_in[i] narrowed to the storage type - give scale_in values that type represents exactly -
 * and apply scale_out / sqrt(d) to the fp32 sums: every product in a sum is exact and nothing is rounded before the
 * one final narrowing.  For fp32 data everything is fp32.
 */
typedef struct {
    const float*   scale_in;   /* S1 diagonal            [Hkv, d] */
    const int32_t* perm_in;    /* P1 as a gather         [Hkv, d] */
    const int32_t* perm_out;   /* P2 as a gather         [Hkv, d] */
    const float*   scale_out;  /* S2 diagonal (ones = the variant without S2 of Section 7.5)  [Hkv, d] */
} fedrag_structured_key;

/* fedrag_scramble_kv with Phi_KQ^{-T} and Phi_V in structured form; everything else as there. */
fedrag_status fedrag_scramble_kv_structured(const fedrag_shape* shape, int64_t L_kv,
                                            const void* K, const void* V,
                                            const fedrag_structured_key* key_k,
                                            const fedrag_structured_key* key_v,
                                            const int32_t* perm_kv, int32_t n_perm,
                                            void* K_out, void* V_out, void* stream);

/* fedrag_scramble_q with Phi_KQ in structured form. */
fedrag_status fedrag_scramble_q_structured(const fedrag_shape* shape, int64_t L_q, const void* Q,
                                           const fedrag_structured_key* key_q, const int32_t* perm_q,
                                           void* Q_out, void* stream);

/* fedrag_unscramble with Phi_V^{-1} in structured form (fp32 throughout). */
fedrag_status fedrag_unscramble_structured(const fedrag_shape* shape, int64_t L_q, const float* O_scr,
                                           const fedrag_structured_key* key_v_inv, const int32_t* perm_q,
                                           float* O_out, void* stream);

/*
 * Transport codec (Section 7.5: affine min-max quantisation of the states sent between nodes), per token row.
 * X : n_rows rows of d values of storage type `dtype` (any [.., d] tensor of the path, e.g. K', V', Q').
 * Per row: lo = min, hi = max, levels = 2^bits - 1, scale = (hi - lo) / levels, steps = levels / (hi - lo),
 *     code = clamp(floor(fma(x - lo, steps, 1/2)), 0, levels)  (all 0 for a constant row);
 *     dequantised value = fma(code, scale, lo), narrowed once (RNE) to `dtype`.
 * All of it in IEEE single precision, operation by operation: codes and params are bit-exact functions of X.
 * codes  : uint8 [n_rows, d * bits / 8]; 4-bit codes two per byte, channel 2k in the low half.
 * params : fp32  [n_rows, 2] = (scale, lo), 8-byte aligned.
 * d in {64, 128}; bits in {8, 4} (else FEDRAG_ERR_UNSUPPORTED).  Out of place; X must be finite.
 */
fedrag_status fedrag_quantize_rows(int64_t n_rows, int32_t d, fedrag_dtype dtype, int32_t bits,
                                   const void* X, uint8_t* codes, float* params, void* stream);
fedrag_status fedrag_dequantize_rows(int64_t n_rows, int32_t d, fedrag_dtype dtype, int32_t bits,
                                     const uint8_t* codes, const float* params, void* X_out, void* stream);

/*
 * fedrag_scramble_kv / fedrag_scramble_kv_structured with the transport codec as the epilogue (Section 7.5: the
 * scrambled K', V' are what travels to the Compute Node): each row of K', V' is narrowed to the storage type as
 * usual and then quantised exactly as fedrag_quantize_rows would quantise it, so the outputs equal
 * fedrag_quantize_rows(fedrag_scramble_kv(...)) bit for bit while K', V' are never written in 16 bits.
 * K_codes, V_codes : uint8 [B,Hkv,L,d*bits/8];  K_params, V_params : fp32 [B,Hkv,L,2].  16-bit storage only
 * (FEDRAG_F32: FEDRAG_ERR_UNSUPPORTED); bits in {8, 4}.  Other arguments and errors as the unquantised calls.
 */
fedrag_status fedrag_scramble_kv_quantized(const fedrag_shape* shape, int64_t L_kv,
                                           const void* K, const void* V,
                                           const void* phi_k, const void* phi_v,
                                           const int32_t* perm_kv, int32_t n_perm, int32_t bits,
                                           uint8_t* K_codes, float* K_params,
                                           uint8_t* V_codes, float* V_params, void* stream);
fedrag_status fedrag_scramble_kv_structured_quantized(const fedrag_shape* shape, int64_t L_kv,
                                                      const void* K, const void* V,
                                                      const fedrag_structured_key* key_k,
                                                      const fedrag_structured_key* key_v,
                                                      const int32_t* perm_kv, int32_t n_perm, int32_t bits,
                                                      uint8_t* K_codes, float* K_params,
                                                      uint8_t* V_codes, float* V_params, void* stream);

/*
 * fedrag_partial_attn on K', V' as they arrive through the transport codec (Section 7.5): the Compute Node reads
 * the codes and dequantises them on the fly, so only d * bits / 8 + 8 bytes per key row are read instead of 2 d.
 * Every element is reconstructed exactly as fedrag_dequantize_rows would (fp32 fma, one narrowing to the storage
 * type), so the call works on the same values as fedrag_partial_attn(fedrag_dequantize_rows(...)); the two results
 * differ only by the order in which fp32 sums are formed (a few 1e-6 for decode shapes, where probabilities enter the
 * second product as two storage-type terms; within the 16-bit bounds of fedrag_partial_attn otherwise).
 * Qs : [B,Hq,L_q,d] storage type (16-bit; FEDRAG_F32 is FEDRAG_ERR_UNSUPPORTED);  K_codes, V_codes : uint8
 * [B,Hkv,L_kv,d*bits/8];  K_params, V_params : fp32 [B,Hkv,L_kv,2] (8-byte aligned).  bits in {8, 4}.
 * Any L_q: decode shapes ((n_q_heads / n_kv_heads) * L_q <= 16, d = 128) stream the codes; everything else - the
 * re-ranker's and the prefill shapes of Sections 5.2 and 5.3 - rebuilds each key tile in on-chip memory.
 * Workspace rule as fedrag_partial_attn.
 */
fedrag_status fedrag_partial_attn_quantized(const fedrag_shape* shape, int64_t L_q, int64_t L_kv, const void* Qs,
                                            const uint8_t* K_codes, const float* K_params,
                                            const uint8_t* V_codes, const float* V_params, int32_t bits,
                                            float softmax_scale, float* O_part, float* lse,
                                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * fedrag_partial_attn_varlen on transport codes: the re-ranker's padded batch of query-document pairs (Section 5.2)
 * with K', V' travelling at 8 or 4 bits (Section 7.5 recommends 4 bits for the re-ranking phase).  kv_lens, q_lens
 * as in fedrag_partial_attn_varlen (rows of the code and parameter tensors past kv_lens[b] are never used and may
 * hold anything); the other arguments as in fedrag_partial_attn_quantized.
 */
fedrag_status fedrag_partial_attn_varlen_quantized(const fedrag_shape* shape, int64_t L_q, int64_t L_kv,
                                                   const void* Qs, const uint8_t* K_codes, const float* K_params,
                                                   const uint8_t* V_codes, const float* V_params, int32_t bits,
                                                   const int32_t* kv_lens, const int32_t* q_lens,
                                                   float softmax_scale, float* O_part, float* lse,
                                                   void* workspace, size_t workspace_bytes, void* stream);

/* inv_out[perm[j]] = j for j in [0, L): the gather array that undoes `perm`.  Device pointers. */
fedrag_status fedrag_invert_perm(const int32_t* perm, int64_t L, int32_t* inv_out, void* stream);

/*
 * Debug aid for the key holders (the token-permutation paragraph of Section 4.2 needs P_Q, P_KV to be permutations;
 * the calls above take that on trust and gather / scatter through the indices unchecked): checks that each of the
 * n_perm rows of perm ([n_perm, L] int32, DEVICE) holds every index 0..L-1 exactly once.
 * marks    : DEVICE scratch of n_perm * L int32 (contents destroyed), 4-byte aligned.
 * flag_out : DEVICE int32; receives 0 when every row is a permutation, else bit 0 = some index lies outside
 *            [0, L), bit 1 = some index occurs more than once.
 * Enqueues two small kernels and returns; read flag_out after synchronising with the stream.  n_perm >= 1, L >= 0
 * (L == 0: flag_out = 0), n_perm * L < 2^40, else FEDRAG_ERR_SHAPE.
 */
fedrag_status fedrag_validate_perm(const int32_t* perm, int32_t n_perm, int64_t L, int32_t* marks, int32_t* flag_out,
                                   void* stream);

/* Static, human-readable name of a status code (host pointer, never NULL). */
const char* fedrag_status_string(fedrag_status status);

/* Library version, major * 10000 + minor * 100 + patch. */
int fedrag_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FEDRAG_H */
