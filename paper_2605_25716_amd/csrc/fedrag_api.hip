// C-ABI entry points (include/fedrag.h): host-side argument validation, then kernel launches.
// Every check below runs before the first HIP call, so the error paths work on a machine without a GPU.
#include "fedrag_host.h"

using namespace fedrag;

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t elem_size(int dtype) { return dtype == FEDRAG_F32 ? 4 : 2; }

bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
    if (!a || !b || na == 0 || nb == 0) return false;
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + nb && b0 < a0 + na;
}

fedrag_status check_shape(const fedrag_shape* s, bool need_dtype) {
    if (!s) return FEDRAG_ERR_NULL;
    if (s->batch < 0 || s->n_q_heads <= 0 || s->n_kv_heads <= 0) return FEDRAG_ERR_SHAPE;
    if (s->n_q_heads % s->n_kv_heads != 0) return FEDRAG_ERR_SHAPE;
    if (s->d_head != 64 && s->d_head != 128) return FEDRAG_ERR_UNSUPPORTED;
    if (need_dtype && s->dtype != FEDRAG_F32 && s->dtype != FEDRAG_BF16 && s->dtype != FEDRAG_F16)
        return FEDRAG_ERR_UNSUPPORTED;
    return FEDRAG_OK;
}

// number of elements of a [B, H, L, d] tensor; false on int64 overflow
bool tensor_elems(int64_t B, int64_t H, int64_t L, int64_t d, int64_t* out) {
    int64_t n = 1;
    const int64_t f[4] = {B, H, L, d};
    for (int i = 0; i < 4; ++i) {
        if (f[i] < 0) return false;
        if (f[i] != 0 && n > INT64_MAX / 8 / f[i]) return false;
        n *= f[i];
    }
    *out = n;
    return true;
}

fedrag_status dev(hipError_t e) { return e == hipSuccess ? FEDRAG_OK : FEDRAG_ERR_DEVICE; }

fedrag_status check_key(const fedrag_structured_key* k) {
    if (!k || !k->scale_in || !k->perm_in || !k->perm_out || !k->scale_out) return FEDRAG_ERR_NULL;
    const uintptr_t bits = reinterpret_cast<uintptr_t>(k->scale_in) | reinterpret_cast<uintptr_t>(k->perm_in) |
                           reinterpret_cast<uintptr_t>(k->perm_out) | reinterpret_cast<uintptr_t>(k->scale_out);
    return (bits & 3u) ? FEDRAG_ERR_ALIAS : FEDRAG_OK;
}

void set_key(RowsJob& j, int i, const fedrag_structured_key* k) {
    j.structured = true;
    j.s_in[i] = k->scale_in;
    j.p_in[i] = k->perm_in;
    j.p_out[i] = k->perm_out;
    j.s_out[i] = k->scale_out;
}

}  // namespace

extern "C" {

fedrag_status fedrag_scramble_kv(const fedrag_shape* shape, int64_t L_kv, const void* K, const void* V,
                                 const void* phi_k, const void* phi_v, const int32_t* perm_kv, int32_t n_perm,
                                 void* K_out, void* V_out, void* stream) {
    fedrag_status st = check_shape(shape, true);
    if (st != FEDRAG_OK) return st;
    if (L_kv < 0 || L_kv > INT32_MAX) return FEDRAG_ERR_SHAPE;  // gather indices are int32
    if (L_kv == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!K || !V || !phi_k || !phi_v || !K_out || !V_out) return FEDRAG_ERR_NULL;
    if (perm_kv && n_perm != 1 && n_perm != shape->batch) return FEDRAG_ERR_SHAPE;
    int64_t n;
    if (!tensor_elems(shape->batch, shape->n_kv_heads, L_kv, shape->d_head, &n)) return FEDRAG_ERR_SHAPE;
    const size_t bytes = (size_t)n * elem_size(shape->dtype);
    if (!aligned16(K) || !aligned16(V) || !aligned16(phi_k) || !aligned16(phi_v) || !aligned16(K_out) ||
        !aligned16(V_out) || (reinterpret_cast<uintptr_t>(perm_kv) & 3u))
        return FEDRAG_ERR_ALIAS;
    if (overlaps(K_out, bytes, K, bytes) || overlaps(K_out, bytes, V, bytes) || overlaps(V_out, bytes, K, bytes) ||
        overlaps(V_out, bytes, V, bytes) || overlaps(K_out, bytes, V_out, bytes))
        return FEDRAG_ERR_ALIAS;
    RowsJob j{};
    j.n_jobs = 2;
    j.X[0] = K; j.Phi[0] = phi_k; j.Y[0] = K_out;
    j.X[1] = V; j.Phi[1] = phi_v; j.Y[1] = V_out;
    j.perm = perm_kv;
    j.perm_batch_stride = (perm_kv && n_perm > 1) ? L_kv : 0;
    j.BH = (int64_t)shape->batch * shape->n_kv_heads;
    j.H = shape->n_kv_heads;
    j.G = 1;
    j.L = L_kv;
    j.D = shape->d_head;
    j.dtype = shape->dtype;
    j.scatter = false;
    return dev(launch_rows_transform(j, (hipStream_t)stream));
}

fedrag_status fedrag_scramble_q(const fedrag_shape* shape, int64_t L_q, const void* Q, const void* phi_q,
                                const int32_t* perm_q, void* Q_out, void* stream) {
    fedrag_status st = check_shape(shape, true);
    if (st != FEDRAG_OK) return st;
    if (L_q < 0 || L_q > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!Q || !phi_q || !Q_out) return FEDRAG_ERR_NULL;
    int64_t n;
    if (!tensor_elems(shape->batch, shape->n_q_heads, L_q, shape->d_head, &n)) return FEDRAG_ERR_SHAPE;
    const size_t bytes = (size_t)n * elem_size(shape->dtype);
    if (!aligned16(Q) || !aligned16(phi_q) || !aligned16(Q_out) || (reinterpret_cast<uintptr_t>(perm_q) & 3u))
        return FEDRAG_ERR_ALIAS;
    if (overlaps(Q_out, bytes, Q, bytes)) return FEDRAG_ERR_ALIAS;
    RowsJob j{};
    j.n_jobs = 1;
    j.X[0] = Q; j.Phi[0] = phi_q; j.Y[0] = Q_out;
    j.X[1] = Q; j.Phi[1] = phi_q; j.Y[1] = Q_out;
    j.perm = perm_q;
    j.perm_batch_stride = 0;
    j.BH = (int64_t)shape->batch * shape->n_q_heads;
    j.H = shape->n_q_heads;
    j.G = shape->n_q_heads / shape->n_kv_heads;
    j.L = L_q;
    j.D = shape->d_head;
    j.dtype = shape->dtype;
    j.scatter = false;
    return dev(launch_rows_transform(j, (hipStream_t)stream));
}

size_t fedrag_partial_attn_workspace_bytes(const fedrag_shape* shape, int64_t L_q, int64_t L_kv) {
    if (check_shape(shape, true) != FEDRAG_OK || L_q < 0 || L_kv < 0) return 0;
    return attn_workspace_bytes(shape->batch, shape->n_q_heads, shape->n_kv_heads, shape->d_head, shape->dtype, L_q,
                                L_kv);
}

fedrag_status fedrag_partial_attn(const fedrag_shape* shape, int64_t L_q, int64_t L_kv, const void* Qs,
                                  const void* Ks, const void* Vs, float softmax_scale, float* O_part, float* lse,
                                  void* workspace, size_t workspace_bytes, void* stream) {
    fedrag_status st = check_shape(shape, true);
    if (st != FEDRAG_OK) return st;
    if (L_q < 0 || L_kv < 0 || L_q > INT32_MAX || L_kv > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!Qs || !O_part || !lse) return FEDRAG_ERR_NULL;
    if (L_kv > 0 && (!Ks || !Vs)) return FEDRAG_ERR_NULL;
    int64_t nq, nk;
    if (!tensor_elems(shape->batch, shape->n_q_heads, L_q, shape->d_head, &nq) ||
        !tensor_elems(shape->batch, shape->n_kv_heads, L_kv, shape->d_head, &nk))
        return FEDRAG_ERR_SHAPE;
    if (!(softmax_scale > 0.0f) || softmax_scale - softmax_scale != 0.0f) return FEDRAG_ERR_SHAPE;  // finite, > 0
    if (!aligned16(Qs) || !aligned16(Ks) || !aligned16(Vs) || !aligned16(O_part) ||
        (reinterpret_cast<uintptr_t>(lse) & 3u) || !aligned16(workspace))
        return FEDRAG_ERR_ALIAS;
    const size_t need = attn_workspace_bytes(shape->batch, shape->n_q_heads, shape->n_kv_heads, shape->d_head,
                                             shape->dtype, L_q, L_kv);
    if (need > 0 && (!workspace || workspace_bytes < need)) return FEDRAG_ERR_WORKSPACE;
    AttnProblem p{};
    p.B = shape->batch; p.Hq = shape->n_q_heads; p.Hkv = shape->n_kv_heads; p.D = shape->d_head;
    p.dtype = shape->dtype;
    p.Lq = L_q; p.Lkv = L_kv;
    p.Q = Qs; p.K = Ks; p.V = Vs;
    p.scale = softmax_scale;
    p.O = O_part; p.lse = lse;
    p.workspace = workspace; p.workspace_bytes = workspace_bytes;
    return dev(launch_partial_attn(p, (hipStream_t)stream));
}

fedrag_status fedrag_partial_attn_static(const fedrag_shape* shape, int64_t L_q, int64_t L_kv, const void* Qs,
                                         const void* Ks, const void* Vs, float softmax_scale, float* O_part,
                                         float* lse, void* stream) {
    fedrag_status st = check_shape(shape, true);
    if (st != FEDRAG_OK) return st;
    if (L_q < 0 || L_kv < 0 || L_q > INT32_MAX || L_kv > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!Qs || !O_part || !lse) return FEDRAG_ERR_NULL;
    if (L_kv > 0 && (!Ks || !Vs)) return FEDRAG_ERR_NULL;
    int64_t nq, nk;
    if (!tensor_elems(shape->batch, shape->n_q_heads, L_q, shape->d_head, &nq) ||
        !tensor_elems(shape->batch, shape->n_kv_heads, L_kv, shape->d_head, &nk))
        return FEDRAG_ERR_SHAPE;
    if (!(softmax_scale > 0.0f) || softmax_scale - softmax_scale != 0.0f) return FEDRAG_ERR_SHAPE;  // finite, > 0
    if (!aligned16(Qs) || !aligned16(Ks) || !aligned16(Vs) || !aligned16(O_part) ||
        (reinterpret_cast<uintptr_t>(lse) & 3u))
        return FEDRAG_ERR_ALIAS;
    const size_t need = attn_workspace_bytes(shape->batch, shape->n_q_heads, shape->n_kv_heads, shape->d_head,
                                             shape->dtype, L_q, L_kv);
    if (need > (size_t)FEDRAG_STATIC_SCRATCH_BYTES) return FEDRAG_ERR_WORKSPACE;  // beyond the static array
    void* scratch_ptr = nullptr;
    if (need > 0 && attn_static_scratch(&scratch_ptr) != hipSuccess) {
        (void)hipGetLastError();
        return FEDRAG_ERR_DEVICE;
    }
    AttnProblem p{};
    p.B = shape->batch; p.Hq = shape->n_q_heads; p.Hkv = shape->n_kv_heads; p.D = shape->d_head;
    p.dtype = shape->dtype;
    p.Lq = L_q; p.Lkv = L_kv;
    p.Q = Qs; p.K = Ks; p.V = Vs;
    p.scale = softmax_scale;
    p.O = O_part; p.lse = lse;
    p.workspace = scratch_ptr; p.workspace_bytes = need > 0 ? (size_t)FEDRAG_STATIC_SCRATCH_BYTES : 0;
    return dev(launch_partial_attn(p, (hipStream_t)stream));
}

size_t fedrag_partial_attn_shards_workspace_bytes(const fedrag_shape* shape, int64_t L_q, int32_t n_shards,
                                                  const int64_t* L_kv) {
    if (check_shape(shape, true) != FEDRAG_OK || L_q < 0 || n_shards < 1 || n_shards > kMaxShards || !L_kv) return 0;
    for (int i = 0; i < n_shards; ++i)
        if (L_kv[i] < 0 || L_kv[i] > INT32_MAX) return 0;
    return attn_workspace_bytes(shape->batch, shape->n_q_heads, shape->n_kv_heads, shape->d_head, shape->dtype, L_q,
                                n_shards, L_kv);
}

fedrag_status fedrag_partial_attn_shards(const fedrag_shape* shape, int64_t L_q, int32_t n_shards, const int64_t* L_kv,
                                         const void* const* Ks, const void* const* Vs, const void* Qs,
                                         float softmax_scale, float* O, float* lse, void* workspace,
                                         size_t workspace_bytes, void* stream) {
    fedrag_status st = check_shape(shape, true);
    if (st != FEDRAG_OK) return st;
    if (n_shards < 1 || n_shards > kMaxShards) return FEDRAG_ERR_SHAPE;
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!L_kv || !Ks || !Vs || !Qs || !O || !lse) return FEDRAG_ERR_NULL;
    if (L_q < 0 || L_q > INT32_MAX) return FEDRAG_ERR_SHAPE;
    int64_t nq, nk;
    if (!tensor_elems(shape->batch, shape->n_q_heads, L_q, shape->d_head, &nq)) return FEDRAG_ERR_SHAPE;
    for (int i = 0; i < n_shards; ++i) {
        if (L_kv[i] < 0 || L_kv[i] > INT32_MAX) return FEDRAG_ERR_SHAPE;
        if (!tensor_elems(shape->batch, shape->n_kv_heads, L_kv[i], shape->d_head, &nk)) return FEDRAG_ERR_SHAPE;
        if (L_kv[i] > 0 && (!Ks[i] || !Vs[i])) return FEDRAG_ERR_NULL;
        if (!aligned16(Ks[i]) || !aligned16(Vs[i])) return FEDRAG_ERR_ALIAS;
    }
    if (!(softmax_scale > 0.0f) || softmax_scale - softmax_scale != 0.0f) return FEDRAG_ERR_SHAPE;  // finite, > 0
    if (!aligned16(Qs) || !aligned16(O) || (reinterpret_cast<uintptr_t>(lse) & 3u) || !aligned16(workspace))
        return FEDRAG_ERR_ALIAS;
    const size_t need = attn_workspace_bytes(shape->batch, shape->n_q_heads, shape->n_kv_heads, shape->d_head,
                                             shape->dtype, L_q, n_shards, L_kv);
    if (need > 0 && (!workspace || workspace_bytes < need)) return FEDRAG_ERR_WORKSPACE;
    AttnProblem p{};
    p.B = shape->batch; p.Hq = shape->n_q_heads; p.Hkv = shape->n_kv_heads; p.D = shape->d_head;
    p.dtype = shape->dtype;
    p.Lq = L_q;
    p.Q = Qs;
    p.scale = softmax_scale;
    p.O = O; p.lse = lse;
    p.workspace = workspace; p.workspace_bytes = workspace_bytes;
    if (n_shards == 1) {
        p.Lkv = L_kv[0]; p.K = Ks[0]; p.V = Vs[0];
    } else {
        p.n_shards = n_shards;
        for (int i = 0; i < n_shards; ++i) { p.Ks[i] = Ks[i]; p.Vs[i] = Vs[i]; p.Ls[i] = L_kv[i]; }
    }
    return dev(launch_partial_attn(p, (hipStream_t)stream));
}

fedrag_status fedrag_partial_attn_varlen(const fedrag_shape* shape, int64_t L_q, int64_t L_kv, const void* Qs,
                                         const void* Ks, const void* Vs, const int32_t* kv_lens,
                                         const int32_t* q_lens, float softmax_scale, float* O_part, float* lse,
                                         void* workspace, size_t workspace_bytes, void* stream) {
    fedrag_status st = check_shape(shape, true);
    if (st != FEDRAG_OK) return st;
    if (L_q < 0 || L_kv < 0 || L_q > INT32_MAX || L_kv > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!Qs || !O_part || !lse || !kv_lens) return FEDRAG_ERR_NULL;
    if (L_kv > 0 && (!Ks || !Vs)) return FEDRAG_ERR_NULL;
    int64_t nq, nk;
    if (!tensor_elems(shape->batch, shape->n_q_heads, L_q, shape->d_head, &nq) ||
        !tensor_elems(shape->batch, shape->n_kv_heads, L_kv, shape->d_head, &nk))
        return FEDRAG_ERR_SHAPE;
    if (!(softmax_scale > 0.0f) || softmax_scale - softmax_scale != 0.0f) return FEDRAG_ERR_SHAPE;  // finite, > 0
    if (!aligned16(Qs) || !aligned16(Ks) || !aligned16(Vs) || !aligned16(O_part) ||
        (reinterpret_cast<uintptr_t>(lse) & 3u) || (reinterpret_cast<uintptr_t>(kv_lens) & 3u) ||
        (reinterpret_cast<uintptr_t>(q_lens) & 3u) || !aligned16(workspace))
        return FEDRAG_ERR_ALIAS;
    const size_t need = attn_workspace_bytes(shape->batch, shape->n_q_heads, shape->n_kv_heads, shape->d_head,
                                             shape->dtype, L_q, L_kv);
    if (need > 0 && (!workspace || workspace_bytes < need)) return FEDRAG_ERR_WORKSPACE;
    AttnProblem p{};
    p.B = shape->batch; p.Hq = shape->n_q_heads; p.Hkv = shape->n_kv_heads; p.D = shape->d_head;
    p.dtype = shape->dtype;
    p.Lq = L_q; p.Lkv = L_kv;
    p.Q = Qs; p.K = Ks; p.V = Vs;
    p.kv_lens = kv_lens;
    p.q_lens = q_lens;
    p.scale = softmax_scale;
    p.O = O_part; p.lse = lse;
    p.workspace = workspace; p.workspace_bytes = workspace_bytes;
    return dev(launch_partial_attn(p, (hipStream_t)stream));
}

// fedrag_partial_attn / fedrag_partial_attn_varlen on transport codes; kv_lens == NULL and !lens_required: every key.
static fedrag_status attn_on_codes(const fedrag_shape* shape, int64_t L_q, int64_t L_kv, const void* Qs,
                                   const uint8_t* K_codes, const float* K_params, const uint8_t* V_codes,
                                   const float* V_params, int32_t bits, const int32_t* kv_lens, const int32_t* q_lens,
                                   bool lens_required, float softmax_scale, float* O_part, float* lse, void* workspace,
                                   size_t workspace_bytes, void* stream) {
    fedrag_status st = check_shape(shape, true);
    if (st != FEDRAG_OK) return st;
    if (bits != 8 && bits != 4) return FEDRAG_ERR_UNSUPPORTED;
    if (shape->dtype == FEDRAG_F32) return FEDRAG_ERR_UNSUPPORTED;  // the codec travels with 16-bit storage
    if (L_q < 0 || L_kv < 0 || L_q > INT32_MAX || L_kv > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!Qs || !O_part || !lse || (lens_required && !kv_lens)) return FEDRAG_ERR_NULL;
    if (L_kv > 0 && (!K_codes || !K_params || !V_codes || !V_params)) return FEDRAG_ERR_NULL;
    int64_t nq, nk;
    if (!tensor_elems(shape->batch, shape->n_q_heads, L_q, shape->d_head, &nq) ||
        !tensor_elems(shape->batch, shape->n_kv_heads, L_kv, shape->d_head, &nk))
        return FEDRAG_ERR_SHAPE;
    if (!(softmax_scale > 0.0f) || softmax_scale - softmax_scale != 0.0f) return FEDRAG_ERR_SHAPE;  // finite, > 0
    if (!aligned16(Qs) || !aligned16(K_codes) || !aligned16(V_codes) || !aligned16(O_part) ||
        (reinterpret_cast<uintptr_t>(K_params) & 7u) || (reinterpret_cast<uintptr_t>(V_params) & 7u) ||
        (reinterpret_cast<uintptr_t>(lse) & 3u) || (reinterpret_cast<uintptr_t>(kv_lens) & 3u) ||
        (reinterpret_cast<uintptr_t>(q_lens) & 3u) || !aligned16(workspace))
        return FEDRAG_ERR_ALIAS;
    const size_t need = attn_workspace_bytes(shape->batch, shape->n_q_heads, shape->n_kv_heads, shape->d_head,
                                             shape->dtype, L_q, L_kv);
    if (need > 0 && (!workspace || workspace_bytes < need)) return FEDRAG_ERR_WORKSPACE;
    AttnProblem p{};
    p.B = shape->batch; p.Hq = shape->n_q_heads; p.Hkv = shape->n_kv_heads; p.D = shape->d_head;
    p.dtype = shape->dtype;
    p.Lq = L_q; p.Lkv = L_kv;
    p.Q = Qs; p.K = K_codes; p.V = V_codes;
    p.K_params = K_params; p.V_params = V_params;
    p.quant_bits = bits;
    p.kv_lens = kv_lens;
    p.q_lens = q_lens;
    p.scale = softmax_scale;
    p.O = O_part; p.lse = lse;
    p.workspace = workspace; p.workspace_bytes = workspace_bytes;
    return dev(launch_partial_attn(p, (hipStream_t)stream));
}

fedrag_status fedrag_partial_attn_quantized(const fedrag_shape* shape, int64_t L_q, int64_t L_kv, const void* Qs,
                                            const uint8_t* K_codes, const float* K_params, const uint8_t* V_codes,
                                            const float* V_params, int32_t bits, float softmax_scale, float* O_part,
                                            float* lse, void* workspace, size_t workspace_bytes, void* stream) {
    return attn_on_codes(shape, L_q, L_kv, Qs, K_codes, K_params, V_codes, V_params, bits, nullptr, nullptr, false,
                         softmax_scale, O_part, lse, workspace, workspace_bytes, stream);
}

fedrag_status fedrag_partial_attn_varlen_quantized(const fedrag_shape* shape, int64_t L_q, int64_t L_kv,
                                                   const void* Qs, const uint8_t* K_codes, const float* K_params,
                                                   const uint8_t* V_codes, const float* V_params, int32_t bits,
                                                   const int32_t* kv_lens, const int32_t* q_lens, float softmax_scale,
                                                   float* O_part, float* lse, void* workspace, size_t workspace_bytes,
                                                   void* stream) {
    return attn_on_codes(shape, L_q, L_kv, Qs, K_codes, K_params, V_codes, V_params, bits, kv_lens, q_lens, true,
                         softmax_scale, O_part, lse, workspace, workspace_bytes, stream);
}

fedrag_status fedrag_local_attn(const fedrag_shape* shape, int64_t L_q, int64_t L_kv, const void* Q, const void* K,
                                const void* V, float softmax_scale, float* O_part, float* lse, void* workspace,
                                size_t workspace_bytes, void* stream) {
    fedrag_status st = check_shape(shape, true);
    if (st != FEDRAG_OK) return st;
    if (L_q < 0 || L_kv < L_q || L_kv > INT32_MAX) return FEDRAG_ERR_SHAPE;  // the queries are among the local tokens
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!Q || !O_part || !lse) return FEDRAG_ERR_NULL;
    if (L_kv > 0 && (!K || !V)) return FEDRAG_ERR_NULL;
    int64_t nq, nk;
    if (!tensor_elems(shape->batch, shape->n_q_heads, L_q, shape->d_head, &nq) ||
        !tensor_elems(shape->batch, shape->n_kv_heads, L_kv, shape->d_head, &nk))
        return FEDRAG_ERR_SHAPE;
    if (!(softmax_scale > 0.0f) || softmax_scale - softmax_scale != 0.0f) return FEDRAG_ERR_SHAPE;  // finite, > 0
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O_part) ||
        (reinterpret_cast<uintptr_t>(lse) & 3u) || !aligned16(workspace))
        return FEDRAG_ERR_ALIAS;
    // only a single query per sequence (decoding) can take the KV-split path that needs the workspace
    const size_t need = L_q == 1 ? attn_workspace_bytes(shape->batch, shape->n_q_heads, shape->n_kv_heads,
                                                        shape->d_head, shape->dtype, L_q, L_kv)
                                 : 0;
    if (need > 0 && (!workspace || workspace_bytes < need)) return FEDRAG_ERR_WORKSPACE;
    AttnProblem p{};
    p.B = shape->batch; p.Hq = shape->n_q_heads; p.Hkv = shape->n_kv_heads; p.D = shape->d_head;
    p.dtype = shape->dtype;
    p.Lq = L_q; p.Lkv = L_kv;
    p.Q = Q; p.K = K; p.V = V;
    p.scale = softmax_scale;
    p.causal = true;
    p.O = O_part; p.lse = lse;
    p.workspace = workspace; p.workspace_bytes = workspace_bytes;
    return dev(launch_partial_attn(p, (hipStream_t)stream));
}

fedrag_status fedrag_unpermute_lse(const fedrag_shape* shape, int64_t L_q, const float* lse_scr, const int32_t* perm_q,
                                   float* lse_out, void* stream) {
    fedrag_status st = check_shape(shape, false);
    if (st != FEDRAG_OK) return st;
    if (L_q < 0 || L_q > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!lse_scr || !lse_out) return FEDRAG_ERR_NULL;
    const int64_t n_bh = (int64_t)shape->batch * shape->n_q_heads;
    if (L_q != 0 && n_bh > INT64_MAX / 8 / L_q) return FEDRAG_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(lse_scr) | reinterpret_cast<uintptr_t>(lse_out) |
         reinterpret_cast<uintptr_t>(perm_q)) & 3u)
        return FEDRAG_ERR_ALIAS;
    if (overlaps(lse_out, (size_t)(n_bh * L_q) * 4, lse_scr, (size_t)(n_bh * L_q) * 4)) return FEDRAG_ERR_ALIAS;
    return dev(launch_scatter_rows_f32(lse_scr, perm_q, n_bh, L_q, lse_out, (hipStream_t)stream));
}

fedrag_status fedrag_lse_merge(const fedrag_shape* shape, int64_t L_q, int32_t n_shards, const float* O_parts,
                               const float* lses, float* O_out, float* lse_out, void* stream) {
    fedrag_status st = check_shape(shape, false);
    if (st != FEDRAG_OK) return st;
    if (L_q < 0 || n_shards < 1) return FEDRAG_ERR_SHAPE;
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!O_parts || !lses || !O_out || !lse_out) return FEDRAG_ERR_NULL;
    int64_t n;
    if (!tensor_elems(shape->batch, shape->n_q_heads, L_q, shape->d_head, &n)) return FEDRAG_ERR_SHAPE;
    if (n > INT64_MAX / 8 / n_shards) return FEDRAG_ERR_SHAPE;
    const int64_t rows = n / shape->d_head;
    if (!aligned16(O_parts) || !aligned16(O_out) || (reinterpret_cast<uintptr_t>(lses) & 3u) ||
        (reinterpret_cast<uintptr_t>(lse_out) & 3u))
        return FEDRAG_ERR_ALIAS;
    if (overlaps(O_out, (size_t)n * 4, O_parts, (size_t)n * 4 * n_shards) ||
        overlaps(lse_out, (size_t)rows * 4, lses, (size_t)rows * 4 * n_shards))
        return FEDRAG_ERR_ALIAS;
    return dev(launch_lse_merge(O_parts, lses, n_shards, rows, shape->d_head, O_out, lse_out, (hipStream_t)stream));
}

fedrag_status fedrag_unscramble(const fedrag_shape* shape, int64_t L_q, const float* O_scr, const float* phi_v_inv,
                                const int32_t* perm_q, float* O_out, void* stream) {
    fedrag_status st = check_shape(shape, false);
    if (st != FEDRAG_OK) return st;
    if (L_q < 0 || L_q > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!O_scr || !phi_v_inv || !O_out) return FEDRAG_ERR_NULL;
    int64_t n;
    if (!tensor_elems(shape->batch, shape->n_q_heads, L_q, shape->d_head, &n)) return FEDRAG_ERR_SHAPE;
    if (!aligned16(O_scr) || !aligned16(phi_v_inv) || !aligned16(O_out) || (reinterpret_cast<uintptr_t>(perm_q) & 3u))
        return FEDRAG_ERR_ALIAS;
    if (overlaps(O_out, (size_t)n * 4, O_scr, (size_t)n * 4)) return FEDRAG_ERR_ALIAS;
    RowsJob j{};
    j.n_jobs = 1;
    j.X[0] = O_scr; j.Phi[0] = phi_v_inv; j.Y[0] = O_out;
    j.X[1] = O_scr; j.Phi[1] = phi_v_inv; j.Y[1] = O_out;
    j.perm = perm_q;
    j.perm_batch_stride = 0;
    j.BH = (int64_t)shape->batch * shape->n_q_heads;
    j.H = shape->n_q_heads;
    j.G = shape->n_q_heads / shape->n_kv_heads;
    j.L = L_q;
    j.D = shape->d_head;
    j.dtype = FEDRAG_F32;
    j.scatter = true;
    return dev(launch_rows_transform(j, (hipStream_t)stream));
}

fedrag_status fedrag_unscramble_merge(const fedrag_shape* shape, int64_t L_q, const float* O_scr, const float* lse_scr,
                                      const float* phi_v_inv, const int32_t* perm_q, const float* O_local,
                                      const float* lse_local, float* O_out, float* lse_out, void* stream) {
    fedrag_status st = check_shape(shape, false);
    if (st != FEDRAG_OK) return st;
    if (L_q < 0 || L_q > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!O_scr || !lse_scr || !phi_v_inv || !O_local || !lse_local || !O_out || !lse_out) return FEDRAG_ERR_NULL;
    int64_t n;
    if (!tensor_elems(shape->batch, shape->n_q_heads, L_q, shape->d_head, &n)) return FEDRAG_ERR_SHAPE;
    const size_t ob = (size_t)n * 4, lb = (size_t)(n / shape->d_head) * 4;
    if (!aligned16(O_scr) || !aligned16(phi_v_inv) || !aligned16(O_out) || !aligned16(O_local) ||
        (reinterpret_cast<uintptr_t>(perm_q) & 3u) || (reinterpret_cast<uintptr_t>(lse_scr) & 3u) ||
        (reinterpret_cast<uintptr_t>(lse_local) & 3u) || (reinterpret_cast<uintptr_t>(lse_out) & 3u))
        return FEDRAG_ERR_ALIAS;
    if (overlaps(O_out, ob, O_scr, ob) || overlaps(O_out, ob, O_local, ob) || overlaps(lse_out, lb, lse_scr, lb) ||
        overlaps(lse_out, lb, lse_local, lb))
        return FEDRAG_ERR_ALIAS;
    RowsJob j{};
    j.n_jobs = 1;
    j.X[0] = O_scr; j.Phi[0] = phi_v_inv; j.Y[0] = O_out;
    j.X[1] = O_scr; j.Phi[1] = phi_v_inv; j.Y[1] = O_out;
    j.perm = perm_q;
    j.perm_batch_stride = 0;
    j.BH = (int64_t)shape->batch * shape->n_q_heads;
    j.H = shape->n_q_heads;
    j.G = shape->n_q_heads / shape->n_kv_heads;
    j.L = L_q;
    j.D = shape->d_head;
    j.dtype = FEDRAG_F32;
    j.scatter = true;
    j.merge = RowsMerge{lse_scr, O_local, lse_local, lse_out};
    return dev(launch_rows_transform(j, (hipStream_t)stream));
}

fedrag_status fedrag_scramble_kv_structured(const fedrag_shape* shape, int64_t L_kv, const void* K, const void* V,
                                            const fedrag_structured_key* key_k, const fedrag_structured_key* key_v,
                                            const int32_t* perm_kv, int32_t n_perm, void* K_out, void* V_out,
                                            void* stream) {
    fedrag_status st = check_shape(shape, true);
    if (st != FEDRAG_OK) return st;
    if (L_kv < 0 || L_kv > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (L_kv == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!K || !V || !K_out || !V_out) return FEDRAG_ERR_NULL;
    if ((st = check_key(key_k)) != FEDRAG_OK || (st = check_key(key_v)) != FEDRAG_OK) return st;
    if (perm_kv && n_perm != 1 && n_perm != shape->batch) return FEDRAG_ERR_SHAPE;
    int64_t n;
    if (!tensor_elems(shape->batch, shape->n_kv_heads, L_kv, shape->d_head, &n)) return FEDRAG_ERR_SHAPE;
    const size_t bytes = (size_t)n * elem_size(shape->dtype);
    if (!aligned16(K) || !aligned16(V) || !aligned16(K_out) || !aligned16(V_out) ||
        (reinterpret_cast<uintptr_t>(perm_kv) & 3u))
        return FEDRAG_ERR_ALIAS;
    if (overlaps(K_out, bytes, K, bytes) || overlaps(K_out, bytes, V, bytes) || overlaps(V_out, bytes, K, bytes) ||
        overlaps(V_out, bytes, V, bytes) || overlaps(K_out, bytes, V_out, bytes))
        return FEDRAG_ERR_ALIAS;
    RowsJob j{};
    j.n_jobs = 2;
    j.X[0] = K; j.Y[0] = K_out;
    j.X[1] = V; j.Y[1] = V_out;
    set_key(j, 0, key_k);
    set_key(j, 1, key_v);
    j.perm = perm_kv;
    j.perm_batch_stride = (perm_kv && n_perm > 1) ? L_kv : 0;
    j.BH = (int64_t)shape->batch * shape->n_kv_heads;
    j.H = shape->n_kv_heads;
    j.G = 1;
    j.L = L_kv;
    j.D = shape->d_head;
    j.dtype = shape->dtype;
    j.scatter = false;
    return dev(launch_rows_transform(j, (hipStream_t)stream));
}

fedrag_status fedrag_scramble_q_structured(const fedrag_shape* shape, int64_t L_q, const void* Q,
                                           const fedrag_structured_key* key_q, const int32_t* perm_q, void* Q_out,
                                           void* stream) {
    fedrag_status st = check_shape(shape, true);
    if (st != FEDRAG_OK) return st;
    if (L_q < 0 || L_q > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!Q || !Q_out) return FEDRAG_ERR_NULL;
    if ((st = check_key(key_q)) != FEDRAG_OK) return st;
    int64_t n;
    if (!tensor_elems(shape->batch, shape->n_q_heads, L_q, shape->d_head, &n)) return FEDRAG_ERR_SHAPE;
    const size_t bytes = (size_t)n * elem_size(shape->dtype);
    if (!aligned16(Q) || !aligned16(Q_out) || (reinterpret_cast<uintptr_t>(perm_q) & 3u)) return FEDRAG_ERR_ALIAS;
    if (overlaps(Q_out, bytes, Q, bytes)) return FEDRAG_ERR_ALIAS;
    RowsJob j{};
    j.n_jobs = 1;
    j.X[0] = j.X[1] = Q;
    j.Y[0] = j.Y[1] = Q_out;
    set_key(j, 0, key_q);
    set_key(j, 1, key_q);
    j.perm = perm_q;
    j.perm_batch_stride = 0;
    j.BH = (int64_t)shape->batch * shape->n_q_heads;
    j.H = shape->n_q_heads;
    j.G = shape->n_q_heads / shape->n_kv_heads;
    j.L = L_q;
    j.D = shape->d_head;
    j.dtype = shape->dtype;
    j.scatter = false;
    return dev(launch_rows_transform(j, (hipStream_t)stream));
}

fedrag_status fedrag_unscramble_structured(const fedrag_shape* shape, int64_t L_q, const float* O_scr,
                                           const fedrag_structured_key* key_v_inv, const int32_t* perm_q, float* O_out,
                                           void* stream) {
    fedrag_status st = check_shape(shape, false);
    if (st != FEDRAG_OK) return st;
    if (L_q < 0 || L_q > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (L_q == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!O_scr || !O_out) return FEDRAG_ERR_NULL;
    if ((st = check_key(key_v_inv)) != FEDRAG_OK) return st;
    int64_t n;
    if (!tensor_elems(shape->batch, shape->n_q_heads, L_q, shape->d_head, &n)) return FEDRAG_ERR_SHAPE;
    if (!aligned16(O_scr) || !aligned16(O_out) || (reinterpret_cast<uintptr_t>(perm_q) & 3u)) return FEDRAG_ERR_ALIAS;
    if (overlaps(O_out, (size_t)n * 4, O_scr, (size_t)n * 4)) return FEDRAG_ERR_ALIAS;
    RowsJob j{};
    j.n_jobs = 1;
    j.X[0] = j.X[1] = O_scr;
    j.Y[0] = j.Y[1] = O_out;
    set_key(j, 0, key_v_inv);
    set_key(j, 1, key_v_inv);
    j.perm = perm_q;
    j.perm_batch_stride = 0;
    j.BH = (int64_t)shape->batch * shape->n_q_heads;
    j.H = shape->n_q_heads;
    j.G = shape->n_q_heads / shape->n_kv_heads;
    j.L = L_q;
    j.D = shape->d_head;
    j.dtype = FEDRAG_F32;
    j.scatter = true;
    return dev(launch_rows_transform(j, (hipStream_t)stream));
}

// Enc of a KV shard with the transport codec as its epilogue; exactly one of (phi_k, phi_v) / (key_k, key_v) is given.
static fedrag_status scramble_kv_quantized(const fedrag_shape* shape, int64_t L_kv, const void* K, const void* V,
                                           const void* phi_k, const void* phi_v, const fedrag_structured_key* key_k,
                                           const fedrag_structured_key* key_v, const int32_t* perm_kv, int32_t n_perm,
                                           int32_t bits, uint8_t* K_codes, float* K_params, uint8_t* V_codes,
                                           float* V_params, void* stream) {
    fedrag_status st = check_shape(shape, true);
    if (st != FEDRAG_OK) return st;
    if (shape->dtype == FEDRAG_F32) return FEDRAG_ERR_UNSUPPORTED;  // the codec epilogue is for 16-bit storage
    if (bits != 8 && bits != 4) return FEDRAG_ERR_UNSUPPORTED;
    if (L_kv < 0 || L_kv > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (L_kv == 0 || shape->batch == 0) return FEDRAG_OK;  // no rows: nothing to do, tensor pointers may be NULL
    if (!K || !V || !K_codes || !K_params || !V_codes || !V_params) return FEDRAG_ERR_NULL;
    const bool structured = key_k != nullptr || key_v != nullptr;
    if (structured) {
        if ((st = check_key(key_k)) != FEDRAG_OK || (st = check_key(key_v)) != FEDRAG_OK) return st;
    } else {
        if (!phi_k || !phi_v) return FEDRAG_ERR_NULL;
        if (!aligned16(phi_k) || !aligned16(phi_v)) return FEDRAG_ERR_ALIAS;
    }
    if (perm_kv && n_perm != 1 && n_perm != shape->batch) return FEDRAG_ERR_SHAPE;
    int64_t n;
    if (!tensor_elems(shape->batch, shape->n_kv_heads, L_kv, shape->d_head, &n)) return FEDRAG_ERR_SHAPE;
    const size_t xb = (size_t)n * 2, cb = (size_t)n * bits / 8, pb = (size_t)(n / shape->d_head) * 8;
    if (!aligned16(K) || !aligned16(V) || !aligned16(K_codes) || !aligned16(V_codes) ||
        (reinterpret_cast<uintptr_t>(K_params) & 7u) || (reinterpret_cast<uintptr_t>(V_params) & 7u) ||
        (reinterpret_cast<uintptr_t>(perm_kv) & 3u))
        return FEDRAG_ERR_ALIAS;
    const void* outs[4] = {K_codes, V_codes, K_params, V_params};
    const size_t out_bytes[4] = {cb, cb, pb, pb};
    for (int a = 0; a < 4; ++a) {
        if (overlaps(outs[a], out_bytes[a], K, xb) || overlaps(outs[a], out_bytes[a], V, xb)) return FEDRAG_ERR_ALIAS;
        for (int b = a + 1; b < 4; ++b)
            if (overlaps(outs[a], out_bytes[a], outs[b], out_bytes[b])) return FEDRAG_ERR_ALIAS;
    }
    RowsJob j{};
    j.n_jobs = 2;
    j.X[0] = K; j.Phi[0] = phi_k; j.Y[0] = K_codes; j.params[0] = K_params;
    j.X[1] = V; j.Phi[1] = phi_v; j.Y[1] = V_codes; j.params[1] = V_params;
    if (structured) {
        set_key(j, 0, key_k);
        set_key(j, 1, key_v);
    }
    j.quant_bits = bits;
    j.perm = perm_kv;
    j.perm_batch_stride = (perm_kv && n_perm > 1) ? L_kv : 0;
    j.BH = (int64_t)shape->batch * shape->n_kv_heads;
    j.H = shape->n_kv_heads;
    j.G = 1;
    j.L = L_kv;
    j.D = shape->d_head;
    j.dtype = shape->dtype;
    j.scatter = false;
    return dev(launch_rows_transform(j, (hipStream_t)stream));
}

fedrag_status fedrag_scramble_kv_quantized(const fedrag_shape* shape, int64_t L_kv, const void* K, const void* V,
                                           const void* phi_k, const void* phi_v, const int32_t* perm_kv, int32_t n_perm,
                                           int32_t bits, uint8_t* K_codes, float* K_params, uint8_t* V_codes,
                                           float* V_params, void* stream) {
    return scramble_kv_quantized(shape, L_kv, K, V, phi_k, phi_v, nullptr, nullptr, perm_kv, n_perm, bits, K_codes,
                                 K_params, V_codes, V_params, stream);
}

fedrag_status fedrag_scramble_kv_structured_quantized(const fedrag_shape* shape, int64_t L_kv, const void* K,
                                                      const void* V, const fedrag_structured_key* key_k,
                                                      const fedrag_structured_key* key_v, const int32_t* perm_kv,
                                                      int32_t n_perm, int32_t bits, uint8_t* K_codes, float* K_params,
                                                      uint8_t* V_codes, float* V_params, void* stream) {
    if (!key_k || !key_v) return FEDRAG_ERR_NULL;
    return scramble_kv_quantized(shape, L_kv, K, V, nullptr, nullptr, key_k, key_v, perm_kv, n_perm, bits, K_codes,
                                 K_params, V_codes, V_params, stream);
}

static fedrag_status codec_call(bool quantize, int64_t n_rows, int32_t d, fedrag_dtype dtype, int32_t bits,
                                const void* X, const void* codes, const void* params, void* stream) {
    if (n_rows < 0 || n_rows > INT64_MAX / 1024) return FEDRAG_ERR_SHAPE;
    if (d != 64 && d != 128) return FEDRAG_ERR_UNSUPPORTED;
    if (bits != 8 && bits != 4) return FEDRAG_ERR_UNSUPPORTED;
    if (dtype != FEDRAG_F32 && dtype != FEDRAG_BF16 && dtype != FEDRAG_F16) return FEDRAG_ERR_UNSUPPORTED;
    if (n_rows == 0) return FEDRAG_OK;  // nothing to do
    if (!X || !codes || !params) return FEDRAG_ERR_NULL;
    if (!aligned16(X) || !aligned16(codes) || (reinterpret_cast<uintptr_t>(params) & 7u)) return FEDRAG_ERR_ALIAS;
    const size_t xb = (size_t)n_rows * d * elem_size(dtype), cb = (size_t)n_rows * d * bits / 8, pb = (size_t)n_rows * 8;
    if (overlaps(X, xb, codes, cb) || overlaps(X, xb, params, pb) || overlaps(codes, cb, params, pb))
        return FEDRAG_ERR_ALIAS;
    CodecJob j{};
    j.quantize = quantize;
    j.n_rows = n_rows;
    j.D = d;
    j.dtype = dtype;
    j.bits = bits;
    j.X = const_cast<void*>(X);
    j.codes = (uint8_t*)const_cast<void*>(codes);
    j.params = (float*)const_cast<void*>(params);
    return dev(launch_codec(j, (hipStream_t)stream));
}

fedrag_status fedrag_quantize_rows(int64_t n_rows, int32_t d, fedrag_dtype dtype, int32_t bits, const void* X,
                                   uint8_t* codes, float* params, void* stream) {
    return codec_call(true, n_rows, d, dtype, bits, X, codes, params, stream);
}

fedrag_status fedrag_dequantize_rows(int64_t n_rows, int32_t d, fedrag_dtype dtype, int32_t bits,
                                     const uint8_t* codes, const float* params, void* X_out, void* stream) {
    return codec_call(false, n_rows, d, dtype, bits, X_out, codes, params, stream);
}

fedrag_status fedrag_invert_perm(const int32_t* perm, int64_t L, int32_t* inv_out, void* stream) {
    if (L < 0 || L > INT32_MAX) return FEDRAG_ERR_SHAPE;
    if (!perm || !inv_out) return FEDRAG_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(perm) & 3u) || (reinterpret_cast<uintptr_t>(inv_out) & 3u)) return FEDRAG_ERR_ALIAS;
    if (overlaps(perm, (size_t)L * 4, inv_out, (size_t)L * 4)) return FEDRAG_ERR_ALIAS;
    return dev(launch_invert_perm(perm, L, inv_out, (hipStream_t)stream));
}

fedrag_status fedrag_validate_perm(const int32_t* perm, int32_t n_perm, int64_t L, int32_t* marks, int32_t* flag_out,
                                   void* stream) {
    if (n_perm < 1 || L < 0 || L > INT32_MAX || (int64_t)n_perm * L >= ((int64_t)1 << 40)) return FEDRAG_ERR_SHAPE;
    if (!flag_out || (L > 0 && (!perm || !marks))) return FEDRAG_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(perm) | reinterpret_cast<uintptr_t>(marks) |
         reinterpret_cast<uintptr_t>(flag_out)) & 3u)
        return FEDRAG_ERR_ALIAS;
    const size_t nb = (size_t)n_perm * (size_t)L * 4;
    if (overlaps(perm, nb, marks, nb) || overlaps(flag_out, 4, marks, nb) || overlaps(flag_out, 4, perm, nb))
        return FEDRAG_ERR_ALIAS;
    return dev(launch_validate_perm(perm, n_perm, L, marks, flag_out, (hipStream_t)stream));
}

const char* fedrag_status_string(fedrag_status status) {
    switch (status) {
        case FEDRAG_OK: return "ok";
        case FEDRAG_ERR_NULL: return "a required pointer is NULL";
        case FEDRAG_ERR_SHAPE: return "invalid shape or size argument";
        case FEDRAG_ERR_UNSUPPORTED: return "unsupported d_head or dtype";
        case FEDRAG_ERR_WORKSPACE: return "workspace missing or too small";
        case FEDRAG_ERR_ALIAS: return "output overlaps an input, or a pointer is misaligned";
        case FEDRAG_ERR_DEVICE: return "HIP launch failed";
    }
    return "unknown status";
}

int fedrag_version(void) { return 100; }

}  // extern "C"
