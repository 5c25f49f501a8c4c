/* Walks the host side of every entry point - argument checks, the key-run planner, the workspace queries - without
 * ever passing a call that would reach a kernel launch: every call below either has an invalid argument or no rows.
 * Built together with the library's sources under AddressSanitizer and UndefinedBehaviorSanitizer (host code only)
 * by tests/test_boundary_cpu.py; the pointers are fake, aligned addresses that the host code must never read. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "fedrag.h"

static int failures = 0;
#define EXPECT(call, want)                                                                          \
    do {                                                                                            \
        const int got_ = (int)(call);                                                               \
        if (got_ != (int)(want)) {                                                                  \
            printf("line %d: %s -> %d, expected %d\n", __LINE__, #call, got_, (int)(want));         \
            ++failures;                                                                             \
        }                                                                                           \
    } while (0)

#define P(n) ((void*)(uintptr_t)(0x10000u * (n)))            /* fake device pointers, 16-byte aligned, far apart */
#define PF(n) ((float*)(uintptr_t)(0x10000u * (n)))
#define PI(n) ((int32_t*)(uintptr_t)(0x10000u * (n)))
#define PU(n) ((uint8_t*)(uintptr_t)(0x10000u * (n)))

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(uint32_t n) {  /* splitmix64 */
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return (uint32_t)((z ^ (z >> 31)) % n);
}

int main(void) {
    fedrag_shape s = {2, 8, 2, 128, FEDRAG_BF16};
    fedrag_shape bad_heads = {2, 8, 3, 128, FEDRAG_BF16}, bad_d = {2, 8, 2, 96, FEDRAG_BF16}, bad_t = {2, 8, 2, 128, 7};
    fedrag_shape f32 = {2, 8, 2, 128, FEDRAG_F32}, neg = {-1, 8, 2, 128, FEDRAG_BF16}, none = {0, 8, 2, 128, FEDRAG_BF16};
    fedrag_structured_key key = {PF(20), PI(21), PI(22), PF(23)}, key_null = {PF(20), NULL, PI(22), PF(23)};
    fedrag_structured_key key_odd = {(float*)(uintptr_t)0x200002u, PI(21), PI(22), PF(23)};
    const float sc = 0.088f;

    /* ---- Enc */
    EXPECT(fedrag_scramble_kv(NULL, 8, P(1), P(2), P(3), P(4), NULL, 0, P(5), P(6), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_scramble_kv(&bad_heads, 8, P(1), P(2), P(3), P(4), NULL, 0, P(5), P(6), NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_scramble_kv(&bad_d, 8, P(1), P(2), P(3), P(4), NULL, 0, P(5), P(6), NULL), FEDRAG_ERR_UNSUPPORTED);
    EXPECT(fedrag_scramble_kv(&bad_t, 8, P(1), P(2), P(3), P(4), NULL, 0, P(5), P(6), NULL), FEDRAG_ERR_UNSUPPORTED);
    EXPECT(fedrag_scramble_kv(&neg, 8, P(1), P(2), P(3), P(4), NULL, 0, P(5), P(6), NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_scramble_kv(&s, -1, P(1), P(2), P(3), P(4), NULL, 0, P(5), P(6), NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_scramble_kv(&s, (int64_t)1 << 40, P(1), P(2), P(3), P(4), NULL, 0, P(5), P(6), NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_scramble_kv(&s, 8, NULL, P(2), P(3), P(4), NULL, 0, P(5), P(6), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_scramble_kv(&s, 8, P(1), P(2), P(3), P(4), PI(7), 3, P(5), P(6), NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_scramble_kv(&s, 8, (char*)P(1) + 2, P(2), P(3), P(4), NULL, 0, P(5), P(6), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_scramble_kv(&s, 8, P(1), P(2), P(3), P(4), NULL, 0, P(1), P(6), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_scramble_kv(&s, 8, P(1), P(2), P(3), P(4), NULL, 0, P(5), P(5), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_scramble_kv(&s, 0, NULL, NULL, NULL, NULL, NULL, 0, NULL, NULL, NULL), FEDRAG_OK);
    EXPECT(fedrag_scramble_kv(&none, 8, NULL, NULL, NULL, NULL, NULL, 0, NULL, NULL, NULL), FEDRAG_OK);
    EXPECT(fedrag_scramble_q(&s, 4, NULL, P(2), NULL, P(3), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_scramble_q(&s, 4, P(1), P(2), (int32_t*)((char*)P(4) + 1), P(3), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_scramble_q(&s, 4, P(1), P(2), NULL, P(1), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_scramble_q(&s, 0, NULL, NULL, NULL, NULL, NULL), FEDRAG_OK);
    EXPECT(fedrag_scramble_kv_structured(&s, 8, P(1), P(2), &key, &key_null, NULL, 0, P(5), P(6), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_scramble_kv_structured(&s, 8, P(1), P(2), &key, &key_odd, NULL, 0, P(5), P(6), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_scramble_kv_structured(&s, 8, P(1), P(2), NULL, &key, NULL, 0, P(5), P(6), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_scramble_q_structured(&s, 4, P(1), &key_null, NULL, P(3), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_unscramble_structured(&s, 4, PF(1), &key, NULL, PF(1), NULL), FEDRAG_ERR_ALIAS);

    /* ---- attention */
    EXPECT(fedrag_partial_attn(&s, 1, 64, NULL, P(2), P(3), sc, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_partial_attn(&s, 1, 64, P(1), NULL, P(3), sc, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_partial_attn(&s, -1, 64, P(1), P(2), P(3), sc, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_partial_attn(&s, 1, 64, P(1), P(2), P(3), 0.0f, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_partial_attn(&s, 1, 64, P(1), P(2), P(3), -1.0f, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_partial_attn(&s, 1, 64, P(1), P(2), P(3), sc / 0.0f, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_partial_attn(&s, 1, 1 << 16, P(1), P(2), P(3), sc, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_WORKSPACE);
    EXPECT(fedrag_partial_attn(&s, 1, 1 << 16, P(1), P(2), P(3), sc, PF(4), PF(5), P(9), 64, NULL), FEDRAG_ERR_WORKSPACE);
    EXPECT(fedrag_partial_attn(&s, 1, 64, P(1), P(2), P(3), sc, (float*)((char*)P(4) + 4), PF(5), NULL, 0, NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_partial_attn(&s, 0, 64, NULL, NULL, NULL, sc, NULL, NULL, NULL, 0, NULL), FEDRAG_OK);
    EXPECT(fedrag_partial_attn_static(&s, 1, 64, NULL, P(2), P(3), sc, PF(4), PF(5), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_partial_attn_static(&s, 1, 64, P(1), P(2), P(3), sc, NULL, PF(5), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_partial_attn_static(&bad_d, 1, 64, P(1), P(2), P(3), sc, PF(4), PF(5), NULL), FEDRAG_ERR_UNSUPPORTED);
    EXPECT(fedrag_partial_attn_static(&s, 1, -3, P(1), P(2), P(3), sc, PF(4), PF(5), NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_partial_attn_static(&s, 1, 64, P(1), P(2), P(3), 0.0f, PF(4), PF(5), NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_partial_attn_static(&s, 1, 64, (char*)P(1) + 8, P(2), P(3), sc, PF(4), PF(5), NULL), FEDRAG_ERR_ALIAS);
    {   /* a 128-token segment of 32 heads against 8192 keys: more key-run partials than the static array holds */
        fedrag_shape seg = {1, 32, 8, 128, FEDRAG_BF16};
        if (fedrag_partial_attn_workspace_bytes(&seg, 128, 8192) <= FEDRAG_STATIC_SCRATCH_BYTES) {
            printf("line %d: expected a workspace above the static array's size\n", __LINE__);
            ++failures;
        }
        EXPECT(fedrag_partial_attn_static(&seg, 128, 8192, P(1), P(2), P(3), sc, PF(4), PF(5), NULL), FEDRAG_ERR_WORKSPACE);
    }
    EXPECT(fedrag_partial_attn_static(&s, 0, 64, NULL, NULL, NULL, sc, NULL, NULL, NULL), FEDRAG_OK);
    EXPECT(fedrag_partial_attn_static(&none, 5, 64, NULL, NULL, NULL, sc, NULL, NULL, NULL), FEDRAG_OK);
    EXPECT(fedrag_local_attn(&s, 8, 4, P(1), P(2), P(3), sc, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_local_attn(&s, 4, 8, P(1), NULL, P(3), sc, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_partial_attn_varlen(&s, 4, 8, P(1), P(2), P(3), NULL, NULL, sc, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_partial_attn_varlen(&s, 4, 8, P(1), P(2), P(3), (int32_t*)((char*)P(6) + 2), NULL, sc, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_partial_attn_quantized(&s, 1, 64, P(1), PU(2), PF(3), PU(4), PF(5), 5, sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_UNSUPPORTED);
    EXPECT(fedrag_partial_attn_quantized(&f32, 1, 64, P(1), PU(2), PF(3), PU(4), PF(5), 8, sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_UNSUPPORTED);
    EXPECT(fedrag_partial_attn_quantized(&s, 1, 64, P(1), PU(2), NULL, PU(4), PF(5), 8, sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_partial_attn_quantized(&s, 300, 64, P(1), PU(2), PF(3), PU(4), PF(5), 8, 0.0f, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_partial_attn_varlen_quantized(&s, 300, 64, P(1), PU(2), PF(3), PU(4), PF(5), 4, NULL, NULL, sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_partial_attn_varlen_quantized(&s, 300, 64, P(1), PU(2), PF(3), PU(4), PF(5), 6, PI(8), NULL, sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_UNSUPPORTED);
    EXPECT(fedrag_partial_attn_varlen_quantized(&f32, 300, 64, P(1), PU(2), PF(3), PU(4), PF(5), 4, PI(8), NULL, sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_UNSUPPORTED);
    EXPECT(fedrag_partial_attn_varlen_quantized(&s, 300, 64, P(1), PU(2), (float*)((char*)P(3) + 4), PU(4), PF(5), 4, PI(8), NULL, sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_partial_attn_varlen_quantized(&s, 0, 64, NULL, NULL, NULL, NULL, NULL, 4, NULL, NULL, sc, NULL, NULL, NULL, 0, NULL), FEDRAG_OK);
    {
        int64_t L[3] = {4096, 0, 4096}, Lneg[2] = {5, -1};
        const void* Ks[3] = {P(2), NULL, P(3)};
        const void* Vs[3] = {P(4), NULL, P(5)};
        const void* Kn[3] = {P(2), NULL, NULL};
        EXPECT(fedrag_partial_attn_shards(&s, 1, 0, L, Ks, Vs, P(1), sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_SHAPE);
        EXPECT(fedrag_partial_attn_shards(&s, 1, FEDRAG_MAX_SHARDS + 1, L, Ks, Vs, P(1), sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_SHAPE);
        EXPECT(fedrag_partial_attn_shards(&s, 1, 2, Lneg, Ks, Vs, P(1), sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_SHAPE);
        EXPECT(fedrag_partial_attn_shards(&s, 1, 3, L, Kn, Vs, P(1), sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_NULL);
        EXPECT(fedrag_partial_attn_shards(&s, 1, 3, L, Ks, Vs, P(1), sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_WORKSPACE);
        EXPECT(fedrag_partial_attn_shards(&s, 1, 3, NULL, Ks, Vs, P(1), sc, PF(6), PF(7), NULL, 0, NULL), FEDRAG_ERR_NULL);
        EXPECT(fedrag_partial_attn_shards_workspace_bytes(&s, 1, 2, Lneg), 0);
        EXPECT(fedrag_partial_attn_shards_workspace_bytes(&s, 1, 0, L), 0);
    }

    /* ---- aggregation, Dec, codec, permutations */
    EXPECT(fedrag_lse_merge(&s, 4, 0, PF(1), PF(2), PF(3), PF(4), NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_lse_merge(&s, 4, 2, PF(1), PF(2), PF(1), PF(4), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_lse_merge(&s, 4, 2, NULL, PF(2), PF(3), PF(4), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_unscramble(&s, 4, PF(1), PF(2), NULL, PF(1), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_unscramble(&s, 4, PF(1), NULL, NULL, PF(3), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_unscramble_merge(&s, 4, PF(1), PF(2), PF(3), NULL, PF(4), PF(5), PF(4), PF(7), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_unscramble_merge(&s, 4, PF(1), NULL, PF(3), NULL, PF(4), PF(5), PF(6), PF(7), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_unpermute_lse(&s, 4, PF(1), NULL, PF(1), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_quantize_rows(16, 96, FEDRAG_BF16, 8, P(1), PU(2), PF(3), NULL), FEDRAG_ERR_UNSUPPORTED);
    EXPECT(fedrag_quantize_rows(16, 128, FEDRAG_BF16, 3, P(1), PU(2), PF(3), NULL), FEDRAG_ERR_UNSUPPORTED);
    EXPECT(fedrag_quantize_rows(-1, 128, FEDRAG_BF16, 8, P(1), PU(2), PF(3), NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_quantize_rows(16, 128, FEDRAG_BF16, 8, P(1), PU(1), PF(3), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_dequantize_rows(16, 128, FEDRAG_F16, 4, PU(2), NULL, P(1), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_dequantize_rows(0, 128, FEDRAG_F16, 4, NULL, NULL, NULL, NULL), FEDRAG_OK);
    EXPECT(fedrag_scramble_kv_quantized(&f32, 8, P(1), P(2), P(3), P(4), NULL, 0, 8, PU(5), PF(6), PU(7), PF(8), NULL), FEDRAG_ERR_UNSUPPORTED);
    EXPECT(fedrag_scramble_kv_quantized(&s, 8, P(1), P(2), P(3), P(4), NULL, 0, 8, PU(5), PF(6), PU(5), PF(8), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_scramble_kv_structured_quantized(&s, 8, P(1), P(2), NULL, &key, NULL, 0, 8, PU(5), PF(6), PU(7), PF(8), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_invert_perm(PI(1), -1, PI(2), NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_invert_perm(PI(1), 8, PI(1), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_invert_perm(NULL, 8, PI(1), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_validate_perm(PI(1), 0, 8, PI(2), PI(3), NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_validate_perm(PI(1), 1, -8, PI(2), PI(3), NULL), FEDRAG_ERR_SHAPE);
    EXPECT(fedrag_validate_perm(PI(1), 1, 8, PI(2), NULL, NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_validate_perm(NULL, 1, 8, PI(2), PI(3), NULL), FEDRAG_ERR_NULL);
    EXPECT(fedrag_validate_perm(PI(1), 1, 8, PI(1), PI(3), NULL), FEDRAG_ERR_ALIAS);
    EXPECT(fedrag_validate_perm(PI(1), 1, 8, (int32_t*)((char*)P(2) + 2), PI(3), NULL), FEDRAG_ERR_ALIAS);

    /* ---- the key-run planner over many shapes: sizes must be finite, consistent and never smaller for one shard
     * given as a list than given alone */
    for (int it = 0; it < 20000; ++it) {
        fedrag_shape r;
        const int g = 1 << rnd(4);
        r.n_kv_heads = 1 + (int32_t)rnd(8);
        r.n_q_heads = r.n_kv_heads * g;
        r.batch = (int32_t)rnd(70);
        r.d_head = rnd(2) ? 128 : 64;
        r.dtype = (int32_t)rnd(3);
        const int64_t Lq = (int64_t)(rnd(3) ? rnd(9) : rnd(5000));
        const int n = 1 + (int)rnd(FEDRAG_MAX_SHARDS);
        int64_t L[FEDRAG_MAX_SHARDS];
        for (int i = 0; i < n; ++i) L[i] = rnd(4) ? (int64_t)rnd(1 << (4 + rnd(16))) : 0;
        const size_t all = fedrag_partial_attn_shards_workspace_bytes(&r, Lq, n, L);
        const size_t rows = (size_t)r.batch * (size_t)r.n_q_heads * (size_t)Lq;
        const size_t per_run = rows * (size_t)(r.d_head + 1) * 4;
        if (per_run && all % per_run != 0) {
            printf("iteration %d: workspace %zu is not a whole number of partials of %zu bytes\n", it, all, per_run);
            ++failures;
        }
        if (per_run && all / per_run > 4096) {
            printf("iteration %d: %zu runs planned\n", it, all / per_run);
            ++failures;
        }
        const size_t one = fedrag_partial_attn_workspace_bytes(&r, Lq, L[0]);
        const size_t one_as_list = fedrag_partial_attn_shards_workspace_bytes(&r, Lq, 1, L);
        if (one != one_as_list) {
            printf("iteration %d: one shard plans %zu bytes alone and %zu as a list\n", it, one, one_as_list);
            ++failures;
        }
    }
    /* sizes at the edge of the supported range */
    {
        fedrag_shape big = {64, 64, 8, 128, FEDRAG_BF16};
        int64_t L[2] = {INT32_MAX, INT32_MAX};
        (void)fedrag_partial_attn_workspace_bytes(&big, 1, INT32_MAX);
        (void)fedrag_partial_attn_workspace_bytes(&big, INT32_MAX, INT32_MAX);
        (void)fedrag_partial_attn_shards_workspace_bytes(&big, 1, 2, L);
        EXPECT(fedrag_partial_attn(&big, (int64_t)INT32_MAX + 1, 8, P(1), P(2), P(3), sc, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_SHAPE);
        EXPECT(fedrag_partial_attn(&big, 1, INT32_MAX, P(1), P(2), P(3), sc, PF(4), PF(5), NULL, 0, NULL), FEDRAG_ERR_WORKSPACE);
    }
    if (failures) {
        printf("%d host-path check(s) failed\n", failures);
        return 1;
    }
    printf("host paths ok\n");
    return 0;
}
