/* A C99 translation unit that uses the library through its header alone: the boundary is plain C.
 * Calls only what needs no GPU: version, status strings, the workspace query and argument checks. */
#include <stdio.h>
#include <string.h>

#include "fedrag.h"

int main(void) {
    fedrag_shape s;
    s.batch = 16; s.n_q_heads = 32; s.n_kv_heads = 8; s.d_head = 128; s.dtype = FEDRAG_BF16;
    if (fedrag_version() <= 0) return 1;
    if (strlen(fedrag_status_string(FEDRAG_ERR_WORKSPACE)) == 0) return 2;
    if (fedrag_partial_attn_workspace_bytes(&s, 1, 8192) == 0) return 3;      /* decode: key runs need scratch */
    if (fedrag_partial_attn_workspace_bytes(&s, 2048, 16384) != 0) return 4;  /* enough query tiles: none */
    /* argument checks happen on the host before anything is enqueued */
    if (fedrag_partial_attn(&s, 1, 8192, NULL, NULL, NULL, 0.088f, NULL, NULL, NULL, 0, NULL) != FEDRAG_ERR_NULL) return 5;
    s.d_head = 100;
    if (fedrag_scramble_q(&s, 1, (const void*)16, (const void*)32, NULL, (void*)48, NULL) != FEDRAG_ERR_UNSUPPORTED) return 6;
    {
        int64_t L[2] = {4096, 4096};
        s.d_head = 128;
        if (fedrag_partial_attn_shards_workspace_bytes(&s, 1, 2, L) == 0) return 7;
        if (fedrag_partial_attn_shards(&s, 1, 0, L, NULL, NULL, NULL, 0.088f, NULL, NULL, NULL, 0, NULL) != FEDRAG_ERR_SHAPE) return 8;
    }
    printf("abi ok, version %d\n", (int)fedrag_version());
    return 0;
}
