/* A plain C99 caller of the library's host-only entry points: the boundary is C, not C++.
 * Built and run by tests/test_abi_host.py (no GPU needed: the context has no device). */
#include <stdio.h>
#include <string.h>
#include "rotatek.h"

int main(void)
{
    rk_ctx* ctx = NULL;
    rk_layout lay;
    int32_t n_splits = 0, tokens = 0;
    size_t kb = 0, vb = 0, ws;

    if (rk_create(&ctx, RK_DEVICE_NONE) != RK_OK || !ctx) return 1;
    memset(&lay, 0, sizeof lay);
    lay.batch = 2; lay.n_q_heads = 8; lay.n_kv_heads = 2; lay.head_dim = 128; lay.keep = 64;
    lay.dtype = RK_BF16; lay.capacity = 1024; lay.max_seq_len = 1000;
    if (rk_validate_layout(&lay) != RK_OK) return 2;
    if (rk_cache_bytes(&lay, &kb, &vb) != RK_OK || kb != 2u * 2 * 1024 * 64 * 2 || vb != 2u * 2 * 1024 * 128 * 2) return 3;
    ws = rk_decode_workspace_size(ctx, &lay);
    if (ws == 0 || rk_decode_plan(ctx, &lay, &n_splits, &tokens) != RK_OK || n_splits < 1) return 4;
    /* a compute call on a context without a device is refused after validation, nothing is launched */
    if (rk_decode_attn(ctx, &lay, (void*)4096, (void*)4096, (void*)4096, (const float*)4096, NULL, 0.0f,
                       (void*)4096, (void*)4096, ws, NULL) != RK_ERR_INVALID_ARG) return 5;   /* seq_len is NULL */
    lay.seq_len = (const int32_t*)4096;
    if (rk_decode_attn(ctx, &lay, (void*)4096, (void*)4096, (void*)4096, (const float*)4096, NULL, 0.0f,
                       (void*)4096, (void*)4096, ws, NULL) != RK_ERR_NO_DEVICE) return 6;
    lay.head_dim = 64;
    if (rk_validate_layout(&lay) != RK_ERR_UNSUPPORTED) return 7;
    printf("%s|%d|%d|%lu\n", rk_status_str(RK_ERR_NO_DEVICE), (int)n_splits, (int)tokens, (unsigned long)ws);
    return rk_destroy(ctx) == RK_OK ? 0 : 8;
}
