/* Every entry point of the library on a context without a device, with valid arguments (refused only
 * for the missing device), with each kind of invalid argument, and with the largest layouts the header
 * allows: the host side -- validation, size arithmetic, split planning, error text -- runs in full and
 * nothing is launched.  Built with -fsanitize=address,undefined against a library whose host code is
 * built the same way, and run by tests/test_sanitizers.py.  Exit code = number of the failed check. */
#include <stdio.h>
#include <string.h>
#include "rotatek.h"

#define P ((void*)4096)                 /* a non-NULL, 16-byte aligned "device pointer": never dereferenced */
#define PF ((float*)4096)
#define PI ((int32_t*)4096)
static int n_checks = 0;
#define CHECK(cond) do { ++n_checks; if (!(cond)) { printf("check %d failed: %s (last error: %s)\n", n_checks, #cond, rk_last_error(ctx)); return n_checks; } } while (0)

static rk_layout make_layout(int B, int Hq, int Hkv, int r, int dtype, int cap, int maxlen)
{
    rk_layout L;
    memset(&L, 0, sizeof L);
    L.batch = B; L.n_q_heads = Hq; L.n_kv_heads = Hkv; L.head_dim = 128; L.keep = r; L.dtype = dtype;
    L.capacity = cap; L.max_seq_len = maxlen; L.seq_len = PI;
    return L;
}

static rk_rows make_rows(int n, int Hkv, int cap)
{
    rk_rows R;
    memset(&R, 0, sizeof R);
    R.data = P; R.n_tokens = n; R.stride_t = 128; R.stride_h = (int64_t)cap * 128; R.stride_b = R.stride_h * Hkv;
    return R;
}

int main(void)
{
    rk_ctx* ctx = NULL;
    size_t kb, vb, ws, fws;
    int32_t ns, tps;
    int i;
    if (rk_create(&ctx, RK_DEVICE_NONE) != RK_OK || !ctx) return 1000;
    for (i = 0; i <= 7; ++i) CHECK(rk_status_str((rk_status)i) != NULL && strlen(rk_status_str((rk_status)i)) > 0);
    CHECK(rk_last_error(NULL) != NULL);

    /* shapes: the five stated workloads and the extremes of every field */
    {
        const int shapes[][7] = {
            {1, 2, 2, 32, RK_F32, 544, 512},       {1, 8, 8, 64, RK_BF16, 4096, 4096},
            {8, 28, 4, 64, RK_BF16, 16448, 16384}, {16, 32, 32, 64, RK_BF16, 32768, 32768},
            {1, 32, 32, 48, RK_BF16, 32896, 32768}, {1, 1, 1, 1, RK_F32, 32, 0},
            {4096, 64, 64, 128, RK_BF16, 1 << 20, 1 << 20}, {3, 16, 1, 37, RK_BF16, 96, 70},
            {65535, 128, 1, 127, RK_F32, 32, 32},
        };
        for (i = 0; i < (int)(sizeof shapes / sizeof shapes[0]); ++i) {
            const int* s = shapes[i];
            rk_layout L = make_layout(s[0], s[1], s[2], s[3], s[4], s[5], s[6]);
            rk_rows K = make_rows(s[6], s[2], s[5]);
            rk_fit_out out;
            rk_subspace sub;
            rk_text text;
            CHECK(rk_validate_layout(&L) == RK_OK);
            CHECK(rk_cache_bytes(&L, &kb, &vb) == RK_OK && vb >= kb && kb > 0);
            ws = rk_decode_workspace_size(ctx, &L);
            fws = rk_fit_workspace_size(&L, s[6]);
            CHECK(ws > 0 && fws > 0);
            CHECK(rk_decode_plan(ctx, &L, &ns, &tps) == RK_OK && ns >= 1 && tps % 128 == 0);
            memset(&out, 0, sizeof out);
            out.R = PF; out.eigvals = PF; out.mask = (uint8_t*)P; out.keep_idx = PI; out.R_r = PF; out.mu = PF; out.delta_mu = PF;
            CHECK(rk_fit_rotation(ctx, &L, &K, NULL, RK_FIT_CENTER, &out, P, fws, NULL) == RK_ERR_NO_DEVICE);
            CHECK(rk_fit_rotation(ctx, &L, &K, PF, 0, &out, P, fws - 1, NULL) == RK_ERR_WORKSPACE);
            sub.v0 = PF; sub.iterations = 5; sub.ridge = 1e-6;
            CHECK(rk_fit_subspace(ctx, &L, &K, NULL, RK_FIT_CENTER, &sub, PF, PF, PF, NULL, NULL, P, fws, NULL) ==
                  (s[3] <= 104 ? RK_ERR_NO_DEVICE : RK_ERR_UNSUPPORTED));
            CHECK(rk_gather_rotation(ctx, &L, PF, PI, PF, NULL) == RK_ERR_NO_DEVICE);
            CHECK(rk_compress(ctx, &L, &K, PF, P, &K, P, PI, NULL) == RK_ERR_NO_DEVICE);
            CHECK(rk_compress(ctx, &L, &K, PF, P, NULL, NULL, PI, NULL) == RK_ERR_NO_DEVICE);
            CHECK(rk_unpack_cache(ctx, &L, P, P, P, P, NULL) == RK_ERR_NO_DEVICE);
            CHECK(rk_query_sigma(ctx, &L, P, (int64_t)s[1] * 32 * 128, 32 * 128, 128, 32, PF, NULL) == RK_ERR_NO_DEVICE);
            CHECK(rk_decode_attn(ctx, &L, P, P, P, PF, PF, 0.0f, P, P, ws, NULL) == RK_ERR_NO_DEVICE);
            CHECK(rk_decode_attn(ctx, &L, P, P, P, PF, NULL, 0.5f, P, P, ws - 1, NULL) == RK_ERR_WORKSPACE);
            CHECK(rk_decode_attn(ctx, &L, (char*)P + 2, P, P, PF, NULL, 0.0f, P, P, ws, NULL) == RK_ERR_INVALID_ARG);
            {
                rk_status st = rk_decode_attn_static(ctx, &L, P, P, P, PF, PF, 0.0f, P, NULL);
                CHECK(st == (ws <= RK_STATIC_SCRATCH_BYTES ? RK_ERR_NO_DEVICE : RK_ERR_WORKSPACE));
            }
            if (s[6] < s[5]) {
                CHECK(rk_append(ctx, &L, P, P, PF, P, P, PI, NULL) == RK_ERR_NO_DEVICE);
                CHECK(rk_append_decode_attn(ctx, &L, P, P, P, PF, PF, P, P, PI, 0.0f, P, P, ws * 2 + 4096, NULL) == RK_ERR_NO_DEVICE);
            } else {
                CHECK(rk_append(ctx, &L, P, P, PF, P, P, PI, NULL) == RK_ERR_CAPACITY);
            }
            memset(&text, 0, sizeof text);
            text.k = P; text.v = P; text.stride_t = 128; text.stride_h = 128 * 128; text.stride_b = (int64_t)s[2] * 128 * 128;
            text.capacity = 128; text.max_len = 64; text.len = PI;
            {
                rk_status st = rk_decode_attn_dual(ctx, &L, P, P, P, PF, PF, &text, 0.0f, P, P, (size_t)1 << 40, NULL);
                CHECK(st == RK_ERR_NO_DEVICE || st == RK_ERR_UNSUPPORTED);
                st = rk_append_text(ctx, &L, &text, P, P, NULL);
                CHECK(st == RK_ERR_NO_DEVICE || st == RK_ERR_UNSUPPORTED);
                st = rk_append_text_decode_attn_dual(ctx, &L, P, P, P, P, P, PF, PF, &text, 0.0f, P, P, (size_t)1 << 40, NULL);
                CHECK(st == RK_ERR_NO_DEVICE || st == RK_ERR_UNSUPPORTED);
                text.max_len = 129;
                CHECK(rk_decode_attn_dual(ctx, &L, P, P, P, PF, PF, &text, 0.0f, P, P, (size_t)1 << 40, NULL) == RK_ERR_INVALID_ARG);
            }
        }
    }
    /* invalid layouts and rows: each refused, none crashes */
    {
        rk_layout L = make_layout(2, 8, 2, 64, RK_BF16, 1024, 1000), M;
        rk_rows K = make_rows(1000, 2, 1024), Q;
        M = L; M.head_dim = 64;          CHECK(rk_validate_layout(&M) == RK_ERR_UNSUPPORTED);
        M = L; M.dtype = 9;              CHECK(rk_validate_layout(&M) == RK_ERR_UNSUPPORTED);
        M = L; M.n_kv_heads = 3;         CHECK(rk_validate_layout(&M) == RK_ERR_INVALID_ARG);
        M = L; M.keep = 0;               CHECK(rk_validate_layout(&M) == RK_ERR_INVALID_ARG);
        M = L; M.keep = 129;             CHECK(rk_validate_layout(&M) == RK_ERR_INVALID_ARG);
        M = L; M.capacity = 1000;        CHECK(rk_validate_layout(&M) != RK_OK);
        M = L; M.batch = -1;             CHECK(rk_validate_layout(&M) == RK_ERR_INVALID_ARG);
        M = L; M.max_seq_len = 2048;     CHECK(rk_decode_attn(ctx, &M, P, P, P, PF, NULL, 0.0f, P, P, (size_t)1 << 40, NULL) == RK_ERR_CAPACITY);
        M = L; M.max_seq_len = -1;       CHECK(rk_validate_layout(&M) == RK_ERR_INVALID_ARG);
        M = L; M.batch = 0x7fffffff;     CHECK(rk_validate_layout(&M) == RK_ERR_INVALID_ARG);
        M = L; M.batch = 65535; M.n_q_heads = M.n_kv_heads = 65535; M.keep = 128; M.capacity = RK_MAX_TOKENS; M.max_seq_len = RK_MAX_TOKENS;
        CHECK(rk_validate_layout(&M) == RK_OK && rk_cache_bytes(&M, &kb, &vb) == RK_OK && kb > 0 && vb >= kb);
        CHECK(rk_decode_plan(ctx, &M, &ns, &tps) == RK_OK && ns >= 1);
        CHECK(rk_decode_workspace_size(ctx, &M) > 0 && rk_fit_workspace_size(&M, RK_MAX_TOKENS) > 0);
        M.capacity = RK_MAX_TOKENS + 32;  CHECK(rk_validate_layout(&M) == RK_ERR_INVALID_ARG);
        Q = K; Q.n_tokens = RK_MAX_TOKENS + 1; CHECK(rk_compress(ctx, &L, &Q, PF, P, NULL, NULL, PI, NULL) == RK_ERR_INVALID_ARG);
        CHECK(rk_validate_layout(NULL) == RK_ERR_INVALID_ARG);
        CHECK(rk_cache_bytes(NULL, &kb, &vb) == RK_ERR_INVALID_ARG && rk_cache_bytes(&L, NULL, &vb) == RK_OK);
        CHECK(rk_fit_workspace_size(&L, -1) == 0 && rk_fit_workspace_size(NULL, 10) == 0);
        CHECK(rk_decode_plan(ctx, &L, NULL, &tps) == RK_ERR_INVALID_ARG);
        Q = K; Q.data = NULL;            CHECK(rk_compress(ctx, &L, &Q, PF, P, NULL, NULL, PI, NULL) == RK_ERR_INVALID_ARG);
        Q = K; Q.n_tokens = 2000;        CHECK(rk_compress(ctx, &L, &Q, PF, P, NULL, NULL, PI, NULL) == RK_ERR_CAPACITY);
        Q = K; Q.stride_t = 64;          CHECK(rk_compress(ctx, &L, &Q, PF, P, NULL, NULL, PI, NULL) == RK_ERR_INVALID_ARG);
        Q = K; Q.tok_idx = PI;           CHECK(rk_compress(ctx, &L, &Q, PF, P, NULL, NULL, PI, NULL) == RK_ERR_INVALID_ARG);
        Q = K; Q.n_tokens = -5;          CHECK(rk_compress(ctx, &L, &Q, PF, P, NULL, NULL, PI, NULL) == RK_ERR_INVALID_ARG);
        CHECK(rk_compress(NULL, &L, &K, PF, P, NULL, NULL, PI, NULL) == RK_ERR_INVALID_ARG);
        CHECK(rk_stream_read(ctx, NULL, 1024, NULL) == RK_ERR_INVALID_ARG);
        CHECK(rk_stream_read(ctx, P, 1 << 20, NULL) == RK_ERR_NO_DEVICE);
    }
    /* options: accepted values change the plan, rejected ones leave a message */
    {
        rk_layout L = make_layout(8, 28, 4, 64, RK_BF16, 16448, 16384);
        int32_t ns0;
        CHECK(rk_decode_plan(ctx, &L, &ns0, &tps) == RK_OK);
        CHECK(rk_set_option(ctx, RK_OPT_DECODE_SPLITS, 5) == RK_OK);
        CHECK(rk_decode_plan(ctx, &L, &ns, &tps) == RK_OK && ns >= 1 && ns <= 5);
        CHECK(rk_set_option(ctx, RK_OPT_DECODE_SPLITS, 0) == RK_OK);
        CHECK(rk_decode_plan(ctx, &L, &ns, &tps) == RK_OK && ns == ns0);
        CHECK(rk_set_option(ctx, RK_OPT_DECODE_SPLITS, -1) == RK_ERR_INVALID_ARG && strlen(rk_last_error(ctx)) > 0);
        CHECK(rk_set_option(ctx, RK_OPT_FORCE_GENERIC, 1) == RK_OK && rk_set_option(ctx, RK_OPT_FORCE_GENERIC, 0) == RK_OK);
        CHECK(rk_set_option(ctx, RK_OPT_FUSE_MERGE, 0) == RK_OK && rk_set_option(ctx, RK_OPT_FUSE_MERGE, 1) == RK_OK);
        CHECK(rk_set_option(ctx, 12345, 1) == RK_ERR_INVALID_ARG);
        CHECK(rk_set_option(NULL, RK_OPT_FORCE_GENERIC, 1) == RK_ERR_INVALID_ARG);
    }
    printf("%d checks passed\n", n_checks);
    return rk_destroy(ctx) == RK_OK ? 0 : 1001;
}
