/*
 * rotatek.h -- C ABI of the RotateK hot path on AMD MI355X (gfx950).
 *
 * RotateK (arXiv 2605.19218) prunes Key-cache channels head-wise after an
 * orthogonal PCA rotation R of the channel space.  This library implements
 * the prefill-side construction of the rotated, pruned cache (Alg. 1 with the
 * full eigendecomposition of Sec. 3.2 as the solver) and the decode-step
 * attention over it (Alg. 2 steps 1-3 and 6, realised as the split-K /
 * merge pair of App. C).
 *
 * Conventions
 *   - Every tensor argument is a DEVICE pointer owned by the caller.  The
 *     library never allocates, frees or retains tensor memory; scratch comes
 *     from a caller-provided workspace sized by rk_*_workspace_size().  The
 *     only device memory of its own is what a context holds from rk_create to
 *     rk_destroy (512 KB of counters) and the fixed scratch array behind
 *     rk_decode_attn_static; no other call allocates or frees.
 *   - A context holds small device counters that rk_append, rk_decode_attn and
 *     rk_append_decode_attn use and leave at zero.  Calls on ONE context must
 *     therefore not overlap in time on the GPU (use one stream per context, or
 *     one context per stream); calls on different contexts are independent.
 *   - All kernels are enqueued on the caller's stream (`stream` is a
 *     hipStream_t passed as void*; NULL = the default stream).  Calls are
 *     asynchronous.  Argument validation is synchronous and precedes any launch.
 *   - Every function returns rk_status; no C++ exception crosses the boundary.
 *   - head_dim d must be 128.  `keep` (the paper's k, App. C's d_keep) is
 *     1..128.  dtype is the storage type of K, V, q, out and of the packed
 *     cache; R, R_r, mu, delta_mu, eigenvalues and all scratch are fp32.
 *   - Query head h reads KV head h / (n_q_heads / n_kv_heads) (App. C: R is
 *     indexed [B, H_kv, d, d_keep]).
 *   - Cache layout: the packed rotated keys K~ and the values V live in two
 *     caller-allocated buffers of rk_cache_bytes() bytes whose INTERNAL layout is
 *     fragment-major (tiled so that the decode kernel's matrix-core operands are
 *     contiguous 1 KB pieces of HBM): per (b, h_kv) slab of `capacity` tokens
 *     (from 4096 tokens on, consecutive slabs are spaced up to 255 tokens further
 *     apart than `capacity`, which keeps the decode's concurrent streams on
 *     different memory channels; rk_cache_bytes() includes that spacing),
 *       K~ element (token t, channel c):  [t/16][c/8][t%16][c%8], keep padded to 16
 *       V  element (token t, channel c):  [t/32][c/16][g][c%16][jj],
 *                                         g = (t%16)/4, jj = 4*((t%32)/16) + t%4
 *     Only rk_compress and rk_append write them; rk_unpack_cache converts a cache
 *     back to row-major [B, H_kv, capacity, keep] / [B, H_kv, capacity, d] for
 *     inspection.  capacity must be a multiple of 32.
 *   - Sequence lengths live on the device (int32 seq_len[B]); the host gives
 *     an upper bound max_seq_len that sizes the grids.  Kernels never read or
 *     write rows >= min(seq_len[b], capacity).
 */
#ifndef ROTATEK_H
#define ROTATEK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RK_OK = 0,
    RK_ERR_INVALID_ARG = 1,   /* NULL pointer, non-positive size, H_q % H_kv != 0, ... */
    RK_ERR_UNSUPPORTED = 2,   /* head_dim != 128, unknown dtype                        */
    RK_ERR_CAPACITY = 3,      /* more rows than `capacity`                             */
    RK_ERR_WORKSPACE = 4,     /* workspace NULL or smaller than rk_*_workspace_size()  */
    RK_ERR_HIP = 5,           /* a HIP call failed; text in rk_last_error()            */
    RK_ERR_NO_DEVICE = 6      /* arguments are valid but the context has no device     */
} rk_status;

enum { RK_F32 = 0, RK_BF16 = 1 };

/* Largest token count per sequence that any size field may hold (capacity, max_seq_len, n_tokens). */
#define RK_MAX_TOKENS (1 << 30)

/* rk_fit_rotation flags */
enum {
    RK_FIT_CENTER = 1u        /* subtract the per-head channel mean (Alg. 1 steps 1-2).
                                 Without it the scatter is the literal K^T K.          */
};

/* rk_set_option keys */
enum {
    RK_OPT_FORCE_GENERIC = 1, /* value != 0: use the plain (non-MFMA) kernels everywhere  */
    RK_OPT_DECODE_SPLITS = 2, /* value > 0: fix the split-K factor N_s; 0 = automatic     */
    RK_OPT_FUSE_MERGE = 3     /* value == 0: rk_decode_attn always merges its partials in a
                                 second launch (default 1: inside the split launch where
                                 the shape allows it)                                    */
};

#define RK_DEVICE_NONE (-1)

typedef struct rk_ctx rk_ctx;

/* Shape of one attention layer's cache; shared by all calls. */
typedef struct {
    int32_t batch;            /* B                                                    */
    int32_t n_q_heads;        /* H_q                                                  */
    int32_t n_kv_heads;       /* H_kv, divides H_q                                    */
    int32_t head_dim;         /* d = 128                                              */
    int32_t keep;             /* r: kept channels per head, 1..d                      */
    int32_t dtype;            /* RK_F32 | RK_BF16                                     */
    int32_t capacity;         /* tokens allocated per (b, h_kv) in K~ and V; multiple of 32, <= RK_MAX_TOKENS */
    int32_t max_seq_len;      /* host upper bound on seq_len[b]                       */
    const int32_t* seq_len;   /* device [B]: tokens currently cached per sequence     */
} rk_layout;

/* Where the unrotated prefill Keys (or Values) come from.
 * Row t of head (b, h) is at data + b*stride_b + h*stride_h + row*stride_t
 * (strides in ELEMENTS, channels contiguous), where
 *   row = t                                if tok_idx == NULL, t < n_b
 *   row = tok_idx[tok_off[b] + t]          otherwise,          t < n_b
 * and n_b = tok_off[b+1]-tok_off[b] (token list), else n_tokens_dev[b]
 * (if given), else n_tokens.  n_tokens is always a host upper bound on n_b.
 * The token list is the stand-in for a token pruner's keep set (Fig. 3a).    */
typedef struct {
    const void* data;
    int64_t stride_b, stride_h, stride_t;
    int32_t n_tokens;
    const int32_t* n_tokens_dev;   /* device [B] or NULL  */
    const int32_t* tok_idx;        /* device or NULL      */
    const int64_t* tok_off;        /* device [B+1]; required with tok_idx */
} rk_rows;

/* The unrotated, full-width prompt/text segment of the cache (Alg. 2 inputs
 * K_pt [M x d] and the text rows of V; Fig. 3(b)): element (b, h, t, c) of both
 * k and v is at data[b*stride_b + h*stride_h + t*stride_t + c], L->dtype, device
 * memory, caller-owned.  Bases 16-byte aligned and strides multiples of 8
 * elements.  Sequence b holds len[b] <= max_len rows (len device [B]; NULL =
 * max_len for every sequence, rk_decode_attn_dual only); max_len is the host's
 * upper bound of them and capacity the rows allocated per (b, h).            */
typedef struct {
    void* k;
    void* v;
    int64_t stride_b, stride_h, stride_t;
    int32_t capacity;
    int32_t max_len;
    int32_t* len;
} rk_text;

/* Outputs of rk_fit_rotation (all device, fp32 unless noted). */
typedef struct {
    float* R;            /* [B,H_kv,d,d]  column c = eigenvector of eigvals[c] (solver order) */
    float* eigvals;      /* [B,H_kv,d]    eigenvalues of C_q, same column order                */
    uint8_t* mask;       /* [B,H_kv,d]    1 = column kept (its eigenvalue ranks among the top r) */
    int32_t* keep_idx;   /* [B,H_kv,r]    keep_idx[j] = column whose eigenvalue has rank j      */
    float* R_r;          /* [B,H_kv,d,r]  R_r[:, j] = R[:, keep_idx[j]]  (the paper's R_k)      */
    float* mu;           /* [B,H_kv,d]    per-head channel mean of the fitted Keys             */
    float* delta_mu;     /* [B,H_kv,d]    mu - R_r R_r^T mu  (Alg. 1 step 15)                   */
    float* cov;          /* optional [B,H_kv,d,d]: the un-weighted scatter of Alg. 1 step 3     */
    int32_t* sweeps;     /* optional [B,H_kv] (int32): Jacobi sweeps the eigensolver used; 20 (its limit)
                          * means that the off-diagonal norm was still above 2e-8 ||C_q||_F: not converged */
} rk_fit_out;

/* ---- context ------------------------------------------------------------- */
/* Create a context bound to HIP device `device`.  RK_DEVICE_NONE makes a
 * host-only context: every entry point then validates its arguments exactly
 * as usual and returns RK_ERR_NO_DEVICE in place of launching.               */
rk_status rk_create(rk_ctx** out, int device);
rk_status rk_destroy(rk_ctx* ctx);
const char* rk_status_str(rk_status s);
const char* rk_last_error(const rk_ctx* ctx);          /* text of the last failure */
rk_status rk_set_option(rk_ctx* ctx, int32_t key, int64_t value);

/* Validate a layout on the host (also done inside every entry point). */
rk_status rk_validate_layout(const rk_layout* L);

/* Bytes the caller must allocate for the packed-Key cache and the Value cache. */
rk_status rk_cache_bytes(const rk_layout* L, size_t* k_packed_bytes, size_t* v_cache_bytes);

/* Bytes of workspace rk_fit_rotation / rk_fit_subspace need for at most max_tokens rows per sequence
 * (0 for an invalid layout or max_tokens outside 0..RK_MAX_TOKENS).  At least 1.3 MB per (b, h_kv):
 * the eigensolver records its rotations there (up to 20 sweeps) after the covariance partials,
 * 64 KB per 2048 rows, are no longer needed. */
size_t rk_fit_workspace_size(const rk_layout* L, int32_t max_tokens);
/* Bytes of workspace rk_decode_attn needs (depends on batch, heads, max_seq_len). */
size_t rk_decode_workspace_size(const rk_ctx* ctx, const rk_layout* L);
/* The split-K plan rk_decode_attn will use: N_s and the tokens of the largest split
 * (the 128-token tiles are shared out evenly, split sizes differ by at most one
 * tile).  App. C: N_s = max(1, min(ceil(S_v / BLOCK_N), 64)) on the A100; here it
 * is sized to fill 256 compute units.                                         */
rk_status rk_decode_plan(const rk_ctx* ctx, const rk_layout* L, int32_t* n_splits, int32_t* tokens_per_split);

/* ---- measurement helper: streaming-read ceiling --------------------------------
 * Reads `bytes` (a positive multiple of 16) of device memory at `src` (16-byte
 * aligned) once with plain streaming loads and keeps nothing.  The decode step is
 * bound by how fast the cache can be streamed from HBM (Sec. 4, "memory IO"); a
 * benchmark times this call on a buffer of the cache's size to get the rate the
 * device actually sustains for such a read, next to the datasheet peak.
 * Errors: INVALID_ARG, NO_DEVICE, HIP.                                          */
rk_status rk_stream_read(rk_ctx* ctx, const void* src, size_t bytes, void* stream);

/* ---- Alg. 1 steps 1-13 with the full eigendecomposition + keep-mask ---------
 * Per (b, h_kv): mu and the centered scatter C = (K-mu)^T (K-mu) of the rows
 * described by `keys` (Alg. 1 steps 1-3); C_q = (sigma sigma^T) .* C (step 5,
 * Eq. 4; sigma [B,H_kv,d] fp32 device or NULL = ones); all d eigenpairs of
 * C_q ("Query-Weighted PCA": R = eigenvectors of C_q); rank of every
 * eigenvalue (descending, ties -> lower column) -> mask, keep_idx, R_r;
 * delta_mu (step 15).  n_b = 0 gives mu = 0, C = 0 (R = I).
 * The eigensolver is a parallel Jacobi iteration that stops when the off-diagonal
 * Frobenius norm is at most 2e-8 ||C_q||_F, or after 20 sweeps (see `sweeps`).
 * Errors: INVALID_ARG (NULL required pointer, bad strides/sizes), UNSUPPORTED,
 * WORKSPACE, HIP.                                                             */
rk_status rk_fit_rotation(rk_ctx* ctx, const rk_layout* L, const rk_rows* keys,
                          const float* sigma, uint32_t flags, const rk_fit_out* out,
                          void* workspace, size_t workspace_bytes, void* stream);

/* ---- Alg. 1 step 4: query-window channel weights ---------------------------------
 * sigma[b, h_kv, j] = l2 norm over the `window` most recent prefill queries of channel
 * j (Sec. 3.2, W = 32 in the paper), pooled over the G = H_q / H_kv query heads that
 * share the KV head (the paper states the per-head formula; under grouped-query
 * attention one rotation serves G heads, so their windows are stacked).  q_window:
 * device, L->dtype, element (b, h_q, w, c) at b*stride_b + h_q*stride_h + w*stride_w
 * + c.  sigma: device fp32 [B,H_kv,d], the `sigma` argument of rk_fit_rotation and
 * rk_fit_subspace.  Errors: INVALID_ARG, HIP.                                      */
rk_status rk_query_sigma(rk_ctx* ctx, const rk_layout* L, const void* q_window, int64_t stride_b,
                         int64_t stride_h, int64_t stride_w, int32_t window, float* sigma, void* stream);

/* Parameters of the subspace solver (Alg. 1 inputs T and epsilon, and the draw of step 6). */
typedef struct {
    const float* v0;      /* device [B,H_kv,d,keep] fp32: the start basis V^(0), i.i.d. N(0,1), drawn by the caller */
    int32_t iterations;   /* T >= 1 (the paper uses 5)                                                             */
    double ridge;         /* epsilon >= 0 of the trace-scaled ridge rho = epsilon tr(G) / k                         */
} rk_subspace;

/* ---- Alg. 1 with the Cholesky-based subspace iteration as the solver (steps 1-13, 16; App. E)
 * mu and the scatter as in rk_fit_rotation (same rows, sigma and flags), then T
 * rounds of V <- C_q V, G = V^T V, L = chol(G + rho I), V <- V L^{-T}, all in one
 * launch and in fp64.  Outputs (device, fp32): R_r [B,H_kv,d,keep] = V^(T) (a basis
 * of the leading subspace, orthonormal up to the ridge, NOT eigenvectors one by
 * one: there are no eigenvalues, mask or keep_idx on this route); mu, delta_mu
 * [B,H_kv,d]; optionally cov [B,H_kv,d,d] and status [B,H_kv] (int32: 0, or t+1 if
 * iteration t met a non-positive Cholesky pivot, in which case that head's R_r and
 * delta_mu are undefined).  keep <= 104 (the basis and the Gram matrix stay in LDS
 * as doubles); larger keep: RK_ERR_UNSUPPORTED, use rk_fit_rotation.  Workspace as
 * rk_fit_rotation.  Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP.          */
rk_status rk_fit_subspace(rk_ctx* ctx, const rk_layout* L, const rk_rows* keys, const float* sigma,
                          uint32_t flags, const rk_subspace* solver, float* R_r, float* mu,
                          float* delta_mu, float* cov, int32_t* status, void* workspace,
                          size_t workspace_bytes, void* stream);

/* R_r[:, j] = R[:, keep_idx[j]] for every (b, h_kv): re-derives the d x r form
 * the kernels read from the canonical (R, keep_idx) state.                    */
rk_status rk_gather_rotation(rk_ctx* ctx, const rk_layout* L, const float* R,
                             const int32_t* keep_idx, float* R_r, void* stream);

/* ---- Alg. 1 step 14: K~ = K R_k, rounded once to the cache dtype ------------
 * Writes tokens [0, n_b) of k_packed[b, h] (n_b as defined at rk_rows; must be
 * <= capacity, checked on the host against keys->n_tokens).  If `values` is
 * non-NULL its rows (gathered through the same token list) are re-tiled into
 * v_cache; this is how the Value cache is built.  If seq_len_out is non-NULL it
 * receives n_b per sequence.
 * Errors: INVALID_ARG, UNSUPPORTED, CAPACITY, HIP.                            */
rk_status rk_compress(rk_ctx* ctx, const rk_layout* L, const rk_rows* keys, const float* R_r,
                      void* k_packed, const rk_rows* values, void* v_cache,
                      int32_t* seq_len_out, void* stream);

/* Inspection helper: caches -> row-major k_rows [B,H_kv,capacity,keep] and/or
 * v_rows [B,H_kv,capacity,d] (either may be NULL).  Not on the hot path.        */
rk_status rk_unpack_cache(rk_ctx* ctx, const rk_layout* L, const void* k_packed, const void* v_cache,
                          void* k_rows, void* v_rows, void* stream);

/* ---- frozen-R append of one token per sequence ------------------------------
 * k~ = k_new R_r (R is fitted once at the end of prefill and reused, Sec. 3.2
 * Step (1)); writes token seq_len[b] of k_packed and v_cache for every KV head,
 * then seq_len[b] += 1 on the device (one launch; calls on one context must not
 * overlap on different streams).  k_new, v_new: [B,H_kv,d] in L->dtype.
 * Returns RK_ERR_CAPACITY if L->max_seq_len + 1 > capacity (nothing is
 * launched); on the device a sequence already at capacity is left untouched.  */
rk_status rk_append(rk_ctx* ctx, const rk_layout* L, const void* k_new, const void* v_new,
                    const float* R_r, void* k_packed, void* v_cache, int32_t* seq_len, void* stream);

/* ---- Alg. 2 steps 1-3, 6 over the packed cache (App. C phases 1 and 2) ------
 * q~ = q R_r, b = q . delta_mu (delta_mu NULL = no bias), scores
 * (q~ . K~_n + b) * scale with scale = 1/sqrt(d) when `scale` <= 0, softmax over
 * the seq_len[b] cached tokens, out = P V.  q, out: [B,H_q,d] in L->dtype; q and
 * both caches 16-byte aligned (the kernels read them in 16-byte pieces).
 * A sequence with seq_len[b] = 0 yields zeros.  Two launches (split-K, merge) as
 * in App. C, one when the plan has a single split.
 * Errors: INVALID_ARG, UNSUPPORTED, CAPACITY (max_seq_len > capacity),
 * WORKSPACE, HIP.                                                             */
rk_status rk_decode_attn(rk_ctx* ctx, const rk_layout* L, const void* q, const void* k_packed,
                         const void* v_cache, const float* R_r, const float* delta_mu, float scale,
                         void* out, void* workspace, size_t workspace_bytes, void* stream);

/* ---- rk_decode_attn for callers that cannot allocate ---------------------------
 * For code that may not call hipMalloc or hand over a buffer of its own making:
 * work under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation.  Same arguments, kernels and results as rk_decode_attn, without the
 * workspace: the split-K partials go to a scratch array built into the library
 * (RK_STATIC_SCRATCH_BYTES of device memory that every GPU the library runs on
 * holds until the process ends).  The call allocates and frees nothing.
 * A shape whose rk_decode_workspace_size() exceeds RK_STATIC_SCRATCH_BYTES is
 * refused with RK_ERR_WORKSPACE (text in rk_last_error) and nothing is launched.
 * All calls on one GPU share that GPU's array, from every context and stream:
 * calls that overlap in time on one GPU race on it and must be ordered by the
 * caller (calls on one stream are).  The array keeps the last call's partials;
 * nothing in it needs clearing between calls.
 * Errors: as rk_decode_attn.                                                    */
#define RK_STATIC_SCRATCH_BYTES (8u << 20)
rk_status rk_decode_attn_static(rk_ctx* ctx, const rk_layout* L, const void* q, const void* k_packed,
                                const void* v_cache, const float* R_r, const float* delta_mu, float scale,
                                void* out, void* stream);

/* ---- rk_append followed by rk_decode_attn, fused ------------------------------
 * One decode step of a layer whose new token joins the rotated cache (Sec. 3.2
 * Step (1) then Alg. 2): row seq_len[b] of k_packed / v_cache receives
 * k_new R_r / v_new, the softmax runs over seq_len[b] + 1 tokens (the new one
 * included), and seq_len[b] += 1 on the device.  Results equal rk_append then
 * rk_decode_attn up to fp32 rounding order (the stored row may differ from
 * rk_append's by one unit in the last place of the storage type plus the fp32
 * accumulation bound).  On the matrix-core path with H_q/H_kv < 16 the append
 * rides in the decode's own launches (k_new takes a free column of the
 * q~ = q R_r product): one launch where rk_decode_attn is one launch, else the
 * split and the merge launch; otherwise the call issues rk_append's and
 * rk_decode_attn's launches.  Calls on one context that overlap in time (two
 * streams) share the context's counters and must not be made.
 * L->max_seq_len bounds seq_len[b] BEFORE the call; L->seq_len is ignored in
 * favour of `seq_len` (device [B], read and written).  k_new, v_new: [B,H_kv,d],
 * q, out: [B,H_q,d], all L->dtype; q, k_new and v_new 16-byte aligned.  Workspace:
 * rk_decode_workspace_size of the layout with max_seq_len + 1.  A sequence
 * already at capacity is left untouched and attends over what it has.
 * Errors: INVALID_ARG, CAPACITY (max_seq_len + 1 > capacity; nothing is
 * launched), UNSUPPORTED, WORKSPACE, HIP.                                      */
rk_status rk_append_decode_attn(rk_ctx* ctx, const rk_layout* L, const void* k_new, const void* v_new,
                                const void* q, const float* R_r, const float* delta_mu, void* k_packed,
                                void* v_cache, int32_t* seq_len, float scale, void* out, void* workspace,
                                size_t workspace_bytes, void* stream);

/* ---- Alg. 2 in full: steps 1-6 with the prompt/text segment (App. C phase 2) --
 * As rk_decode_attn for the visual segment; in addition the len[b] rows of
 * `text` are scored with the unrotated query, s_pt = q . K_pt * scale (no
 * bias), and ONE softmax runs over the concatenation [s_vis; s_pt]; out =
 * P [V_vis; V_pt].  The bias therefore matters here: it shifts the visual
 * scores against the text scores.  Either segment may be empty per sequence;
 * both empty yields zeros.  On the matrix-core path the text attention runs in
 * extra work-groups of the split-K launch, in slices of about 512 rows that
 * each leave a partial of their own, and visual and text partials are folded
 * alike, inside that launch where rk_decode_attn folds its own, else by the
 * merge kernel; with fp32 storage or the plain kernels
 * the second kernel runs the text attention itself and then folds the visual
 * partials (the fusion App. C describes).  Same workspace as rk_decode_attn.
 * Errors: as rk_decode_attn, plus INVALID_ARG for a malformed `text`
 * (NULL pointers, misaligned base or strides, max_len > capacity).            */
rk_status rk_decode_attn_dual(rk_ctx* ctx, const rk_layout* L, const void* q, const void* k_packed,
                              const void* v_cache, const float* R_r, const float* delta_mu,
                              const rk_text* text, float scale, void* out, void* workspace,
                              size_t workspace_bytes, void* stream);

/* Append one full-width token per sequence to the text segment (the paper keeps
 * tokens that arrive after prefill unrotated; they are the K_pt rows of Alg. 2):
 * row len[b] of text->k / text->v receives k_new / v_new [B,H_kv,d] (L->dtype)
 * for every KV head, then len[b] += 1 on the device.  text->len must be given.
 * Returns RK_ERR_CAPACITY if text->max_len + 1 > text->capacity (nothing is
 * launched); on the device a sequence already at capacity is left untouched.  */
rk_status rk_append_text(rk_ctx* ctx, const rk_layout* L, const rk_text* text, const void* k_new,
                         const void* v_new, void* stream);

/* ---- rk_append_text followed by rk_decode_attn_dual, fused ---------------------
 * One decode step of a layer whose new token joins the unrotated text segment
 * (the paper's handling of tokens that arrive after prefill, Alg. 2 input
 * K_pt): row len[b] of text->k / text->v receives k_new / v_new [B,H_kv,d],
 * len[b] += 1 on the device, and the softmax of this step already includes the
 * new row.  Same results as the two calls (the rows are copied, the attention
 * arithmetic is the same code); the same launches as rk_decode_attn_dual, the
 * copy riding in the first.  text->len must be given; text->max_len bounds
 * len[b] BEFORE the call.  k_new, v_new 16-byte aligned.  A sequence whose text
 * segment is already full is left untouched and attends over what it has.
 * Errors: as rk_decode_attn_dual, plus CAPACITY if text->max_len + 1 >
 * text->capacity (nothing is launched).                                       */
rk_status rk_append_text_decode_attn_dual(rk_ctx* ctx, const rk_layout* L, const void* k_new, const void* v_new,
                                          const void* q, const void* k_packed, const void* v_cache,
                                          const float* R_r, const float* delta_mu, const rk_text* text,
                                          float scale, void* out, void* workspace, size_t workspace_bytes,
                                          void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ROTATEK_H */
