// C ABI of the RotateK hot path: argument validation, workspace carving and
// kernel launches.  See include/rotatek.h for the contract of every entry point.
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "rk_kernels.hpp"
#include "rotatek.h"

struct rk_ctx {
    int device;           // RK_DEVICE_NONE: host-only validation context
    int n_cu;
    int force_generic;
    int decode_splits;
    int fuse_merge;       // fold the split-K merge into the split launch where the shape allows it
    int xcd_deal_ok;      // work-groups with equal (linear index mod 8) share an XCD on this device (probed)
    int32_t* tickets;     // device: APP_TICKETS zero-initialised counters (one per batch item, rk_append)
    void* static_scratch; // this device's copy of `scratch` below (its device address), for rk_decode_attn_static
    char err[256];
};

// Split-K partials of rk_decode_attn_static, for callers that cannot hand over a workspace they
// allocated.  Every GPU the library runs on holds its own copy until the process ends.  In host code
// this name is only a stand-in for the symbol: the device address of a GPU's copy comes from
// hipGetSymbolAddress (rk_create, with that device current) and is what kernels and copies receive.
// Nothing in it has to start at zero: the merge kernel reads exactly the partial slots that the split
// kernel of the same call has written.
static __device__ __align__(256) unsigned char scratch[RK_STATIC_SCRATCH_BYTES];

namespace {

using namespace rk;

rk_status fail(rk_ctx* ctx, rk_status s, const char* fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return s;
}

rk_status hip_fail(rk_ctx* ctx, hipError_t e, const char* what)
{
    return fail(ctx, RK_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

constexpr int APP_TICKETS = 1 << 16;   // >= batch
constexpr int DEC_COUNTERS = 1 << 16;  // units (b, h_kv, head group) whose split-K merge can ride in the split launch

size_t elem_size(int dtype) { return dtype == RK_F32 ? 4 : 2; }
size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

rk_status check_layout(rk_ctx* ctx, const rk_layout* L)
{
    if (!L) return fail(ctx, RK_ERR_INVALID_ARG, "layout is NULL");
    if (L->head_dim != D) return fail(ctx, RK_ERR_UNSUPPORTED, "head_dim %d: only 128 is supported", L->head_dim);
    if (L->dtype != RK_F32 && L->dtype != RK_BF16) return fail(ctx, RK_ERR_UNSUPPORTED, "unknown dtype %d", L->dtype);
    if (L->batch < 1 || L->n_q_heads < 1 || L->n_kv_heads < 1)
        return fail(ctx, RK_ERR_INVALID_ARG, "batch/head counts must be positive");
    if (L->batch > 65535 || L->n_q_heads > 65535) return fail(ctx, RK_ERR_INVALID_ARG, "batch/head counts exceed 65535");
    if (L->n_q_heads % L->n_kv_heads != 0)
        return fail(ctx, RK_ERR_INVALID_ARG, "n_q_heads %d is not a multiple of n_kv_heads %d", L->n_q_heads, L->n_kv_heads);
    if (L->keep < 1 || L->keep > D) return fail(ctx, RK_ERR_INVALID_ARG, "keep %d outside 1..128", L->keep);
    if (L->capacity < 32 || L->capacity % 32 != 0)
        return fail(ctx, RK_ERR_INVALID_ARG, "capacity %d must be a positive multiple of 32", L->capacity);
    if (L->max_seq_len < 0) return fail(ctx, RK_ERR_INVALID_ARG, "max_seq_len is negative");
    // token counts stay below 2^30, so that rounding one up to a tile never leaves the range of int
    if (L->capacity > RK_MAX_TOKENS || L->max_seq_len > RK_MAX_TOKENS)
        return fail(ctx, RK_ERR_INVALID_ARG, "capacity / max_seq_len exceed %d tokens", RK_MAX_TOKENS);
    return RK_OK;
}

rk_status check_rows(rk_ctx* ctx, const rk_layout* L, const rk_rows* r, const char* name)
{
    if (!r || !r->data) return fail(ctx, RK_ERR_INVALID_ARG, "%s: NULL", name);
    if (r->n_tokens < 0) return fail(ctx, RK_ERR_INVALID_ARG, "%s: n_tokens is negative", name);
    if (r->n_tokens > RK_MAX_TOKENS) return fail(ctx, RK_ERR_INVALID_ARG, "%s: n_tokens exceeds %d", name, RK_MAX_TOKENS);
    if (r->tok_idx && !r->tok_off) return fail(ctx, RK_ERR_INVALID_ARG, "%s: tok_idx given without tok_off", name);
    if (r->stride_t < D || r->stride_b < 0 || r->stride_h < 0)
        return fail(ctx, RK_ERR_INVALID_ARG, "%s: bad strides", name);
    const int64_t ea = 16 / (int64_t)elem_size(L->dtype);    // elements per 16 bytes
    if (((uintptr_t)r->data & 15) || r->stride_t % ea || r->stride_b % ea || r->stride_h % ea)
        return fail(ctx, RK_ERR_INVALID_ARG, "%s: rows must be 16-byte aligned", name);
    return RK_OK;
}

RowsDev to_dev(const rk_rows* r)
{
    RowsDev d;
    d.data = r->data; d.sb = r->stride_b; d.sh = r->stride_h; d.st = r->stride_t;
    d.n_tokens = r->n_tokens; d.n_dev = r->n_tokens_dev; d.tok_idx = r->tok_idx; d.tok_off = r->tok_off;
    return d;
}

int cov_chunks(int max_tokens) { int n = (max_tokens + COV_CHUNK - 1) / COV_CHUNK; return n < 1 ? 1 : n; }

// The covariance partials are dead once the covariance is reduced: the eigensolver's recorded
// rotations reuse their space (the region is sized for the larger of the two).
struct FitWs { size_t part_S, part_sum, cov, sweeps, total; };
FitWs fit_ws(const rk_layout* L, int max_tokens)
{
    size_t U = (size_t)L->batch * L->n_kv_heads, nc = (size_t)cov_chunks(max_tokens);
    FitWs w;
    w.part_S = 0;
    size_t first = U * nc * D * D * sizeof(float);
    if (first < eig_rotation_bytes(U)) first = eig_rotation_bytes(U);
    w.part_sum = align_up(w.part_S + first, 256);
    w.cov = align_up(w.part_sum + U * nc * D * sizeof(float), 256);
    w.sweeps = align_up(w.cov + U * D * D * sizeof(float), 256);
    w.total = align_up(w.sweeps + U * sizeof(int32_t), 256);
    return w;
}

bool use_mfma_decode(const rk_ctx* ctx, const rk_layout* L)
{
    return !(ctx && ctx->force_generic) && decode_mfma_supported(L->dtype, L->keep);
}

rk_status check_text(rk_ctx* ctx, const rk_text* t, bool need_len)
{
    if (!t->k || !t->v) return fail(ctx, RK_ERR_INVALID_ARG, "text: NULL k or v");
    if (((uintptr_t)t->k & 15) || ((uintptr_t)t->v & 15))
        return fail(ctx, RK_ERR_INVALID_ARG, "text: k and v must be 16-byte aligned");
    if (t->stride_b < 0 || t->stride_h < 0 || t->stride_t < D || (t->stride_b % 8) || (t->stride_h % 8) ||
        (t->stride_t % 8))
        return fail(ctx, RK_ERR_INVALID_ARG, "text: strides must be non-negative multiples of 8 elements, stride_t >= %d", D);
    if (t->capacity < 0 || t->max_len < 0) return fail(ctx, RK_ERR_INVALID_ARG, "text: negative capacity or max_len");
    if (t->max_len > t->capacity)
        return fail(ctx, RK_ERR_INVALID_ARG, "text: max_len %d exceeds capacity %d", t->max_len, t->capacity);
    if (need_len && !t->len) return fail(ctx, RK_ERR_INVALID_ARG, "text: len is NULL");
    return RK_OK;
}

// N_s and the number of 128-token tiles they share (split s gets floor(tiles / N_s) tiles, the
// last tiles % N_s splits one more)
void decode_plan(const rk_ctx* ctx, const rk_layout* L, int* S_out, int* tiles_out)
{
    const int G = L->n_q_heads / L->n_kv_heads;
    const bool mfma = use_mfma_decode(ctx, L);
    const long units = mfma ? (long)L->batch * L->n_kv_heads * ((G + 15) / 16) : (long)L->batch * L->n_q_heads;
    const int maxL = L->max_seq_len > 0 ? L->max_seq_len : 1;
    const int tiles = (maxL + 127) / 128;
    const int n_cu = ctx ? ctx->n_cu : 256;
    int S;
    if (ctx && ctx->decode_splits > 0) S = ctx->decode_splits;
    else {
        // one 4-wave work-group per compute unit: a second one gets its memory requests served only
        // after the first one's (measured: its prologue then ends 10 us later), and every work-group
        // pays its own prologue and partial
        // (rounded down: a few work-groups more than compute units would run as a second round)
        long target = n_cu;
        S = (int)(target / units);
        if (S < 1) {
            // more units than compute units: a partly filled last round costs a whole round (320 units:
            // 186 us unsplit, 162 us with four splits); take the split count 1..4 that wastes least of it
            S = 1;
            double best = 1e30;
            for (int c = 1; c <= 4; ++c) {
                const double cost = (double)((units * c + target - 1) / target) / c;
                if (cost < best - 1e-9) { best = cost; S = c; }
            }
        }
        if (S > 64) S = 64;
        // a split shorter than 512 tokens (four 32-token tiles per wave) no longer amortises its
        // prologue and its partial: measured optimum on short caches and small batches.  Very short
        // caches (under 2K tokens) still gain from up to four splits of 256 tokens or more
        // (32 heads x 1024 tokens: 9.4 us with two splits, 8.2 us with four).
        const int cap_long = tiles / 4, cap_short = tiles / 2 < 4 ? tiles / 2 : 4;
        const int cap = cap_long > cap_short ? cap_long : cap_short;
        if (S > cap) S = cap;
    }
    if (S > tiles) S = tiles;
    if (S < 1) S = 1;
    *S_out = S;
    *tiles_out = tiles;
}

hipStream_t as_stream(void* s) { return (hipStream_t)s; }

// Makes `device` current for the duration of a call and puts the caller's device back
// afterwards: the library must not change the calling thread's current device.
struct DeviceGuard {
    int prev = -1;
    hipError_t status;
    explicit DeviceGuard(int device)
    {
        status = hipGetDevice(&prev);
        if (status == hipSuccess && prev != device) status = hipSetDevice(device);
        else if (status == hipSuccess) prev = -1;          // nothing to restore
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
    DeviceGuard(const DeviceGuard&) = delete;
    DeviceGuard& operator=(const DeviceGuard&) = delete;
};

}  // namespace

extern "C" {

const char* rk_status_str(rk_status s)
{
    switch (s) {
        case RK_OK: return "ok";
        case RK_ERR_INVALID_ARG: return "invalid argument";
        case RK_ERR_UNSUPPORTED: return "unsupported configuration";
        case RK_ERR_CAPACITY: return "cache capacity exceeded";
        case RK_ERR_WORKSPACE: return "workspace missing or too small";
        case RK_ERR_HIP: return "HIP error";
        case RK_ERR_NO_DEVICE: return "context has no device";
    }
    return "unknown status";
}

rk_status rk_create(rk_ctx** out, int device)
{
    if (!out) return RK_ERR_INVALID_ARG;
    *out = nullptr;
    rk_ctx* c = new (std::nothrow) rk_ctx();
    if (!c) return RK_ERR_INVALID_ARG;
    memset(c, 0, sizeof(*c));
    c->device = device;
    c->n_cu = 256;
    c->fuse_merge = 1;
    if (device != RK_DEVICE_NONE) {
        if (device < 0) { delete c; return RK_ERR_INVALID_ARG; }
        hipDeviceProp_t prop;
        hipError_t e = hipGetDeviceProperties(&prop, device);
        if (e != hipSuccess) { delete c; return RK_ERR_HIP; }
        c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        const size_t tb = (size_t)(APP_TICKETS + DEC_COUNTERS) * sizeof(int32_t);
        DeviceGuard dev(device);
        if (dev.status != hipSuccess || hipMalloc((void**)&c->tickets, tb) != hipSuccess) {
            delete c;
            return RK_ERR_HIP;
        }
        if (hipMemset(c->tickets, 0, tb) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
            (void)hipFree(c->tickets);
            delete c;
            return RK_ERR_HIP;
        }
        // the folded merge needs all work-groups of a unit behind one L2: check how this device deals them
        bool same_xcd = false;
        if (probe_xcd_deal(c->tickets, &same_xcd) != hipSuccess) {
            (void)hipFree(c->tickets);
            delete c;
            return RK_ERR_HIP;
        }
        c->xcd_deal_ok = same_xcd ? 1 : 0;
        // this device's copy of the static scratch array (each GPU has its own, at its own address)
        if (hipGetSymbolAddress(&c->static_scratch, HIP_SYMBOL(scratch)) != hipSuccess || !c->static_scratch) {
            (void)hipFree(c->tickets);
            delete c;
            return RK_ERR_HIP;
        }
    }
    *out = c;
    return RK_OK;
}

rk_status rk_destroy(rk_ctx* ctx)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    if (ctx->tickets) {
        DeviceGuard dev(ctx->device);
        (void)hipFree(ctx->tickets);
    }
    delete ctx;
    return RK_OK;
}

const char* rk_last_error(const rk_ctx* ctx) { return ctx ? ctx->err : "context is NULL"; }

rk_status rk_set_option(rk_ctx* ctx, int32_t key, int64_t value)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    switch (key) {
        case RK_OPT_FORCE_GENERIC: ctx->force_generic = value != 0; return RK_OK;
        case RK_OPT_FUSE_MERGE: ctx->fuse_merge = value != 0; return RK_OK;
        case RK_OPT_DECODE_SPLITS:
            if (value < 0 || value > 4096) return fail(ctx, RK_ERR_INVALID_ARG, "decode splits %lld outside 0..4096", (long long)value);
            ctx->decode_splits = (int)value;
            return RK_OK;
        default: return fail(ctx, RK_ERR_INVALID_ARG, "unknown option %d", key);
    }
}

rk_status rk_validate_layout(const rk_layout* L) { return check_layout(nullptr, L); }

size_t rk_fit_workspace_size(const rk_layout* L, int32_t max_tokens)
{
    if (check_layout(nullptr, L) != RK_OK || max_tokens < 0 || max_tokens > RK_MAX_TOKENS) return 0;
    return fit_ws(L, max_tokens).total;
}

size_t rk_decode_workspace_size(const rk_ctx* ctx, const rk_layout* L)
{
    if (check_layout(nullptr, L) != RK_OK) return 0;
    int S, tiles;
    decode_plan(ctx, L, &S, &tiles);
    // (m, l, acc[d]) per split and per text slice of the dual path, plus one score per row for a fused append
    return align_up((size_t)L->batch * L->n_q_heads * ((size_t)(S + DECODE_TEXT_SLICES_MAX) * (D + 2) + 1) * sizeof(float), 256);
}

rk_status rk_decode_plan(const rk_ctx* ctx, const rk_layout* L, int32_t* n_splits, int32_t* tokens_per_split)
{
    rk_status s = check_layout(nullptr, L);
    if (s != RK_OK) return s;
    if (!n_splits || !tokens_per_split) return RK_ERR_INVALID_ARG;
    int S, tiles;
    decode_plan(ctx, L, &S, &tiles);
    *n_splits = S;
    *tokens_per_split = 128 * ((tiles + S - 1) / S);      // the largest split
    return RK_OK;
}

rk_status rk_cache_bytes(const rk_layout* L, size_t* k_packed_bytes, size_t* v_cache_bytes)
{
    rk_status s = check_layout(nullptr, L);
    if (s != RK_OK) return s;
    const size_t slabs = (size_t)L->batch * L->n_kv_heads * slab_tokens(L->capacity);       // slabs are spaced, see slab_tokens()
    if (k_packed_bytes) *k_packed_bytes = slabs * keep_padded(L->keep) * elem_size(L->dtype);
    if (v_cache_bytes) *v_cache_bytes = slabs * D * elem_size(L->dtype);
    return RK_OK;
}

rk_status rk_unpack_cache(rk_ctx* ctx, const rk_layout* L, const void* k_packed, const void* v_cache,
                          void* k_rows, void* v_rows, void* stream)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    rk_status s = check_layout(ctx, L);
    if (s != RK_OK) return s;
    if ((k_rows && !k_packed) || (v_rows && !v_cache) || (!k_rows && !v_rows))
        return fail(ctx, RK_ERR_INVALID_ARG, "unpack: nothing to do or source missing");
    if (ctx->device == RK_DEVICE_NONE) return fail(ctx, RK_ERR_NO_DEVICE, "valid arguments, but the context has no device");
    DeviceGuard dev(ctx->device);
    hipError_t e = dev.status;
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    e = launch_unpack(L->dtype, L->batch * L->n_kv_heads, L->capacity, L->keep, k_packed, v_cache, k_rows, v_rows,
                      as_stream(stream));
    if (e != hipSuccess) return hip_fail(ctx, e, "unpack launch");
    return RK_OK;
}

rk_status rk_stream_read(rk_ctx* ctx, const void* src, size_t bytes, void* stream)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    if (!src || ((uintptr_t)src & 15) || bytes == 0 || (bytes & 15))
        return fail(ctx, RK_ERR_INVALID_ARG, "stream_read: src must be non-NULL and 16-byte aligned, bytes a positive multiple of 16");
    if (ctx->device == RK_DEVICE_NONE) return fail(ctx, RK_ERR_NO_DEVICE, "valid arguments, but the context has no device");
    DeviceGuard dev(ctx->device);
    hipError_t e = dev.status;
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    e = launch_stream_read(src, bytes, ctx->n_cu, nullptr, as_stream(stream));
    if (e != hipSuccess) return hip_fail(ctx, e, "stream_read launch");
    return RK_OK;
}

rk_status rk_fit_rotation(rk_ctx* ctx, const rk_layout* L, const rk_rows* keys, const float* sigma,
                          uint32_t flags, const rk_fit_out* out, void* workspace, size_t workspace_bytes,
                          void* stream)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    rk_status s = check_layout(ctx, L);
    if (s != RK_OK) return s;
    s = check_rows(ctx, L, keys, "keys");
    if (s != RK_OK) return s;
    if (!out || !out->R || !out->eigvals || !out->mask || !out->keep_idx || !out->R_r || !out->mu || !out->delta_mu)
        return fail(ctx, RK_ERR_INVALID_ARG, "fit outputs: a required pointer is NULL");
    if (flags & ~(uint32_t)RK_FIT_CENTER) return fail(ctx, RK_ERR_INVALID_ARG, "unknown fit flags 0x%x", flags);
    const FitWs w = fit_ws(L, keys->n_tokens);
    if (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace & 255))
        return fail(ctx, RK_ERR_WORKSPACE, "fit workspace: need %zu bytes, 256-byte aligned", w.total);
    if (ctx->device == RK_DEVICE_NONE) return fail(ctx, RK_ERR_NO_DEVICE, "valid arguments, but the context has no device");

    DeviceGuard dev(ctx->device);
    hipError_t e = dev.status;
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    const int B = L->batch, Hkv = L->n_kv_heads, U = B * Hkv;
    const int ct = cov_chunk_tokens(L->dtype, !ctx->force_generic);
    int nc = (keys->n_tokens + ct - 1) / ct;        // never more than the workspace was sized for
    if (nc < 1) nc = 1;
    char* ws = (char*)workspace;
    float* part_S = (float*)(ws + w.part_S);
    float* part_sum = (float*)(ws + w.part_sum);
    float* cov = out->cov ? out->cov : (float*)(ws + w.cov);
    const RowsDev rows = to_dev(keys);
    hipStream_t st = as_stream(stream);
    e = launch_cov_partial(L->dtype, !ctx->force_generic, rows, B, Hkv, nc, part_S, part_sum, st);
    if (e != hipSuccess) return hip_fail(ctx, e, "covariance launch");
    e = launch_cov_finalize(rows, B, Hkv, nc, (flags & RK_FIT_CENTER) != 0, ct == cov_chunk_tokens(RK_BF16, true),
                            part_S, part_sum, cov, out->mu, st);
    if (e != hipSuccess) return hip_fail(ctx, e, "covariance reduction launch");
    e = launch_eig(U, cov, sigma, out->mu, L->keep, out->R, out->eigvals, out->mask, out->keep_idx, out->R_r,
                   out->delta_mu, out->sweeps, ws + w.part_S, (int32_t*)(ws + w.sweeps), st);
    if (e != hipSuccess) return hip_fail(ctx, e, "eigensolver launch");
    return RK_OK;
}

rk_status rk_query_sigma(rk_ctx* ctx, const rk_layout* L, const void* q_window, int64_t stride_b, int64_t stride_h,
                         int64_t stride_w, int32_t window, float* sigma, void* stream)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    rk_status s = check_layout(ctx, L);
    if (s != RK_OK) return s;
    if (!q_window || !sigma) return fail(ctx, RK_ERR_INVALID_ARG, "query_sigma: NULL pointer");
    if (window < 1) return fail(ctx, RK_ERR_INVALID_ARG, "query_sigma: window must be >= 1");
    if (stride_b < 0 || stride_h < 0 || stride_w < D)
        return fail(ctx, RK_ERR_INVALID_ARG, "query_sigma: strides must be non-negative, stride_w >= %d", D);
    if (ctx->device == RK_DEVICE_NONE) return fail(ctx, RK_ERR_NO_DEVICE, "valid arguments, but the context has no device");
    DeviceGuard dev(ctx->device);
    hipError_t e = dev.status;
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    e = launch_sigma_window(L->dtype, q_window, stride_b, stride_h, stride_w, L->batch, L->n_q_heads, L->n_kv_heads,
                            window, sigma, as_stream(stream));
    if (e != hipSuccess) return hip_fail(ctx, e, "query_sigma launch");
    return RK_OK;
}

rk_status rk_fit_subspace(rk_ctx* ctx, const rk_layout* L, const rk_rows* keys, const float* sigma, uint32_t flags,
                          const rk_subspace* solver, float* R_r, float* mu, float* delta_mu, float* cov_out,
                          int32_t* status, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    rk_status s = check_layout(ctx, L);
    if (s != RK_OK) return s;
    s = check_rows(ctx, L, keys, "keys");
    if (s != RK_OK) return s;
    if (!solver || !solver->v0) return fail(ctx, RK_ERR_INVALID_ARG, "fit_subspace: solver or its start basis is NULL");
    if (solver->iterations < 1 || !(solver->ridge >= 0.0))
        return fail(ctx, RK_ERR_INVALID_ARG, "fit_subspace: iterations must be >= 1 and ridge >= 0");
    if (!R_r || !mu || !delta_mu) return fail(ctx, RK_ERR_INVALID_ARG, "fit_subspace: a required output is NULL");
    if (flags & ~(uint32_t)RK_FIT_CENTER) return fail(ctx, RK_ERR_INVALID_ARG, "unknown fit flags 0x%x", flags);
    if (L->keep > subspace_max_keep())
        return fail(ctx, RK_ERR_UNSUPPORTED, "fit_subspace: keep %d exceeds %d; use rk_fit_rotation", L->keep,
                    subspace_max_keep());
    const FitWs w = fit_ws(L, keys->n_tokens);
    if (!workspace || workspace_bytes < w.total || ((uintptr_t)workspace & 255))
        return fail(ctx, RK_ERR_WORKSPACE, "fit workspace: need %zu bytes, 256-byte aligned", w.total);
    if (ctx->device == RK_DEVICE_NONE) return fail(ctx, RK_ERR_NO_DEVICE, "valid arguments, but the context has no device");

    DeviceGuard dev(ctx->device);
    hipError_t e = dev.status;
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    const int B = L->batch, Hkv = L->n_kv_heads, U = B * Hkv;
    const int ct = cov_chunk_tokens(L->dtype, !ctx->force_generic);
    int nc = (keys->n_tokens + ct - 1) / ct;
    if (nc < 1) nc = 1;
    char* ws = (char*)workspace;
    float* part_S = (float*)(ws + w.part_S);
    float* part_sum = (float*)(ws + w.part_sum);
    float* cov = cov_out ? cov_out : (float*)(ws + w.cov);
    const RowsDev rows = to_dev(keys);
    hipStream_t st = as_stream(stream);
    e = launch_cov_partial(L->dtype, !ctx->force_generic, rows, B, Hkv, nc, part_S, part_sum, st);
    if (e != hipSuccess) return hip_fail(ctx, e, "covariance launch");
    e = launch_cov_finalize(rows, B, Hkv, nc, (flags & RK_FIT_CENTER) != 0, ct == cov_chunk_tokens(RK_BF16, true),
                            part_S, part_sum, cov, mu, st);
    if (e != hipSuccess) return hip_fail(ctx, e, "covariance reduction launch");
    e = launch_subspace(U, cov, sigma, mu, solver->v0, L->keep, solver->iterations, solver->ridge, R_r, delta_mu,
                        status, st);
    if (e != hipSuccess) return hip_fail(ctx, e, "subspace iteration launch");
    return RK_OK;
}

rk_status rk_gather_rotation(rk_ctx* ctx, const rk_layout* L, const float* R, const int32_t* keep_idx,
                             float* R_r, void* stream)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    rk_status s = check_layout(ctx, L);
    if (s != RK_OK) return s;
    if (!R || !keep_idx || !R_r) return fail(ctx, RK_ERR_INVALID_ARG, "gather_rotation: NULL pointer");
    if (ctx->device == RK_DEVICE_NONE) return fail(ctx, RK_ERR_NO_DEVICE, "valid arguments, but the context has no device");
    DeviceGuard dev(ctx->device);
    hipError_t e = dev.status;
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    e = launch_gather_rotation(L->batch * L->n_kv_heads, L->keep, R, keep_idx, R_r, as_stream(stream));
    if (e != hipSuccess) return hip_fail(ctx, e, "gather launch");
    return RK_OK;
}

rk_status rk_compress(rk_ctx* ctx, const rk_layout* L, const rk_rows* keys, const float* R_r, void* k_packed,
                      const rk_rows* values, void* v_cache, int32_t* seq_len_out, void* stream)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    rk_status s = check_layout(ctx, L);
    if (s != RK_OK) return s;
    s = check_rows(ctx, L, keys, "keys");
    if (s != RK_OK) return s;
    if (!R_r || !k_packed) return fail(ctx, RK_ERR_INVALID_ARG, "compress: R_r or k_packed is NULL");
    if ((uintptr_t)k_packed & 15) return fail(ctx, RK_ERR_INVALID_ARG, "compress: k_packed must be 16-byte aligned");
    if (values) {
        s = check_rows(ctx, L, values, "values");
        if (s != RK_OK) return s;
        if (!v_cache || ((uintptr_t)v_cache & 15))
            return fail(ctx, RK_ERR_INVALID_ARG, "compress: values given but v_cache is NULL or misaligned");
        if (values->n_tokens != keys->n_tokens || values->tok_idx != keys->tok_idx ||
            values->tok_off != keys->tok_off || values->n_tokens_dev != keys->n_tokens_dev)
            return fail(ctx, RK_ERR_INVALID_ARG, "compress: values must use the same row selection as keys");
    }
    if (keys->n_tokens > L->capacity)
        return fail(ctx, RK_ERR_CAPACITY, "compress: %d rows exceed capacity %d", keys->n_tokens, L->capacity);
    if (ctx->device == RK_DEVICE_NONE) return fail(ctx, RK_ERR_NO_DEVICE, "valid arguments, but the context has no device");

    DeviceGuard dev(ctx->device);
    hipError_t e = dev.status;
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    hipStream_t st = as_stream(stream);
    e = launch_compress(L->dtype, !ctx->force_generic, to_dev(keys), L->batch, L->n_kv_heads, L->capacity, L->keep,
                        R_r, k_packed, seq_len_out, st);
    if (e != hipSuccess) return hip_fail(ctx, e, "compress launch");
    if (values) {
        e = launch_v_retile(L->dtype, to_dev(values), L->batch, L->n_kv_heads, L->capacity, v_cache, st);
        if (e != hipSuccess) return hip_fail(ctx, e, "value re-tiling launch");
    }
    return RK_OK;
}

rk_status rk_append(rk_ctx* ctx, const rk_layout* L, const void* k_new, const void* v_new, const float* R_r,
                    void* k_packed, void* v_cache, int32_t* seq_len, void* stream)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    rk_status s = check_layout(ctx, L);
    if (s != RK_OK) return s;
    if (!k_new || !v_new || !R_r || !k_packed || !v_cache || !seq_len)
        return fail(ctx, RK_ERR_INVALID_ARG, "append: NULL pointer");
    if (L->max_seq_len + 1 > L->capacity)
        return fail(ctx, RK_ERR_CAPACITY, "append: %d + 1 rows exceed capacity %d", L->max_seq_len, L->capacity);
    if (L->batch > APP_TICKETS) return fail(ctx, RK_ERR_UNSUPPORTED, "append: batch too large");
    if (ctx->device == RK_DEVICE_NONE) return fail(ctx, RK_ERR_NO_DEVICE, "valid arguments, but the context has no device");
    DeviceGuard dev(ctx->device);
    hipError_t e = dev.status;
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    e = launch_append(L->dtype, L->batch, L->n_kv_heads, L->capacity, L->keep, k_new, v_new, R_r, k_packed,
                      v_cache, seq_len, ctx->tickets, as_stream(stream));
    if (e != hipSuccess) return hip_fail(ctx, e, "append launch");
    return RK_OK;
}

// tk_new / tv_new non-null: one row per sequence joins the text segment inside the same launches
static rk_status decode_common(rk_ctx* ctx, const rk_layout* L, const void* q, const void* k_packed,
                               const void* v_cache, const float* R_r, const float* delta_mu, const rk_text* text,
                               const void* tk_new, const void* tv_new, float scale, void* out, void* workspace,
                               size_t workspace_bytes, void* stream, bool use_static = false)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    rk_status s = check_layout(ctx, L);
    if (s != RK_OK) return s;
    if (!q || !k_packed || !v_cache || !R_r || !out || !L->seq_len)
        return fail(ctx, RK_ERR_INVALID_ARG, "decode: NULL pointer (q, k_packed, v_cache, R_r, out, seq_len)");
    if (((uintptr_t)k_packed & 15) || ((uintptr_t)v_cache & 15) || ((uintptr_t)q & 15))
        return fail(ctx, RK_ERR_INVALID_ARG, "decode: q and the caches must be 16-byte aligned");
    if (L->max_seq_len > L->capacity)
        return fail(ctx, RK_ERR_CAPACITY, "decode: max_seq_len %d exceeds capacity %d", L->max_seq_len, L->capacity);
    TextDev td{};
    TextAppendDev ta{};
    if (text) {
        s = check_text(ctx, text, tk_new != nullptr);
        if (s != RK_OK) return s;
        td = TextDev{text->k, text->v, text->stride_b, text->stride_h, text->stride_t, text->len, text->max_len};
        if (tk_new) {
            if (!tv_new || ((uintptr_t)tk_new & 15) || ((uintptr_t)tv_new & 15))
                return fail(ctx, RK_ERR_INVALID_ARG, "append_text_decode: k_new, v_new must be non-NULL, 16-byte aligned");
            if (text->max_len + 1 > text->capacity)
                return fail(ctx, RK_ERR_CAPACITY, "append_text_decode: %d + 1 rows exceed capacity %d", text->max_len,
                            text->capacity);
            td.max_len = text->max_len + 1;
            ta = TextAppendDev{text->k, text->v, tk_new, tv_new, text->stride_b, text->stride_h, text->stride_t,
                               text->len, text->capacity};
        }
    }
    const size_t need = rk_decode_workspace_size(ctx, L);
    if (use_static) {
        if (need > (size_t)RK_STATIC_SCRATCH_BYTES)
            return fail(ctx, RK_ERR_WORKSPACE, "decode (static scratch): this shape needs %zu bytes of partials, the "
                        "built-in scratch holds %zu; use rk_decode_attn with a workspace", need,
                        (size_t)RK_STATIC_SCRATCH_BYTES);
        if (ctx->device == RK_DEVICE_NONE) return fail(ctx, RK_ERR_NO_DEVICE, "valid arguments, but the context has no device");
        workspace = ctx->static_scratch;            // the device address taken at rk_create, never the symbol
    } else if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15))
        return fail(ctx, RK_ERR_WORKSPACE, "decode workspace: need %zu bytes, 16-byte aligned", need);
    if (ctx->device == RK_DEVICE_NONE) return fail(ctx, RK_ERR_NO_DEVICE, "valid arguments, but the context has no device");

    DeviceGuard dev(ctx->device);
    hipError_t e = dev.status;
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    int S, tiles;
    decode_plan(ctx, L, &S, &tiles);
    const float sc = scale > 0.f ? scale : 1.0f / sqrtf((float)L->head_dim);
    e = launch_decode(L->dtype, use_mfma_decode(ctx, L), L->batch, L->n_q_heads, L->n_kv_heads, L->capacity,
                      L->keep, S, tiles, q, k_packed, v_cache, R_r, delta_mu, L->seq_len, text ? &td : nullptr, nullptr,
                      tk_new ? &ta : nullptr, sc, out, (float*)workspace,
                      ctx->fuse_merge && ctx->xcd_deal_ok ? ctx->tickets + APP_TICKETS : nullptr, DEC_COUNTERS,
                      L->batch <= APP_TICKETS ? ctx->tickets : nullptr, as_stream(stream));
    if (e != hipSuccess) return hip_fail(ctx, e, "decode launch");
    return RK_OK;
}

rk_status rk_decode_attn(rk_ctx* ctx, const rk_layout* L, const void* q, const void* k_packed,
                         const void* v_cache, const float* R_r, const float* delta_mu, float scale, void* out,
                         void* workspace, size_t workspace_bytes, void* stream)
{
    return decode_common(ctx, L, q, k_packed, v_cache, R_r, delta_mu, nullptr, nullptr, nullptr, scale, out,
                         workspace, workspace_bytes, stream);
}

rk_status rk_decode_attn_static(rk_ctx* ctx, const rk_layout* L, const void* q, const void* k_packed,
                                const void* v_cache, const float* R_r, const float* delta_mu, float scale,
                                void* out, void* stream)
{
    return decode_common(ctx, L, q, k_packed, v_cache, R_r, delta_mu, nullptr, nullptr, nullptr, scale, out,
                         nullptr, 0, stream, true);
}

rk_status rk_decode_attn_dual(rk_ctx* ctx, const rk_layout* L, const void* q, const void* k_packed,
                              const void* v_cache, const float* R_r, const float* delta_mu, const rk_text* text,
                              float scale, void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    if (!text) return fail(ctx, RK_ERR_INVALID_ARG, "decode (dual): text is NULL");
    return decode_common(ctx, L, q, k_packed, v_cache, R_r, delta_mu, text, nullptr, nullptr, scale, out, workspace,
                         workspace_bytes, stream);
}

rk_status rk_append_text_decode_attn_dual(rk_ctx* ctx, const rk_layout* L, const void* k_new, const void* v_new,
                                          const void* q, const void* k_packed, const void* v_cache,
                                          const float* R_r, const float* delta_mu, const rk_text* text, float scale,
                                          void* out, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    if (!text) return fail(ctx, RK_ERR_INVALID_ARG, "append_text_decode: text is NULL");
    if (!k_new || !v_new) return fail(ctx, RK_ERR_INVALID_ARG, "append_text_decode: NULL pointer (k_new, v_new)");
    return decode_common(ctx, L, q, k_packed, v_cache, R_r, delta_mu, text, k_new, v_new, scale, out, workspace,
                         workspace_bytes, stream);
}

rk_status rk_append_decode_attn(rk_ctx* ctx, const rk_layout* L, const void* k_new, const void* v_new, const void* q,
                                const float* R_r, const float* delta_mu, void* k_packed, void* v_cache,
                                int32_t* seq_len, float scale, void* out, void* workspace, size_t workspace_bytes,
                                void* stream)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    rk_status s = check_layout(ctx, L);
    if (s != RK_OK) return s;
    if (!k_new || !v_new || !q || !R_r || !k_packed || !v_cache || !seq_len || !out)
        return fail(ctx, RK_ERR_INVALID_ARG, "append_decode: NULL pointer");
    if (((uintptr_t)k_packed & 15) || ((uintptr_t)v_cache & 15) || ((uintptr_t)k_new & 15) || ((uintptr_t)v_new & 15) ||
        ((uintptr_t)q & 15))
        return fail(ctx, RK_ERR_INVALID_ARG, "append_decode: q, k_new, v_new and the caches must be 16-byte aligned");
    if (L->max_seq_len + 1 > L->capacity)
        return fail(ctx, RK_ERR_CAPACITY, "append_decode: %d + 1 rows exceed capacity %d", L->max_seq_len,
                    L->capacity);
    if (L->batch > APP_TICKETS) return fail(ctx, RK_ERR_UNSUPPORTED, "append_decode: batch too large");
    // everything below is planned for the length after the append
    rk_layout La = *L;
    La.max_seq_len = L->max_seq_len + 1;
    La.seq_len = seq_len;
    const size_t need = rk_decode_workspace_size(ctx, &La);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15))
        return fail(ctx, RK_ERR_WORKSPACE, "append_decode workspace: need %zu bytes, 16-byte aligned", need);
    if (ctx->device == RK_DEVICE_NONE) return fail(ctx, RK_ERR_NO_DEVICE, "valid arguments, but the context has no device");

    DeviceGuard dev(ctx->device);
    hipError_t e = dev.status;
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    hipStream_t st = as_stream(stream);
    int S, tiles;
    decode_plan(ctx, &La, &S, &tiles);
    const float sc = scale > 0.f ? scale : 1.0f / sqrtf((float)L->head_dim);
    const bool mfma = use_mfma_decode(ctx, L);
    const AppendDev app{k_new, v_new, seq_len};
    const bool fused = decode_append_fusable(L->dtype, mfma, L->n_q_heads, L->n_kv_heads, L->keep);
    if (!fused) {
        // no free matrix-core column (G >= 16) or the plain kernels: the two steps run
        // as the launches of rk_append and rk_decode_attn
        e = launch_append(L->dtype, L->batch, L->n_kv_heads, L->capacity, L->keep, k_new, v_new, R_r, k_packed,
                          v_cache, seq_len, ctx->tickets, st);
        if (e != hipSuccess) return hip_fail(ctx, e, "append launch");
    }
    e = launch_decode(L->dtype, mfma, L->batch, L->n_q_heads, L->n_kv_heads, L->capacity, L->keep, S, tiles, q,
                      k_packed, v_cache, R_r, delta_mu, seq_len, nullptr, fused ? &app : nullptr, nullptr, sc, out,
                      (float*)workspace, ctx->fuse_merge && ctx->xcd_deal_ok ? ctx->tickets + APP_TICKETS : nullptr,
                      DEC_COUNTERS, ctx->tickets, st);
    if (e != hipSuccess) return hip_fail(ctx, e, "decode launch");
    return RK_OK;
}

rk_status rk_append_text(rk_ctx* ctx, const rk_layout* L, const rk_text* text, const void* k_new,
                         const void* v_new, void* stream)
{
    if (!ctx) return RK_ERR_INVALID_ARG;
    rk_status s = check_layout(ctx, L);
    if (s != RK_OK) return s;
    if (!text) return fail(ctx, RK_ERR_INVALID_ARG, "append_text: text is NULL");
    s = check_text(ctx, text, true);
    if (s != RK_OK) return s;
    if (!k_new || !v_new) return fail(ctx, RK_ERR_INVALID_ARG, "append_text: NULL pointer (k_new, v_new)");
    if (text->max_len + 1 > text->capacity)
        return fail(ctx, RK_ERR_CAPACITY, "append_text: %d + 1 rows exceed capacity %d", text->max_len,
                    text->capacity);
    if (ctx->device == RK_DEVICE_NONE) return fail(ctx, RK_ERR_NO_DEVICE, "valid arguments, but the context has no device");
    DeviceGuard dev(ctx->device);
    hipError_t e = dev.status;
    if (e != hipSuccess) return hip_fail(ctx, e, "hipSetDevice");
    e = launch_append_text(L->dtype, L->batch, L->n_kv_heads, text->capacity, k_new, v_new, text->k, text->v,
                           text->stride_b, text->stride_h, text->stride_t, text->len, as_stream(stream));
    if (e != hipSuccess) return hip_fail(ctx, e, "append_text launch");
    return RK_OK;
}

}  // extern "C"
