// Host-side launch wrappers of the RotateK kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "rk_device.hpp"

namespace rk {

// ---- rk_fit.hip ------------------------------------------------------------
// Partials are [U, n_chunks, d*d] + [U, n_chunks, d]; n_chunks = ceil(tokens / cov_chunk_tokens()).
constexpr int COV_CHUNK = 512;             // tokens per work-group of the plain kernel (the smaller chunk)
int cov_chunk_tokens(int dtype, bool mfma);
hipError_t launch_cov_partial(int dtype, bool mfma, const RowsDev& rows, int B, int Hkv, int n_chunks,
                              float* part_S, float* part_sum, hipStream_t st);
// tiled: the partials were written by the MFMA kernel (10 upper-triangular tiles in register layout)
hipError_t launch_cov_finalize(const RowsDev& rows, int B, int Hkv, int n_chunks, bool center, bool tiled,
                               const float* part_S, const float* part_sum, float* cov, float* mu,
                               hipStream_t st);
// rotations: eig_rotation_bytes(U) bytes of device scratch (the recorded Jacobi rotations),
// sweeps_ws: U ints of device scratch; sweeps (optional) receives the sweep counts
size_t eig_rotation_bytes(size_t U);
hipError_t launch_eig(int U, const float* cov, const float* sigma, const float* mu, int r, float* R,
                      float* lam, uint8_t* mask, int32_t* keep_idx, float* Rr, float* dmu, int32_t* sweeps,
                      void* rotations, int32_t* sweeps_ws, hipStream_t st);
// Cholesky-based subspace iteration (Alg. 1 steps 6-13): V0 [U,d,k] -> Rr [U,d,k], dmu [U,d];
// status [U] (optional): 0, or t+1 if iteration t met a non-positive pivot.
int subspace_max_keep();
hipError_t launch_subspace(int U, const float* cov, const float* sigma, const float* mu, const float* V0, int k,
                           int T, double eps, float* Rr, float* dmu, int32_t* status, hipStream_t st);
// sigma [B,Hkv,d] from a query window [B,Hq,W,d] with element strides (sb, sh, sw)
hipError_t launch_sigma_window(int dtype, const void* qw, int64_t sb, int64_t sh, int64_t sw, int B, int Hq,
                               int Hkv, int W, float* sigma, hipStream_t st);
hipError_t launch_gather_rotation(int U, int r, const float* R, const int32_t* keep_idx, float* Rr,
                                  hipStream_t st);

// ---- rk_compress.hip -------------------------------------------------------
hipError_t launch_compress(int dtype, bool mfma, const RowsDev& rows, int B, int Hkv, int cap, int r,
                           const float* Rr, void* Kp, int32_t* seq_len_out, hipStream_t st);
hipError_t launch_v_retile(int dtype, const RowsDev& rows, int B, int Hkv, int cap, void* dst, hipStream_t st);
// tickets: B zero-initialised ints, left at zero on completion
hipError_t launch_append(int dtype, int B, int Hkv, int cap, int r, const void* k_new, const void* v_new,
                         const float* Rr, void* Kp, void* Vc, int32_t* seq_len, int32_t* tickets, hipStream_t st);
hipError_t launch_unpack(int dtype, int U, int cap, int r, const void* Kp, const void* Vc, void* k_rows,
                         void* v_rows, hipStream_t st);

// ---- rk_decode.hip ---------------------------------------------------------
// Partials: m [B,Hq,S], l [B,Hq,S], acc [B,Hq,S,d]; m is in the log2 domain.
bool decode_mfma_supported(int dtype, int r);
// Unrotated full-width prompt/text segment (Alg. 2 input K_pt and its Value rows).
struct TextDev {
    const void* k;
    const void* v;
    int64_t sb, sh, st;      // element strides of [B, H_kv, token, d], shared by k and v
    const int32_t* len;      // device [B] or null (= max_len)
    int max_len;
};
// One token per sequence appended with the frozen R inside the decode launches (Sec. 3.2 Step (1)).
struct AppendDev {
    const void* k_new;       // [B, H_kv, d]
    const void* v_new;       // [B, H_kv, d]
    int32_t* seq_len;        // the same array the decode reads, writable: bumped by the merge kernel, or by the
                             // split launch itself when the merge is folded into it
};
// One full-width token per sequence appended to the text segment inside the split kernel.
struct TextAppendDev {
    void* k;                 // text segment (null = no append), strides as in TextDev
    void* v;
    const void* k_new;       // [B, H_kv, d]
    const void* v_new;
    int64_t sb, sh, st;
    int32_t* len;            // device [B], bumped by the one wave that copies the rows
    int capacity;
};
// Dual path on the matrix-core kernels: the text attention runs as up to this
// many slices in work-groups of the split launch, each writing a partial of its own (the workspace holds
// S + DECODE_TEXT_SLICES_MAX partials per row); otherwise the text rows are handled by the merge kernel.
constexpr int DECODE_TEXT_SLICES_MAX = 8;
// whether launch_decode can take `app` for this shape (MFMA kernel with a free column: G < 16)
bool decode_append_fusable(int dtype, bool mfma, int Hq, int Hkv, int r);
// text == nullptr: visual segment only; otherwise the text segment joins the softmax in the merge kernel
// app != nullptr: the new token is written to row seq_len[b] of both caches (which must then be writable),
//                 joins the softmax, and seq_len[b] += 1; needs decode_append_fusable and text == nullptr
// tapp != nullptr (needs text): row text.len[b] of the text segment receives k_new / v_new and the length is
//                 bumped before the merge kernel reads it; text->max_len must already count the new row
// tiles_all: 128-token tiles of the longest sequence; split s takes a balanced share of them
// ws: partials, ((S + DECODE_TEXT_SLICES_MAX) (d + 2) + 1) floats per (b, h_q)
// counters: n_counters ints that are zero between launches (or null): lets a plain matrix-core decode
//           fold its partials inside the split launch (one counter per (b, h_kv, head group)).  Only
//           valid on a device that deals work-groups to its XCDs round-robin by linear index
//           (probe_xcd_deal)
// batch_tickets: B ints that are zero between launches (or null): with them a fused append is folded
//           the same way and the launch bumps seq_len itself
hipError_t launch_decode(int dtype, bool mfma, int B, int Hq, int Hkv, int cap, int r, int S, int tiles_all,
                         const void* q, const void* Kp, const void* Vc, const float* Rr, const float* dmu,
                         const int32_t* seq_len, const TextDev* text, const AppendDev* app, const TextAppendDev* tapp,
                         float scale, void* out, float* ws, int32_t* counters, int n_counters, int32_t* batch_tickets,
                         hipStream_t st);
// Whether work-groups whose linear indices agree modulo 8 run on the same XCD (true on MI355X in every
// partition mode).  Launches a tiny kernel that records each work-group's XCD and synchronises;
// scratch: 64 ints of device memory, left zeroed.
hipError_t probe_xcd_deal(int32_t* scratch, bool* same_xcd);
// plain streaming read of `bytes` (a multiple of 16) of device memory; sink: one writable int (or null)
hipError_t launch_stream_read(const void* src, size_t bytes, int n_cu, int32_t* sink, hipStream_t st);
hipError_t launch_append_text(int dtype, int B, int Hkv, int capacity, const void* k_new, const void* v_new,
                              void* kt, void* vt, int64_t sb, int64_t sh, int64_t st_, int32_t* len,
                              hipStream_t st);

}  // namespace rk
