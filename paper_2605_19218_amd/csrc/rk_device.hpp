// Internal device-side helpers shared by the RotateK kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rk {

constexpr int D = 128;                 // head dim the kernels are written for
typedef uint16_t bf16_t;               // raw bfloat16 storage

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// round-to-nearest-even (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    __bf16 h = (__bf16)f;
    return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ float ld_elem(const float* p) { return *p; }
__device__ __forceinline__ float ld_elem(const bf16_t* p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void st_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_elem(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// split an fp32 value into a bf16 head and a bf16 remainder: x ~= hi + lo to ~2^-17
__device__ __forceinline__ void split_bf16(float x, __bf16& hi, __bf16& lo) {
    hi = (__bf16)x;
    lo = (__bf16)(x - (float)hi);
}

// Orders this wave's LDS writes before its later LDS reads by other lanes.  DS
// operations of one wave execute in issue order, so only the compiler has to be
// kept from moving them.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Device view of rk_rows (see rotatek.h).
struct RowsDev {
    const void* data;
    int64_t sb, sh, st;
    int32_t n_tokens;
    const int32_t* n_dev;
    const int32_t* tok_idx;
    const int64_t* tok_off;
};

__device__ __forceinline__ int rows_count(const RowsDev& r, int b) {
    int n;
    if (r.tok_idx) n = (int)(r.tok_off[b + 1] - r.tok_off[b]);
    else if (r.n_dev) n = r.n_dev[b];
    else n = r.n_tokens;
    n = n < 0 ? 0 : n;
    return n < r.n_tokens ? n : r.n_tokens;
}

// element offset of logical row t of head (b, h)
__device__ __forceinline__ int64_t rows_offset(const RowsDev& r, int b, int h, int t) {
    int64_t row = r.tok_idx ? (int64_t)r.tok_idx[r.tok_off[b] + t] : (int64_t)t;
    return (int64_t)b * r.sb + (int64_t)h * r.sh + row * r.st;
}
// Branch-free form for the streaming kernels (GATHER is a template parameter there, so a
// sequence of row loads stays one basic block and the load counters are tracked exactly).
// head_base = b * sb + h * sh, list = tok_idx + tok_off[b].
template <bool GATHER>
__device__ __forceinline__ int64_t row_off(int64_t head_base, int64_t st, const int32_t* __restrict__ list, int t) {
    const int64_t row = GATHER ? (int64_t)list[t] : (int64_t)t;
    return head_base + row * st;
}

// ---------------------------------------------------------------------------
// Cache layouts (element indices within one (batch item, KV head) slab).  Both
// caches are tiled so that a wave's MFMA operand fragment is ONE contiguous
// 1 KB piece of HBM (lane l reads bytes [16 l, 16 l + 16)):
//
//  packed Keys K~: blocks of 16 tokens; inside a block channel octets are the
//    slow axis:   [t / 16][c / 8][t % 16][c % 8]        (r padded to a multiple of 16 with
//    zero channels, so that every r runs on the 16-wide MFMA blocks; every writer of the
//    cache stores the zeros)
//    A 16x16x32 MFMA A-fragment of k-step i is octets 4i..4i+3 of a block:
//    lane (g, n) holds token n, channels 32 i + 8 g ..+7.
//
//  Values V: blocks of 32 tokens:  [t / 32][c / 16][g][c % 16][jj]  where the
//    token's position in its block, tl = t % 32, maps to k-slot (g, jj) with
//    g = (tl % 16) / 4,  jj = 4 (tl / 16) + tl % 4.  This is exactly how the score
//    MFMA hands the softmax weights of 32 tokens to lane group g, so P feeds the
//    P.V MFMA as produced and lane (g, n) reads V's B-fragment for channel block
//    cb as one 16-byte piece.
__host__ __device__ __forceinline__ int keep_padded(int r) { return (r + 15) & ~15; }
// Tokens from one (batch item, KV head) slab to the next inside either cache.  Every work-group of a decode
// launch streams its own contiguous piece of some slab, all at the same pace, so the distance between the slabs
// decides which memory channels the pieces share at any moment: with the slabs `capacity` tokens apart a
// capacity of 16384 + 128 took 45 us per decode step where 16384 + 64 took 36.5 us (+ 96 and + 160: 39-40 us).
// Larger caches therefore space their slabs at the next count that is 64 above a multiple of 256 tokens (at
// most 255 tokens, i.e. at most 6 %, of padding per slab); rk_cache_bytes() includes it.
__host__ __device__ __forceinline__ size_t slab_tokens(int cap)
{
    return cap < 4096 ? (size_t)cap : (size_t)((cap - 64 + 255) / 256) * 256 + 64;
}
__host__ __device__ __forceinline__ size_t kidx(int t, int c, int rp) {
    return (size_t)(t >> 4) * (16 * (size_t)rp) + (size_t)(c >> 3) * 128 + (size_t)(t & 15) * 8 + (c & 7);
}
__host__ __device__ __forceinline__ size_t vidx(int t, int c) {
    int tl = t & 31;
    int g = (tl & 15) >> 2, jj = ((tl >> 4) << 2) | (tl & 3);
    return (size_t)(t >> 5) * 4096 + (size_t)(c >> 4) * 512 + (size_t)g * 128 + (size_t)(c & 15) * 8 + jj;
}

// 16-byte non-temporal (streaming) accesses: data that is written once and read once by a later
// kernel, or read exactly once, should not displace anything in the caches
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void nt_store16(void* p, uint4 v) {
    __builtin_nontemporal_store((u32x4){v.x, v.y, v.z, v.w}, (u32x4*)p);
}
__device__ __forceinline__ void nt_store8(void* p, uint2 v) {
    __builtin_nontemporal_store((u32x2){v.x, v.y}, (u32x2*)p);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

}  // namespace rk
