// Rotate + gather + pack of the Key cache (Alg. 1 step 14: K~ = K R_k, stored in
// place of K, rounded once to the cache dtype) and the frozen-R append of new
// tokens (the rotation is fitted once at the end of prefill and reused,
// Sec. 3.2 Step (1)).
#include "rk_kernels.hpp"

namespace rk {

// ---------------------------------------------------------------------------
// Plain kernel, any dtype and any r: 64 tokens per block, K tile in LDS as fp32,
// thread (t, j) accumulates over the 128 channels in ascending order.
template <typename T>
__global__ __launch_bounds__(256) void compress_generic(RowsDev rows, int Hkv, int cap, int r,
                                                        const float* __restrict__ Rr, T* __restrict__ Kp,
                                                        int32_t* __restrict__ seq_len_out)
{
    const int h = blockIdx.y, b = blockIdx.z, u = b * Hkv + h;
    const int tid = threadIdx.x;
    const int n_b = min(rows_count(rows, b), cap);
    if (blockIdx.x == 0 && h == 0 && tid == 0 && seq_len_out) seq_len_out[b] = n_b;
    const int t0 = blockIdx.x * 64;
    if (t0 >= n_b) return;
    const int nt = min(64, n_b - t0);
    const T* base = (const T*)rows.data;
    __shared__ float tile[64][D];
    for (int idx = tid; idx < nt * D; idx += 256) {
        int t = idx >> 7, c = idx & 127;
        tile[t][c] = ld_elem(base + rows_offset(rows, b, h, t0 + t) + c);
    }
    __syncthreads();
    const float* Ru = Rr + (size_t)u * D * r;
    for (int o = tid; o < nt * r; o += 256) {
        int t = o / r, j = o - t * r;
        float a = 0.f;
        for (int c = 0; c < D; ++c) a = fmaf(tile[t][c], Ru[c * r + j], a);
        st_elem(Kp + ((size_t)u * cap + t0 + t) * r + j, a);
    }
}

// ---------------------------------------------------------------------------
// MFMA kernel (bf16, r a multiple of 16).  Per wave: D^T[j, token] = R_r^T . K^T
// with v_mfma_f32_16x16x32_bf16; the B operand (lane (g, n): token n, channels
// 32 i + 8 g ..+7) is a plain 16-byte load of a Key row, so Keys go from HBM
// straight into MFMA registers.  R_r is split into bf16 head + remainder
// (two MFMAs) to keep ~fp32 accuracy of the fp32 rotation.  The rows of the A
// operand are permuted so that lane (g, n) ends up holding the r/4 CONTIGUOUS
// output channels g*r/4 .. of token n: each wave then writes one contiguous
// 16-token x r block of the packed cache.
template <int R>
struct CompressCfg {
    static constexpr int JB = R / 16;                 // 16-wide output-channel blocks
    static constexpr int TT = (R <= 64) ? 4 : 2;      // 16-token tiles in flight per wave
    static constexpr int TOK_PER_BLOCK = 4 * TT * 16; // 4 waves
    static constexpr size_t LDS_BYTES = (size_t)JB * 4 * 2 * 64 * 16;   // A fragments, hi+lo
};

template <int R>
__global__ __launch_bounds__(256) void compress_mfma(RowsDev rows, int Hkv, int cap,
                                                     const float* __restrict__ Rr, bf16_t* __restrict__ Kp,
                                                     int32_t* __restrict__ seq_len_out)
{
    typedef CompressCfg<R> Cfg;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16x8* frag = (bf16x8*)smem_raw;       // [JB][4][2][64]

    const int h = blockIdx.y, b = blockIdx.z, u = b * Hkv + h;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, n = lane & 15;
    const int n_b = min(rows_count(rows, b), cap);
    if (blockIdx.x == 0 && h == 0 && tid == 0 && seq_len_out) seq_len_out[b] = n_b;
    const int blk0 = blockIdx.x * Cfg::TOK_PER_BLOCK;
    if (blk0 >= n_b) return;

    // A fragments: block jb, k-step i, lane (gk, a): rows a <-> output channel
    // (a/4)*(R/4) + 4 jb + a%4 ; k slots <-> input channels 32 i + 8 gk + jj.
    const float* Ru = Rr + (size_t)u * D * R;
    for (int f = tid; f < Cfg::JB * 4 * 64; f += 256) {
        int l = f & 63, i = (f >> 6) & 3, jb = f >> 8;
        int gk = l >> 4, a = l & 15;
        int j = (a >> 2) * (R / 4) + 4 * jb + (a & 3);
        bf16x8 hi, lo;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            float x = Ru[(32 * i + 8 * gk + jj) * R + j];
            __bf16 xh, xl;
            split_bf16(x, xh, xl);
            hi[jj] = xh;
            lo[jj] = xl;
        }
        frag[((jb * 4 + i) * 2 + 0) * 64 + l] = hi;
        frag[((jb * 4 + i) * 2 + 1) * 64 + l] = lo;
    }
    __syncthreads();

    const bf16_t* base = (const bf16_t*)rows.data;
    const int w0 = blk0 + wave * (Cfg::TT * 16);
    if (w0 >= n_b) return;

    bf16x8 kb[Cfg::TT][4];
#pragma unroll
    for (int tt = 0; tt < Cfg::TT; ++tt) {
        int tok = min(w0 + tt * 16 + n, n_b - 1);
        const bf16_t* row = base + rows_offset(rows, b, h, tok);
#pragma unroll
        for (int i = 0; i < 4; ++i) kb[tt][i] = *(const bf16x8*)(row + 32 * i + 8 * g);
    }
    f32x4 acc[Cfg::TT][Cfg::JB];
#pragma unroll
    for (int tt = 0; tt < Cfg::TT; ++tt)
#pragma unroll
        for (int jb = 0; jb < Cfg::JB; ++jb) acc[tt][jb] = (f32x4){0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int jb = 0; jb < Cfg::JB; ++jb) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            bf16x8 ah = frag[((jb * 4 + i) * 2 + 0) * 64 + lane];
            bf16x8 al = frag[((jb * 4 + i) * 2 + 1) * 64 + lane];
#pragma unroll
            for (int tt = 0; tt < Cfg::TT; ++tt) {
                acc[tt][jb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, kb[tt][i], acc[tt][jb], 0, 0, 0);
                acc[tt][jb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, kb[tt][i], acc[tt][jb], 0, 0, 0);
            }
        }
    }
    // lane (g, n): acc[tt][jb][ii] = channel g*R/4 + 4 jb + ii of token w0 + 16 tt + n
#pragma unroll
    for (int tt = 0; tt < Cfg::TT; ++tt) {
        int tok = w0 + tt * 16 + n;
        if (tok < n_b) {
            bf16_t* dst = Kp + ((size_t)u * cap + tok) * R + g * (R / 4);
#pragma unroll
            for (int jb = 0; jb < Cfg::JB; ++jb) {
                uint2 pk;
                pk.x = (uint32_t)f32_to_bf16(acc[tt][jb][0]) | ((uint32_t)f32_to_bf16(acc[tt][jb][1]) << 16);
                pk.y = (uint32_t)f32_to_bf16(acc[tt][jb][2]) | ((uint32_t)f32_to_bf16(acc[tt][jb][3]) << 16);
                *(uint2*)(dst + 4 * jb) = pk;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Row copy / gather (Values follow the same token list as the Keys): 16 threads
// per 128-channel row, 16-byte pieces.
template <typename T>
__global__ __launch_bounds__(256) void row_copy(RowsDev rows, int Hkv, int cap, T* __restrict__ dst)
{
    const int h = blockIdx.y, b = blockIdx.z, u = b * Hkv + h;
    const int n_b = min(rows_count(rows, b), cap);
    const int t = blockIdx.x * 16 + (threadIdx.x >> 4);
    if (t >= n_b) return;
    constexpr int PIECES = (int)(D * sizeof(T) / 16 / 16);   // 16-byte pieces per thread
    const uint4* s = (const uint4*)((const T*)rows.data + rows_offset(rows, b, h, t));
    uint4* d = (uint4*)(dst + ((size_t)u * cap + t) * D);
    const int c = threadIdx.x & 15;
#pragma unroll
    for (int p = 0; p < PIECES; ++p) d[c + 16 * p] = s[c + 16 * p];
}

// ---------------------------------------------------------------------------
// Append: block (h, b), 128 threads.  k~_j = sum_c k_new[c] R_r[c][j].
template <typename T>
__global__ __launch_bounds__(128) void append_rows(int Hkv, int cap, int r, const T* __restrict__ k_new,
                                                   const T* __restrict__ v_new, const float* __restrict__ Rr,
                                                   T* __restrict__ Kp, T* __restrict__ Vc,
                                                   const int32_t* __restrict__ seq_len)
{
    const int h = blockIdx.x, b = blockIdx.y, u = b * Hkv + h;
    const int tid = threadIdx.x;
    const int len = seq_len[b];
    if (len < 0 || len >= cap) return;
    __shared__ float kn[D];
    kn[tid] = ld_elem(k_new + (size_t)u * D + tid);
    __syncthreads();
    if (tid < r) {
        const float* Ru = Rr + (size_t)u * D * r;
        float a = 0.f;
        for (int c = 0; c < D; ++c) a = fmaf(kn[c], Ru[c * r + tid], a);
        st_elem(Kp + ((size_t)u * cap + len) * r + tid, a);
    }
    Vc[((size_t)u * cap + len) * D + tid] = v_new[(size_t)u * D + tid];
}

// runs after append_rows on the same stream: every head has read the old length
__global__ void bump_lengths(int B, int cap, int32_t* __restrict__ seq_len)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) {
        int len = seq_len[b];
        if (len >= 0 && len < cap) seq_len[b] = len + 1;
    }
}

// ---------------------------------------------------------------------------
template <int R>
static hipError_t launch_compress_mfma_r(const RowsDev& rows, int B, int Hkv, int cap, const float* Rr,
                                         bf16_t* Kp, int32_t* seq_len_out, hipStream_t st)
{
    typedef CompressCfg<R> Cfg;
    int nblk = (rows.n_tokens + Cfg::TOK_PER_BLOCK - 1) / Cfg::TOK_PER_BLOCK;
    if (nblk < 1) nblk = 1;
    hipLaunchKernelGGL(compress_mfma<R>, dim3(nblk, Hkv, B), dim3(256), Cfg::LDS_BYTES, st, rows, Hkv, cap, Rr,
                       Kp, seq_len_out);
    return hipGetLastError();
}

hipError_t launch_compress(int dtype, bool mfma, const RowsDev& rows, int B, int Hkv, int cap, int r,
                           const float* Rr, void* Kp, int32_t* seq_len_out, hipStream_t st)
{
    if (mfma && dtype == 1 && r % 16 == 0) {
        bf16_t* kp = (bf16_t*)Kp;
        switch (r) {
            case 16: return launch_compress_mfma_r<16>(rows, B, Hkv, cap, Rr, kp, seq_len_out, st);
            case 32: return launch_compress_mfma_r<32>(rows, B, Hkv, cap, Rr, kp, seq_len_out, st);
            case 48: return launch_compress_mfma_r<48>(rows, B, Hkv, cap, Rr, kp, seq_len_out, st);
            case 64: return launch_compress_mfma_r<64>(rows, B, Hkv, cap, Rr, kp, seq_len_out, st);
            case 80: return launch_compress_mfma_r<80>(rows, B, Hkv, cap, Rr, kp, seq_len_out, st);
            case 96: return launch_compress_mfma_r<96>(rows, B, Hkv, cap, Rr, kp, seq_len_out, st);
            case 112: return launch_compress_mfma_r<112>(rows, B, Hkv, cap, Rr, kp, seq_len_out, st);
            case 128: return launch_compress_mfma_r<128>(rows, B, Hkv, cap, Rr, kp, seq_len_out, st);
            default: break;
        }
    }
    int nblk = (rows.n_tokens + 63) / 64;
    if (nblk < 1) nblk = 1;
    dim3 grid(nblk, Hkv, B);
    if (dtype == 0)
        hipLaunchKernelGGL(compress_generic<float>, grid, dim3(256), 0, st, rows, Hkv, cap, r, Rr, (float*)Kp,
                           seq_len_out);
    else
        hipLaunchKernelGGL(compress_generic<bf16_t>, grid, dim3(256), 0, st, rows, Hkv, cap, r, Rr, (bf16_t*)Kp,
                           seq_len_out);
    return hipGetLastError();
}

hipError_t launch_row_copy(int dtype, const RowsDev& rows, int B, int Hkv, int cap, void* dst, hipStream_t st)
{
    int nblk = (rows.n_tokens + 15) / 16;
    if (nblk < 1) nblk = 1;
    dim3 grid(nblk, Hkv, B);
    if (dtype == 0) hipLaunchKernelGGL(row_copy<float>, grid, dim3(256), 0, st, rows, Hkv, cap, (float*)dst);
    else hipLaunchKernelGGL(row_copy<bf16_t>, grid, dim3(256), 0, st, rows, Hkv, cap, (bf16_t*)dst);
    return hipGetLastError();
}

hipError_t launch_append(int dtype, int B, int Hkv, int cap, int r, const void* k_new, const void* v_new,
                         const float* Rr, void* Kp, void* Vc, int32_t* seq_len, hipStream_t st)
{
    dim3 grid(Hkv, B);
    if (dtype == 0)
        hipLaunchKernelGGL(append_rows<float>, grid, dim3(128), 0, st, Hkv, cap, r, (const float*)k_new,
                           (const float*)v_new, Rr, (float*)Kp, (float*)Vc, seq_len);
    else
        hipLaunchKernelGGL(append_rows<bf16_t>, grid, dim3(128), 0, st, Hkv, cap, r, (const bf16_t*)k_new,
                           (const bf16_t*)v_new, Rr, (bf16_t*)Kp, (bf16_t*)Vc, seq_len);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bump_lengths, dim3((B + 63) / 64), dim3(64), 0, st, B, cap, seq_len);
    return hipGetLastError();
}

}  // namespace rk
