// Decode-step attention over the rotated, channel-pruned Key cache (Alg. 2 steps
// 1-3 and 6 of the RotateK paper, realised as the split-K + merge pair of
// App. C): per split, q~ = q R_k and the bias q . delta_mu are computed in the
// kernel's prologue, the packed Keys and full-width Values are streamed once
// with an online softmax, and a partial (m, l, acc) goes to scratch; the merge
// kernel folds the N_s partials.
//
// Differences from the paper's Triton design, made for CDNA4:
//   - one work-group per (batch item, KV head, split) serves all G = H_q/H_kv
//     query heads of the group, so the K/V stream is read once per KV head;
//   - scores and P.V run on v_mfma_f32_16x16x32_bf16 with the G heads padded to
//     16 MFMA columns; K~ rows are loaded from HBM directly in MFMA operand
//     layout; V tiles are staged through a wave-private LDS buffer (no
//     work-group barrier in the streaming loop);
//   - q~ and P are fed as bf16 head + remainder pairs so that the fp32 rotation
//     and the softmax weights keep ~2^-17 relative accuracy.
#include "rk_kernels.hpp"

namespace rk {

constexpr float NEG_INF = -__builtin_huge_valf();

// ---------------------------------------------------------------------------
// Plain kernel: one block of 128 threads per (split, query head, batch item).
template <typename T>
__global__ __launch_bounds__(128) void decode_split_generic(
    const T* __restrict__ q, const T* __restrict__ Kp, const T* __restrict__ Vc, const float* __restrict__ Rr,
    const float* __restrict__ dmu, const int32_t* __restrict__ seq_len, int Hq, int Hkv, int cap, int r, int tps,
    float scale_log2, float* __restrict__ ws_m, float* __restrict__ ws_l, float* __restrict__ ws_acc, int S)
{
    const int split = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
    const int G = Hq / Hkv, hk = hq / G, u = b * Hkv + hk;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int L = min(max(seq_len[b], 0), cap);
    const int t0 = split * tps, t1 = min(t0 + tps, L);
    const size_t pidx = ((size_t)b * Hq + hq) * S + split;
    if (t0 >= t1) {
        if (tid == 0) { ws_m[pidx] = NEG_INF; ws_l[pidx] = 0.f; }
        ws_acc[pidx * D + tid] = 0.f;
        return;
    }
    __shared__ float qs[D], qt[D], ps[128], red[4];
    qs[tid] = ld_elem(q + ((size_t)b * Hq + hq) * D + tid);
    __syncthreads();
    if (tid < r) {
        const float* Ru = Rr + (size_t)u * D * r;
        float a = 0.f;
        for (int c = 0; c < D; ++c) a = fmaf(qs[c], Ru[c * r + tid], a);
        qt[tid] = a * scale_log2;
    }
    float bpart = dmu ? qs[tid] * dmu[(size_t)u * D + tid] : 0.f;
    bpart = wave_sum(bpart);
    if (lane == 0) red[wave] = bpart;
    __syncthreads();
    const float bias = (red[0] + red[1]) * scale_log2;
    __syncthreads();

    float m = NEG_INF, l = 0.f, acc = 0.f;
    const T* Ku = Kp + (size_t)u * cap * r;
    const T* Vu = Vc + (size_t)u * cap * D;
    for (int base = t0; base < t1; base += 128) {
        const int tok = base + tid;
        const bool valid = tok < t1;
        float s = NEG_INF;
        if (valid) {
            const T* row = Ku + (size_t)tok * r;
            float a = 0.f;
            for (int j = 0; j < r; ++j) a = fmaf(qt[j], ld_elem(row + j), a);
            s = a + bias;
        }
        float mt = wave_max(s);
        if (lane == 0) red[wave] = mt;
        __syncthreads();
        mt = fmaxf(red[0], red[1]);
        const float m_new = fmaxf(m, mt);
        const float alpha = exp2f(m - m_new);
        const float p = valid ? exp2f(s - m_new) : 0.f;
        ps[tid] = p;
        float lsum = wave_sum(p);
        if (lane == 0) red[2 + wave] = lsum;
        __syncthreads();
        l = l * alpha + (red[2] + red[3]);
        acc *= alpha;
        const int nv = min(128, t1 - base);
        for (int t = 0; t < nv; ++t) acc = fmaf(ps[t], ld_elem(Vu + (size_t)(base + t) * D + tid), acc);
        m = m_new;
        __syncthreads();
    }
    if (tid == 0) { ws_m[pidx] = m; ws_l[pidx] = l; }
    ws_acc[pidx * D + tid] = acc;
}

// ---------------------------------------------------------------------------
// Merge of the N_s partials (App. C phase 2, merge part): out = sum_i acc_i w_i / sum_i l_i w_i,
// w_i = 2^(m_i - M).  An all-empty row (M = -inf) gives zeros.
template <typename T>
__global__ __launch_bounds__(128) void decode_merge(const float* __restrict__ ws_m, const float* __restrict__ ws_l,
                                                    const float* __restrict__ ws_acc, int S, T* __restrict__ out)
{
    const size_t row = blockIdx.x;         // b * Hq + hq
    const int tid = threadIdx.x;
    const float* m = ws_m + row * S;
    const float* l = ws_l + row * S;
    float M = NEG_INF;
    for (int i = 0; i < S; ++i) M = fmaxf(M, m[i]);
    float o = 0.f;
    if (M > NEG_INF) {
        float den = 0.f, num = 0.f;
        for (int i = 0; i < S; ++i) {
            float mi = m[i];
            float w = (mi > NEG_INF) ? exp2f(mi - M) : 0.f;
            den = fmaf(l[i], w, den);
            num = fmaf(ws_acc[(row * S + i) * D + tid], w, num);
        }
        o = num / den;
    }
    st_elem(out + row * D + tid, o);
}

// ---------------------------------------------------------------------------
// MFMA split-K kernel (bf16 cache, r a multiple of 16).  256 threads = 4 waves;
// grid (split, H_kv * head groups of 16, B).  Each wave walks its own 32-token
// tiles (tile index = wave, wave + 4, ...) with a private online-softmax state;
// the four states are merged through LDS at the end.
//
// Lane (g = lane / 16, n = lane % 16) register layouts:
//   S^T = K~ Q~^T  : A = K~ rows (token n of a 16-token block, channels
//                    32 i + 8 g ..+7: one 16-byte HBM load), B = q~ of head n;
//                    result s[tb][ii] = score(token 16 tb + 4 g + ii, head n).
//   O = P V        : A = P as produced (head n, k-slots (g, jj) <-> tokens
//                    4 g + jj and 16 + 4 g + jj - 4), B = V[token(g, jj)][16 cb + n]
//                    read back from LDS; result O[cb][ii] = out(head 4 g + ii,
//                    channel 16 cb + n).
constexpr int DEC_VROW = 272;               // bytes per staged V row (256 + 16 pad)
constexpr int DEC_VTILE = 32 * DEC_VROW;    // 8704 B per wave, also holds 16x128 fp32 at the end

// One 32-token tile: K~ rows in MFMA A-operand layout (lane (g, n): token n of each
// 16-token block, channels 32 i + 8 g ..+7, plus 4 channels of a k = 16 tail) and
// 8 KB of V as 16-byte pieces (row 4 u8 + g, piece n).  Rows past the split's end
// are clamped to its last valid row; their scores are masked later.
template <int R>
__device__ __forceinline__ void load_tile(const bf16_t* __restrict__ Ku, const bf16_t* __restrict__ Vu, int tb0,
                                          int t1, int g, int n, bf16x8 (&kf)[2][(R / 32) > 0 ? (R / 32) : 1],
                                          s16x4 (&kt)[2], uint4 (&vf)[8])
{
    constexpr int NF = R / 32;
    constexpr bool TAIL = (R % 32) != 0;
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        int tok = min(tb0 + 16 * tb + n, t1 - 1);
        const bf16_t* kr = Ku + (size_t)tok * R;
#pragma unroll
        for (int i = 0; i < NF; ++i) kf[tb][i] = *(const bf16x8*)(kr + 32 * i + 8 * g);
        if (TAIL) kt[tb] = *(const s16x4*)(kr + 32 * NF + 4 * g);
    }
#pragma unroll
    for (int u8 = 0; u8 < 8; ++u8) {
        int tok = min(tb0 + 4 * u8 + g, t1 - 1);
        vf[u8] = *(const uint4*)(Vu + (size_t)tok * D + 8 * n);
    }
}

template <int R>
__global__ __launch_bounds__(256, 2) void decode_split_mfma(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ Kp, const bf16_t* __restrict__ Vc,
    const float* __restrict__ Rr, const float* __restrict__ dmu, const int32_t* __restrict__ seq_len, int Hq,
    int Hkv, int cap, int tps, float scale_log2, float* __restrict__ ws_m, float* __restrict__ ws_l,
    float* __restrict__ ws_acc, int S)
{
    constexpr int NF = R / 32;                 // k = 32 steps over the kept channels
    constexpr bool TAIL = (R % 32) != 0;       // plus one k = 16 step
    constexpr int NFA = NF > 0 ? NF : 1;

    __shared__ __attribute__((aligned(16))) unsigned char vt[4][DEC_VTILE];
    __shared__ float qs[16][D];
    __shared__ float qt[16][R];
    __shared__ float sbias[16];
    __shared__ __attribute__((aligned(16))) float salpha[4][16];
    __shared__ float sm_m[4][16], sm_l[4][16];

    const int G = Hq / Hkv;
    const int ngrp = (G + 15) >> 4;
    const int split = blockIdx.x, b = blockIdx.z;
    const int hk = blockIdx.y / ngrp, grp = blockIdx.y - hk * ngrp;
    const int h0 = hk * G + grp * 16;          // first query head of this group
    const int Gc = min(16, G - grp * 16);
    const int u = b * Hkv + hk;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, n = lane & 15;

    const int L = min(max(seq_len[b], 0), cap);
    const int t0 = split * tps, t1 = min(t0 + tps, L);
    if (t0 >= t1) {
        for (int idx = tid; idx < Gc * D; idx += 256) {
            int hh = idx >> 7, c = idx & 127;
            size_t pidx = ((size_t)b * Hq + h0 + hh) * S + split;
            ws_acc[pidx * D + c] = 0.f;
            if (c == 0) { ws_m[pidx] = NEG_INF; ws_l[pidx] = 0.f; }
        }
        return;
    }

    const bf16_t* Ku = Kp + (size_t)u * cap * R;
    const bf16_t* Vu = Vc + (size_t)u * cap * D;
    const int ntiles = (t1 - t0 + 31) >> 5;

    // ---- tile loads (issued before the prologue so HBM latency overlaps it) ----
    bf16x8 kf[2][NFA];
    s16x4 kt[2];
    uint4 vf[8];
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
        kt[tb] = (s16x4){0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < NFA; ++i) kf[tb][i] = (bf16x8){0, 0, 0, 0, 0, 0, 0, 0};
    }
#pragma unroll
    for (int u8 = 0; u8 < 8; ++u8) vf[u8] = make_uint4(0, 0, 0, 0);
    if (wave < ntiles) load_tile<R>(Ku, Vu, t0 + wave * 32, t1, g, n, kf, kt, vf);

    // ---- prologue: q~ = q R_r (scaled into the log2 domain), bias ---------------
    for (int idx = tid; idx < 16 * D; idx += 256) {
        int hh = idx >> 7, c = idx & 127;
        qs[hh][c] = hh < Gc ? bf16_to_f32(q[((size_t)b * Hq + h0 + hh) * D + c]) : 0.f;
    }
    __syncthreads();
    {
        const float* Ru = Rr + (size_t)u * D * R;
        for (int idx = tid; idx < 16 * R; idx += 256) {
            int hh = idx / R, j = idx - hh * R;
            float a = 0.f;
            if (hh < Gc) {
#pragma unroll 8
                for (int c = 0; c < D; ++c) a = fmaf(qs[hh][c], Ru[c * R + j], a);
            }
            qt[hh][j] = a * scale_log2;
        }
        if (tid < 16) {
            float a = 0.f;
            if (tid < Gc && dmu) {
                const float* dm = dmu + (size_t)u * D;
                for (int c = 0; c < D; ++c) a = fmaf(qs[tid][c], dm[c], a);
            }
            sbias[tid] = a * scale_log2;
        }
    }
    __syncthreads();

    // B operands of the score MFMAs: q~ of head n, split into bf16 head + remainder
    bf16x8 qh[NFA], ql[NFA];
    s16x4 qth, qtl;
#pragma unroll
    for (int i = 0; i < NF; ++i) {
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            __bf16 hi, lo;
            split_bf16(qt[n][32 * i + 8 * g + jj], hi, lo);
            qh[i][jj] = hi;
            ql[i][jj] = lo;
        }
    }
    if (TAIL) {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            __bf16 hi, lo;
            split_bf16(qt[n][32 * NF + 4 * g + jj], hi, lo);
            qth[jj] = __builtin_bit_cast(short, hi);
            qtl[jj] = __builtin_bit_cast(short, lo);
        }
    }

    float m_run = NEG_INF, l_run = 0.f;
    f32x4 O[8];
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) O[cb] = (f32x4){0.f, 0.f, 0.f, 0.f};
    unsigned char* vw = vt[wave];

    for (int tile = wave; tile < ntiles; tile += 4) {
        const int tb0 = t0 + tile * 32;
        // stage this tile's V rows (row 4 u8 + g, 16-byte piece n) and free the registers
#pragma unroll
        for (int u8 = 0; u8 < 8; ++u8) *(uint4*)(vw + (4 * u8 + g) * DEC_VROW + 16 * n) = vf[u8];

        // scores
        f32x4 s[2];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) {
            s[tb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < NF; ++i) {
                s[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tb][i], qh[i], s[tb], 0, 0, 0);
                s[tb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tb][i], ql[i], s[tb], 0, 0, 0);
            }
            if (TAIL) {
                s[tb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(kt[tb], qth, s[tb], 0, 0, 0);
                s[tb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(kt[tb], qtl, s[tb], 0, 0, 0);
            }
        }
        // K~ registers are consumed: prefetch the wave's next tile
        if (tile + 4 < ntiles) load_tile<R>(Ku, Vu, tb0 + 128, t1, g, n, kf, kt, vf);

        // online softmax for head n over this lane's 8 tokens
        float mt = NEG_INF;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) {
                int tok = tb0 + 16 * tb + 4 * g + ii;
                float sv = tok < t1 ? s[tb][ii] : NEG_INF;
                s[tb][ii] = sv;
                mt = fmaxf(mt, sv);
            }
        mt = fmaxf(mt, __shfl_xor(mt, 16));
        mt = fmaxf(mt, __shfl_xor(mt, 32));
        const float m_new = fmaxf(m_run, mt);
        const float alpha = exp2f(m_run - m_new);
        float psum = 0.f;
        bf16x8 ph, pl;
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int ii = 0; ii < 4; ++ii) {
                float p = exp2f(s[tb][ii] - m_new);
                psum += p;
                __bf16 hi, lo;
                split_bf16(p, hi, lo);
                ph[4 * tb + ii] = hi;
                pl[4 * tb + ii] = lo;
            }
        l_run = fmaf(l_run, alpha, psum);
        if (__any(m_new > m_run)) {
            // alpha lives in lanes (., n = head); the accumulators need alpha[4 g + ii]
            if (g == 0) salpha[wave][n] = alpha;
            wave_lds_fence();
            f32x4 a4 = *(const f32x4*)&salpha[wave][4 * g];
#pragma unroll
            for (int cb = 0; cb < 8; ++cb) O[cb] *= a4;
        }
        m_run = m_new;
        wave_lds_fence();

        // O += P V
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) {
            bf16x8 vb;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                int tl = jj < 4 ? 4 * g + jj : 16 + 4 * g + (jj - 4);
                vb[jj] = *(const __bf16*)(vw + tl * DEC_VROW + 2 * (16 * cb + n));
            }
            O[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ph, vb, O[cb], 0, 0, 0);
            O[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pl, vb, O[cb], 0, 0, 0);
        }
        wave_lds_fence();
    }

    // ---- merge the four waves' states, write the split's partial -----------------
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    float* ow = (float*)vw;                   // [16 heads][128 channels]
#pragma unroll
    for (int cb = 0; cb < 8; ++cb)
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) ow[(4 * g + ii) * D + 16 * cb + n] = O[cb][ii];
    if (g == 0) { sm_m[wave][n] = m_run; sm_l[wave][n] = l_run; }
    __syncthreads();
    for (int idx = tid; idx < Gc * D; idx += 256) {
        int hh = idx >> 7, c = idx & 127;
        float M = fmaxf(fmaxf(sm_m[0][hh], sm_m[1][hh]), fmaxf(sm_m[2][hh], sm_m[3][hh]));
        float lsum = 0.f, a = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            float mw = sm_m[w][hh];
            float wgt = (mw > NEG_INF) ? exp2f(mw - M) : 0.f;
            lsum = fmaf(sm_l[w][hh], wgt, lsum);
            a = fmaf(((const float*)vt[w])[hh * D + c], wgt, a);
        }
        size_t pidx = ((size_t)b * Hq + h0 + hh) * S + split;
        ws_acc[pidx * D + c] = a;
        if (c == 0) { ws_m[pidx] = M + sbias[hh]; ws_l[pidx] = lsum; }
    }
}

// ---------------------------------------------------------------------------
bool decode_mfma_supported(int dtype, int r) { return dtype == 1 && r % 16 == 0 && r >= 16 && r <= 128; }

template <int R>
static void launch_decode_mfma_r(dim3 grid, hipStream_t st, const bf16_t* q, const bf16_t* Kp, const bf16_t* Vc,
                                 const float* Rr, const float* dmu, const int32_t* seq_len, int Hq, int Hkv,
                                 int cap, int tps, float sl2, float* m, float* l, float* acc, int S)
{
    hipLaunchKernelGGL(decode_split_mfma<R>, grid, dim3(256), 0, st, q, Kp, Vc, Rr, dmu, seq_len, Hq, Hkv, cap,
                       tps, sl2, m, l, acc, S);
}

hipError_t launch_decode(int dtype, bool mfma, int B, int Hq, int Hkv, int cap, int r, int S, int tps,
                         const void* q, const void* Kp, const void* Vc, const float* Rr, const float* dmu,
                         const int32_t* seq_len, float scale, void* out, float* ws, hipStream_t st)
{
    const size_t rows = (size_t)B * Hq;
    float* ws_m = ws;
    float* ws_l = ws_m + rows * S;
    float* ws_acc = ws_l + rows * S;
    const float sl2 = scale * 1.4426950408889634f;    // scores in the log2 domain
    if (mfma && decode_mfma_supported(dtype, r)) {
        const int G = Hq / Hkv;
        dim3 grid(S, Hkv * ((G + 15) / 16), B);
        const bf16_t *q_ = (const bf16_t*)q, *k_ = (const bf16_t*)Kp, *v_ = (const bf16_t*)Vc;
#define RK_CASE(RV)                                                                                        \
    case RV:                                                                                               \
        launch_decode_mfma_r<RV>(grid, st, q_, k_, v_, Rr, dmu, seq_len, Hq, Hkv, cap, tps, sl2, ws_m, ws_l, \
                                 ws_acc, S);                                                               \
        break;
        switch (r) {
            RK_CASE(16) RK_CASE(32) RK_CASE(48) RK_CASE(64) RK_CASE(80) RK_CASE(96) RK_CASE(112) RK_CASE(128)
            default: return hipErrorInvalidValue;
        }
#undef RK_CASE
    } else {
        dim3 grid(S, Hq, B);
        if (dtype == 0)
            hipLaunchKernelGGL(decode_split_generic<float>, grid, dim3(128), 0, st, (const float*)q,
                               (const float*)Kp, (const float*)Vc, Rr, dmu, seq_len, Hq, Hkv, cap, r, tps, sl2,
                               ws_m, ws_l, ws_acc, S);
        else
            hipLaunchKernelGGL(decode_split_generic<bf16_t>, grid, dim3(128), 0, st, (const bf16_t*)q,
                               (const bf16_t*)Kp, (const bf16_t*)Vc, Rr, dmu, seq_len, Hq, Hkv, cap, r, tps, sl2,
                               ws_m, ws_l, ws_acc, S);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (dtype == 0)
        hipLaunchKernelGGL(decode_merge<float>, dim3((unsigned)rows), dim3(128), 0, st, ws_m, ws_l, ws_acc, S,
                           (float*)out);
    else
        hipLaunchKernelGGL(decode_merge<bf16_t>, dim3((unsigned)rows), dim3(128), 0, st, ws_m, ws_l, ws_acc, S,
                           (bf16_t*)out);
    return hipGetLastError();
}

}  // namespace rk
