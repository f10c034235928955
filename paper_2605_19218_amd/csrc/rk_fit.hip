// Prefill-side rotation construction (Alg. 1 of the RotateK paper, with the full
// eigendecomposition of Sec. 3.2 "Query-Weighted PCA" as the solver):
//   cov_partial_*   : per token chunk, S = sum x x^T and column sums   (Alg. 1 steps 1-3)
//   cov_finalize    : mu, C = S - n mu mu^T, reduced over chunks in fp64
//   eig_jacobi      : C_q = (sigma sigma^T) .* C (step 5 / Eq. 4), all eigenpairs by
//                     parallel two-sided Jacobi resident in LDS, then the keep-mask,
//                     R_r and delta_mu (step 15)
#include <mutex>
#include <set>
#include <utility>
#include "rk_kernels.hpp"

namespace rk {

// Kernels that use more than 64 KB of dynamic LDS need the limit raised once per (device,
// kernel); launches may come from several host threads and contexts.
static hipError_t allow_dynamic_lds(const void* kernel, size_t bytes)
{
    static std::mutex mu;
    static std::set<std::pair<int, const void*>> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (done.count({dev, kernel})) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) done.insert({dev, kernel});
    return e;
}


// ---------------------------------------------------------------------------
// Plain covariance partial: 256 threads, thread (ty, tx) owns the 8x8 outputs
// (ty + 16 i, tx + 16 j); a 16-token tile is staged in LDS as fp32.
template <typename T>
__global__ __launch_bounds__(256) void cov_partial_generic(RowsDev rows, int Hkv, int n_chunks,
                                                           float* __restrict__ part_S,
                                                           float* __restrict__ part_sum)
{
    const int chunk = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int u = b * Hkv + h;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int n_b = rows_count(rows, b);
    const int t0 = chunk * COV_CHUNK;
    const int t1 = min(t0 + COV_CHUNK, n_b);
    const T* base = (const T*)rows.data;

    __shared__ float tile[16][D];
    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
    float csum = 0.f;

    for (int tt = t0; tt < t1; tt += 16) {
        {   // stage 16 rows x 128 channels; thread loads 8 consecutive channels of one row
            int rr = tt + ty;
            int c0 = tx * 8;
            if (rr < t1) {
                const T* src = base + rows_offset(rows, b, h, rr) + c0;
#pragma unroll
                for (int e = 0; e < 8; ++e) tile[ty][c0 + e] = ld_elem(src + e);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) tile[ty][c0 + e] = 0.f;
            }
        }
        __syncthreads();
        if (tid < D) {
#pragma unroll
            for (int t = 0; t < 16; ++t) csum += tile[t][tid];
        }
#pragma unroll 4
        for (int t = 0; t < 16; ++t) {
            float a[8], bb[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) { a[i] = tile[t][ty + 16 * i]; bb[i] = tile[t][tx + 16 * i]; }
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] = fmaf(a[i], bb[j], acc[i][j]);
        }
        __syncthreads();
    }
    float* S = part_S + ((size_t)u * n_chunks + chunk) * (D * D);
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) S[(ty + 16 * i) * D + tx + 16 * j] = acc[i][j];
    if (tid < D) part_sum[((size_t)u * n_chunks + chunk) * D + tid] = csum;
}

// ---------------------------------------------------------------------------
// MFMA covariance partial (bf16 Keys): S = K^T K over a 2048-token chunk with
// v_mfma_f32_32x32x16_bf16, contraction index = tokens.  The matrix core wants, per
// lane, 8 consecutive TOKENS of one channel, while memory holds 8 consecutive
// CHANNELS of one token.  No LDS staging is used: lane (g2, m) loads the 8x8 block
// (tokens 8 g2 ..+7) x (channels 8 (m%16) ..+7) as eight 16-byte row pieces and
// transposes it in registers with v_perm; lanes m and m+16 share a block and take
// the even / odd channels of it.  The channel held by MFMA row m of block cbk is
// therefore ch(cbk, m) = 8 (m % 16) + 2 cbk + m / 16 -- a permutation that is undone
// when the 128x128 partial is written.  Each wave accumulates the 10 upper-triangular
// 32x32 tiles for its own 512 tokens (160 accumulator registers); the four waves are
// summed through LDS in a fixed order, each wave folding and storing a quarter.
constexpr int COVM_TOK_PER_WAVE = 512;
constexpr int COVM_CHUNK = 4 * COVM_TOK_PER_WAVE;
constexpr int COVM_STAGES = 4;             // 16-token k-steps of loads in flight per wave (16 KB; 3 to 5 time alike, 6 and 8 slower)
constexpr size_t COVM_LDS_BYTES = (size_t)(4 * 30 * 4 * 64 + 4 * D) * sizeof(float);   // 4 x 30 parked groups + column sums

// rows >= t_end contribute zeros; the address is clamped to row t_last (always a valid row)
// all 8 rows known to be valid: plain loads, nothing for the compiler to predicate.  Without
// a token list the row address is lane_ptr + (tok0 + jj) * st with st wave-uniform, so the
// only per-lane work is one 64-bit add per row (no per-lane 64-bit multiplies).
template <bool GATHER>
__device__ __forceinline__ void covm_load_full(uint4 (&r)[8], const bf16_t* __restrict__ base, int64_t head_base,
                                               int64_t st, const int32_t* __restrict__ list, int tok0, int o,
                                               const bf16_t* __restrict__ lane_ptr, int tok_rel)
{
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
        if (GATHER) r[jj] = *(const uint4*)(base + row_off<true>(head_base, st, list, tok0 + jj) + 8 * o);
        else {
            // read-once stream: non-temporal, so the rows do not displace each other in the L2
            const u32x4 v = __builtin_nontemporal_load((const u32x4*)(lane_ptr + (int64_t)(tok_rel + jj) * st));
            r[jj] = make_uint4(v.x, v.y, v.z, v.w);
        }
    }
}

// Token-list form: the row numbers of a k-step (eight per lane) and the rows they address are
// two loads in a chain.  The row numbers are requested a whole turn of the stage ring ahead of
// their rows, so that the wait for them does not drain the rows in flight.
__device__ __forceinline__ void covm_load_idx(int (&ix)[8], const int32_t* __restrict__ list, int tok0, int t_last)
{
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) ix[jj] = list[min(tok0 + jj, t_last)];
}
__device__ __forceinline__ void covm_load_rows(uint4 (&r)[8], const bf16_t* __restrict__ base, int64_t head_base,
                                               int64_t st, const int (&ix)[8], int o)
{
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) r[jj] = *(const uint4*)(base + head_base + (int64_t)ix[jj] * st + 8 * o);
}

template <bool GATHER>
__device__ __forceinline__ void covm_load(uint4 (&r)[8], const bf16_t* __restrict__ base, int64_t head_base,
                                          int64_t st, const int32_t* __restrict__ list, int tok0, int t_end,
                                          int t_last, int o)
{
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
        const int tok = tok0 + jj;
        const uint4 v = *(const uint4*)(base + row_off<GATHER>(head_base, st, list, min(tok, t_last)) + 8 * o);
        r[jj] = tok < t_end ? v : make_uint4(0, 0, 0, 0);
    }
}

__device__ __forceinline__ uint32_t dw(const uint4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

__device__ __forceinline__ void covm_step(const uint4 (&r)[8], uint32_t sel, f32x16 (&acc)[10], float (&csum)[4])
{
    bf16x8 frag[4];
#pragma unroll
    for (int cbk = 0; cbk < 4; ++cbk) {
        uint4 d;
        // token pair (2 tp, 2 tp + 1) of channel 2 cbk + parity: low or high halves of dword cbk
        d.x = __builtin_amdgcn_perm(dw(r[1], cbk), dw(r[0], cbk), sel);
        d.y = __builtin_amdgcn_perm(dw(r[3], cbk), dw(r[2], cbk), sel);
        d.z = __builtin_amdgcn_perm(dw(r[5], cbk), dw(r[4], cbk), sel);
        d.w = __builtin_amdgcn_perm(dw(r[7], cbk), dw(r[6], cbk), sel);
        frag[cbk] = __builtin_bit_cast(bf16x8, d);
        // column sums: v_dot2 of each token pair with (1, 1), fp32 accumulate
        const bf16x2 one2 = {(__bf16)1.0f, (__bf16)1.0f};
        float s = csum[cbk];
        s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, d.x), one2, s, false);
        s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, d.y), one2, s, false);
        s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, d.z), one2, s, false);
        s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, d.w), one2, s, false);
        csum[cbk] = s;
    }
    int t = 0;
#pragma unroll
    for (int bi = 0; bi < 4; ++bi)
#pragma unroll
        for (int bj = bi; bj < 4; ++bj) {
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[bi], frag[bj], acc[t], 0, 0, 0);
            ++t;
        }
}

// End-of-chunk reduction over the four waves of a work-group.  park area: [wave][30][lane]
// 16-byte groups, wave w's group g (not one of its own) at slot g - (g > 10 w ? 10 : 0).
constexpr int COVM_OWN = 10, COVM_PARKED = 30;
__device__ __forceinline__ constexpr int covm_slot(int w, int g) { return w * COVM_PARKED + (g < COVM_OWN * w ? g : g - COVM_OWN); }

template <int W>
__device__ __forceinline__ void covm_park(const f32x16 (&acc)[10], f32x4* __restrict__ park, int lane)
{
#pragma unroll
    for (int g = 0; g < 40; ++g)
        if (g / COVM_OWN != W)
            park[covm_slot(W, g) * 64 + lane] =
                (f32x4){acc[g >> 2][4 * (g & 3)], acc[g >> 2][4 * (g & 3) + 1], acc[g >> 2][4 * (g & 3) + 2], acc[g >> 2][4 * (g & 3) + 3]};
}

// partial layout written here: [g][lane][4] floats (element e of group g is accumulator
// i = 4 (g % 4) + e of tile g / 4)
template <int W>
__device__ __forceinline__ void covm_fold_store(const f32x16 (&acc)[10], const f32x4* __restrict__ park, int lane,
                                                f32x4* __restrict__ S4)
{
    f32x4 p[4][COVM_OWN];
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int k = 0; k < COVM_OWN; ++k) {
            const int g = COVM_OWN * W + k;
            if (w == W) p[w][k] = (f32x4){acc[g >> 2][4 * (g & 3)], acc[g >> 2][4 * (g & 3) + 1], acc[g >> 2][4 * (g & 3) + 2], acc[g >> 2][4 * (g & 3) + 3]};
            else p[w][k] = park[covm_slot(w, g) * 64 + lane];
        }
#pragma unroll
    for (int k = 0; k < COVM_OWN; ++k) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = ((p[0][k][e] + p[1][k][e]) + p[2][k][e]) + p[3][k][e];
        S4[(COVM_OWN * W + k) * 64 + lane] = v;
    }
}

template <bool GATHER>
__global__ __launch_bounds__(256) void cov_partial_mfma(RowsDev rows, int Hkv, int n_chunks,
                                                        float* __restrict__ part_S, float* __restrict__ part_sum)
{
    // the chunk number is rotated by head and batch item: with a chunk count that is a multiple of 8 an
    // XCD (work-groups are dealt to the XCDs by linear index) would otherwise own one chunk position of
    // every sequence, and ragged batches have few sequences with the last positions
    const int h = blockIdx.y, b = blockIdx.z;
    const int chunk = (int)((blockIdx.x + blockIdx.y + blockIdx.z) % gridDim.x);
    const int u = b * Hkv + h;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: loop control stays scalar
    const int g2 = lane >> 5, m = lane & 31, o = m & 15, par = m >> 4;
    const uint32_t sel = par ? 0x07060302u : 0x05040100u;
    const int n_b = rows_count(rows, b);
    const int t0 = chunk * COVM_CHUNK, t1 = min(t0 + COVM_CHUNK, n_b);
    const int tw0 = t0 + wave * COVM_TOK_PER_WAVE, tw1 = min(tw0 + COVM_TOK_PER_WAVE, t1);
    const int nks = tw1 > tw0 ? (tw1 - tw0 + 15) >> 4 : 0;      // 16-token k-steps, the last may be partial
    const int nfull = tw1 > tw0 ? (tw1 - tw0) >> 4 : 0;         // k-steps with all 16 tokens valid
    const bf16_t* base = (const bf16_t*)rows.data;
    const int64_t hb = (int64_t)b * rows.sb + (int64_t)h * rows.sh, rst = rows.st;
    const int32_t* list = GATHER ? rows.tok_idx + rows.tok_off[b] : nullptr;
    // this lane's first row piece: token tw0 + 8 g2, channels 8 o ..+7 (used when there is no token list)
    const bf16_t* lane_ptr = base + hb + (int64_t)(tw0 + 8 * g2) * rst + 8 * o;

    extern __shared__ __attribute__((aligned(16))) float cov_smem[];
    f32x4* bufv = (f32x4*)cov_smem;             // parked accumulator groups: [wave][30][lane]
    float (*ssum)[D] = (float (*)[D])(cov_smem + 4 * 30 * 4 * 64);

    f32x16 acc[10];
#pragma unroll
    for (int t = 0; t < 10; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
    float csum[4] = {0.f, 0.f, 0.f, 0.f};

    if (nks > 0) {
        uint4 st[COVM_STAGES][8];
        int ks = 0;
        // Every wave owns a 128 KB run of rows at a 128 KB-aligned offset; walking them all from
        // the start would keep the 1024 waves of the grid on the same few HBM channels at any
        // instant.  A full wave (32 k-steps) therefore starts at a wave/chunk/head dependent
        // k-step and wraps around (the sum is order-independent up to fp32 rounding, and the
        // order is still fixed for a given launch shape).
        constexpr int NKW = COVM_TOK_PER_WAVE / 16;
        const int shift = (nfull == NKW) ? ((wave * 8 + chunk * 5 + u * 11) & (NKW - 1)) : 0;
#define KSTEP_TOK(i) (16 * (((i) + shift) & (NKW - 1)))
        if (GATHER && nfull >= 2 * COVM_STAGES) {
            int ix[COVM_STAGES][8];
#pragma unroll
            for (int s = 0; s < COVM_STAGES; ++s) covm_load_idx(ix[s], list, tw0 + KSTEP_TOK(s) + 8 * g2, tw1 - 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < COVM_STAGES; ++s) {
                covm_load_rows(st[s], base, hb, rst, ix[s], o);
                covm_load_idx(ix[s], list, tw0 + KSTEP_TOK(s + COVM_STAGES) + 8 * g2, tw1 - 1);
                __builtin_amdgcn_sched_barrier(0);
            }
            for (; ks + 2 * COVM_STAGES <= nfull; ks += COVM_STAGES) {
#pragma unroll
                for (int s = 0; s < COVM_STAGES; ++s) {
                    covm_step(st[s], sel, acc, csum);
                    covm_load_rows(st[s], base, hb, rst, ix[s], o);           // k-step ks + s + STAGES
                    covm_load_idx(ix[s], list, tw0 + KSTEP_TOK(ks + s + 2 * COVM_STAGES) + 8 * g2, tw1 - 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else if (nfull >= 2 * COVM_STAGES) {
            // Long chunk (the normal case).  The fill and the steady loop use plain loads of
            // full k-steps with no branch anywhere near them, so every wait on them is exact
            // (a conservative wait-count state entering the loop would be paid every iteration).
#pragma unroll
            for (int s = 0; s < COVM_STAGES; ++s) {
                covm_load_full<GATHER>(st[s], base, hb, rst, list, tw0 + KSTEP_TOK(s) + 8 * g2, o, lane_ptr, KSTEP_TOK(s));
                __builtin_amdgcn_sched_barrier(0);      // stage 0 must be the OLDEST load on loop entry
            }
            for (; ks + 2 * COVM_STAGES <= nfull; ks += COVM_STAGES) {
#pragma unroll
                for (int s = 0; s < COVM_STAGES; ++s) {
                    covm_step(st[s], sel, acc, csum);
                    covm_load_full<GATHER>(st[s], base, hb, rst, list, tw0 + KSTEP_TOK(ks + s + COVM_STAGES) + 8 * g2, o,
                                           lane_ptr, KSTEP_TOK(ks + s + COVM_STAGES));
                    // keep "consume stage s, refill stage s" together: without this the scheduler
                    // hoists all four stages' math above all 32 loads and the pipeline collapses
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < COVM_STAGES; ++s)
                covm_load<GATHER>(st[s], base, hb, rst, list, tw0 + 16 * s + 8 * g2, s < nks ? tw1 : 0, tw1 - 1, o);
        }
        // remaining k-steps (at most 2 STAGES - 1 after a steady loop), the last possibly partial
        for (; ks < nks; ks += COVM_STAGES) {
#pragma unroll
            for (int s = 0; s < COVM_STAGES; ++s) {
                if (ks + s < nks) {
                    covm_step(st[s], sel, acc, csum);
                    if (ks + s + COVM_STAGES < nks)
                        covm_load<GATHER>(st[s], base, hb, rst, list,
                                          tw0 + (shift ? KSTEP_TOK(ks + s + COVM_STAGES) : 16 * (ks + s + COVM_STAGES)) + 8 * g2,
                                          tw1, tw1 - 1, o);
                }
            }
        }
    }

#undef KSTEP_TOK
    // ---- sum the four waves, every element as ((w0 + w1) + w2) + w3 ----------------------
    // The 160 accumulators of a lane form 40 groups of four, g = 4 tile + i / 4.  Wave w owns
    // groups [10 w, 10 w + 10): it parks the 30 groups it does not own, and after ONE barrier
    // adds the three parked copies of its own groups to its registers (all 30 reads issued
    // before the first add) and stores its quarter of the chunk's partial, 16 bytes per lane.
#pragma unroll
    for (int cbk = 0; cbk < 4; ++cbk) {
        float s = csum[cbk] + __shfl_xor(csum[cbk], 32);
        if (g2 == 0) ssum[wave][8 * o + 2 * cbk + par] = s;
    }
    switch (wave) {
    case 0: covm_park<0>(acc, bufv, lane); break;
    case 1: covm_park<1>(acc, bufv, lane); break;
    case 2: covm_park<2>(acc, bufv, lane); break;
    default: covm_park<3>(acc, bufv, lane); break;
    }
    __syncthreads();
    f32x4* S4 = (f32x4*)(part_S + ((size_t)u * n_chunks + chunk) * (D * D));
    switch (wave) {
    case 0: covm_fold_store<0>(acc, bufv, lane, S4); break;
    case 1: covm_fold_store<1>(acc, bufv, lane, S4); break;
    case 2: covm_fold_store<2>(acc, bufv, lane, S4); break;
    default: covm_fold_store<3>(acc, bufv, lane, S4); break;
    }
    if (tid < D)
        part_sum[((size_t)u * n_chunks + chunk) * D + tid] = ((ssum[0][tid] + ssum[1][tid]) + ssum[2][tid]) + ssum[3][tid];
}

// ---------------------------------------------------------------------------
// Reduce the chunk partials in fp64 and apply the centering correction
// C = S - n mu mu^T (equal to (K-mu)^T (K-mu)).  grid (8, U): block x covers rows
// [16x, 16x+16).
__global__ __launch_bounds__(256) void cov_finalize(RowsDev rows, int Hkv, int n_chunks, int center,
                                                    const float* __restrict__ part_S,
                                                    const float* __restrict__ part_sum,
                                                    float* __restrict__ cov, float* __restrict__ mu_out)
{
    const int u = blockIdx.y, b = u / Hkv;
    const int tid = threadIdx.x;
    const int n_b = rows_count(rows, b);
    __shared__ double smu[D];
    // sum over chunks in ascending order; loads are issued 8 at a time (independent), adds stay ordered
    auto chunk_sum = [&](const float* __restrict__ p, size_t stride) {
        double s = 0.0;
        int ch = 0;
        for (; ch + 8 <= n_chunks; ch += 8) {
            float v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = p[(size_t)(ch + k) * stride];
#pragma unroll
            for (int k = 0; k < 8; ++k) s += (double)v[k];
        }
        for (; ch < n_chunks; ++ch) s += (double)p[(size_t)ch * stride];
        return s;
    };
    if (tid < D) {
        double s = chunk_sum(part_sum + (size_t)u * n_chunks * D + tid, D);
        double m = n_b > 0 ? s / (double)n_b : 0.0;
        smu[tid] = m;
        if (blockIdx.x == 0) mu_out[(size_t)u * D + tid] = (float)m;
    }
    __syncthreads();
    const int j = tid & (D - 1);
    for (int ri = 0; ri < 8; ++ri) {
        int i = blockIdx.x * 16 + ri * 2 + (tid >> 7);
        const int pos = i * D + j;
        double s = chunk_sum(part_S + (size_t)u * n_chunks * (D * D) + pos, (size_t)D * D);
        if (center) s -= (double)n_b * (smu[i] * smu[j]);
        cov[(size_t)u * D * D + i * D + j] = (float)s;
    }
}

// Reduction of tile-format partials (written by cov_partial_mfma) in their own order: thread =
// one (tile, i, lane) position, so every load is coalesced across the wave and all chunks of a
// position are in flight together; the element goes to cov[r][c] and, for off-diagonal tiles
// and off-diagonal elements of diagonal tiles, cov[c][r] is written by its own position or
// mirrored here.  Grid (40, U): 10 tiles x 1024 positions per (b, h_kv).
__global__ __launch_bounds__(256) void cov_finalize_tiled(RowsDev rows, int Hkv, int n_chunks, int center,
                                                          const float* __restrict__ part_S,
                                                          const float* __restrict__ part_sum,
                                                          float* __restrict__ cov, float* __restrict__ mu_out)
{
    const int u = blockIdx.y, b = u / Hkv;
    const int tid = threadIdx.x;
    const int n_b = rows_count(rows, b);
    __shared__ double smu[D];
    const int posn = blockIdx.x * 256 + tid;            // [tile][i / 4][lane][i % 4], 0 .. 10239
    const float* pS = part_S + (size_t)u * n_chunks * (D * D) + posn;
    // the first 8 chunks of this position: requested before the mean is formed
    float v0[8];
    const int first = min(n_chunks, 8);
#pragma unroll
    for (int k = 0; k < 8; ++k) v0[k] = pS[(size_t)min(k, first - 1) * (D * D)];
    if (tid < D) {
        // column sums of the chunks, eight loads in flight at a time (one at a time this loop was most of
        // the kernel: eight dependent round trips), added in ascending chunk order
        const float* ps = part_sum + (size_t)u * n_chunks * D + tid;
        double s = 0.0;
        for (int ch = 0; ch < n_chunks; ch += 8) {
            float v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = ps[(size_t)min(ch + k, n_chunks - 1) * D];
#pragma unroll
            for (int k = 0; k < 8; ++k) s += ch + k < n_chunks ? (double)v[k] : 0.0;
        }
        const double m = n_b > 0 ? s / (double)n_b : 0.0;
        smu[tid] = m;
        if (blockIdx.x == 0) mu_out[(size_t)u * D + tid] = (float)m;
    }
    __syncthreads();
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < 8; ++k) acc += k < first ? (double)v0[k] : 0.0;          // ascending chunk order
    for (int ch = 8; ch < n_chunks; ch += 8) {
        float v[8];
        const int last = n_chunks - 1;
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = pS[(size_t)min(ch + k, last) * (D * D)];
#pragma unroll
        for (int k = 0; k < 8; ++k) acc += ch + k < n_chunks ? (double)v[k] : 0.0;
    }
    // position -> (row channel, column channel): the MFMA output layout and the channel permutation undone
    const int t = posn >> 10, i = 4 * ((posn >> 8) & 3) + (posn & 3), lane = (posn >> 2) & 63;
    int br = 0, rem = t;
    while (rem >= 4 - br) { rem -= 4 - br; ++br; }
    const int bc = br + rem;
    const int mr = 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3), mc = lane & 31;
    const int rch = ((mr & 15) << 3) | (br << 1) | (mr >> 4);
    const int cch = ((mc & 15) << 3) | (bc << 1) | (mc >> 4);
    if (center) acc -= (double)n_b * (smu[rch] * smu[cch]);
    float* Cu = cov + (size_t)u * D * D;
    Cu[rch * D + cch] = (float)acc;
    if (br != bc) Cu[cch * D + rch] = (float)acc;       // diagonal tiles hold both (r, c) and (c, r)
}

// ---------------------------------------------------------------------------
// Batched symmetric eigensolver: parallel two-sided Jacobi with a round-robin ordering (a sweep is
// 127 rounds of 64 disjoint pairs), in three launches.
//   eig_jacobi_rotations  one 1024-thread work-group per 128x128 matrix iterates on A alone and
//                         records the 64 rotations (sin, sin / (1 + cos)) of every round;
//   eig_apply_rotations   replays the recorded rotations on V = I.  Rows of V are independent, so
//                         this half of the arithmetic leaves the one compute unit that holds A and
//                         spreads over the chip, four rows per wave, in registers;
//   eig_finish            gathers R_r and forms delta_mu.
// Pairs are taken by POSITION: position 2 k and 2 k + 1 form pair k, and after every round the rows
// and columns move to new positions (position 0 stays, 1 -> 2, even positions move up by two,
// 126 -> 127, odd positions move down by two): the 127 moving positions form one cycle, every two
// indices meet exactly once in 127 rounds, and after a sweep every index is back where it started,
// so eigenvalue c is the final A[c][c] and its vector is V[:, c].  Because the pairing is fixed in
// position space, every thread reads and writes the same LDS addresses in every round: the rotated
// 2x2 block is written straight to its next position in a second copy of A (two copies, row stride
// 130 floats), there is no index arithmetic in the loop, and only the part of A on or above the
// diagonal (by pair, then by position) is kept: a rotated element is stored once, at (r, c) or (c, r),
// whichever lies there.  The LDS pipeline is the bound of a round (about five cycles per wave-wide
// instruction, whatever its width up to 8 bytes per lane), so the loop is written for few LDS
// instructions: 7 per block.
constexpr int EIG_THREADS = 1024;
constexpr int EIG_MAX_SWEEPS = 20;
constexpr int EIG_ROUNDS = D - 1;
constexpr int EIG_LD = D + 2;             // row stride of the LDS copies of A (even: a 2x2 block is two 8-byte reads)
constexpr int EIG_ROT_ROUNDS = EIG_MAX_SWEEPS * EIG_ROUNDS;     // recorded rounds per matrix
constexpr int EIG_FUSE_V_FROM = 192;      // matrices per call from which V is carried inside the A kernel
                                          // (measured: 128 matrices 1.29 ms carried / 1.17 ms replayed, 256: 1.41 / 1.53, 512: 2.48 / 3.0)
constexpr size_t EIG_LDS_BYTES = (size_t)(2 * D * EIG_LD + 4 * 64 + 32 + D) * sizeof(float);

// LDS offset of the kept copy of element (r, c) = (c, r): pairs in ascending order, then positions
__device__ __forceinline__ constexpr int eig_upper(int r, int c)
{
    return ((r >> 1) < (c >> 1) || ((r >> 1) == (c >> 1) && r <= c)) ? r * (D + 2) + c : c * (D + 2) + r;
}

size_t eig_rotation_bytes(size_t U) { return U * EIG_ROT_ROUNDS * 64 * sizeof(float2); }

// position of a row / column after one round
__host__ __device__ constexpr int eig_next_pos(int p)
{
    return p == 0 ? 0 : p == 1 ? 2 : p == D - 2 ? D - 1 : (p & 1) ? p - 2 : p + 2;
}

// Rotation that annihilates the (p, q) element: t = tan, s = sin, tau = s / (1 + c).  One square
// root and hardware reciprocals with a Newton step each: the chain sits between the two barriers of
// every round, and the IEEE division and square-root sequences are several times as long.
// (s, tau) is applied as x' = x - s (y + tau x), y' = y + s (x - tau y), which is orthogonal to the
// accuracy of tau = s / (1 + c) alone, so a last-place error in t only moves the angle.
__device__ __forceinline__ float rcp_nr(float x)
{
    float r = __builtin_amdgcn_rcpf(x);
    return fmaf(r, fmaf(-x, r, 1.f), r);
}
__device__ __forceinline__ void jacobi_params(float app, float aqq, float apq, float thr_skip, float& s, float& tau,
                                              float& t)
{
    s = 0.f; tau = 0.f; t = 0.f;
    if (fabsf(apq) > thr_skip) {
        // t = sgn(theta) / (|theta| + sqrt(theta^2 + 1)), theta = (aqq - app) / (2 apq), without forming theta
        const float al = aqq - app, be = 2.f * apq;
        const float h = __builtin_amdgcn_sqrtf(fmaf(al, al, be * be));
        t = (al >= 0.f) ? be * rcp_nr(al + h) : be * rcp_nr(al - h);
        const float d = fmaf(t, t, 1.f);
        float c = __builtin_amdgcn_rsqf(d);
        c = c * fmaf(-0.5f * d * c, c, 1.5f);          // one Newton step on 1/sqrt(d)
        s = t * c;
        tau = s * rcp_nr(1.f + c);
    }
}

// whole-wave lane shifts by one (data-parallel-primitive moves; the end lane has no source and keeps `keep`)
__device__ __forceinline__ float lane_from_below(float keep, float v)      // lane i <- lane i - 1; lane 0 keeps `keep`
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, keep), __builtin_bit_cast(int, v),
                                                                 0x138, 0xf, 0xf, false));
}
__device__ __forceinline__ float lane_from_above(float keep, float v)      // lane i <- lane i + 1; lane 63 keeps `keep`
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, keep), __builtin_bit_cast(int, v),
                                                                 0x130, 0xf, 0xf, false));
}

template <bool B>
struct EigBool { static constexpr bool value = B; };

// WITH_V: the rows of V are updated in this kernel as well (waves 1-15, nine rows each, in registers, as
// in eig_apply_rotations) and R is written at the end; nothing is recorded.  A round is then bound by
// vector issue (about 2000 cycles instead of 1400), which pays once there are enough matrices to fill
// the chip: the replay kernel is throughput-bound, this one is not.
constexpr int EIGV_FUSED_ROWS = 9;
template <bool WITH_V>
__global__ __launch_bounds__(EIG_THREADS) void eig_jacobi_rotations(const float* __restrict__ cov,
                                                                    const float* __restrict__ sigma, int r,
                                                                    float* __restrict__ lam_out,
                                                                    uint8_t* __restrict__ mask_out,
                                                                    int32_t* __restrict__ keep_out,
                                                                    float2* __restrict__ rot,
                                                                    int32_t* __restrict__ sweeps_ws,
                                                                    int32_t* __restrict__ sweeps_out,
                                                                    float* __restrict__ R_out)
{
    extern __shared__ float sm[];
    float* A2 = sm;                                   // [2][128][129]: the two copies of A
    float2* prm = (float2*)(A2 + 2 * D * EIG_LD);     // [2][64] (sin, sin / (1 + cos)) of this round and the next
    float* red = (float*)(prm + 128);                 // [32] reduction scratch
    float* slam = red + 32;                           // [128]
    constexpr int BUF = D * EIG_LD;

    const int u = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // 16 waves
    const float* C = cov + (size_t)u * D * D;
    const float* sg = sigma ? sigma + (size_t)u * D : nullptr;
    float2* rot_u = rot + (size_t)u * EIG_ROT_ROUNDS * 64;

    // load C_q = sigma_i sigma_j C_ij and ||C_q||_F^2
    float nrm = 0.f;
    for (int idx = tid; idx < D * D; idx += EIG_THREADS) {
        int i = idx >> 7, j = idx & 127;
        float v = C[idx];
        if (sg) v *= sg[i] * sg[j];
        A2[i * EIG_LD + j] = v;
        nrm = fmaf(v, v, nrm);
    }
    nrm = wave_sum(nrm);
    if (lane == 0) red[wave] = nrm;
    __syncthreads();
    float normF2 = 0.f;
    for (int w = 0; w < 16; ++w) normF2 += red[w];
    const float normF = sqrtf(normF2);
    const float thr_skip = 1e-12f * normF;
    const float tol2 = (2e-8f * 2e-8f) * normF2;
    __syncthreads();

    // The 2016 blocks above the diagonal as 32 wave-wide tasks, two per wave: task j covers row
    // pair j (63 - j blocks) in its first lanes and row pair 62 - j (j + 1 blocks) in the rest;
    // task 31 is the 32 blocks of row pair 31 alone.  A thread's two blocks never change.
    // Stores: one instruction stores an even column from lanes with bit 4 clear and an odd column from
    // the others (and the second instruction the other way round), so that the 32 lanes the LDS serves
    // together spread over all 32 banks instead of the 16 of one column parity.
    const bool hi16 = (lane & 16) != 0;
    int rd[2], rd1[2], pk[2], pkp[2], wa[2][2], wb[2][2];
    bool act[2];
#pragma unroll
    for (int ts = 0; ts < 2; ++ts) {
        const int j = ts == 0 ? wave : 31 - wave;
        const int split = 63 - j;
        const int k = lane < split ? j : 62 - j;
        const int kp = lane < split ? j + 1 + lane : 63 - j + (lane - split);
        act[ts] = !(j == 31 && lane >= 32);
        rd[ts] = 2 * k * EIG_LD + 2 * kp;
        rd1[ts] = rd[ts] + EIG_LD;
        asm volatile("" : "+v"(rd1[ts]));      // two 8-byte reads: measured at 7 cycles per wave against 10 for one two-address read
        pk[ts] = k;
        pkp[ts] = kp;
        const int r0 = eig_next_pos(2 * k), r1 = eig_next_pos(2 * k + 1);
        const int c0 = eig_next_pos(2 * kp), c1 = eig_next_pos(2 * kp + 1);
        // pairs (x0, x1) = (e00, e01) and (e10, e11): first store takes x0 in the low lanes and x1 in the
        // high lanes, second store the rest
        const int w00 = eig_upper(r0, c0), w01 = eig_upper(r0, c1), w10 = eig_upper(r1, c0), w11 = eig_upper(r1, c1);
        wa[ts][0] = hi16 ? w01 : w00; wb[ts][0] = hi16 ? w00 : w01;
        wa[ts][1] = hi16 ? w11 : w10; wb[ts][1] = hi16 ? w10 : w11;
    }
    // Wave 0, lane k, owns pair k: its diagonal block and its rotation.  The rotation of round n + 1 is
    // computed DURING round n, so that no wave ever waits for it: after round n the new diagonal
    // block of pair k holds the old (rotated) diagonal elements of pairs k - 1 and k + 1 -- known to
    // this wave -- and one off-diagonal element of the block (k - 1, k + 1), which the lane rotates
    // for itself from the current copy of A (lanes 0, 1 and 63 sit at the ends of the cycle and take
    // their three elements from the neighbouring places instead).
    const int lk = lane;
    const int lrow = lk <= 1 ? 0 : lk == 63 ? 62 : lk - 1;              // row pair of the look-ahead block
    const int lcol = lk == 0 ? 1 : lk == 63 ? 63 : lk + 1;              // its column pair
    const int lrd = 2 * lrow * EIG_LD + 2 * lcol;
    int lrd1 = lrd + EIG_LD;
    asm volatile("" : "+v"(lrd1));
    const int dn0 = eig_next_pos(2 * lk), dn1 = eig_next_pos(2 * lk + 1);
    float ps = 0.f, ptau = 0.f, dE00 = 0.f, dE11 = 0.f, dOff = 0.f;    // pair k: rotation and rotated diagonal block
    if (wave == 0) __builtin_amdgcn_s_setprio(3);     // its dependent chain is the critical path of every round (740 -> 727 us)
    if (wave == 0) {
        const int dg = 2 * lk * EIG_LD + 2 * lk;
        const float app = A2[dg], apq = A2[dg + 1], aqq = A2[dg + EIG_LD + 1];
        float tn;
        jacobi_params(app, aqq, apq, thr_skip, ps, ptau, tn);
        prm[lk] = make_float2(ps, ptau);
        if (!WITH_V) rot_u[lk] = lk == 0 ? make_float2(-ps, -ptau) : make_float2(ps, ptau);   // pair 0: see eig_apply_rotations
        dOff = (ps == 0.f) ? apq : 0.f;                    // left as it is when the rotation is skipped
        dE00 = app - tn * apq;
        dE11 = aqq + tn * apq;
    }
    __syncthreads();
    // WITH_V: wave w >= 1 holds rows 9 (w - 1) .. + 8 of V (rows >= 128 are padding), lane k the elements at
    // positions 2 k and 2 k + 1
    float vtop[EIGV_FUSED_ROWS], vbot[EIGV_FUSED_ROWS];
    const int vrow0 = (wave - 1) * EIGV_FUSED_ROWS;
    if (WITH_V) {
#pragma unroll
        for (int i = 0; i < EIGV_FUSED_ROWS; ++i) {
            // lane 0 holds its pair exchanged (position 1 on top): see eig_apply_rotations
            vtop[i] = (wave > 0 && vrow0 + i == (lane == 0 ? 1 : 2 * lane)) ? 1.f : 0.f;
            vbot[i] = (wave > 0 && vrow0 + i == (lane == 0 ? 0 : 2 * lane + 1)) ? 1.f : 0.f;
        }
    }

    // One round: from copy FROM1 of A to the other one; rotations of this round in prm[FROM1].
    // Rotations are applied as x' = x - s (y + tau x), y' = y + s (x - tau y) with tau = s / (1 + c):
    // 1 - c is then carried to relative precision, so small angles (c rounding to 1) do not inflate
    // the column norms of V.
    auto round_step = [&](auto from1, int t) {
        constexpr int F = decltype(from1)::value ? 1 : 0;
        const float* cur = A2 + F * BUF;
        float* nxt = A2 + (1 - F) * BUF;
        const float2* pcur = prm + 64 * F;
        float2* pnext = prm + 64 * (1 - F);
        if (wave == 0) {
            // this round's rotated diagonal blocks, at their next positions
            nxt[dn0 * EIG_LD + dn0] = dE00;
            nxt[dn1 * EIG_LD + dn1] = dE11;
            nxt[eig_upper(dn0, dn1)] = dOff;
            // next round's pair k
            const float2 ltop = *(const float2*)(cur + lrd), lbot = *(const float2*)(cur + lrd1);
            const float a00 = ltop.x, a01 = ltop.y, a10 = lbot.x, a11 = lbot.y;
            const float s1 = lane_from_below(ps, ps), tau1 = lane_from_below(ptau, ptau);      // pair k - 1 (lane 0: its own)
            const float s2 = lane_from_above(ps, ps), tau2 = lane_from_above(ptau, ptau);      // pair k + 1 (lane 63: its own)
            const float b00 = a00 - s1 * (a10 + tau1 * a00), b01 = a01 - s1 * (a11 + tau1 * a01);
            const float b10 = a10 + s1 * (a00 - tau1 * a10), b11 = a11 + s1 * (a01 - tau1 * a11);
            const float e00 = b00 - s2 * (b01 + tau2 * b00), e01 = b01 + s2 * (b00 - tau2 * b01);
            const float e11 = b11 + s2 * (b10 - tau2 * b11);
            const float apq = lk == 1 ? e11 : lk == 63 ? e00 : e01;
            const float below00 = lane_from_below(dE00, dE00), below11 = lane_from_below(dE11, dE11);
            const float app = lk == 1 ? below11 : below00;                 // lane 0: its own dE00
            const float aqq = lane_from_above(dE00, dE11);                 // lane 63: its own dE00
            float tn;
            jacobi_params(app, aqq, apq, thr_skip, ps, ptau, tn);
            pnext[lk] = make_float2(ps, ptau);
            if (!WITH_V && t + 1 < EIG_ROT_ROUNDS)
                rot_u[(size_t)(t + 1) * 64 + lk] = lk == 0 ? make_float2(-ps, -ptau) : make_float2(ps, ptau);
            dOff = (ps == 0.f) ? apq : 0.f;
            dE00 = app - tn * apq;
            dE11 = aqq + tn * apq;
        }
        float2 pv = make_float2(0.f, 0.f);
        if (WITH_V && wave != 0) {
            pv = pcur[lane];
            if (lane == 0) pv = make_float2(-pv.x, -pv.y);
        }
        float a[2][4];
        float2 p1[2], p2[2];
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) {
            const float2 top = *(const float2*)(cur + rd[ts]), bot = *(const float2*)(cur + rd1[ts]);
            a[ts][0] = top.x; a[ts][1] = top.y; a[ts][2] = bot.x; a[ts][3] = bot.y;
            p1[ts] = pcur[pk[ts]];
            p2[ts] = pcur[pkp[ts]];
        }
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) {
            const float s1 = p1[ts].x, tau1 = p1[ts].y, s2 = p2[ts].x, tau2 = p2[ts].y;
            const float a00 = a[ts][0], a01 = a[ts][1], a10 = a[ts][2], a11 = a[ts][3];
            // rows 2 k, 2 k + 1 : J^T from the left
            const float b00 = a00 - s1 * (a10 + tau1 * a00), b01 = a01 - s1 * (a11 + tau1 * a01);
            const float b10 = a10 + s1 * (a00 - tau1 * a10), b11 = a11 + s1 * (a01 - tau1 * a11);
            // columns 2 k', 2 k' + 1 : J from the right
            const float e00 = b00 - s2 * (b01 + tau2 * b00), e01 = b01 + s2 * (b00 - tau2 * b01);
            const float e10 = b10 - s2 * (b11 + tau2 * b10), e11 = b11 + s2 * (b10 - tau2 * b11);
            const float xa0 = hi16 ? e01 : e00, xb0 = hi16 ? e00 : e01;
            const float xa1 = hi16 ? e11 : e10, xb1 = hi16 ? e10 : e11;
            if (act[ts]) { nxt[wa[ts][0]] = xa0; nxt[wb[ts][0]] = xb0; nxt[wa[ts][1]] = xa1; nxt[wb[ts][1]] = xb1; }
        }
        if (WITH_V && wave != 0) {                      // V <- V J, then the columns move (see eig_apply_rotations)
            const bool lane0 = lane == 0;
#pragma unroll
            for (int i = 0; i < EIGV_FUSED_ROWS; ++i) {
                const float x = vtop[i], y = vbot[i];
                const float xn = x - pv.x * (y + pv.y * x), yn = y + pv.x * (x - pv.y * y);
                const float b_dn = lane_from_above(xn, yn);
                vtop[i] = lane_from_below(b_dn, xn);
                vbot[i] = lane0 ? yn : b_dn;
            }
        }
        __syncthreads();
    };
    // One sweep that starts in copy START1 (and ends in the other one: 127 is odd).
    auto sweep_from = [&](auto start1, int t0) {
        constexpr bool S1 = decltype(start1)::value;
#pragma unroll 1
        for (int round = 0; round < EIG_ROUNDS - 1; round += 2) {
            round_step(EigBool<S1>{}, t0 + round);
            round_step(EigBool<!S1>{}, t0 + round + 1);
        }
        round_step(EigBool<S1>{}, t0 + EIG_ROUNDS - 1);
    };

    int sweeps_done = 0;
    for (int sweep = 0; sweep < EIG_MAX_SWEEPS; ++sweep) {
        // off-diagonal norm (every index is at its own position between sweeps)
        const float* cur = A2 + (sweeps_done & 1) * BUF;
        float off = 0.f;
        for (int idx = tid; idx < D * D; idx += EIG_THREADS) {
            int i = idx >> 7, j = idx & 127;
            float v = cur[i * EIG_LD + j];
            if (i < j) off = fmaf(2.f * v, v, off);             // only the upper triangle is kept
        }
        off = wave_sum(off);
        if (lane == 0) red[16 + wave] = off;
        __syncthreads();
        float off2 = 0.f;
        for (int w = 0; w < 16; ++w) off2 += red[16 + w];
        __syncthreads();
        if (!(off2 > tol2)) break;      // uniform across the block
        if (sweeps_done & 1) sweep_from(EigBool<true>{}, sweeps_done * EIG_ROUNDS);
        else sweep_from(EigBool<false>{}, sweeps_done * EIG_ROUNDS);
        ++sweeps_done;
    }

    // ---- eigenvalues, rank, mask (integer logic) -----------------------------
    const float* Af = A2 + (sweeps_done & 1) * BUF;
    if (tid == 0) {
        sweeps_ws[u] = sweeps_done;
        if (sweeps_out) sweeps_out[u] = sweeps_done;
    }
    if (tid < D) slam[tid] = Af[tid * EIG_LD + tid];
    if (WITH_V && wave != 0) {
#pragma unroll
        for (int i = 0; i < EIGV_FUSED_ROWS; ++i)
            if (vrow0 + i < D)
                *(float2*)(R_out + (size_t)u * D * D + (size_t)(vrow0 + i) * D + 2 * lane) =
                    lane == 0 ? make_float2(vbot[i], vtop[i]) : make_float2(vtop[i], vbot[i]);
    }
    __syncthreads();
    if (tid < D) {
        float lc = slam[tid];
        int rank = 0;
        for (int i = 0; i < D; ++i) {
            float li = slam[i];
            rank += (li > lc || (li == lc && i < tid)) ? 1 : 0;
        }
        lam_out[(size_t)u * D + tid] = lc;
        mask_out[(size_t)u * D + tid] = (uint8_t)(rank < r);
        if (rank < r) keep_out[(size_t)u * r + rank] = tid;
    }
}

// V <- V J_1 J_2 ... over the recorded rounds, V = I at the start.  Wave = four rows of V; lane k
// holds the elements at positions 2 k ("top") and 2 k + 1 ("bottom") of each row -- except lane 0,
// which holds its pair exchanged (position 1 on top, the position 0 that never moves at the bottom;
// its recorded rotation is stored negated, which is the same rotation with the two roles swapped).
// A round rotates every lane's pair and then moves the columns to their next positions.  With lane 0
// exchanged the 127 moving positions form one ring through the registers: up the tops from lane 0 to
// lane 63, down the bottoms from lane 63 to lane 1, and back into lane 0's top.  That is two whole-wave
// shifts by one lane (data-parallel-primitive moves, no LDS) -- the bottoms move down, lane 63 taking
// its own top; the tops move up, lane 0 taking what came down to it -- and one select that puts the
// fixed element back: 7 vector instructions per row and round.  Grid (8, U), 256 threads.
constexpr int EIGV_ROWS = 4;
__global__ __launch_bounds__(256) void eig_apply_rotations(const float2* __restrict__ rot,
                                                           const int32_t* __restrict__ sweeps_ws,
                                                           float* __restrict__ R_out)
{
    const int u = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row0 = (blockIdx.x * 4 + wave) * EIGV_ROWS;
    const float2* rot_u = rot + (size_t)u * EIG_ROT_ROUNDS * 64 + lane;
    const int n_rounds = min(max(sweeps_ws[u], 0), EIG_MAX_SWEEPS) * EIG_ROUNDS;
    float top[EIGV_ROWS], bot[EIGV_ROWS];
#pragma unroll
    for (int i = 0; i < EIGV_ROWS; ++i) {
        top[i] = (row0 + i == (lane == 0 ? 1 : 2 * lane)) ? 1.f : 0.f;
        bot[i] = (row0 + i == (lane == 0 ? 0 : 2 * lane + 1)) ? 1.f : 0.f;
    }
    const bool lane0 = lane == 0;
    auto apply = [&](float2 p) {
#pragma unroll
        for (int i = 0; i < EIGV_ROWS; ++i) {
            const float x = top[i], y = bot[i];
            const float xn = x - p.x * (y + p.y * x), yn = y + p.x * (x - p.y * y);
            const float b_dn = lane_from_above(xn, yn);      // lane k <- bottom of lane k + 1; lane 63 <- its own top
            top[i] = lane_from_below(b_dn, xn);              // lane k <- top of lane k - 1; lane 0 <- what came down to it
            bot[i] = lane0 ? yn : b_dn;                      // position 0 stays
        }
    };
    constexpr int PF = 8;                                  // rounds of rotations requested ahead
    float2 nx[PF];
    int t = 0;
    if (n_rounds >= PF) {
#pragma unroll
        for (int i = 0; i < PF; ++i) nx[i] = rot_u[(size_t)i * 64];
        for (; t + 2 * PF <= n_rounds; t += PF) {
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                const float2 p = nx[i];
                nx[i] = rot_u[(size_t)(t + PF + i) * 64];
                apply(p);
            }
        }
#pragma unroll
        for (int i = 0; i < PF; ++i) apply(nx[i]);
        t += PF;
    }
    for (; t < n_rounds; ++t) apply(rot_u[(size_t)t * 64]);
#pragma unroll
    for (int i = 0; i < EIGV_ROWS; ++i)
        *(float2*)(R_out + (size_t)u * D * D + (size_t)(row0 + i) * D + 2 * lane) =
            lane == 0 ? make_float2(bot[i], top[i]) : make_float2(top[i], bot[i]);
}

// R_r = R[:, keep] and delta_mu = mu - R_r R_r^T mu (Alg. 1 step 14 and 16), one work-group per matrix;
// R is staged in LDS (row stride 129) so that the column reads below do not go to memory one by one.
constexpr int EIGF_LD = D + 1;
constexpr int EIGF_THREADS = 1024, EIGF_PARTS = EIGF_THREADS / D;
constexpr size_t EIGF_LDS_BYTES = (size_t)(D * EIGF_LD + EIGF_PARTS * D + 2 * D) * sizeof(float) + D * sizeof(int);
__global__ __launch_bounds__(EIGF_THREADS) void eig_finish(int r, const float* __restrict__ R,
                                                           const int32_t* __restrict__ keep_idx,
                                                           const float* __restrict__ mu_in, float* __restrict__ Rr_out,
                                                           float* __restrict__ dmu_out)
{
    extern __shared__ float fsm[];
    float* Vs = fsm;                          // [128][129]
    float* part = Vs + D * EIGF_LD;           // [parts][128] partial sums
    float* sw = part + EIGF_PARTS * D;        // [128] R_r^T mu
    float* smu = sw + D;                      // [128]
    int* skeep = (int*)(smu + D);             // [128]
    const int u = blockIdx.x, tid = threadIdx.x;
    const float* V = R + (size_t)u * D * D;
    for (int idx = tid; idx < D * D / 4; idx += EIGF_THREADS) {
        const float4 v = *(const float4*)(V + 4 * idx);
        float* d = Vs + (idx >> 5) * EIGF_LD + 4 * (idx & 31);
        d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
    }
    if (tid < D) smu[tid] = mu_in[(size_t)u * D + tid];
    if (tid < r) skeep[tid] = min(max(keep_idx[(size_t)u * r + tid], 0), D - 1);
    __syncthreads();
    for (int idx = tid; idx < D * r; idx += EIGF_THREADS) {
        int c = idx / r, j = idx - c * r;
        Rr_out[(size_t)u * D * r + idx] = Vs[c * EIGF_LD + skeep[j]];
    }
    const int pt = tid >> 7, x = tid & (D - 1);
    {                                          // w_j = sum_c V[c][keep_j] mu[c], the rows in EIGF_PARTS ranges
        float w = 0.f;
        if (x < r) {
            const int col = skeep[x];
            constexpr int RP = D / EIGF_PARTS;
            for (int c = RP * pt; c < RP * pt + RP; ++c) w = fmaf(Vs[c * EIGF_LD + col], smu[c], w);
        }
        part[pt * D + x] = w;
    }
    __syncthreads();
    if (tid < r) {
        float w = 0.f;
#pragma unroll
        for (int k = 0; k < EIGF_PARTS; ++k) w += part[k * D + tid];
        sw[tid] = w;
    }
    __syncthreads();
    {                                          // delta_mu[c] = mu[c] - sum_j V[c][keep_j] w_j, the kept columns in ranges
        float pr = 0.f;
        const int per = (r + EIGF_PARTS - 1) / EIGF_PARTS, j0 = min(pt * per, r), j1 = min(j0 + per, r);
        for (int j = j0; j < j1; ++j) pr = fmaf(Vs[x * EIGF_LD + skeep[j]], sw[j], pr);
        part[pt * D + x] = pr;
    }
    __syncthreads();
    if (tid < D) {
        float pr = 0.f;
#pragma unroll
        for (int k = 0; k < EIGF_PARTS; ++k) pr += part[k * D + tid];
        dmu_out[(size_t)u * D + tid] = smu[tid] - pr;
    }
}

__global__ __launch_bounds__(256) void gather_rotation_kernel(int r, const float* __restrict__ R,
                                                              const int32_t* __restrict__ keep_idx,
                                                              float* __restrict__ Rr)
{
    const int u = blockIdx.x;
    for (int idx = threadIdx.x; idx < D * r; idx += 256) {
        int c = idx / r, j = idx - c * r;
        int col = keep_idx[(size_t)u * r + j];
        col = min(max(col, 0), D - 1);
        Rr[(size_t)u * D * r + idx] = R[(size_t)u * D * D + c * D + col];
    }
}

// ---------------------------------------------------------------------------
int cov_chunk_tokens(int dtype, bool mfma) { return (mfma && dtype == 1) ? COVM_CHUNK : COV_CHUNK; }

hipError_t launch_cov_partial(int dtype, bool mfma, const RowsDev& rows, int B, int Hkv, int n_chunks,
                              float* part_S, float* part_sum, hipStream_t st)
{
    dim3 grid(n_chunks, Hkv, B);
    if (mfma && dtype == 1) {
        hipError_t e = allow_dynamic_lds(rows.tok_idx ? (const void*)cov_partial_mfma<true>
                                                      : (const void*)cov_partial_mfma<false>, COVM_LDS_BYTES);
        if (e != hipSuccess) return e;
        if (rows.tok_idx)
            hipLaunchKernelGGL(cov_partial_mfma<true>, grid, dim3(256), COVM_LDS_BYTES, st, rows, Hkv, n_chunks, part_S,
                               part_sum);
        else
            hipLaunchKernelGGL(cov_partial_mfma<false>, grid, dim3(256), COVM_LDS_BYTES, st, rows, Hkv, n_chunks,
                               part_S, part_sum);
        return hipGetLastError();
    }
    if (dtype == 0)
        hipLaunchKernelGGL(cov_partial_generic<float>, grid, dim3(256), 0, st, rows, Hkv, n_chunks, part_S, part_sum);
    else
        hipLaunchKernelGGL(cov_partial_generic<bf16_t>, grid, dim3(256), 0, st, rows, Hkv, n_chunks, part_S, part_sum);
    return hipGetLastError();
}

hipError_t launch_cov_finalize(const RowsDev& rows, int B, int Hkv, int n_chunks, bool center, bool tiled,
                               const float* part_S, const float* part_sum, float* cov, float* mu,
                               hipStream_t st)
{
    if (tiled)
        hipLaunchKernelGGL(cov_finalize_tiled, dim3(40, B * Hkv), dim3(256), 0, st, rows, Hkv, n_chunks,
                           center ? 1 : 0, part_S, part_sum, cov, mu);
    else
        hipLaunchKernelGGL(cov_finalize, dim3(8, B * Hkv), dim3(256), 0, st, rows, Hkv, n_chunks, center ? 1 : 0,
                           part_S, part_sum, cov, mu);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Cholesky-based subspace iteration (Alg. 1 steps 6-13, App. E), one work-group
// per (b, h_kv), the whole T-step loop in one launch (the paper's four kernels
// per iteration exist to cut dispatch count; here there is nothing to dispatch).
// All arithmetic is fp64: the Gram matrix of C_q V has the squared condition of
// C_q's leading block, which fp32 cannot factor reliably; the fp64 vector rate of
// this part is half its fp32 rate, which does not matter at this size.
//
// LDS (doubles): W [128][ks] (the basis, row stride ks = k padded so that ks % 32 == 8:
// eight consecutive rows then start 16 banks apart), G packed lower triangle
// [k(k+1)/2], per-column pivots, sigma, a k-vector, the published pivot row (x2).
//
// One iteration:
//   W <- diag(sigma) C diag(sigma) W   register-tiled: thread = 4 rows x RJ columns
//                                      (adjacent pairs), C read from global/L2 as
//                                      float4 broadcasts, in place via registers;
//   G <- W^T W (lower, 2x2 blocks), rho = eps tr(G) / k added to the diagonal;
//   right-looking elimination of the stacked matrix [W; G], one barrier per column,
//   with the rows held in registers (see elim_step): step j uses row j of G (final
//   since step j-1) to update columns > j,
//       G[a][b] -= G[a][j] G[j][b] / G[j][j],   W[i][b] -= W[i][j] G[j][b] / G[j][j];
//   this is the Cholesky factorisation and the solve V L^{-T} at once, with the
//   square roots deferred: V[i][j] = W[i][j] / sqrt(pivot_j) at the end.
constexpr int SUB_THREADS = 1024;
constexpr int SUB_MAX_K = 104;

__host__ __device__ inline int sub_row_stride(int k)
{
    int ks = k;
    while (ks % 32 != 8) ++ks;
    return ks;
}
__host__ __device__ inline size_t sub_lds_bytes(int k)
{
    const size_t kpad = 16 * (size_t)((k + 15) / 16) + 8;      // one published pivot row: 4 parts x (columns / 4 + 2)
    return sizeof(double) * ((size_t)D * sub_row_stride(k) + (size_t)k * (k + 1) / 2 + 2 * (size_t)(k + 4) + D + 2 * kpad + 2);
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// 1 / g for g > 0 in double: hardware estimate + two Newton steps (the full IEEE division
// sequence is four times as long and sits on the critical path of every elimination step)
__device__ __forceinline__ double fast_rcp_f64(double g)
{
    double r = __builtin_amdgcn_rcp(g);
    double e = fma(-g, r, 1.0);
    r = fma(r, e, r);
    e = fma(-g, r, 1.0);
    return fma(r, e, r);
}

// Two doubles as one 16-byte LDS access: a true vector type keeps the access whole (the struct double2 is loaded
// member by member, and the pair then comes back as a two-address 8-byte read, which takes almost twice as long).
typedef double f64x2 __attribute__((ext_vector_type(2)));

// value of lane (quad base + PJ) for every lane of the quad
template <int PJ>
__device__ __forceinline__ double quad_bcast(double v)
{
    constexpr int ctrl = PJ | (PJ << 2) | (PJ << 4) | (PJ << 6);       // DPP quad_perm [PJ, PJ, PJ, PJ]
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_mov_dpp(lo, ctrl, 0xf, 0xf, true);
    hi = __builtin_amdgcn_mov_dpp(hi, ctrl, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

// Right-looking elimination of the stacked matrix [W; G] with the rows in registers: thread
// (row, part) holds x[c] = element (row, part + 4 c); rows 0..127 are W, rows 128.. are G (k
// padded to a multiple of 4 with an identity block, so that every step exists).  Step
// j = 4 CJ + PJ: the four owners of stack row 128 + j (= row j of G, final since step j-1)
// publish it scaled by 1 / G[j][j] (the raw pivot goes to slot j), one barrier, then every
// thread subtracts (its own column-j element) x (the published row) from its columns > j.
// The code is straight-line per block of four steps; a pivot that is not positive is only
// recorded, the remaining steps then run on meaningless numbers and the caller discards the
// result (early exits here made the register allocator spill the whole row).
// The published row is laid out by part: element (part, c) = column part + 4 c at rb[part * (NCOL + 2) + c],
// so that a thread's columns are consecutive doubles and two of them come with one 16-byte LDS read
// (the LDS pipeline issues about one wave-wide instruction per five cycles whatever its width, and a
// step is little else than these reads); the stride NCOL + 2 keeps the four parts of a wave in
// different banks and every even c 16-byte aligned.
template <int NCOL, int CJ, int PJ>
__device__ __forceinline__ void elim_step(double (&x)[NCOL], double* __restrict__ rb, double* __restrict__ piv,
                                          int row, int part, int tid, bool& bad)
{
    constexpr int j = 4 * CJ + PJ, RS = NCOL + 2;
    double* rbp = rb + part * RS;
    if (row == D + j) {
        const double gjj = quad_bcast<PJ>(x[CJ]);
        const double rinv = fast_rcp_f64(gjj);
        if (part == PJ) rbp[CJ] = gjj;
        else if (part > PJ) rbp[CJ] = x[CJ] * rinv;
#pragma unroll
        for (int c = CJ + 1; c < NCOL; ++c) rbp[c] = x[c] * rinv;
    }
    __syncthreads();
    // The wave that holds stack row 128 + j + 1 publishes next: its reads, its update and the reciprocal are the
    // dependent chain between this barrier and the next one, so it issues ahead of the others.
    if (__builtin_amdgcn_readfirstlane(tid >> 6) == ((D + j + 1) >> 4)) __builtin_amdgcn_s_setprio(3);
    else __builtin_amdgcn_s_setprio(0);
    const double gjj = rb[PJ * RS + CJ];
    bad = bad || !(gjj > 0.0);
    if (tid == 0) piv[j] = gjj;
    const double f = -quad_bcast<PJ>(x[CJ]);
    if (part > PJ) x[CJ] = fma(f, rbp[CJ], x[CJ]);
    constexpr int c0 = CJ + 1, c1 = (c0 + 1) & ~1;          // c1: first even column index from c0 on
    if constexpr ((c0 & 1) != 0 && c0 < NCOL) x[c0] = fma(f, rbp[c0], x[c0]);
#pragma unroll
    for (int c = c1; c + 1 < NCOL; c += 2) {
        const f64x2 v = *(const f64x2*)(rbp + c);
        x[c] = fma(f, v.x, x[c]);
        x[c + 1] = fma(f, v.y, x[c + 1]);
    }
}

// Blocks CJ, CJ + 1, ... while they exist (4 CJ < kp4, uniform); nested so that the register
// values only merge once, after the last block.
template <int NCOL, int CJ>
__device__ __forceinline__ void elim_block(double (&x)[NCOL], double* __restrict__ rowbuf2, double* __restrict__ piv,
                                           int kp4, int kpad, int row, int part, int tid, bool& bad)
{
    if constexpr (CJ < NCOL) {
        if (4 * CJ < kp4) {
            elim_step<NCOL, CJ, 0>(x, rowbuf2, piv, row, part, tid, bad);
            elim_step<NCOL, CJ, 1>(x, rowbuf2 + kpad, piv, row, part, tid, bad);
            elim_step<NCOL, CJ, 2>(x, rowbuf2, piv, row, part, tid, bad);
            elim_step<NCOL, CJ, 3>(x, rowbuf2 + kpad, piv, row, part, tid, bad);
            elim_block<NCOL, CJ + 1>(x, rowbuf2, piv, kp4, kpad, row, part, tid, bad);
        }
    }
}

template <int KB>
__global__ __launch_bounds__(SUB_THREADS) void subspace_iter(const float* __restrict__ cov,
                                                             const float* __restrict__ sigma,
                                                             const float* __restrict__ mu,
                                                             const float* __restrict__ V0, int k, int T,
                                                             double eps, float* __restrict__ Rr,
                                                             float* __restrict__ dmu, int32_t* __restrict__ status)
{
    extern __shared__ __attribute__((aligned(16))) double sub_lds[];
    const int ks = sub_row_stride(k);
    double* W = sub_lds;                                  // [D][ks]
    double* G = W + (size_t)D * ks;                       // packed lower triangle
    double* piv = G + (size_t)k * (k + 1) / 2;            // [k + 4] (k padded to a multiple of 4)
    double* tv = piv + k + 4;                             // [k + 4]
    double* sig = tv + k + 4;                             // [D]
    double* rowbuf2 = sig + D;                            // [2][kpad]: the published pivot row, double-buffered
    rowbuf2 += ((uintptr_t)rowbuf2 >> 3) & 1;             // 16-byte aligned (the packed triangle has k (k + 1) / 2 doubles)
    constexpr int RJ = (KB + 1) / 2;                      // GEMM columns per thread (32 apart)
    constexpr int NCOL = 4 * KB;                          // elimination: columns per thread (4 apart)
    const int kpad = 4 * (NCOL + 2);                      // one published row: [part][NCOL + 2]

    const int u = blockIdx.x, tid0 = threadIdx.x, tid = tid0;
    const float* C = cov + (size_t)u * D * D;
    const bool weighted = sigma != nullptr;

    for (int idx = tid; idx < D * k; idx += SUB_THREADS) {
        const int i = idx / k, j = idx - i * k;
        W[i * ks + j] = (double)V0[(size_t)u * D * k + idx];
    }
    for (int idx = tid; idx < D * (ks - k); idx += SUB_THREADS) {     // padding columns: keep them finite
        const int i = idx / (ks - k), j = k + idx - i * (ks - k);
        W[i * ks + j] = 0.0;
    }
    if (tid < D) sig[tid] = weighted ? (double)sigma[(size_t)u * D + tid] : 1.0;
    __syncthreads();

    int fail = 0;
    for (int t = 0; t < T; ++t) {
        // The thread index is made opaque once per iteration and per phase: otherwise every address and
        // mask derived from it (a few dozen) is computed before the loop, held in registers through all
        // phases, and spilled.
        int tid = tid0;
        asm volatile("" : "+v"(tid));
        int ib = tid >> 5, jb = tid & 31;                  // GEMM tile: rows 4 ib .. +3, columns gemm_col(c)
        // ---- W <- C_q W ----
        if (weighted) {
            for (int idx = tid; idx < D * k; idx += SUB_THREADS) {
                const int i = idx / k, j = idx - i * k;
                W[i * ks + j] *= sig[i];
            }
            __syncthreads();
        }
        double acc[4][RJ];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < RJ; ++c) acc[r][c] = 0.0;
        // a thread's columns come in adjacent pairs, 64 c' + 2 jb and + 1 (c' = 0 .. RJ / 2 - 1), so that a pair is
        // one 16-byte LDS read, plus the single column 64 (RJ / 2) + jb when RJ is odd; reads of surplus threads
        // are clamped onto the end of the padded row, and they store nothing
        auto gemm_col = [&](int c) { return c < (RJ & ~1) ? 64 * (c >> 1) + 2 * jb + (c & 1) : 64 * (RJ >> 1) + jb; };
#pragma unroll 2
        for (int m0 = 0; m0 < D; m0 += 4) {          // bounded unroll: a full unroll hoists 512 registers of C
            float4 c4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) c4[r] = *(const float4*)(C + (size_t)(4 * ib + r) * D + m0);
#pragma unroll
            for (int mm = 0; mm < 4; ++mm) {
                double wv[RJ];
                const double* wrow = W + (m0 + mm) * ks;
#pragma unroll
                for (int c = 0; c + 1 < RJ; c += 2) {
                    const f64x2 w2 = *(const f64x2*)(wrow + min(gemm_col(c), (ks - 2) & ~1));
                    wv[c] = w2.x;
                    wv[c + 1] = w2.y;
                }
                if (RJ & 1) wv[RJ - 1] = wrow[min(gemm_col(RJ - 1), ks - 1)];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float cf = mm == 0 ? c4[r].x : mm == 1 ? c4[r].y : mm == 2 ? c4[r].z : c4[r].w;
                    const double cd = (double)cf;
#pragma unroll
                    for (int c = 0; c < RJ; ++c) acc[r][c] = fma(cd, wv[c], acc[r][c]);
                }
            }
        }
        __syncthreads();                                   // every thread has read the old basis
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < RJ; ++c)
                if (gemm_col(c) < k) W[(4 * ib + r) * ks + gemm_col(c)] = acc[r][c] * sig[4 * ib + r];
        __syncthreads();

        // ---- G <- W^T W (lower triangle, 2 x 2 blocks) ----
        const int K2 = (k + 1) >> 1, nblk = K2 * (K2 + 1) / 2;
        for (int blk = tid; blk < nblk; blk += SUB_THREADS) {
            int pa = (int)((sqrtf(8.f * (float)blk + 1.f) - 1.f) * 0.5f);
            while (pa * (pa + 1) / 2 > blk) --pa;
            while ((pa + 1) * (pa + 2) / 2 <= blk) ++pa;
            const int pb = blk - pa * (pa + 1) / 2;
            double s00 = 0.0, s01 = 0.0, s10 = 0.0, s11 = 0.0;
            for (int i = 0; i < D; ++i) {
                const f64x2 wa = *(const f64x2*)(W + i * ks + 2 * pa);
                const f64x2 wb = *(const f64x2*)(W + i * ks + 2 * pb);
                s00 = fma(wa.x, wb.x, s00);
                s01 = fma(wa.x, wb.y, s01);
                s10 = fma(wa.y, wb.x, s10);
                s11 = fma(wa.y, wb.y, s11);
            }
            const int a0 = 2 * pa, a1 = a0 + 1, b0 = 2 * pb, b1 = b0 + 1;
            G[a0 * (a0 + 1) / 2 + b0] = s00;
            if (pa > pb) G[a0 * (a0 + 1) / 2 + b1] = s01;
            if (a1 < k) {
                G[a1 * (a1 + 1) / 2 + b0] = s10;
                G[a1 * (a1 + 1) / 2 + b1] = s11;          // b1 <= a1 < k
            }
        }
        __syncthreads();
        if (tid < 64) {                                    // rho = eps tr(G) / k
            double tr = 0.0;
            for (int a = tid; a < k; a += 64) tr += G[a * (a + 1) / 2 + a];
            tr = wave_sum_f64(tr);
            const double rho = eps * tr / (double)k;
            for (int a = tid; a < k; a += 64) G[a * (a + 1) / 2 + a] += rho;
        }
        __syncthreads();

        // ---- elimination of [W; G] with the rows in registers, one barrier per column ----
        {
            asm volatile("" : "+v"(tid));
            int row = tid >> 2, part = tid & 3;            // stacked row: W rows 0..127, then G rows
            const int kp4 = (k + 3) & ~3;                  // G padded with an identity block to a multiple of 4
            double x[NCOL];
#pragma unroll
            for (int c = 0; c < NCOL; ++c) {
                const int bcol = part + 4 * c;
                double v = 0.0;
                if (row < D) {
                    if (bcol < k) v = W[row * ks + bcol];
                } else if (row < D + kp4) {
                    const int a = row - D, hi = max(a, bcol), lo = min(a, bcol);
                    if (hi < k) v = G[hi * (hi + 1) / 2 + lo];
                    else if (a == bcol) v = 1.0;
                }
                x[c] = v;
            }
            bool bad = false;
            elim_block<NCOL, 0>(x, rowbuf2, piv, kp4, kpad, row, part, tid, bad);
            __builtin_amdgcn_s_setprio(0);
            if (bad) { fail = t + 1; break; }              // uniform: every thread saw the same pivots
            __syncthreads();                               // piv complete
            if (tid < k) tv[tid] = 1.0 / sqrt(piv[tid]);
            __syncthreads();
            asm volatile("" : "+v"(row), "+v"(part), "+v"(tid));      // recompute the column numbers: keeping them costs NCOL registers
            if (row < D) {
#pragma unroll
                for (int c = 0; c < NCOL; ++c) {
                    const int bcol = part + 4 * c;
                    if (bcol < k) W[row * ks + bcol] = x[c] * tv[bcol];
                }
            }
            __syncthreads();
        }
    }

    // ---- outputs: R_k = V, delta_mu = mu - V V^T mu (Alg. 1 steps 14, 16) ----
    if (tid == 0 && status) status[u] = fail;
    for (int idx = tid; idx < D * k; idx += SUB_THREADS) {
        const int i = idx / k, j = idx - i * k;
        Rr[(size_t)u * D * k + idx] = (float)W[i * ks + j];
    }
    if (tid < k) {
        double a = 0.0;
        for (int i = 0; i < D; ++i) a = fma(W[i * ks + tid], (double)mu[(size_t)u * D + i], a);
        tv[tid] = a;
    }
    __syncthreads();
    if (tid < D) {
        double a = (double)mu[(size_t)u * D + tid];
        for (int j = 0; j < k; ++j) a = fma(-W[tid * ks + j], tv[j], a);
        dmu[(size_t)u * D + tid] = (float)a;
    }
}

// ---------------------------------------------------------------------------
// Alg. 1 step 4: sigma_j = ||(Q_W)_{:,j}||_2 over the window of recent queries, pooled
// over the G query heads that share a KV head.  One block per (b, h_kv), thread =
// channel; rows are coalesced 256- or 512-byte reads.
template <typename T>
__global__ __launch_bounds__(128) void sigma_window_kernel(const T* __restrict__ qw, int64_t sb, int64_t sh,
                                                           int64_t sw, int Hq, int Hkv, int W,
                                                           float* __restrict__ sigma)
{
    const int u = blockIdx.x, b = u / Hkv, hk = u % Hkv, G = Hq / Hkv, c = threadIdx.x;
    float a0 = 0.f, a1 = 0.f;
    for (int g = 0; g < G; ++g) {
        const T* base = qw + (int64_t)b * sb + (int64_t)(hk * G + g) * sh + c;
        int w = 0;
        for (; w + 2 <= W; w += 2) {
            const float x0 = ld_elem(base + (int64_t)w * sw), x1 = ld_elem(base + (int64_t)(w + 1) * sw);
            a0 = fmaf(x0, x0, a0);
            a1 = fmaf(x1, x1, a1);
        }
        if (w < W) {
            const float x0 = ld_elem(base + (int64_t)w * sw);
            a0 = fmaf(x0, x0, a0);
        }
    }
    sigma[(size_t)u * D + c] = sqrtf(a0 + a1);
}

hipError_t launch_eig(int U, const float* cov, const float* sigma, const float* mu, int r, float* R,
                      float* lam, uint8_t* mask, int32_t* keep_idx, float* Rr, float* dmu, int32_t* sweeps,
                      void* rotations, int32_t* sweeps_ws, hipStream_t st)
{
    // Few matrices: one compute unit each iterates on A and the whole chip replays the rotations on V.
    // From three quarters of a chip of matrices on, the replay (throughput-bound) costs more than carrying V along.
    hipError_t e;
    if (U >= EIG_FUSE_V_FROM) {
        e = allow_dynamic_lds((const void*)eig_jacobi_rotations<true>, EIG_LDS_BYTES);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(eig_jacobi_rotations<true>, dim3(U), dim3(EIG_THREADS), EIG_LDS_BYTES, st, cov, sigma, r, lam,
                           mask, keep_idx, (float2*)rotations, sweeps_ws, sweeps, R);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    } else {
        e = allow_dynamic_lds((const void*)eig_jacobi_rotations<false>, EIG_LDS_BYTES);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(eig_jacobi_rotations<false>, dim3(U), dim3(EIG_THREADS), EIG_LDS_BYTES, st, cov, sigma, r, lam,
                           mask, keep_idx, (float2*)rotations, sweeps_ws, sweeps, R);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(eig_apply_rotations, dim3(D / (4 * EIGV_ROWS), U), dim3(256), 0, st, (const float2*)rotations,
                           sweeps_ws, R);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    e = allow_dynamic_lds((const void*)eig_finish, EIGF_LDS_BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(eig_finish, dim3(U), dim3(EIGF_THREADS), EIGF_LDS_BYTES, st, r, R, keep_idx, mu, Rr, dmu);
    return hipGetLastError();
}

int subspace_max_keep() { return SUB_MAX_K; }

hipError_t launch_subspace(int U, const float* cov, const float* sigma, const float* mu, const float* V0, int k,
                           int T, double eps, float* Rr, float* dmu, int32_t* status, hipStream_t st)
{
    if (k < 1 || k > SUB_MAX_K) return hipErrorInvalidValue;
    const size_t lds = sub_lds_bytes(k);
    const int kb = (k + 15) / 16;
#define RK_SUB(KBV)                                                                                          \
    case KBV: {                                                                                              \
        hipError_t e = allow_dynamic_lds((const void*)subspace_iter<KBV>, sub_lds_bytes(SUB_MAX_K));         \
        if (e != hipSuccess) return e;                                                                       \
        hipLaunchKernelGGL(subspace_iter<KBV>, dim3(U), dim3(SUB_THREADS), lds, st, cov, sigma, mu, V0, k, T, eps, \
                           Rr, dmu, status);                                                                 \
        break;                                                                                               \
    }
    switch (kb) {
        RK_SUB(1) RK_SUB(2) RK_SUB(3) RK_SUB(4) RK_SUB(5) RK_SUB(6) RK_SUB(7)
        default: return hipErrorInvalidValue;
    }
#undef RK_SUB
    return hipGetLastError();
}

hipError_t launch_sigma_window(int dtype, const void* qw, int64_t sb, int64_t sh, int64_t sw, int B, int Hq,
                               int Hkv, int W, float* sigma, hipStream_t st)
{
    if (dtype == 0)
        hipLaunchKernelGGL(sigma_window_kernel<float>, dim3(B * Hkv), dim3(128), 0, st, (const float*)qw, sb, sh, sw,
                           Hq, Hkv, W, sigma);
    else
        hipLaunchKernelGGL(sigma_window_kernel<bf16_t>, dim3(B * Hkv), dim3(128), 0, st, (const bf16_t*)qw, sb, sh,
                           sw, Hq, Hkv, W, sigma);
    return hipGetLastError();
}

hipError_t launch_gather_rotation(int U, int r, const float* R, const int32_t* keep_idx, float* Rr,
                                  hipStream_t st)
{
    hipLaunchKernelGGL(gather_rotation_kernel, dim3(U), dim3(256), 0, st, r, R, keep_idx, Rr);
    return hipGetLastError();
}

}  // namespace rk
