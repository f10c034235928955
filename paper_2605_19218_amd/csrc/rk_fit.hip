// Prefill-side rotation construction (Alg. 1 of the RotateK paper, with the full
// eigendecomposition of Sec. 3.2 "Query-Weighted PCA" as the solver):
//   cov_partial_*   : per token chunk, S = sum x x^T and column sums   (Alg. 1 steps 1-3)
//   cov_finalize    : mu, C = S - n mu mu^T, reduced over chunks in fp64
//   eig_jacobi      : C_q = (sigma sigma^T) .* C (step 5 / Eq. 4), all eigenpairs by
//                     parallel two-sided Jacobi resident in LDS, then the keep-mask,
//                     R_r and delta_mu (step 15)
#include "rk_kernels.hpp"

namespace rk {

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
    if (tid < D) {
        double s = 0.0;
        for (int ch = 0; ch < n_chunks; ++ch) s += (double)part_sum[((size_t)u * n_chunks + ch) * D + tid];
        double m = n_b > 0 ? s / (double)n_b : 0.0;
        smu[tid] = m;
        if (blockIdx.x == 0) mu_out[(size_t)u * D + tid] = (float)m;
    }
    __syncthreads();
    const int j = tid & (D - 1);
    for (int ri = 0; ri < 8; ++ri) {
        int i = blockIdx.x * 16 + ri * 2 + (tid >> 7);
        double s = 0.0;
        for (int ch = 0; ch < n_chunks; ++ch)
            s += (double)part_S[((size_t)u * n_chunks + ch) * (D * D) + i * D + j];
        if (center) s -= (double)n_b * (smu[i] * smu[j]);
        cov[(size_t)u * D * D + i * D + j] = (float)s;
    }
}

// ---------------------------------------------------------------------------
// Batched symmetric eigensolver: one 1024-thread work-group per 128x128 matrix,
// A and the accumulated eigenvectors V both resident in LDS (2 x 64 KB).
// Parallel two-sided Jacobi with the round-robin ("circle") ordering: a sweep is
// 127 rounds of 64 disjoint (p, q) pairs.  In a round, thread (k, k') owns the
// 2x2 block A[{p_k,q_k}][{p_k',q_k'}] and applies J_k^T (.) J_k' to it, so row and
// column rotations fuse into one pass with no read/write overlap between threads.
// Columns never move: eigenvalue c is the final A[c][c] and its vector is V[:, c].
constexpr int EIG_THREADS = 1024;
constexpr int EIG_MAX_SWEEPS = 20;
constexpr size_t EIG_LDS_BYTES = (size_t)(2 * D * D + 3 * 64 + 2 * D + 64) * sizeof(float) + D * sizeof(int);

__device__ __forceinline__ void rr_pair(int round, int k, int& p, int& q) {
    // circle method on n-1 = 127 rotating players, player 127 fixed
    if (k == 0) { p = D - 1; q = round; }
    else {
        p = round + k;       if (p >= D - 1) p -= D - 1;
        q = round - k;       if (q < 0) q += D - 1;
    }
}

__global__ __launch_bounds__(EIG_THREADS) void eig_jacobi(const float* __restrict__ cov,
                                                          const float* __restrict__ sigma,
                                                          const float* __restrict__ mu_in, int r,
                                                          float* __restrict__ R_out, float* __restrict__ lam_out,
                                                          uint8_t* __restrict__ mask_out,
                                                          int32_t* __restrict__ keep_out,
                                                          float* __restrict__ Rr_out, float* __restrict__ dmu_out)
{
    extern __shared__ float sm[];
    float* A = sm;                        // [128][128]
    float* V = A + D * D;                 // [128][128]
    float* rs = V + D * D;                // [64] sin
    float* rtau = rs + 64;                // [64] sin / (1 + cos)
    float* rt = rtau + 64;                // [64] tan
    float* slam = rt + 64;                // [128]
    float* sw = slam + D;                 // [128] scratch (R_r^T mu)
    float* red = sw + D;                  // [64] reduction scratch
    int* skeep = (int*)(red + 64);        // [128]

    const int u = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;   // 16 waves
    const float* C = cov + (size_t)u * D * D;
    const float* sg = sigma ? sigma + (size_t)u * D : nullptr;

    // load C_q = sigma_i sigma_j C_ij, V = I, and ||C_q||_F^2
    float nrm = 0.f;
    for (int idx = tid; idx < D * D; idx += EIG_THREADS) {
        int i = idx >> 7, j = idx & 127;
        float v = C[idx];
        if (sg) v *= sg[i] * sg[j];
        A[idx] = v;
        V[idx] = (i == j) ? 1.f : 0.f;
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

    for (int sweep = 0; sweep < EIG_MAX_SWEEPS; ++sweep) {
        // off-diagonal norm
        float off = 0.f;
        for (int idx = tid; idx < D * D; idx += EIG_THREADS) {
            int i = idx >> 7, j = idx & 127;
            float v = A[idx];
            if (i != j) off = fmaf(v, v, off);
        }
        off = wave_sum(off);
        if (lane == 0) red[16 + wave] = off;
        __syncthreads();
        float off2 = 0.f;
        for (int w = 0; w < 16; ++w) off2 += red[16 + w];
        __syncthreads();
        if (!(off2 > tol2)) break;      // uniform across the block

        for (int round = 0; round < D - 1; ++round) {
            if (tid < 64) {
                int p, q;
                rr_pair(round, tid, p, q);
                float app = A[p * D + p], aqq = A[q * D + q], apq = A[p * D + q];
                // Rotations are applied as x' = x - s (y + tau x), y' = y + s (x - tau y) with
                // tau = s / (1 + c): 1 - c is then carried to relative precision, so small
                // angles (c rounding to 1) do not inflate the column norms of V.
                float s = 0.f, tau = 0.f, t = 0.f;
                if (fabsf(apq) > thr_skip) {
                    float th = (aqq - app) / (2.f * apq);
                    t = copysignf(1.f, th) / (fabsf(th) + sqrtf(fmaf(th, th, 1.f)));
                    float c = 1.f / sqrtf(fmaf(t, t, 1.f));
                    s = t * c;
                    tau = s / (1.f + c);
                }
                rs[tid] = s;
                rtau[tid] = tau;
                rt[tid] = t;
            }
            __syncthreads();
            int p2, q2;
            rr_pair(round, lane, p2, q2);
            const float s2 = rs[lane], tau2 = rtau[lane];
            // A <- J^T A J : 64 x 64 blocks, wave handles pair-rows k = wave + 16 it
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                int k = wave + 16 * it;
                int p, q;
                rr_pair(round, k, p, q);
                float s1 = rs[k], tau1 = rtau[k];
                float a00 = A[p * D + p2], a01 = A[p * D + q2];
                float a10 = A[q * D + p2], a11 = A[q * D + q2];
                // rows p, q : J^T from the left
                float b00 = a00 - s1 * (a10 + tau1 * a00), b01 = a01 - s1 * (a11 + tau1 * a01);
                float b10 = a10 + s1 * (a00 - tau1 * a10), b11 = a11 + s1 * (a01 - tau1 * a11);
                // columns p', q' : J from the right
                float e00 = b00 - s2 * (b01 + tau2 * b00), e01 = b01 + s2 * (b00 - tau2 * b01);
                float e10 = b10 - s2 * (b11 + tau2 * b10), e11 = b11 + s2 * (b10 - tau2 * b11);
                if (k == lane) {           // the pair's own block: annihilated exactly
                    float t = rt[k];
                    e00 = a00 - t * a01;
                    e11 = a11 + t * a01;
                    e01 = 0.f;
                    e10 = 0.f;
                }
                A[p * D + p2] = e00; A[p * D + q2] = e01;
                A[q * D + p2] = e10; A[q * D + q2] = e11;
            }
            // V <- V J : 128 rows x 64 pairs
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                int i = wave + 16 * it;
                float v0 = V[i * D + p2], v1 = V[i * D + q2];
                V[i * D + p2] = v0 - s2 * (v1 + tau2 * v0);
                V[i * D + q2] = v1 + s2 * (v0 - tau2 * v1);
            }
            __syncthreads();
        }
    }

    // ---- eigenvalues, rank, mask (integer logic), R, R_r, delta_mu -----------
    if (tid < D) slam[tid] = A[tid * D + tid];
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
        if (rank < r) { skeep[rank] = tid; keep_out[(size_t)u * r + rank] = tid; }
    }
    __syncthreads();
    for (int idx = tid; idx < D * D; idx += EIG_THREADS) R_out[(size_t)u * D * D + idx] = V[idx];
    for (int idx = tid; idx < D * r; idx += EIG_THREADS) {
        int c = idx / r, j = idx - c * r;
        Rr_out[(size_t)u * D * r + idx] = V[c * D + skeep[j]];
    }
    const float* mu = mu_in + (size_t)u * D;
    if (tid < r) {
        int col = skeep[tid];
        float w = 0.f;
        for (int c = 0; c < D; ++c) w = fmaf(V[c * D + col], mu[c], w);
        sw[tid] = w;
    }
    __syncthreads();
    if (tid < D) {
        float pr = 0.f;
        for (int j = 0; j < r; ++j) pr = fmaf(V[tid * D + skeep[j]], sw[j], pr);
        dmu_out[(size_t)u * D + tid] = mu[tid] - pr;
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
hipError_t launch_cov_partial(int dtype, bool mfma, const RowsDev& rows, int B, int Hkv, int n_chunks,
                              float* part_S, float* part_sum, hipStream_t st)
{
    (void)mfma;
    dim3 grid(n_chunks, Hkv, B);
    if (dtype == 0)
        hipLaunchKernelGGL(cov_partial_generic<float>, grid, dim3(256), 0, st, rows, Hkv, n_chunks, part_S, part_sum);
    else
        hipLaunchKernelGGL(cov_partial_generic<bf16_t>, grid, dim3(256), 0, st, rows, Hkv, n_chunks, part_S, part_sum);
    return hipGetLastError();
}

hipError_t launch_cov_finalize(const RowsDev& rows, int B, int Hkv, int n_chunks, bool center,
                               const float* part_S, const float* part_sum, float* cov, float* mu,
                               hipStream_t st)
{
    hipLaunchKernelGGL(cov_finalize, dim3(8, B * Hkv), dim3(256), 0, st, rows, Hkv, n_chunks, center ? 1 : 0,
                       part_S, part_sum, cov, mu);
    return hipGetLastError();
}

hipError_t launch_eig(int U, const float* cov, const float* sigma, const float* mu, int r, float* R,
                      float* lam, uint8_t* mask, int32_t* keep_idx, float* Rr, float* dmu, hipStream_t st)
{
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)eig_jacobi, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)EIG_LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(eig_jacobi, dim3(U), dim3(EIG_THREADS), EIG_LDS_BYTES, st, cov, sigma, mu, r, R, lam,
                       mask, keep_idx, Rr, dmu);
    return hipGetLastError();
}

hipError_t launch_gather_rotation(int U, int r, const float* R, const int32_t* keep_idx, float* Rr,
                                  hipStream_t st)
{
    hipLaunchKernelGGL(gather_rotation_kernel, dim3(U), dim3(256), 0, st, r, R, keep_idx, Rr);
    return hipGetLastError();
}

}  // namespace rk
