// Rotate + gather + pack of the Key cache (Alg. 1 step 14: K~ = K R_k, stored in
// place of K, rounded once to the cache dtype), re-tiling of the Values into the
// decode kernel's fragment-major layout, the frozen-R append of new tokens (the
// rotation is fitted once at the end of prefill and reused, Sec. 3.2 Step (1)),
// and the inverse re-tiling used to inspect a cache.
#include "rk_kernels.hpp"
#include <type_traits>

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
    const int rp = keep_padded(r);
    const T* base = (const T*)rows.data;
    __shared__ float tile[64][D];
    for (int idx = tid; idx < nt * D; idx += 256) {
        int t = idx >> 7, c = idx & 127;
        tile[t][c] = ld_elem(base + rows_offset(rows, b, h, t0 + t) + c);
    }
    __syncthreads();
    const float* Ru = Rr + (size_t)u * D * r;
    T* Ku = Kp + (size_t)u * slab_tokens(cap) * rp;
    for (int o = tid; o < nt * rp; o += 256) {
        int t = o / rp, j = o - t * rp;
        float a = 0.f;
        if (j < r)                                  // channels r .. rp - 1 are the layout's zero padding
            for (int c = 0; c < D; ++c) a = fmaf(tile[t][c], Ru[c * r + j], a);
        st_elem(Ku + kidx(t0 + t, j, rp), a);
    }
}

// ---------------------------------------------------------------------------
// MFMA kernel (bf16; R = r padded to a multiple of 16, columns r .. R - 1 of R_r read as
// zero, which writes the layout's zero padding).  Per wave: D^T[j, token] = R_r^T . K^T
// with v_mfma_f32_16x16x32_bf16; the B operand (lane (g, n): token n, channels
// 32 i + 8 g ..+7) is a plain 16-byte load of a Key row, so Keys go from HBM
// straight into MFMA registers.  R_r is split into bf16 head + remainder
// (two MFMAs) to keep ~fp32 accuracy of the fp32 rotation.  The rows of the A
// operand are permuted so that after output blocks 2i and 2i+1 lane (g, n) holds
// the 8 output channels 32 i + 8 g ..+7 of token n -- one 16-byte piece of the
// packed layout, and consecutive lanes write consecutive pieces.
template <int R, int NP>
struct CompressCfg {
    static constexpr int JB = R / 16;                 // 16-wide output-channel blocks
    static constexpr int NF = R / 32;                 // full 32-channel groups
    static constexpr bool TAIL = (R % 32) != 0;       // one trailing 16-channel block
    static constexpr int TT = 2;                      // 16-token tiles per wave and pass (two passes in flight)
    static constexpr int TOK_PER_PASS = 4 * TT * 16;  // tokens one pass of the 4 waves covers
    static constexpr int PASSES = NP;                  // passes per work-group (amortises the R_r fragment build)
    static constexpr int TOK_PER_BLOCK = PASSES * TOK_PER_PASS;
    static constexpr size_t LDS_BYTES = (size_t)JB * 4 * 2 * 64 * 16;   // A fragments, hi+lo
    // output channel held by A row a of block jb
    __host__ __device__ static constexpr int chan(int jb, int a) {
        return (jb < 2 * NF) ? 32 * (jb >> 1) + 8 * (a >> 2) + 4 * (jb & 1) + (a & 3) : 32 * NF + a;
    }
};

__device__ __forceinline__ uint32_t pack2_bf16(float a, float b) {
    return (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
}

template <int R, bool GATHER, int NP>
__global__ __launch_bounds__(256, 2) void compress_mfma(RowsDev rows, int Hkv, int cap, int r,
                                                     const float* __restrict__ Rr, bf16_t* __restrict__ Kp,
                                                     int32_t* __restrict__ seq_len_out)
{
    typedef CompressCfg<R, NP> Cfg;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16x8* frag = (bf16x8*)smem_raw;       // [JB][4][2][64]

    const int h = blockIdx.y, b = blockIdx.z, u = b * Hkv + h;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, n = lane & 15;
    const int n_b = min(rows_count(rows, b), cap);
    // Work-groups go to the 8 XCDs round-robin by linear index, i.e. by blockIdx.x when the grid's first
    // extent is a multiple of 8: the block number is rotated by head and batch item, so that an XCD
    // does not end up with "block 7 of every sequence" (which only the longest sequences have)
    const int bx = (int)((blockIdx.x + blockIdx.y + blockIdx.z) % gridDim.x);
    if (bx == 0 && h == 0 && tid == 0 && seq_len_out) seq_len_out[b] = n_b;
    const int blk0 = bx * Cfg::TOK_PER_BLOCK;
    if (blk0 >= n_b) return;

    const bf16_t* base = (const bf16_t*)rows.data;
    const int64_t hb = (int64_t)b * rows.sb + (int64_t)h * rows.sh;
    const int32_t* list = GATHER ? rows.tok_idx + rows.tok_off[b] : nullptr;
    bf16_t* Ku = Kp + (size_t)u * slab_tokens(cap) * R;

    // Row numbers of one pass of this wave (token list entries; the token itself without a list).
    // Rows past the end are clamped to the last row (never stored).
    auto load_rows_idx = [&](int (&idx)[Cfg::TT], int w0) {
#pragma unroll
        for (int tt = 0; tt < Cfg::TT; ++tt) {
            const int tok = min(w0 + tt * 16 + n, n_b - 1);
            idx[tt] = GATHER ? list[tok] : tok;
        }
    };
    // Key rows of one pass, straight into B-operand registers.  Every row is read once: non-temporal.
    auto load_keys_at = [&](bf16x8 (&kb)[Cfg::TT][4], const int (&idx)[Cfg::TT]) {
#pragma unroll
        for (int tt = 0; tt < Cfg::TT; ++tt) {
            const bf16_t* row = base + hb + (int64_t)idx[tt] * rows.st;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                kb[tt][i] = __builtin_bit_cast(bf16x8, __builtin_nontemporal_load((const u32x4*)(row + 32 * i + 8 * g)));
        }
    };
    auto load_keys = [&](bf16x8 (&kb)[Cfg::TT][4], int w0) {
        int idx[Cfg::TT];
        load_rows_idx(idx, w0);
        load_keys_at(kb, idx);
    };
    // rotate one pass and store its packed rows
    auto rotate_store = [&](const bf16x8 (&kb)[Cfg::TT][4], int w0, auto all_valid) {
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
            // the fragment reads of one output block at a time: hoisting all of them costs 128 registers
            if (Cfg::JB > 4 && (jb & 1)) __builtin_amdgcn_sched_barrier(0);
        }
        // lane (g, n): blocks 2i, 2i+1 hold channels 32 i + 8 g + (0..3), (4..7) of token w0 + 16 tt + n
#pragma unroll
        for (int tt = 0; tt < Cfg::TT; ++tt) {
            int tok = w0 + tt * 16 + n;
            if (decltype(all_valid)::value || tok < n_b) {
                bf16_t* blk = Ku + (size_t)((w0 >> 4) + tt) * (16 * R);
#pragma unroll
                for (int i = 0; i < Cfg::NF; ++i) {
                    uint4 pk;
                    pk.x = pack2_bf16(acc[tt][2 * i][0], acc[tt][2 * i][1]);
                    pk.y = pack2_bf16(acc[tt][2 * i][2], acc[tt][2 * i][3]);
                    pk.z = pack2_bf16(acc[tt][2 * i + 1][0], acc[tt][2 * i + 1][1]);
                    pk.w = pack2_bf16(acc[tt][2 * i + 1][2], acc[tt][2 * i + 1][3]);
                    nt_store16(blk + (4 * i) * 128 + lane * 8, pk);
                }
                if (Cfg::TAIL) {
                    uint2 pk;
                    pk.x = pack2_bf16(acc[tt][Cfg::JB - 1][0], acc[tt][Cfg::JB - 1][1]);
                    pk.y = pack2_bf16(acc[tt][Cfg::JB - 1][2], acc[tt][Cfg::JB - 1][3]);
                    nt_store8(blk + (4 * Cfg::NF + (g >> 1)) * 128 + n * 8 + 4 * (g & 1), pk);
                }
            }
        }
    };

    // A fragments: block jb, k-step i, lane (gk, a): row a <-> output channel chan(jb, a);
    // k slots <-> input channels 32 i + 8 gk + jj.  Thread tid builds fragment (jb = it, i = tid / 64,
    // lane = tid % 64) for it = 0 .. JB - 1: R_r elements first (all loads of a thread in flight
    // together), the split into bf16 head + remainder after them.
    const float* Ru = Rr + (size_t)u * D * r;
    const int fi = tid >> 6, fgk = lane >> 4, fa = lane & 15;
    float rx[Cfg::JB][8];
    // EXACT: r is the kernel's own width (the common case), so the row stride of R_r is a compile-time
    // constant; otherwise r < R and the columns r .. R - 1 are the zero padding
    auto fetch_Rr = [&](auto exact) {
        constexpr bool EXACT = decltype(exact)::value;
        const int rs = EXACT ? R : r;
#pragma unroll
        for (int jb = 0; jb < Cfg::JB; ++jb) {
            const int j = Cfg::chan(jb, fa);
#pragma unroll
            for (int jj = 0; jj < 8; ++jj)
                rx[jb][jj] = Ru[(32 * fi + 8 * fgk + jj) * rs + (EXACT ? j : min(j, r - 1))];
        }
    };
    auto park_fragments = [&]() {
#pragma unroll
        for (int jb = 0; jb < Cfg::JB; ++jb) {
            const bool pad = Cfg::chan(jb, fa) >= r;
            bf16x8 hi, lo;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                __bf16 xh, xl;
                split_bf16(pad ? 0.f : rx[jb][jj], xh, xl);
                hi[jj] = xh;
                lo[jj] = xl;
            }
            frag[((jb * 4 + fi) * 2 + 0) * 64 + lane] = hi;
            frag[((jb * 4 + fi) * 2 + 1) * 64 + lane] = lo;
        }
    };
    if (r == R) fetch_Rr(std::true_type{});
    else fetch_Rr(std::false_type{});
    __builtin_amdgcn_sched_barrier(0);

    const int w_first = blk0 + wave * (Cfg::TT * 16);
    // Passes in pairs, the Key rows of pass p + 1 requested before pass p is rotated, the first pass
    // before R_r is even split -- R_r's loads are older than the Key loads, so the wait for them does
    // not wait for Keys.  Nothing is loaded conditionally (rows past the end are clamped to the last
    // row and never stored) and the trip count is uniform, so every wait on a load is exact.  A full
    // block makes PASSES passes; the ragged last block of a sequence makes as many as it has rows for,
    // rounded up to a pair.
    static_assert(Cfg::PASSES % 2 == 0 && Cfg::PASSES >= 4, "passes are taken in pairs");
    auto run_block = [&](auto full, int np2) {
        constexpr int TP = Cfg::TOK_PER_PASS;
        bf16x8 ka[Cfg::TT][4], kc[Cfg::TT][4];
        if (!GATHER) {
            load_keys(ka, w_first);
            __builtin_amdgcn_sched_barrier(0);
            park_fragments();
            __syncthreads();
#pragma unroll 1
            for (int p = 0; p < np2 - 2; p += 2) {
                load_keys(kc, w_first + (p + 1) * TP);
                __builtin_amdgcn_sched_barrier(0);
                rotate_store(ka, w_first + p * TP, full);
                load_keys(ka, w_first + (p + 2) * TP);
                __builtin_amdgcn_sched_barrier(0);
                rotate_store(kc, w_first + (p + 1) * TP, full);
            }
            load_keys(kc, w_first + (np2 - 1) * TP);
            __builtin_amdgcn_sched_barrier(0);
            rotate_store(ka, w_first + (np2 - 2) * TP, full);
            rotate_store(kc, w_first + (np2 - 1) * TP, full);
            return;
        }
        // With a token list a row's address comes from a load.  The row numbers of pass p + 2 are
        // requested BEFORE the rows of pass p + 1, so that waiting for them (the oldest loads in flight
        // by then) leaves the rows of the pass in between in flight; requested together with the rows
        // they address, every pass would begin with a full round trip and an empty pipeline.
        int ia[Cfg::TT], ic[Cfg::TT];
        load_rows_idx(ia, w_first);
        load_rows_idx(ic, w_first + TP);
        __builtin_amdgcn_sched_barrier(0);
        load_keys_at(ka, ia);
        __builtin_amdgcn_sched_barrier(0);
        park_fragments();
        __syncthreads();
#pragma unroll 1
        for (int p = 0; p < np2 - 2; p += 2) {
            load_rows_idx(ia, w_first + (p + 2) * TP);
            __builtin_amdgcn_sched_barrier(0);
            load_keys_at(kc, ic);
            __builtin_amdgcn_sched_barrier(0);
            rotate_store(ka, w_first + p * TP, full);
            load_rows_idx(ic, w_first + min(p + 3, np2 - 1) * TP);
            __builtin_amdgcn_sched_barrier(0);
            load_keys_at(ka, ia);
            __builtin_amdgcn_sched_barrier(0);
            rotate_store(kc, w_first + (p + 1) * TP, full);
        }
        load_keys_at(kc, ic);
        __builtin_amdgcn_sched_barrier(0);
        rotate_store(ka, w_first + (np2 - 2) * TP, full);
        rotate_store(kc, w_first + (np2 - 1) * TP, full);
    };
    const int rows_here = min(n_b - blk0, Cfg::TOK_PER_BLOCK);
    run_block(std::false_type{}, (((rows_here + Cfg::TOK_PER_PASS - 1) / Cfg::TOK_PER_PASS) + 1) & ~1);
}

// ---------------------------------------------------------------------------
// Values -> fragment-major V cache: one block per 32-token block, transposed
// through LDS; rows past the sequence end inside the last block are zero-filled.
template <typename T>
struct alignas(16) Oct { T v[8]; };

template <typename T>
__global__ __launch_bounds__(256) void v_retile(RowsDev rows, int Hkv, int cap, T* __restrict__ dst)
{
    const int h = blockIdx.y, b = blockIdx.z, u = b * Hkv + h;
    const int tid = threadIdx.x;
    const int n_b = min(rows_count(rows, b), cap);
    const int t0 = blockIdx.x * 32;
    if (t0 >= n_b) return;
    __shared__ Oct<T> tile[32][17];              // 16 octets per row + 1 pad
    const T* base = (const T*)rows.data;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        int p = tid + 256 * k, row = p >> 4, oc = p & 15;
        Oct<T> x;
        if (t0 + row < n_b) x = *(const Oct<T>*)(base + rows_offset(rows, b, h, t0 + row) + oc * 8);
        else {
#pragma unroll
            for (int e = 0; e < 8; ++e) x.v[e] = (T)0;
        }
        tile[row][oc] = x;
    }
    __syncthreads();
    T* Vu = dst + (size_t)u * slab_tokens(cap) * D + (size_t)blockIdx.x * 4096;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        int o = tid + 256 * k;                   // piece index: [cb][g][n]
        int cb = o >> 6, g = (o >> 4) & 3, n = o & 15;
        int c = 16 * cb + n;
        Oct<T> x;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            int tl = jj < 4 ? 4 * g + jj : 16 + 4 * g + (jj - 4);
            x.v[jj] = tile[tl][c >> 3].v[c & 7];
        }
        if constexpr (sizeof(Oct<T>) == 16) nt_store16(Vu + (size_t)o * 8, __builtin_bit_cast(uint4, x));
        else *(Oct<T>*)(Vu + (size_t)o * 8) = x;
    }
}

// ---------------------------------------------------------------------------
// Append: block (h, b), 256 threads.  k~_j = sum_c k_new[c] R_r[c][j]: thread (cq, j)
// sums one quarter of the channels (its 32 loads of R_r are independent, one memory
// round trip), the four quarters are added in a fixed order.  The block that
// finishes last for a batch item bumps its length (all blocks of the item read the
// old length before taking a ticket).
template <typename T>
__global__ __launch_bounds__(256) void append_rows(int Hkv, int cap, int r, const T* __restrict__ k_new,
                                                   const T* __restrict__ v_new, const float* __restrict__ Rr,
                                                   T* __restrict__ Kp, T* __restrict__ Vc,
                                                   int32_t* __restrict__ seq_len, int32_t* __restrict__ tickets)
{
    const int h = blockIdx.x, b = blockIdx.y, u = b * Hkv + h;
    const int tid = threadIdx.x;
    const int len = seq_len[b];
    const bool ok = len >= 0 && len < cap;
    __shared__ float kn[D];
    __shared__ float part[4][D];
    if (ok) {
        const int rp = keep_padded(r);
        const float* Ru = Rr + (size_t)u * D * r;
        if (tid < D) kn[tid] = ld_elem(k_new + (size_t)u * D + tid);
        const int npass = (4 * r + 255) / 256;                   // 1 or 2, the same for every thread
        for (int pss = 0; pss < npass; ++pss) {
            const int idx = tid + 256 * pss;
            const bool act = idx < 4 * r;
            const int cq = act ? idx / r : 0, j = act ? idx - cq * r : 0;
            float x[32];
#pragma unroll
            for (int c = 0; c < 32; ++c) x[c] = act ? Ru[(32 * cq + c) * r + j] : 0.f;
            if (pss == 0) __syncthreads();                       // kn staged (uniform branch)
            float a = 0.f;
#pragma unroll
            for (int c = 0; c < 32; ++c) a = fmaf(kn[32 * cq + c], x[c], a);
            if (act) part[cq][j] = a;
        }
        __syncthreads();
        if (tid < rp) st_elem(Kp + (size_t)u * slab_tokens(cap) * rp + kidx(len, tid, rp),        // zeros in the padding
                              tid < r ? (part[0][tid] + part[1][tid]) + (part[2][tid] + part[3][tid]) : 0.f);
        if (tid < D) Vc[(size_t)u * slab_tokens(cap) * D + vidx(len, tid)] = v_new[(size_t)u * D + tid];
    }
    __syncthreads();
    if (tid == 0) {
        int old = atomicAdd(&tickets[b], 1);
        if (old == Hkv - 1) {
            tickets[b] = 0;
            if (ok) seq_len[b] = len + 1;
        }
    }
}

// ---------------------------------------------------------------------------
// Inverse re-tiling for inspection: caches -> row-major [B,H_kv,cap,r] / [B,H_kv,cap,d].
template <typename T>
__global__ __launch_bounds__(256) void unpack_cache(int cap, int r, const T* __restrict__ Kp,
                                                    const T* __restrict__ Vc, T* __restrict__ k_rows,
                                                    T* __restrict__ v_rows)
{
    const int u = blockIdx.y;
    const int t0 = blockIdx.x * 32;
    const int rp = keep_padded(r);
    if (k_rows) {
        for (int idx = threadIdx.x; idx < 32 * r; idx += 256) {
            int t = t0 + idx / r, j = idx % r;
            if (t < cap) k_rows[((size_t)u * cap + t) * r + j] = Kp[(size_t)u * slab_tokens(cap) * rp + kidx(t, j, rp)];
        }
    }
    if (v_rows) {
        for (int idx = threadIdx.x; idx < 32 * D; idx += 256) {
            int t = t0 + (idx >> 7), c = idx & 127;
            if (t < cap) v_rows[((size_t)u * cap + t) * D + c] = Vc[(size_t)u * slab_tokens(cap) * D + vidx(t, c)];
        }
    }
}

// ---------------------------------------------------------------------------
template <int R, int NP>
static hipError_t launch_compress_mfma_rp(const RowsDev& rows, int B, int Hkv, int cap, int r, const float* Rr,
                                          bf16_t* Kp, int32_t* seq_len_out, hipStream_t st)
{
    typedef CompressCfg<R, NP> Cfg;
    int nblk = (rows.n_tokens + Cfg::TOK_PER_BLOCK - 1) / Cfg::TOK_PER_BLOCK;
    if (nblk < 1) nblk = 1;
    if (rows.tok_idx)
        hipLaunchKernelGGL((compress_mfma<R, true, NP>), dim3(nblk, Hkv, B), dim3(256), Cfg::LDS_BYTES, st, rows, Hkv,
                           cap, r, Rr, Kp, seq_len_out);
    else
        hipLaunchKernelGGL((compress_mfma<R, false, NP>), dim3(nblk, Hkv, B), dim3(256), Cfg::LDS_BYTES, st, rows, Hkv,
                           cap, r, Rr, Kp, seq_len_out);
    return hipGetLastError();
}

// 2048 tokens per work-group (one R_r fragment build per 2048 rows, one work-group per compute unit at
// the large shapes) when that still gives every one of the 256 compute units a work-group, else 512
template <int R>
static hipError_t launch_compress_mfma_r(const RowsDev& rows, int B, int Hkv, int cap, int r, const float* Rr,
                                         bf16_t* Kp, int32_t* seq_len_out, hipStream_t st)
{
    const int64_t long_blocks = (int64_t)((rows.n_tokens + CompressCfg<R, 16>::TOK_PER_BLOCK - 1) /
                                          CompressCfg<R, 16>::TOK_PER_BLOCK) * Hkv * B;
    if (long_blocks >= 256) return launch_compress_mfma_rp<R, 16>(rows, B, Hkv, cap, r, Rr, Kp, seq_len_out, st);
    return launch_compress_mfma_rp<R, 4>(rows, B, Hkv, cap, r, Rr, Kp, seq_len_out, st);
}

hipError_t launch_compress(int dtype, bool mfma, const RowsDev& rows, int B, int Hkv, int cap, int r,
                           const float* Rr, void* Kp, int32_t* seq_len_out, hipStream_t st)
{
    if (mfma && dtype == 1) {
        bf16_t* kp = (bf16_t*)Kp;
        switch (keep_padded(r)) {
            case 16: return launch_compress_mfma_r<16>(rows, B, Hkv, cap, r, Rr, kp, seq_len_out, st);
            case 32: return launch_compress_mfma_r<32>(rows, B, Hkv, cap, r, Rr, kp, seq_len_out, st);
            case 48: return launch_compress_mfma_r<48>(rows, B, Hkv, cap, r, Rr, kp, seq_len_out, st);
            case 64: return launch_compress_mfma_r<64>(rows, B, Hkv, cap, r, Rr, kp, seq_len_out, st);
            case 80: return launch_compress_mfma_r<80>(rows, B, Hkv, cap, r, Rr, kp, seq_len_out, st);
            case 96: return launch_compress_mfma_r<96>(rows, B, Hkv, cap, r, Rr, kp, seq_len_out, st);
            case 112: return launch_compress_mfma_r<112>(rows, B, Hkv, cap, r, Rr, kp, seq_len_out, st);
            case 128: return launch_compress_mfma_r<128>(rows, B, Hkv, cap, r, Rr, kp, seq_len_out, st);
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

hipError_t launch_v_retile(int dtype, const RowsDev& rows, int B, int Hkv, int cap, void* dst, hipStream_t st)
{
    int nblk = (rows.n_tokens + 31) / 32;
    if (nblk < 1) nblk = 1;
    dim3 grid(nblk, Hkv, B);
    if (dtype == 0) hipLaunchKernelGGL(v_retile<float>, grid, dim3(256), 0, st, rows, Hkv, cap, (float*)dst);
    else hipLaunchKernelGGL(v_retile<bf16_t>, grid, dim3(256), 0, st, rows, Hkv, cap, (bf16_t*)dst);
    return hipGetLastError();
}

hipError_t launch_append(int dtype, int B, int Hkv, int cap, int r, const void* k_new, const void* v_new,
                         const float* Rr, void* Kp, void* Vc, int32_t* seq_len, int32_t* tickets, hipStream_t st)
{
    dim3 grid(Hkv, B);
    if (dtype == 0)
        hipLaunchKernelGGL(append_rows<float>, grid, dim3(256), 0, st, Hkv, cap, r, (const float*)k_new,
                           (const float*)v_new, Rr, (float*)Kp, (float*)Vc, seq_len, tickets);
    else
        hipLaunchKernelGGL(append_rows<bf16_t>, grid, dim3(256), 0, st, Hkv, cap, r, (const bf16_t*)k_new,
                           (const bf16_t*)v_new, Rr, (bf16_t*)Kp, (bf16_t*)Vc, seq_len, tickets);
    return hipGetLastError();
}

hipError_t launch_unpack(int dtype, int U, int cap, int r, const void* Kp, const void* Vc, void* k_rows,
                         void* v_rows, hipStream_t st)
{
    dim3 grid((cap + 31) / 32, U);
    if (dtype == 0)
        hipLaunchKernelGGL(unpack_cache<float>, grid, dim3(256), 0, st, cap, r, (const float*)Kp, (const float*)Vc,
                           (float*)k_rows, (float*)v_rows);
    else
        hipLaunchKernelGGL(unpack_cache<bf16_t>, grid, dim3(256), 0, st, cap, r, (const bf16_t*)Kp,
                           (const bf16_t*)Vc, (bf16_t*)k_rows, (bf16_t*)v_rows);
    return hipGetLastError();
}

}  // namespace rk
