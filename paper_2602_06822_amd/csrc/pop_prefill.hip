// Prefill: gate/up contraction over all m channels and all T prompt tokens, fused with the column-wise
// importance reduction  s2[j] = sum_t H[t][j]^2  (Sec. 3.3 "Prefilling Stage"; Eq. 3: activation norm over
// tokens and samples).  H itself is never written to memory.
//
// bf16: MFMA 32x32x16 tiles.  A workgroup (4 waves, 2 x 2) owns BM tokens (256, or 128 for short prompts) and a
// chunk of up to 96 channels, i.e. up to 192 rows of the B operand (gate and up rows of the channel-major blocks
// w[j] = [gate row | up row | down column]); a wave owns BM/2 tokens x 48 channels = 96 B rows, so each pair of LDS
// fragment reads feeds about two MFMAs, which keeps the LDS port below the matrix cores' demand.  The chunk size is
// chosen so that the tiles divide evenly over the compute units (one or a whole number of tiles each).  The 96 B
// rows of a wave are three fragments: gate of its channels 0..31, up of the same channels (same lane and register
// slot in the two accumulators, so silu(g)*u needs no exchange), and a mixed fragment [gate 32..47 | up 32..47]
// whose halves meet through one cross-lane move in the epilogue.  Each accumulator lane holds 16 token rows of one
// channel column, so the token reduction is in-register adds, one cross-half shuffle and a 2-wave LDS combine.
// Token tiles write separate partial rows that are summed in tile order.
// float32: plain FMA tiles with the same structure (64 tokens x 32 channels per workgroup).
#include "pop_internal.h"

namespace pop {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kPfBMmin = 128;     // smallest token tile (sizes the partial-row buffer)
constexpr int kPfRows = 192;      // B rows per workgroup tile (96 channels: gate + up)
constexpr int kPfChunk = 96;      // channels per workgroup tile at most
constexpr int kPfBK = 64;         // k elements per stage
constexpr int kPfLd = kPfBK + 8;  // padded LDS row stride in elements (144 B): conflict-free 16-byte reads

constexpr int kPf32BM = 64;
constexpr int kPf32BC = 32;
constexpr int kPf32BK = 16;

int prefill_num_tiles(int T, int is_bf16)
{
    return is_bf16 ? (T + kPfBMmin - 1) / kPfBMmin : (T + kPf32BM - 1) / kPf32BM;
}

// Workgroups are dealt round-robin to the 8 XCDs; renumber so that consecutive logical tiles (the token tiles
// of one channel chunk, which share the weight rows) land on the same XCD and meet in its L2.
__device__ __forceinline__ int xcd_logical_block(int bid, int per_xcd) { return (bid % 8) * per_xcd + bid / 8; }

// Channel (relative to the chunk) and matrix (0 gate, 1 up) of B row r of the workgroup tile.
__device__ __forceinline__ void pf_row_channel(int r, int &ch, int &which)
{
    const int half = r / 96, rr = r % 96;
    if (rr < 64) {
        ch = half * 48 + rr % 32;
        which = rr / 32;
    } else {
        ch = half * 48 + 32 + rr % 16;
        which = (rr - 64) / 16;
    }
}

template <int BM, int NW>
__global__ __launch_bounds__(NW * 64) void prefill_bf16_kernel(const uint16_t *__restrict__ w,
                                                           const uint16_t *__restrict__ x, int T, int d, int m,
                                                           int n_ttiles, int chunk, int n_items, int per_xcd,
                                                           float *__restrict__ s2_part)
{
    constexpr int TW = NW / 2;          // waves along the tokens (2 along the B rows)
    constexpr int MT = BM / (32 * TW);  // 32-token fragments per wave
    constexpr int RP = NW * 8;          // rows one staging pass of the workgroup covers
    extern __shared__ __attribute__((aligned(16))) uint16_t pf_lds[];
    uint16_t *As = pf_lds;                       // [2][BM * kPfLd]
    uint16_t *Bs = pf_lds + 2 * BM * kPfLd;      // [2][kPfRows * kPfLd]
    __shared__ float colsum[TW][kPfChunk];

    const int logical = xcd_logical_block(blockIdx.x, per_xcd);
    if (logical >= n_items) return;
    const int ctile = logical / n_ttiles, ttile = logical % n_ttiles;
    const int t0 = ttile * BM, c0 = ctile * chunk;
    const int cn = min(chunk, m - c0);  // channels in this chunk

    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int wm = wave / 2, wn = wave % 2;  // wave tile: tokens wm*BM/TW.., B rows wn*96..

    // global -> LDS staging: 8 vectors of 16 bytes per 64-element row; the workgroup covers RP rows per pass
    const int ld_row = tid / 8, ld_kv = tid % 8;
    constexpr int PA = BM / RP, PB = kPfRows / RP;
    static_assert(BM % RP == 0 && kPfRows % RP == 0, "whole staging passes");
    uint4 ra[PA], rb[PB];
    const uint16_t *pa[PA], *pb[PB];  // row starts (null: a row of zeros)
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        const int t = t0 + ld_row + p * RP;
        pa[p] = t < T ? x + (size_t)t * d : nullptr;
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        int ch, which;
        pf_row_channel(ld_row + p * RP, ch, which);
        pb[p] = ch < cn ? w + ((size_t)(c0 + ch) * 3 + which) * d : nullptr;
    }
    auto load_global = [&](int k0) {
        const int k = k0 + ld_kv * 8;
        const bool k_ok = k < d;
#pragma unroll
        for (int p = 0; p < PA; ++p)
            ra[p] = (k_ok && pa[p]) ? *reinterpret_cast<const uint4 *>(pa[p] + k) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int p = 0; p < PB; ++p)
            rb[p] = (k_ok && pb[p]) ? *reinterpret_cast<const uint4 *>(pb[p] + k) : make_uint4(0, 0, 0, 0);
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int p = 0; p < PA; ++p)
            *reinterpret_cast<uint4 *>(&As[(buf * BM + ld_row + p * RP) * kPfLd + ld_kv * 8]) = ra[p];
#pragma unroll
        for (int p = 0; p < PB; ++p)
            *reinterpret_cast<uint4 *>(&Bs[(buf * kPfRows + ld_row + p * RP) * kPfLd + ld_kv * 8]) = rb[p];
    };

    f32x16_t acc[MT][3];  // [token fragment][0 = gate 0..31, 1 = up 0..31, 2 = gate 32..47 | up 32..47]
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int f = 0; f < 3; ++f)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][f][v] = 0.f;

    const int n_k = (d + kPfBK - 1) / kPfBK;
    const int arow = wm * (BM / TW) + (lane % 32), brow = wn * 96 + (lane % 32), koff = (lane / 32) * 8;
    auto multiply = [&](int buf) {
        const uint16_t *Ab = As + (buf * BM + arow) * kPfLd + koff;
        const uint16_t *Bb = Bs + (buf * kPfRows + brow) * kPfLd + koff;
#pragma unroll
        for (int kk = 0; kk < kPfBK; kk += 16) {
            bf16x8_t bf[3], af[MT];
#pragma unroll
            for (int f = 0; f < 3; ++f) bf[f] = *reinterpret_cast<const bf16x8_t *>(Bb + f * 32 * kPfLd + kk);
#pragma unroll
            for (int a = 0; a < MT; ++a) af[a] = *reinterpret_cast<const bf16x8_t *>(Ab + a * 32 * kPfLd + kk);
#pragma unroll
            for (int a = 0; a < MT; ++a)
#pragma unroll
                for (int f = 0; f < 3; ++f)
                    acc[a][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[f], acc[a][f], 0, 0, 0);
        }
    };
    // step ks multiplies LDS buffer ks % 2 while the rows of step ks + 1 are on their way through registers
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int ks = 0; ks < n_k; ++ks) {
        const int buf = ks & 1;
        if (ks + 1 < n_k) load_global((ks + 1) * kPfBK);
        multiply(buf);
        if (ks + 1 < n_k) store_lds(buf ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds 16 * MT token rows of column (lane % 32) of each fragment; rows of padded tokens and
    // columns of padded channels are exactly 0
    float ss01 = 0.f, ss2 = 0.f;
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float hv = silu_mul(acc[a][0][v], acc[a][1][v]);
            ss01 = fmaf(hv, hv, ss01);
            // mixed fragment: the up value of column c < 16 sits in lane c + 16, same register
            const float g2 = acc[a][2][v];
            const float u2 = __shfl_xor(g2, 16, kWave);
            const float h2 = silu_mul(g2, u2);
            ss2 = fmaf(h2, h2, ss2);
        }
    ss01 += __shfl_xor(ss01, 32, kWave);
    ss2 += __shfl_xor(ss2, 32, kWave);
    if (lane < 32) colsum[wm][wn * 48 + lane] = ss01;
    if (lane < 16) colsum[wm][wn * 48 + 32 + lane] = ss2;
    __syncthreads();
    if (tid < cn) {
        float tot = 0.f;
#pragma unroll
        for (int q = 0; q < TW; ++q) tot += colsum[q][tid];
        s2_part[(size_t)ttile * m + c0 + tid] = tot;
    }
}

// float32: 64 tokens x 32 channels per workgroup; thread (tx = channel, ty = group of 8 tokens).
__global__ __launch_bounds__(256) void prefill_f32_kernel(const float *__restrict__ w, const float *__restrict__ x,
                                                          int T, int d, int m, float *__restrict__ s2_part)
{
    __shared__ float As[kPf32BM][kPf32BK + 1];
    __shared__ float Bg[kPf32BC][kPf32BK + 1];
    __shared__ float Bu[kPf32BC][kPf32BK + 1];
    __shared__ float colsum[8][kPf32BC];
    const int c0 = blockIdx.x * kPf32BC, ttile = blockIdx.y, t0 = ttile * kPf32BM;
    const int tid = threadIdx.x, tx = tid % 32, ty = tid / 32;
    float g[8], u[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) g[i] = u[i] = 0.f;
    for (int k0 = 0; k0 < d; k0 += kPf32BK) {
        for (int i = tid; i < kPf32BM * kPf32BK; i += 256) {
            int r = i / kPf32BK, k = i % kPf32BK;
            As[r][k] = (t0 + r < T && k0 + k < d) ? x[(size_t)(t0 + r) * d + k0 + k] : 0.f;
        }
        for (int i = tid; i < kPf32BC * kPf32BK; i += 256) {
            int r = i / kPf32BK, k = i % kPf32BK;
            bool ok = c0 + r < m && k0 + k < d;
            Bg[r][k] = ok ? w[((size_t)(c0 + r) * 3) * d + k0 + k] : 0.f;
            Bu[r][k] = ok ? w[((size_t)(c0 + r) * 3 + 1) * d + k0 + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kPf32BK; ++k) {
            float wg = Bg[tx][k], wu = Bu[tx][k];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float a = As[ty * 8 + i][k];
                g[i] = fmaf(a, wg, g[i]);
                u[i] = fmaf(a, wu, u[i]);
            }
        }
        __syncthreads();
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float hv = silu_mul(g[i], u[i]);
        ss = fmaf(hv, hv, ss);
    }
    colsum[ty][tx] = ss;
    __syncthreads();
    if (tid < kPf32BC && c0 + tid < m) {
        float tot = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) tot += colsum[q][tid];
        s2_part[(size_t)ttile * m + c0 + tid] = tot;
    }
}

// Token tile: 256 tokens unless the padding to whole tiles would then cost over 15 % more rows than with 128.
static int prefill_token_tile(int T)
{
    const int pad256 = (T + 255) / 256 * 256, pad128 = (T + 127) / 128 * 128;
    return (double)pad256 <= 1.15 * (double)pad128 ? 256 : 128;
}

int prefill_rows_used(int T, int is_bf16)
{
    if (!is_bf16) return (T + kPf32BM - 1) / kPf32BM;
    const int bm = prefill_token_tile(T);
    return (T + bm - 1) / bm;
}

hipError_t launch_prefill_gateup(const void *w, int is_bf16, int d, int m, const void *x, int T, float *s2_part,
                                 int n_cu, hipStream_t s)
{
    if (is_bf16) {
        const int bm = prefill_token_tile(T);
        const int n_tt = (T + bm - 1) / bm;
        // channel chunks of at most kPfChunk channels, as many as make the tiles a whole number per compute unit
        const int min_ct = (m + kPfChunk - 1) / kPfChunk;
        const int per_cu = (min_ct * n_tt + n_cu - 1) / n_cu;
        int n_ct = per_cu * n_cu / n_tt;
        if (n_ct < min_ct) n_ct = min_ct;
        if (n_ct > m) n_ct = m;
        const int chunk = (m + n_ct - 1) / n_ct;
        n_ct = (m + chunk - 1) / chunk;
        const int total = n_tt * n_ct, per_xcd = (total + 7) / 8;
        const size_t lds = (size_t)2 * (bm + kPfRows) * kPfLd * sizeof(uint16_t);
        hipError_t e;
        // 256-token tiles run with 8 waves (two per SIMD: one wave's waits for staging loads, LDS writes and the
        // k-step barrier are covered by the other's products), 128-token tiles with 4
        if (bm == 256) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&prefill_bf16_kernel<256, 8>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((prefill_bf16_kernel<256, 8>), dim3(per_xcd * 8), dim3(512), lds, s, (const uint16_t *)w,
                               (const uint16_t *)x, T, d, m, n_tt, chunk, total, per_xcd, s2_part);
        } else {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&prefill_bf16_kernel<128, 4>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((prefill_bf16_kernel<128, 4>), dim3(per_xcd * 8), dim3(256), lds, s, (const uint16_t *)w,
                               (const uint16_t *)x, T, d, m, n_tt, chunk, total, per_xcd, s2_part);
        }
    } else {
        dim3 grid((m + kPf32BC - 1) / kPf32BC, (T + kPf32BM - 1) / kPf32BM);
        hipLaunchKernelGGL(prefill_f32_kernel, grid, dim3(256), 0, s, (const float *)w, (const float *)x, T, d, m,
                           s2_part);
    }
    return hipGetLastError();
}

// scores[j] = nrm[j] * sqrt(sum over token tiles, in tile order, of s2_part[tile][j])   (Eq. 3)
__global__ __launch_bounds__(256) void scores_from_partials_kernel(const float *__restrict__ s2_part, int n_tiles, int m,
                                                                   const float *__restrict__ nrm,
                                                                   float *__restrict__ scores)
{
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= m) return;
    double acc = 0.0;
    for (int t = 0; t < n_tiles; ++t) acc += (double)s2_part[(size_t)t * m + j];
    scores[j] = (float)((double)nrm[j] * sqrt(acc));
}

hipError_t launch_scores_from_partials(const float *s2_part, int n_tiles, int m, const float *nrm, float *scores,
                                       hipStream_t s)
{
    hipLaunchKernelGGL(scores_from_partials_kernel, dim3((m + 255) / 256), dim3(256), 0, s, s2_part, n_tiles, m, nrm,
                       scores);
    return hipGetLastError();
}

// Stand-alone column reduction of a materialised H[T][m]: a workgroup owns 64 channels; its 4 waves stride the
// tokens (coalesced rows of 64 channels), then combine through LDS in wave order.
template <bool BF16>
__global__ __launch_bounds__(256) void importance_reduce_kernel(const void *__restrict__ h, int T, int m,
                                                                const float *__restrict__ nrm,
                                                                float *__restrict__ scores)
{
    __shared__ float part[4][kWave];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int j = blockIdx.x * kWave + lane;
    float acc = 0.f;
    if (j < m)
        for (int t = wave; t < T; t += 4) {
            float v = BF16 ? __uint_as_float(((uint32_t)((const uint16_t *)h)[(size_t)t * m + j]) << 16)
                           : ((const float *)h)[(size_t)t * m + j];
            acc = fmaf(v, v, acc);
        }
    part[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && j < m) {
        double tot = (double)part[0][lane] + (double)part[1][lane] + (double)part[2][lane] + (double)part[3][lane];
        scores[j] = (float)((double)nrm[j] * sqrt(tot));
    }
}

hipError_t launch_importance_reduce(const void *h, int is_bf16, int T, int m, const float *nrm, float *scores,
                                    hipStream_t s)
{
    dim3 grid((m + kWave - 1) / kWave);
    if (is_bf16)
        hipLaunchKernelGGL(importance_reduce_kernel<true>, grid, dim3(256), 0, s, h, T, m, nrm, scores);
    else
        hipLaunchKernelGGL(importance_reduce_kernel<false>, grid, dim3(256), 0, s, h, T, m, nrm, scores);
    return hipGetLastError();
}

}  // namespace pop
