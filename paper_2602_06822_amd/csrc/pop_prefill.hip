// Prefill: gate/up contraction over all m channels and all T prompt tokens, fused with the column-wise
// importance reduction  s2[j] = sum_t H[t][j]^2  (Sec. 3.3 "Prefilling Stage"; Eq. 3: activation norm over
// tokens and samples).  H itself is never written to memory.
//
// bf16: MFMA 32x32x16 tiles.  A workgroup owns 128 tokens x 64 channels; its B operand is the channel-major
// block w[j] = [gate row | up row | down column], so the gate and up accumulators of one (token, channel) pair sit in
// the same lane and register slot and silu(g)*u is formed without any exchange.  Each accumulator lane holds
// 16 token rows of one channel column, so the token reduction is in-register adds, one cross-half shuffle
// and a 2-wave LDS combine.  Token tiles write separate partial rows that are summed in tile order.
// float32: plain FMA tiles with the same structure (64 tokens x 32 channels per workgroup).
#include "pop_internal.h"

namespace pop {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kPfBM = 128;        // tokens per workgroup tile
constexpr int kPfBC = 64;         // channels per workgroup tile (128 B-operand rows: gate + up)
constexpr int kPfBK = 64;         // k elements per stage
constexpr int kPfLd = kPfBK + 8;  // padded LDS row stride in elements (144 B): conflict-free 16-byte reads

constexpr int kPf32BM = 64;
constexpr int kPf32BC = 32;
constexpr int kPf32BK = 16;

int prefill_num_tiles(int T, int is_bf16) { return is_bf16 ? (T + kPfBM - 1) / kPfBM : (T + kPf32BM - 1) / kPf32BM; }

// Workgroups are dealt round-robin to the 8 XCDs; renumber so that consecutive logical tiles (the token tiles
// of one channel tile, which share the weight block) land on the same XCD and meet in its L2.
__device__ __forceinline__ int xcd_logical_block(int bid, int per_xcd) { return (bid % 8) * per_xcd + bid / 8; }

__global__ __launch_bounds__(256) void prefill_bf16_kernel(const uint16_t *__restrict__ w,
                                                           const uint16_t *__restrict__ x, int T, int d, int m,
                                                           int n_ttiles, int n_tiles_total, int per_xcd,
                                                           float *__restrict__ s2_part)
{
    __shared__ __attribute__((aligned(16))) uint16_t As[2][kPfBM * kPfLd];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][2 * kPfBC * kPfLd];
    __shared__ float colsum[2][kPfBC];

    const int logical = xcd_logical_block(blockIdx.x, per_xcd);
    if (logical >= n_tiles_total) return;
    const int ctile = logical / n_ttiles, ttile = logical % n_ttiles;
    const int t0 = ttile * kPfBM, c0 = ctile * kPfBC;

    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int wm = wave / 2, wn = wave % 2;  // wave tile: tokens wm*64..+64, channels wn*32..+32

    // global -> LDS staging: 8 vectors of 16 bytes per 64-element row; 256 threads cover 32 rows per pass
    const int ld_row = tid / 8, ld_kv = tid % 8;
    uint4 ra[4], rb[4];

    auto load_global = [&](int k0) {
        const int k = k0 + ld_kv * 8;
        const bool k_ok = k < d;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = ld_row + p * 32;  // 0..127
            const int t = t0 + r;
            ra[p] = (k_ok && t < T) ? *reinterpret_cast<const uint4 *>(x + (size_t)t * d + k) : make_uint4(0, 0, 0, 0);
            // B rows 0..63: gate of channel c0+r; rows 64..127: up of channel c0+r-64
            const int ch = c0 + (r % kPfBC), which = r / kPfBC;
            rb[p] = (k_ok && ch < m) ? *reinterpret_cast<const uint4 *>(w + ((size_t)ch * 3 + which) * d + k)
                                     : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = ld_row + p * 32;
            *reinterpret_cast<uint4 *>(&As[buf][r * kPfLd + ld_kv * 8]) = ra[p];
            *reinterpret_cast<uint4 *>(&Bs[buf][r * kPfLd + ld_kv * 8]) = rb[p];
        }
    };

    f32x16_t acc[2][2];  // [token block][0 = gate, 1 = up]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    const int n_k = (d + kPfBK - 1) / kPfBK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int ks = 0; ks < n_k; ++ks) {
        const int buf = ks & 1;
        if (ks + 1 < n_k) load_global((ks + 1) * kPfBK);
        const int arow = wm * 64 + (lane % 32), brow = wn * 32 + (lane % 32), koff = (lane / 32) * 8;
#pragma unroll
        for (int kk = 0; kk < kPfBK; kk += 16) {
            bf16x8_t a0 = *reinterpret_cast<const bf16x8_t *>(&As[buf][(arow)*kPfLd + kk + koff]);
            bf16x8_t a1 = *reinterpret_cast<const bf16x8_t *>(&As[buf][(arow + 32) * kPfLd + kk + koff]);
            bf16x8_t bg = *reinterpret_cast<const bf16x8_t *>(&Bs[buf][(brow)*kPfLd + kk + koff]);
            bf16x8_t bu = *reinterpret_cast<const bf16x8_t *>(&Bs[buf][(brow + kPfBC) * kPfLd + kk + koff]);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bg, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bu, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bg, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bu, acc[1][1], 0, 0, 0);
        }
        if (ks + 1 < n_k) store_lds(buf ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds 32 token rows of channel column (lane % 32); rows of padded tokens are exactly 0
    float ss = 0.f;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float hv = silu_mul(acc[a][0][v], acc[a][1][v]);
            ss = fmaf(hv, hv, ss);
        }
    ss += __shfl_xor(ss, 32, kWave);
    if (lane < 32) colsum[wm][wn * 32 + lane] = ss;
    __syncthreads();
    if (tid < kPfBC && c0 + tid < m) s2_part[(size_t)ttile * m + c0 + tid] = colsum[0][tid] + colsum[1][tid];
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

hipError_t launch_prefill_gateup(const void *w, int is_bf16, int d, int m, const void *x, int T, float *s2_part,
                                 hipStream_t s)
{
    if (is_bf16) {
        int n_tt = (T + kPfBM - 1) / kPfBM, n_ct = (m + kPfBC - 1) / kPfBC;
        int total = n_tt * n_ct, per_xcd = (total + 7) / 8;
        hipLaunchKernelGGL(prefill_bf16_kernel, dim3(per_xcd * 8), dim3(256), 0, s, (const uint16_t *)w,
                           (const uint16_t *)x, T, d, m, n_tt, total, per_xcd, s2_part);
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
