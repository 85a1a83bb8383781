// Column-wise importance reduction over materialised activations (Sec. 3.4 Eq. 3):
//     scores[j] = nrm[j] * sqrt( sum over tokens t of H[t][j]^2 ),   H: [T][m] float32 or bf16.
//
// HBM-bound: every element of H is read once.  The tokens are split into chunks so that a prompt-sized H fills
// the chip (a column block alone gives only m/256 workgroups); a workgroup owns 256 adjacent columns of one token
// chunk, a lane one column of each 64-column group (coalesced row segments), eight rows in flight per lane.
//   stage 1  part[chunk][j] = sum over the chunk's tokens of H[t][j]^2, in double (a float32 running sum over a
//            long prompt would lose more than the 1e-5 the scores are held to); the four waves take the chunk's
//            rows round robin and meet through LDS in wave order.
//   stage 2  scores[j] = nrm[j] * sqrt(sum over chunks, in chunk order, of part[chunk][j]).
// The summation order is fixed by (T, m) alone, so the result is bit-reproducible.
// `part` is scratch: [n_chunks][m] doubles beyond the inputs and outputs.
#include <mutex>

#include "pop_internal.h"

namespace pop {

constexpr int kIrCols = 256;      // columns per workgroup
constexpr int kIrWaves = 4;       // waves per workgroup: rows of the chunk round robin
constexpr int kIrRows = 8;        // rows in flight per lane
constexpr int kIrMaxChunks = 32;  // token chunks at most

template <bool BF16>
__device__ __forceinline__ float ir_load(const void *h, size_t i)
{
    return BF16 ? __uint_as_float(((uint32_t)((const uint16_t *)h)[i]) << 16) : ((const float *)h)[i];
}

template <bool BF16>
__global__ __launch_bounds__(kIrWaves * kWave) void importance_partial_kernel(const void *__restrict__ h, int T, int m,
                                                                              int rows_per_chunk,
                                                                              double *__restrict__ part)
{
    __shared__ double red[kIrWaves][kIrCols];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int c0 = blockIdx.x * kIrCols, chunk = blockIdx.y;
    const int t_lo = chunk * rows_per_chunk, t_hi = min(T, t_lo + rows_per_chunk);
    constexpr int G = kIrCols / kWave;  // column groups of a lane
    int col[G];
    bool ok[G];
    double acc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        col[g] = c0 + g * kWave + lane;
        ok[g] = col[g] < m;
        acc[g] = 0.0;
    }
    // wave w takes rows t_lo + w, t_lo + w + 4, ...; kIrRows of them requested together
    for (int t = t_lo + wave; t < t_hi; t += kIrWaves * kIrRows) {
        float v[kIrRows][G];
#pragma unroll
        for (int r = 0; r < kIrRows; ++r) {
            const int tr = t + r * kIrWaves;
#pragma unroll
            for (int g = 0; g < G; ++g) v[r][g] = (tr < t_hi && ok[g]) ? ir_load<BF16>(h, (size_t)tr * m + col[g]) : 0.f;
        }
#pragma unroll
        for (int r = 0; r < kIrRows; ++r)
#pragma unroll
            for (int g = 0; g < G; ++g) acc[g] = fma((double)v[r][g], (double)v[r][g], acc[g]);
    }
#pragma unroll
    for (int g = 0; g < G; ++g) red[wave][g * kWave + lane] = acc[g];
    __syncthreads();
    const int c = c0 + (int)threadIdx.x;
    if (c < m) {
        double tot = 0.0;
#pragma unroll
        for (int w = 0; w < kIrWaves; ++w) tot += red[w][threadIdx.x];
        part[(size_t)chunk * m + c] = tot;
    }
}

__global__ __launch_bounds__(256) void importance_finish_kernel(const double *__restrict__ part, int n_chunks, int m,
                                                                const float *__restrict__ nrm,
                                                                float *__restrict__ scores)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= m) return;
    double tot = 0.0;
    for (int c = 0; c < n_chunks; ++c) tot += part[(size_t)c * m + j];
    scores[j] = (float)((double)nrm[j] * sqrt(tot));
}

// Token chunks for (T, m): enough workgroups to fill the chip a few times over, at least 32 rows per chunk.
static int importance_chunks(int T, int m)
{
    const int col_blocks = (m + kIrCols - 1) / kIrCols;
    int n = (1024 + col_blocks - 1) / col_blocks;
    if (n > kIrMaxChunks) n = kIrMaxChunks;
    if (n > (T + 31) / 32) n = (T + 31) / 32;
    return n < 1 ? 1 : n;
}

size_t importance_reduce_scratch_bytes(int T, int m) { return (size_t)importance_chunks(T, m) * m * sizeof(double); }

hipError_t launch_importance_reduce(const void *h, int is_bf16, int T, int m, const float *nrm, float *scores,
                                    void *scratch, hipStream_t s)
{
    const int n_chunks = importance_chunks(T, m);
    const int rows_per_chunk = (T + n_chunks - 1) / n_chunks;
    double *part = (double *)scratch;
    dim3 grid((m + kIrCols - 1) / kIrCols, n_chunks);
    if (is_bf16)
        hipLaunchKernelGGL(importance_partial_kernel<true>, grid, dim3(kIrWaves * kWave), 0, s, h, T, m, rows_per_chunk,
                           part);
    else
        hipLaunchKernelGGL(importance_partial_kernel<false>, grid, dim3(kIrWaves * kWave), 0, s, h, T, m, rows_per_chunk,
                           part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(importance_finish_kernel, dim3((m + 255) / 256), dim3(256), 0, s, part, n_chunks, m, nrm, scores);
    return hipGetLastError();
}

}  // namespace pop
