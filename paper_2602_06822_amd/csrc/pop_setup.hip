// One-time layer setup: channel-major repack of the three projections and the weight factor of Eq. 3.
//
// A channel j owns row j of W_gate and W_up and column j of W_down (Sec. 3.1).  After the repack it owns
// one contiguous block  w[j] = [gate row | up row | down column]  (3*d elements), so a decode step streams
// whole, contiguous blocks for exactly the active channels.
#include "pop_internal.h"

namespace pop {

// 16-byte copies: row j of gate and up -> w[j][0], w[j][1].  vec_per_row = d * esize / 16.
__global__ __launch_bounds__(256) void repack_gateup_kernel(const uint4 *__restrict__ w_gate,
                                                            const uint4 *__restrict__ w_up,
                                                            uint4 *__restrict__ w, int m, int vec_per_row)
{
    size_t total = (size_t)m * vec_per_row;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        size_t j = i / vec_per_row, c = i % vec_per_row;
        w[(j * 3) * vec_per_row + c] = w_gate[i];
        w[(j * 3 + 1) * vec_per_row + c] = w_up[i];
    }
}

// w[j][2][o] = w_down[o][j] through a 64x64 LDS tile (padded against bank conflicts).
template <typename T>
__global__ __launch_bounds__(256) void transpose_down_kernel(const T *__restrict__ w_down, T *__restrict__ w,
                                                             int d, int m)
{
    __shared__ T tile[64][65];
    int j0 = blockIdx.x * 64, o0 = blockIdx.y * 64;
    int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
    for (int r = ty; r < 64; r += 4) {
        int o = o0 + r, j = j0 + tx;
        if (o < d && j < m) tile[r][tx] = w_down[(size_t)o * m + j];
    }
    __syncthreads();
    for (int r = ty; r < 64; r += 4) {
        int j = j0 + r, o = o0 + tx;
        if (o < d && j < m) w[((size_t)j * 3 + 2) * d + o] = tile[tx][r];
    }
}

// nrm[j] = ||w[j][2][:]||_2: one wave per channel, float64 accumulation, rounded once to float32.
template <bool BF16>
__global__ __launch_bounds__(256) void down_norms_kernel(const void *__restrict__ w, float *__restrict__ nrm,
                                                         int d, int m)
{
    int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    int j = blockIdx.x * 4 + wave;
    if (j >= m) return;
    double acc = 0.0;
    for (int o = lane; o < d; o += kWave) {
        float v;
        if (BF16)
            v = __uint_as_float(((uint32_t)((const uint16_t *)w)[((size_t)j * 3 + 2) * d + o]) << 16);
        else
            v = ((const float *)w)[((size_t)j * 3 + 2) * d + o];
        acc += (double)v * (double)v;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
    if (lane == 0) nrm[j] = (float)sqrt(acc);
}

hipError_t launch_repack(const void *w_gate, const void *w_up, const void *w_down, int d, int m, int esize,
                         void *w, float *nrm, int is_bf16, hipStream_t s)
{
    int vec_per_row = d * esize / 16;
    size_t total = (size_t)m * vec_per_row;
    int grid = (int)((total + 255) / 256);
    if (grid > 8192) grid = 8192;
    hipLaunchKernelGGL(repack_gateup_kernel, dim3(grid), dim3(256), 0, s, (const uint4 *)w_gate, (const uint4 *)w_up,
                       (uint4 *)w, m, vec_per_row);
    dim3 tg((m + 63) / 64, (d + 63) / 64);
    if (is_bf16)
        hipLaunchKernelGGL(transpose_down_kernel<uint16_t>, tg, dim3(256), 0, s, (const uint16_t *)w_down,
                           (uint16_t *)w, d, m);
    else
        hipLaunchKernelGGL(transpose_down_kernel<uint32_t>, tg, dim3(256), 0, s, (const uint32_t *)w_down,
                           (uint32_t *)w, d, m);
    if (is_bf16)
        hipLaunchKernelGGL(down_norms_kernel<true>, dim3((m + 3) / 4), dim3(256), 0, s, w, nrm, d, m);
    else
        hipLaunchKernelGGL(down_norms_kernel<false>, dim3((m + 3) / 4), dim3(256), 0, s, w, nrm, d, m);
    return hipGetLastError();
}

}  // namespace pop
