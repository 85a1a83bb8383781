// Channel importance under the input-side reading of Sec. 3.1 (Eq. 1-2 applied literally to the FFN's first
// projections and the FFN input): I_j = || [W_gate[j,:], W_up[j,:]] * s ||_2 with s_k = ||X[:,k]||_2 over the tokens
// of a prompt, or s_k = |x_k| for a decode token.  Two steps: the squared input norms s2[k] (a column reduction of X,
// deterministic: row groups in a fixed order), then one wave per listed channel streams its gate and up rows and
// forms sqrt(sum_k (wg^2 + wu^2) s2[k]).  HBM-bound on the rows it reads; float32 accumulation of non-negative terms
// (64 per-lane partial sums, then a tree).
#include "pop_internal.h"
#include "pop_vec.h"

namespace pop {

constexpr int kIsRowsPerGroup = 32;

int input_side_groups(int T) { return (T + kIsRowsPerGroup - 1) / kIsRowsPerGroup; }

template <bool BF16>
__device__ __forceinline__ float is_load(const void *x, size_t i)
{
    return BF16 ? __uint_as_float(((uint32_t)((const uint16_t *)x)[i]) << 16) : ((const float *)x)[i];
}

// part[g][k] = sum over the rows t of group g of x[t][k]^2
template <bool BF16>
__global__ __launch_bounds__(256) void colsumsq_part_kernel(const void *__restrict__ x, int T, int d,
                                                            double *__restrict__ part)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= d) return;
    const int t0 = blockIdx.y * kIsRowsPerGroup, t1 = min(T, t0 + kIsRowsPerGroup);
    double acc = 0.0;
    for (int t = t0; t < t1; ++t) {
        const double v = (double)is_load<BF16>(x, (size_t)t * d + k);
        acc += v * v;
    }
    part[(size_t)blockIdx.y * d + k] = acc;
}

// s2[k] = sum over the groups, in group order
__global__ __launch_bounds__(256) void colsumsq_reduce_kernel(const double *__restrict__ part, int n_groups, int d,
                                                              float *__restrict__ s2)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= d) return;
    double acc = 0.0;
    for (int g = 0; g < n_groups; ++g) acc += part[(size_t)g * d + k];
    s2[k] = (float)acc;
}

// s2[b][k] = x[b][k]^2 (decode: every sequence is its own one-token sample)
template <bool BF16>
__global__ __launch_bounds__(256) void square_kernel(const void *__restrict__ x, int n, float *__restrict__ s2)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float v = is_load<BF16>(x, i);
    s2[i] = v * v;
}

hipError_t launch_input_norms(const void *x, int is_bf16, int T, int d, double *part, float *s2, hipStream_t s)
{
    const int n_groups = input_side_groups(T);
    dim3 grid((d + 255) / 256, n_groups);
    if (is_bf16)
        hipLaunchKernelGGL(colsumsq_part_kernel<true>, grid, dim3(256), 0, s, x, T, d, part);
    else
        hipLaunchKernelGGL(colsumsq_part_kernel<false>, grid, dim3(256), 0, s, x, T, d, part);
    hipLaunchKernelGGL(colsumsq_reduce_kernel, dim3((d + 255) / 256), dim3(256), 0, s, part, n_groups, d, s2);
    return hipGetLastError();
}

hipError_t launch_input_squares(const void *x, int is_bf16, int B, int d, float *s2, hipStream_t s)
{
    const int n = B * d;
    if (is_bf16)
        hipLaunchKernelGGL(square_kernel<true>, dim3((n + 255) / 256), dim3(256), 0, s, x, n, s2);
    else
        hipLaunchKernelGGL(square_kernel<false>, dim3((n + 255) / 256), dim3(256), 0, s, x, n, s2);
    return hipGetLastError();
}

template <class V>
__device__ __forceinline__ void is_unpack(const typename V::vec_t &v, float (&f)[8]);
template <>
__device__ __forceinline__ void is_unpack<VecBF16>(const uint4 &v, float (&f)[8])
{
    f[0] = bf16_lo(v.x), f[1] = bf16_hi(v.x), f[2] = bf16_lo(v.y), f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z), f[5] = bf16_hi(v.z), f[6] = bf16_lo(v.w), f[7] = bf16_hi(v.w);
}
template <>
__device__ __forceinline__ void is_unpack<VecF32>(const float4 &v, float (&f)[8])
{
    f[0] = v.x, f[1] = v.y, f[2] = v.z, f[3] = v.w;
    f[4] = f[5] = f[6] = f[7] = 0.f;
}

// out[s][p] = sqrt(sum_k (w_gate[j][k]^2 + w_up[j][k]^2) * s2[s][k]),  j = rows ? rows[p] : p, for p < n_rows and the
// two sequences s = 2 blockIdx.y, 2 blockIdx.y + 1 (< S) whose s2 rows the workgroup holds in LDS.
template <class V>
__global__ __launch_bounds__(256) void input_side_scores_kernel(const typename V::vec_t *__restrict__ w, int nvec,
                                                                const float *__restrict__ s2, int S,
                                                                const int *__restrict__ rows, int n_rows,
                                                                float *__restrict__ out, int out_stride)
{
    typedef typename V::vec_t vec_t;
    constexpr int E = V::kElems;
    extern __shared__ __attribute__((aligned(16))) float is_s2[];  // [2][nvec * E]
    const int d = nvec * E;
    const int s0 = blockIdx.y * 2, ns = min(2, S - s0);
    for (int i = threadIdx.x; i < 2 * d; i += blockDim.x) is_s2[i] = i < ns * d ? s2[(size_t)s0 * d + i] : 0.f;
    __syncthreads();
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int n_waves = gridDim.x * (blockDim.x / kWave);
    for (int p = blockIdx.x * (blockDim.x / kWave) + wave; p < n_rows; p += n_waves) {
        const int j = rows ? rows[p] : p;
        const vec_t *g = w + (size_t)j * 3 * nvec;
        const vec_t *u = g + nvec;
        float a0 = 0.f, a1 = 0.f;
        for (int c = lane; c < nvec; c += kWave) {
            float fg[8], fu[8];
            is_unpack<V>(g[c], fg);
            is_unpack<V>(u[c], fu);
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float ww = fmaf(fg[e], fg[e], fu[e] * fu[e]);
                a0 = fmaf(ww, is_s2[c * E + e], a0);
                a1 = fmaf(ww, is_s2[d + c * E + e], a1);
            }
        }
        a0 = wave_sum(a0);
        a1 = wave_sum(a1);
        if (lane == 0) {
            out[(size_t)s0 * out_stride + p] = sqrtf(a0);
            if (ns > 1) out[(size_t)(s0 + 1) * out_stride + p] = sqrtf(a1);
        }
    }
}

// rows == nullptr: channels 0 .. n_rows-1.  s2: [S][d] float32.  out: [S][out_stride].
hipError_t launch_input_side_scores(const void *w, int is_bf16, int d, const float *s2, int S, const int *rows,
                                    int n_rows, float *out, int out_stride, hipStream_t s)
{
    if (n_rows < 1 || S < 1) return hipSuccess;
    const size_t lds = (size_t)2 * d * sizeof(float);
    int bx = (n_rows + 3) / 4;
    if (bx > 1024) bx = 1024;
    dim3 grid(bx, (S + 1) / 2);
    hipError_t e;
    if (is_bf16) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&input_side_scores_kernel<VecBF16>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(input_side_scores_kernel<VecBF16>, grid, dim3(256), lds, s, (const uint4 *)w, d / 8, s2, S,
                           rows, n_rows, out, out_stride);
    } else {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&input_side_scores_kernel<VecF32>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(input_side_scores_kernel<VecF32>, grid, dim3(256), lds, s, (const float4 *)w, d / 4, s2, S,
                           rows, n_rows, out, out_stride);
    }
    return hipGetLastError();
}

}  // namespace pop
