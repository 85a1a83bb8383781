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

// ---------------------------------------------------------------- the variant that allocates nothing
// Scratch of the variant below: a file-scope device array (every GPU the library runs on holds its own copy until
// the process ends).  Host code never passes the array's name to a kernel: the name is a host-side stand-in, not a
// device address.  Its device address is looked up once per device and used from then on.
namespace {

constexpr int kStaticMaxChannels = 32768;  // largest m of the allocation-free variant
constexpr size_t kStaticScratchBytes = (size_t)pop::kIrMaxChunks * kStaticMaxChannels * sizeof(double);  // 8 MiB
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, once looked up

// Device address of the static scratch on the current device (looked up at the first call on that device).
hipError_t static_scratch(void **ptr)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" int pop_importance_reduce_static(const void *h, pop_dtype_t hdtype, int T, int m, const float *nrm,
                                            float *scores, void *stream)
{
    if (!h || !nrm || !scores) return POP_EINVAL;
    if (hdtype != POP_F32 && hdtype != POP_BF16) return POP_EINVAL;
    if (T < 1 || m < 1) return POP_ESHAPE;
    if (m > kStaticMaxChannels || pop::importance_reduce_scratch_bytes(T, m) > kStaticScratchBytes)
        return POP_EUNSUPPORTED;  // beyond the static scratch: use pop_importance_reduce
    void *ptr = nullptr;
    if (static_scratch(&ptr) != hipSuccess) {
        (void)hipGetLastError();
        return POP_EHIP;
    }
    // stage 1 writes every partial sum that stage 2 reads, so nothing in the array has to start at zero
    const hipError_t e = pop::launch_importance_reduce(h, hdtype == POP_BF16, T, m, nrm, scores, ptr,
                                                       reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return POP_EHIP;
    return POP_OK;
}
