// Measurement aids: bare reads of device memory, the yardstick the decode kernels are held against.
//
// Neither kernel computes anything of the method.  They request the same bytes a decode step streams (Sec. 3.4:
// gate and up rows of the retained and candidate channels, down rows of the retained and selected ones), with
// 16-byte loads, eight rows in flight per thread, and fold them into one word so that the loads cannot be dropped.
// What they take is the time the memory system needs for those bytes on this machine; a decode kernel cannot be
// faster than that.
#include "pop_internal.h"

namespace pop {

constexpr int kProbeInFlight = 8;  // 16-byte loads in flight per thread

// Contiguous read of n_vec 16-byte vectors, workgroups striding the buffer in blocks of kProbeInFlight sweeps.
__global__ __launch_bounds__(512) void probe_read_kernel(const uint4 *__restrict__ p, size_t n_vec,
                                                         unsigned int *__restrict__ sink)
{
    const size_t sweep = (size_t)blockDim.x, chunk = sweep * kProbeInFlight;
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (size_t base = (size_t)blockIdx.x * chunk; base < n_vec; base += (size_t)gridDim.x * chunk) {
        uint4 v[kProbeInFlight];
#pragma unroll
        for (int u = 0; u < kProbeInFlight; ++u) {
            const size_t i = base + u * sweep + threadIdx.x;
            v[u] = p[i < n_vec ? i : 0];
        }
#pragma unroll
        for (int u = 0; u < kProbeInFlight; ++u) acc.x ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc.x == 0x9e3779b9u) atomicOr(sink, 1u);  // (a value the compiler cannot rule out: keeps the loads alive)
}

// Gathered read of the rows of a decode step.  rows of w viewed as [3 m][nvec]: for list entry i < n_gu the gate row
// 3 j and the up row 3 j + 1 of channel j = gu_list[i]; for i < n_dn the down row 3 j + 2 of j = dn_list[i]
// (i < n_dn_ret from dn_ret, the rest from dn_sel).  A workgroup takes whole rows (its threads cover the row's
// vectors), kProbeInFlight rows at a time, the rows dealt round robin over the workgroups.
__global__ __launch_bounds__(512) void probe_step_read_kernel(const uint4 *__restrict__ w, int nvec,
                                                              const int *__restrict__ gu_list, int n_gu,
                                                              const int *__restrict__ dn_ret, int n_dn_ret,
                                                              const int *__restrict__ dn_sel, int n_dn_sel,
                                                              unsigned int *__restrict__ sink)
{
    const int n_rows = 2 * n_gu + n_dn_ret + n_dn_sel;
    auto row_of = [&](int r) -> size_t {  // r-th row of the step -> row number in w
        if (r < 2 * n_gu) return (size_t)gu_list[r >> 1] * 3 + (r & 1);
        r -= 2 * n_gu;
        return (size_t)(r < n_dn_ret ? dn_ret[r] : dn_sel[r - n_dn_ret]) * 3 + 2;
    };
    unsigned int acc = 0;
    for (int r0 = blockIdx.x * kProbeInFlight; r0 < n_rows; r0 += gridDim.x * kProbeInFlight) {
        size_t off[kProbeInFlight];
#pragma unroll
        for (int u = 0; u < kProbeInFlight; ++u) off[u] = row_of(min(r0 + u, n_rows - 1)) * (size_t)nvec;
        for (int c = threadIdx.x; c < nvec; c += blockDim.x) {
            uint4 v[kProbeInFlight];
#pragma unroll
            for (int u = 0; u < kProbeInFlight; ++u) v[u] = w[off[u] + c];
#pragma unroll
            for (int u = 0; u < kProbeInFlight; ++u)
                if (r0 + u < n_rows) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
        }
    }
    if (acc == 0x9e3779b9u) atomicOr(sink, 1u);
}

hipError_t launch_probe_read(const void *buf, size_t bytes, int workgroups, unsigned int *sink, hipStream_t s)
{
    hipLaunchKernelGGL(probe_read_kernel, dim3(workgroups), dim3(512), 0, s, (const uint4 *)buf, bytes / 16, sink);
    return hipGetLastError();
}

hipError_t launch_probe_step_read(const void *w, int nvec, const int *gu_list, int n_gu, const int *dn_ret,
                                  int n_dn_ret, const int *dn_sel, int n_dn_sel, int workgroups, unsigned int *sink,
                                  hipStream_t s)
{
    hipLaunchKernelGGL(probe_step_read_kernel, dim3(workgroups), dim3(512), 0, s, (const uint4 *)w, nvec, gu_list,
                       n_gu, dn_ret, n_dn_ret, dn_sel, n_dn_sel, sink);
    return hipGetLastError();
}

}  // namespace pop
