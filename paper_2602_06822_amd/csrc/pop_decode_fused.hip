// Fused single-sequence decode step (Sec. 3.3 "Decoding Stage", Sec. 3.4 two-step decoding).
//
// One launch streams, exactly once, the weights the step needs: gate+up rows of the retained and candidate
// channels and down columns of the retained and selected channels, each channel's block w[j] = [gate|up|down]
// being contiguous in memory.
//
//   phase A  every workgroup evaluates a share of the candidate channels: h_j = silu(g_j) u_j and the step
//            score I_j(t) = n_j |h_j| (Eq. 3 with one token); results go to global memory.
//   select   workgroup 0 owns no retained rows.  It waits until all workgroups have published their phase A
//            results (bounded spin on a counter; the others never wait for anything before that point), then
//            runs the top-k selection and publishes the selected list and a done flag.
//   phase B  every other workgroup owns a contiguous block of retained channels: gate+up dot products, one wave
//            per row, h kept in LDS (and stored for the caller).
//   phase C  the same workgroup multiplies its block's down columns by those h values.  Waves own 64-vector
//            column chunks, so the workgroup's partial y needs no reduction across waves (or a fixed-order one
//            across row groups when d is small).
//   phase D  down columns of the selected candidates, dealt round-robin to the workgroups, added into the same
//            accumulators.  Needs the selection: a workgroup waits (bounded) for the done flag, which in
//            practice was set long before.  If the bound is ever hit, the workgroup marks its share as
//            deferred and the tail kernel adds it, so the result is correct and every wave still exits.
//   tail     a second small kernel sums the per-workgroup partials in workgroup order (plus deferred shares)
//            and writes y.
//
// Waiting is safe because the launch is sized to be co-resident (host checks the occupancy) and both waits
// are bounded; nothing spins without an exit.
#include "pop_select_dev.h"
#include "pop_vec.h"

namespace pop {

constexpr int kFusedGuUnroll = 8;    // 16-byte loads per matrix in flight per lane in the row dot products
constexpr int kFusedDownUnroll = 8;  // down-column loads in flight per lane
constexpr int kSpinLimit = 1 << 16;

__device__ __forceinline__ bool spin_until(const int *addr, int target, bool ge)
{
    for (int it = 0; it < kSpinLimit; ++it) {
        int v = __hip_atomic_load(addr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (ge ? (v >= target) : (v == target)) return true;
        __builtin_amdgcn_s_sleep(4);
    }
    return false;
}

template <class V, int CPW>
__global__ __launch_bounds__(1024) void decode_fused_kernel(FusedParams p)
{
    typedef typename V::vec_t vec_t;
    constexpr int E = V::kElems;
    extern __shared__ uint4 smem_raw[];
    __shared__ SelShared sh;
    __shared__ int s_flag;

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int nw = blockDim.x / kWave;
    const int b = blockIdx.x, n_wg = gridDim.x;
    const int nvec = p.nvec;
    const vec_t *w = reinterpret_cast<const vec_t *>(p.w);

    // dynamic LDS: x | h_s[rows_per_wg] | j_s[rows_per_wg] | red[(groups-1)][ncw*CPW*64*E]
    vec_t *xs = reinterpret_cast<vec_t *>(smem_raw);
    float *h_s = reinterpret_cast<float *>(xs + nvec);
    int *j_s = reinterpret_cast<int *>(h_s + p.rows_per_wg);
    float *red = reinterpret_cast<float *>(j_s + p.rows_per_wg);

    for (int i = tid; i < nvec; i += blockDim.x) xs[i] = reinterpret_cast<const vec_t *>(p.x)[i];
    // retained rows of this workgroup (workgroup 0 has none)
    const int r_lo = b == 0 ? 0 : min(p.n_ret, (b - 1) * p.rows_per_wg);
    const int r_hi = b == 0 ? 0 : min(p.n_ret, r_lo + p.rows_per_wg);
    const int n_rows = r_hi - r_lo;
    for (int i = tid; i < n_rows; i += blockDim.x) j_s[i] = p.ret_idx[r_lo + i];
    __syncthreads();

    // ---- phase A: candidates c = b, b + n_wg, ...; wave takes every nw-th of them
    for (int i = wave; b + i * n_wg < p.n_cand; i += nw) {
        const int c = b + i * n_wg;
        const int j = p.cand_idx[c];
        const vec_t *g = w + (size_t)j * 3 * nvec;
        typename V::acc_t ag, au;
        row_dot_gate_up<V, kFusedGuUnroll>(g, g + nvec, xs, nvec, lane, ag, au);
        float gs = (float)wave_sum(ag), us = (float)wave_sum(au);
        if (lane == 0) {
            float hv = silu_mul(gs, us);
            p.h[j] = hv;
            p.cscore[c] = p.nrm[j] * fabsf(hv);
        }
    }
    __syncthreads();
    if (b != 0) {
        if (tid == 0) {
            __threadfence();
            atomicAdd(&p.sync[0], 1);
        }
    } else {
        // ---- select (workgroup 0 only)
        if (tid == 0) {
            bool ok = spin_until(&p.sync[0], p.epoch * (n_wg - 1), true);  // the counter only grows within a partition
            if (!ok) p.sync[2] = 1;
            __threadfence();
            s_flag = ok ? 1 : 0;
        }
        __syncthreads();
        if (s_flag) {
            block_select_candidates(p.cscore, p.cand_idx, p.n_cand, p.k, p.mask, p.active_idx + p.n_ret, sh);
            if (tid == 0 && p.n_active) *p.n_active = p.n_ret + p.k;
            __syncthreads();
            if (tid == 0) {
                __threadfence();
                __hip_atomic_store(&p.sync[1], p.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        return;
    }

    // ---- phase B: gate/up of the block's retained rows, one wave per row
    for (int r = wave; r < n_rows; r += nw) {
        const int j = j_s[r];
        const vec_t *g = w + (size_t)j * 3 * nvec;
        typename V::acc_t ag, au;
        row_dot_gate_up<V, kFusedGuUnroll>(g, g + nvec, xs, nvec, lane, ag, au);
        float gs = (float)wave_sum(ag), us = (float)wave_sum(au);
        if (lane == 0) {
            float hv = silu_mul(gs, us);
            h_s[r] = hv;
            p.h[j] = hv;
        }
    }
    __syncthreads();

    // ---- phase C: down columns of the block; wave = (row group grp, chunk-wave cw)
    const int cw = wave % p.ncw, grp = wave / p.ncw;
    const bool down_wave = grp < p.groups;
    float acc[CPW][8];
#pragma unroll
    for (int q = 0; q < CPW; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[q][e] = 0.f;
    int col[CPW];
    bool col_ok[CPW];
#pragma unroll
    for (int q = 0; q < CPW; ++q) {
        col[q] = (cw + q * p.ncw) * kWave + lane;
        col_ok[q] = down_wave && col[q] < nvec;
    }
    if (down_wave) {
        int r = grp;
        for (; r + (kFusedDownUnroll - 1) * p.groups < n_rows; r += kFusedDownUnroll * p.groups) {
            vec_t wv[kFusedDownUnroll][CPW];
            float hv[kFusedDownUnroll];
#pragma unroll
            for (int u = 0; u < kFusedDownUnroll; ++u) {
                const int rr = r + u * p.groups;
                const size_t base = ((size_t)j_s[rr] * 3 + 2) * nvec;
                hv[u] = h_s[rr];
#pragma unroll
                for (int q = 0; q < CPW; ++q) wv[u][q] = col_ok[q] ? w[base + col[q]] : V::zero();
            }
#pragma unroll
            for (int u = 0; u < kFusedDownUnroll; ++u)
#pragma unroll
                for (int q = 0; q < CPW; ++q) V::axpy(hv[u], wv[u][q], acc[q]);
        }
        for (; r < n_rows; r += p.groups) {
            const size_t base = ((size_t)j_s[r] * 3 + 2) * nvec;
            const float hv = h_s[r];
#pragma unroll
            for (int q = 0; q < CPW; ++q) {
                vec_t wv = col_ok[q] ? w[base + col[q]] : V::zero();
                V::axpy(hv, wv, acc[q]);
            }
        }
    }

    // ---- phase D: selected candidates i = (b-1), (b-1) + (n_wg-1), ...; needs the selection
    if (tid == 0) {
        bool ok = spin_until(&p.sync[1], p.epoch, false);
        __threadfence();
        s_flag = ok ? 1 : 0;
        p.deferred[b] = ok ? 0 : 1;
        if (!ok) p.sync[2] = 1;
    }
    __syncthreads();
    if (s_flag && down_wave) {
        const int *sel = p.active_idx + p.n_ret;
        int n_mine = 0;  // index among this workgroup's selected rows, dealt to row groups
        for (int i = b - 1; i < p.k; i += n_wg - 1, ++n_mine) {
            if (n_mine % p.groups != grp) continue;
            const int j = sel[i];
            const float hv = p.h[j];
            const size_t base = ((size_t)j * 3 + 2) * nvec;
#pragma unroll
            for (int q = 0; q < CPW; ++q) {
                vec_t wv = col_ok[q] ? w[base + col[q]] : V::zero();
                V::axpy(hv, wv, acc[q]);
            }
        }
    }

    // ---- partial y of this workgroup: combine row groups in group order, then store
    const int chunk_floats = kWave * E;  // floats per (chunk, wave)
    if (p.groups > 1) {
        if (down_wave && grp > 0) {
#pragma unroll
            for (int q = 0; q < CPW; ++q)
#pragma unroll
                for (int e = 0; e < E; ++e)
                    red[((size_t)(grp - 1) * p.ncw * CPW + cw * CPW + q) * chunk_floats + e * kWave + lane] = acc[q][e];
        }
        __syncthreads();
        if (down_wave && grp == 0) {
            for (int g2 = 1; g2 < p.groups; ++g2)
#pragma unroll
                for (int q = 0; q < CPW; ++q)
#pragma unroll
                    for (int e = 0; e < E; ++e)
                        acc[q][e] += red[((size_t)(g2 - 1) * p.ncw * CPW + cw * CPW + q) * chunk_floats + e * kWave + lane];
        }
    }
    if (down_wave && grp == 0) {
        float *dst = p.partial + (size_t)b * p.d;
#pragma unroll
        for (int q = 0; q < CPW; ++q)
            if (col_ok[q]) {
#pragma unroll
                for (int e = 0; e < E; ++e) dst[(size_t)col[q] * E + e] = acc[q][e];
            }
    }
}

// y[o] = sum over workgroups 1..n_wg-1 (in order) of partial[b][o], plus shares a workgroup deferred.
// A workgroup owns 64 outputs; its 4 waves sum contiguous quarters of the partial rows and combine in wave order.
__global__ __launch_bounds__(256) void decode_tail_kernel(const float *__restrict__ partial, int n_wg, int d,
                                                          const int *__restrict__ deferred,
                                                          const int *__restrict__ sel, int k,
                                                          const float *__restrict__ h, const void *__restrict__ w,
                                                          int m, int is_bf16, void *__restrict__ y, int y_bf16)
{
    __shared__ float part[4][kWave];
    const int lane = threadIdx.x % kWave, q = threadIdx.x / kWave;
    const int o = blockIdx.x * kWave + lane;
    const int n = n_wg - 1, per = (n + 3) / 4;
    const int s0 = 1 + min(n, q * per), s1 = 1 + min(n, q * per + per);
    float acc = 0.f;
    if (o < d) {
        int s = s0;
        for (; s + 8 <= s1; s += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = partial[(size_t)(s + u) * d + o];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; s < s1; ++s) acc += partial[(size_t)s * d + o];
    }
    part[q][lane] = acc;
    __syncthreads();
    if (q == 0 && o < d) {
        float v = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
        for (int b = 1; b < n_wg; ++b) {
            if (!deferred[b]) continue;
            for (int i = b - 1; i < k; i += n_wg - 1) {
                const int j = sel[i];
                if (j < 0 || j >= m) continue;  // selection never ran: the step is flagged invalid, stay in bounds
                const size_t idx = ((size_t)j * 3 + 2) * d + o;
                const float wv = is_bf16 ? __uint_as_float(((uint32_t)((const uint16_t *)w)[idx]) << 16)
                                         : ((const float *)w)[idx];
                v = fmaf(h[j], wv, v);
            }
        }
        if (y_bf16)
            ((uint16_t *)y)[o] = f32_to_bf16(v);
        else
            ((float *)y)[o] = v;
    }
}

// ---------------------------------------------------------------- host side
template <class V, int CPW>
static hipError_t fused_launch(const FusedPlan &pl, FusedParams &p, hipStream_t s)
{
    if (pl.lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&decode_fused_kernel<V, CPW>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((decode_fused_kernel<V, CPW>), dim3(pl.n_wg), dim3(pl.block), pl.lds, s, p);
    return hipGetLastError();
}

template <class V, int CPW>
static hipError_t fused_occupancy(int block, size_t lds, int *blocks_per_cu)
{
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, decode_fused_kernel<V, CPW>, block, lds);
}

int fused_max_workgroups() { return 512; }

// Chooses the launch shape; returns false when this d is not supported by the fused kernel.
bool fused_plan(int d, int is_bf16, int n_ret, int n_cand, int wg_target, FusedPlan *pl)
{
    const int E = is_bf16 ? 8 : 4, nvec = d / E;
    const int n_cc = (nvec + kWave - 1) / kWave;
    int cpw = 1;
    if (n_cc > 16) cpw = 2;
    const int ncw = (n_cc + cpw - 1) / cpw;
    if (ncw > 16) return false;
    int groups = ncw >= 8 ? 1 : 8 / ncw;
    if (groups < 1) groups = 1;
    pl->ncw = ncw;
    pl->groups = groups;
    pl->cpw = cpw;
    pl->block = ncw * groups * kWave;
    int workers = (n_ret + 7) / 8;  // at least ~8 retained rows per workgroup
    const int by_cand = (n_cand + 3) / 4;
    if (by_cand > workers) workers = by_cand;
    if (workers < 1) workers = 1;
    if (workers > wg_target - 1) workers = wg_target - 1;
    pl->n_wg = workers + 1;
    pl->rows_per_wg = n_ret > 0 ? (n_ret + workers - 1) / workers : 1;
    pl->lds = (size_t)nvec * 16 + (size_t)pl->rows_per_wg * 8 +
              (size_t)(groups > 1 ? (groups - 1) : 0) * ncw * cpw * kWave * E * 4;
    return true;
}

hipError_t fused_resident_limit(int is_bf16, const FusedPlan &pl, int n_cu, int *max_wg)
{
    int per_cu = 0;
    hipError_t e;
    if (is_bf16)
        e = pl.cpw == 1 ? fused_occupancy<VecBF16, 1>(pl.block, pl.lds, &per_cu)
                        : fused_occupancy<VecBF16, 2>(pl.block, pl.lds, &per_cu);
    else
        e = pl.cpw == 1 ? fused_occupancy<VecF32, 1>(pl.block, pl.lds, &per_cu)
                        : fused_occupancy<VecF32, 2>(pl.block, pl.lds, &per_cu);
    if (e != hipSuccess) return e;
    *max_wg = per_cu * n_cu;
    return hipSuccess;
}

hipError_t launch_decode_fused(const FusedPlan &pl, int is_bf16, FusedParams &p, hipStream_t s)
{
    p.rows_per_wg = pl.rows_per_wg;
    p.ncw = pl.ncw;
    p.groups = pl.groups;
    if (is_bf16)
        return pl.cpw == 1 ? fused_launch<VecBF16, 1>(pl, p, s) : fused_launch<VecBF16, 2>(pl, p, s);
    return pl.cpw == 1 ? fused_launch<VecF32, 1>(pl, p, s) : fused_launch<VecF32, 2>(pl, p, s);
}

hipError_t launch_decode_tail(const float *partial, int n_wg, int d, const int *deferred, const int *sel, int k,
                              const float *h, const void *w, int m, int is_bf16, void *y, int y_bf16, hipStream_t s)
{
    hipLaunchKernelGGL(decode_tail_kernel, dim3((d + kWave - 1) / kWave), dim3(256), 0, s, partial, n_wg, d, deferred,
                       sel, k, h, w, m, is_bf16, y, y_bf16);
    return hipGetLastError();
}

}  // namespace pop
