// Fused single-sequence decode step (Sec. 3.3 "Decoding Stage", Sec. 3.4 two-step decoding).
//
// One launch streams, exactly once, the weights the step needs: gate+up rows of the retained and candidate
// channels and down columns of the retained and selected channels, each channel's block w[j] = [gate|up|down]
// being contiguous in memory.
//
// Work unit: a "round" of kRB channels handled by one whole workgroup.  The workgroup's threads split the d
// columns (thread t owns 16-byte vector column t), so a channel's gate, up and down rows are each read by one
// coalesced sweep of the workgroup, x and the partial y live in registers (no LDS staging, no reduction of y
// across waves), and the only exchange is the per-row gate/up dot product: wave partials go through LDS, one
// barrier per round.  The next round's rows are loaded into a second register buffer before the current round
// is reduced, so the barrier never drains the memory pipeline.
//
//   phase A  candidate rounds (gate+up only), dealt round-robin to all workgroups: h_j = silu(g_j) u_j and the
//            step score I_j(t) = n_j |h_j| (Eq. 3 with one token) go to global memory.
//   select   workgroup 0 owns no retained rows.  It waits until all workgroups have published their phase A
//            results (bounded spin on a counter; nobody waits for anything before that point), then runs the
//            top-k selection and publishes the selected list and a done flag.
//   phase B  retained rounds, dealt round-robin to workgroups 1..: gate+up dot products -> h, then the down
//            rows of the same round, already in registers, are multiplied by h into the partial y.
//   phase D  down rows of the selected candidates, dealt the same way.  Needs the selection: the workgroup
//            waits (bounded) for the done flag, which in practice was set long before.  If the bound is ever
//            hit, the workgroup marks its share as deferred (and raises sync[3]) and
//            the tail kernel adds it, so the result is correct and every wave still exits.
//   tail     a second small kernel sums the per-workgroup partials in workgroup order (plus deferred shares)
//            and writes y.
//
// Waiting is safe because the launch is sized to be co-resident (host checks the occupancy) and both waits
// are bounded; nothing spins without an exit.
#include <type_traits>

#include "pop_select_dev.h"
#include "pop_vec.h"

namespace pop {

constexpr int kRB = 2;  // channels per round
constexpr int kSpinLimit = 1 << 16;

// Optional per-workgroup timestamps (100 MHz wall clock), compiled in only for profiling builds.
#ifdef POP_TRACE
#define POP_STAMP(slot)                                                                 \
    do {                                                                                \
        if (p.trace && threadIdx.x == 0) p.trace[(size_t)blockIdx.x * 8 + (slot)] = wall_clock64(); \
    } while (0)
#else
#define POP_STAMP(slot) \
    do {                \
    } while (0)
#endif

// Bounded wait until *addr >= target.
__device__ __forceinline__ bool spin_until(const int *addr, int target)
{
    for (int it = 0; it < kSpinLimit; ++it) {
        int v = __hip_atomic_load(addr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (v >= target) return true;
        __builtin_amdgcn_s_sleep(2);
    }
    return false;
}

constexpr int kKeepRounds = 64;              // rounds whose indices / results are staged in LDS at a time
constexpr int kKeep = kKeepRounds * kRB;

template <class V, int PER>
struct RoundBuf {
    typename V::vec_t g[kRB][PER], u[kRB][PER], dn[kRB][PER];
    int j[kRB];  // channel of each slot, -1 when the slot is empty
};

// Loads the rows of one round; js points at the round's kRB staged channel indices (LDS), -1 = empty slot.
template <class V, int PER, bool GU, bool DN>
__device__ __forceinline__ void load_round(RoundBuf<V, PER> &rb, const typename V::vec_t *__restrict__ w, int nvec,
                                           const int *js, const int (&col)[PER], const bool (&ok)[PER])
{
#pragma unroll
    for (int t = 0; t < kRB; ++t) {
        const int j = js[t];
        rb.j[t] = j;
        const typename V::vec_t *row = w + (size_t)(j < 0 ? 0 : j) * 3 * nvec;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const bool ld = ok[q] && j >= 0;
            if (GU) {
                rb.g[t][q] = ld ? row[col[q]] : V::zero();
                rb.u[t][q] = ld ? row[nvec + col[q]] : V::zero();
            }
            if (DN) rb.dn[t][q] = ld ? row[2 * nvec + col[q]] : V::zero();
        }
    }
}

// Sum over the 16 lanes of each DPP row, result in every lane of the row (4 cross-lane adds, no LDS).
__device__ __forceinline__ float dpp_row_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, true));   // quad_perm 1,0,3,2
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, true));   // quad_perm 2,3,0,1
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, true));  // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, true));  // row_mirror
    return v;
}

__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

__device__ __forceinline__ float wave_total(float v)
{
    const float r = dpp_row_sum(v);
    return (lane_value(r, 0) + lane_value(r, 16)) + (lane_value(r, 32) + lane_value(r, 48));
}
__device__ __forceinline__ double wave_total(double v) { return wave_sum(v); }

// Gate/up dot products of the round's rows with x: lane partials -> wave sums -> LDS -> totals in every thread.
// One barrier; `part` ([2*kRB][16], entries of absent waves stay zero) is double-buffered by the caller.
template <class V, int PER>
__device__ __forceinline__ void round_hidden(const RoundBuf<V, PER> &rb, const typename V::vec_t (&xv)[PER],
                                             typename V::acc_t (*part)[kSelMaxWaves], int wave, int lane, int nw,
                                             float (&hv)[kRB])
{
    typedef typename V::acc_t acc_t;
    static_assert(2 * kRB * kSelMaxWaves == kWave, "one LDS word per lane in the cross-wave step");
#pragma unroll
    for (int t = 0; t < kRB; ++t) {
        acc_t ag = 0, au = 0;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            ag = V::dot(rb.g[t][q], xv[q], ag);
            au = V::dot(rb.u[t][q], xv[q], au);
        }
        ag = wave_total(ag);
        au = wave_total(au);
        if (lane == 0) {
            part[2 * t][wave] = ag;
            part[2 * t + 1][wave] = au;
        }
    }
    __syncthreads();
    if constexpr (sizeof(acc_t) == 4) {
        // lane l holds value l/16 of wave l%16; a DPP row sum adds the waves in a fixed tree order
        const float tot = dpp_row_sum((&part[0][0])[lane]);
#pragma unroll
        for (int t = 0; t < kRB; ++t) {
            const float gs = lane_value(tot, 32 * t), us = lane_value(tot, 32 * t + 16);
            hv[t] = rb.j[t] >= 0 ? silu_mul(gs, us) : 0.f;
        }
    } else {
#pragma unroll
        for (int t = 0; t < kRB; ++t) {
            acc_t gs = 0, us = 0;
            for (int wv = 0; wv < nw; ++wv) {
                gs += part[2 * t][wv];
                us += part[2 * t + 1][wv];
            }
            hv[t] = rb.j[t] >= 0 ? silu_mul((float)gs, (float)us) : 0.f;
        }
    }
}

template <class V, int PER>
__global__ __launch_bounds__(1024) void decode_fused_kernel(FusedParams p)
{
    typedef typename V::vec_t vec_t;
    typedef typename V::acc_t acc_t;
    constexpr int E = V::kElems;
    __shared__ SelShared sh;
    __shared__ int s_flag;
    __shared__ acc_t part[2][2 * kRB][kSelMaxWaves];
    __shared__ int j_s[kKeep];    // channel indices of the staged rounds
    __shared__ float h_s[kKeep];  // their hidden activations, flushed to global memory outside the streaming loop

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int nw = blockDim.x / kWave;
    const int b = blockIdx.x, n_wg = gridDim.x, n_workers = n_wg - 1, wb = b - 1;
    const int nvec = p.nvec;
    const vec_t *w = reinterpret_cast<const vec_t *>(p.w);

    POP_STAMP(0);
    if (b == 0 && tid == 0) p.sync[3] = 0;  // "some workgroup deferred its phase D share" flag of this step
    int col[PER];
    bool ok[PER];
    vec_t xv[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        col[q] = tid + q * blockDim.x;
        ok[q] = col[q] < nvec;
        xv[q] = ok[q] ? reinterpret_cast<const vec_t *>(p.x)[col[q]] : V::zero();
    }
    for (int i = tid; i < 2 * 2 * kRB * kSelMaxWaves; i += blockDim.x) (&part[0][0][0])[i] = 0;

    RoundBuf<V, PER> buf_a, buf_b;  // ping-pong: one is reduced while the other's loads are in flight

    // Streams `my_rounds` rounds of a list dealt round-robin (round i of sharer `me` = rows (i*n_sh + me)*kRB + t).
    // No global stores happen inside the streaming loop (a store would make the next wait drain every load in
    // flight, prefetched ones included): h is staged in LDS and flushed per chunk of kKeepRounds rounds.
    auto stream_phase = [&](auto with_down, const int *list, int n_list, int n_sh, int me, int my_rounds, auto consume,
                            auto flush) {
        constexpr bool DN = decltype(with_down)::value;
        for (int base = 0; base < my_rounds; base += kKeepRounds) {
            const int nr = min(kKeepRounds, my_rounds - base);
            for (int e = tid; e < nr * kRB; e += blockDim.x) {
                const int r = ((base + e / kRB) * n_sh + me) * kRB + e % kRB;
                j_s[e] = r < n_list ? list[r] : -1;
            }
            __syncthreads();
            load_round<V, PER, true, DN>(buf_a, w, nvec, j_s, col, ok);
            for (int i = 0; i < nr; i += 2) {
                if (i + 1 < nr) load_round<V, PER, true, DN>(buf_b, w, nvec, j_s + (i + 1) * kRB, col, ok);
                {
                    float hv[kRB];
                    round_hidden<V, PER>(buf_a, xv, part[0], wave, lane, nw, hv);
                    if (tid == 0)
#pragma unroll
                        for (int t = 0; t < kRB; ++t) h_s[i * kRB + t] = hv[t];
                    consume(buf_a, hv);
                }
                if (i + 2 < nr) load_round<V, PER, true, DN>(buf_a, w, nvec, j_s + (i + 2) * kRB, col, ok);
                if (i + 1 < nr) {
                    float hv[kRB];
                    round_hidden<V, PER>(buf_b, xv, part[1], wave, lane, nw, hv);
                    if (tid == 0)
#pragma unroll
                        for (int t = 0; t < kRB; ++t) h_s[(i + 1) * kRB + t] = hv[t];
                    consume(buf_b, hv);
                }
            }
            __syncthreads();
            for (int e = tid; e < nr * kRB; e += blockDim.x)
                if (j_s[e] >= 0) flush(j_s[e], h_s[e], ((base + e / kRB) * n_sh + me) * kRB + e % kRB);
            __syncthreads();
        }
    };

    // ---- phase A: candidate rounds, shared by all n_wg workgroups
    {
        const int my_rounds = (b * kRB < p.n_cand) ? (p.n_cand - b * kRB + n_wg * kRB - 1) / (n_wg * kRB) : 0;
        stream_phase(
            std::false_type{}, p.cand_idx, p.n_cand, n_wg, b, my_rounds, [&](const RoundBuf<V, PER> &, const float(&)[kRB]) {},
            [&](int j, float hv, int c) {
                p.h[j] = hv;
                p.cscore[c] = p.nrm[j] * fabsf(hv);
            });
    }
    __syncthreads();
    POP_STAMP(1);
    if (b != 0) {
        if (tid == 0) {
            __threadfence();
            atomicAdd(&p.sync[0], 1);
        }
    } else {
        // ---- select (workgroup 0 only)
        if (tid == 0) {
            bool ok_a = spin_until(&p.sync[0], n_workers);
            if (!ok_a) p.sync[2] = 1;
            __hip_atomic_store(&p.sync[0], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // all arrivals are in
            __threadfence();
            s_flag = ok_a ? 1 : 0;
        }
        __syncthreads();
        POP_STAMP(2);
        if (s_flag) {
            block_select_candidates(p.cscore, p.cand_idx, p.n_cand, p.k, p.mask, p.active_idx + p.n_ret, sh);
            if (tid == 0 && p.n_active) *p.n_active = p.n_ret + p.k;
            __syncthreads();
            if (tid == 0) {
                __threadfence();
                __hip_atomic_store(&p.sync[1], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        POP_STAMP(3);
        return;
    }

    float acc[PER][8];
#pragma unroll
    for (int q = 0; q < PER; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[q][e] = 0.f;

    // ---- phase B: retained rounds, shared by workgroups 1..n_wg-1
    {
        const int my_rounds =
            (wb * kRB < p.n_ret) ? (p.n_ret - wb * kRB + n_workers * kRB - 1) / (n_workers * kRB) : 0;
        stream_phase(
            std::true_type{}, p.ret_idx, p.n_ret, n_workers, wb, my_rounds,
            [&](const RoundBuf<V, PER> &rb, const float(&hv)[kRB]) {
#pragma unroll
                for (int t = 0; t < kRB; ++t)
#pragma unroll
                    for (int q = 0; q < PER; ++q) V::axpy(hv[t], rb.dn[t][q], acc[q]);
            },
            [&](int j, float hv, int) { p.h[j] = hv; });
    }
    POP_STAMP(2);

    // ---- phase D: selected candidates; needs the selection
    POP_STAMP(3);
    if (tid == 0) {
        bool ok_d = spin_until(&p.sync[1], 1);
        __threadfence();
        s_flag = ok_d ? 1 : 0;
        p.deferred[b] = ok_d ? 0 : 1;
        if (!ok_d) {
            p.sync[2] = 1;
            __hip_atomic_store(&p.sync[3], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // the last workgroup past this point rearms the flags for the next launch
        if (atomicAdd(&p.sync[4], 1) == n_workers - 1) {
            __hip_atomic_store(&p.sync[4], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&p.sync[1], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
    POP_STAMP(4);
    if (s_flag) {
        const int *sel = p.active_idx + p.n_ret;
        const int my_rounds = (wb * kRB < p.k) ? (p.k - wb * kRB + n_workers * kRB - 1) / (n_workers * kRB) : 0;
        for (int base = 0; base < my_rounds; base += kKeepRounds) {
            const int nr = min(kKeepRounds, my_rounds - base);
            for (int e = tid; e < nr * kRB; e += blockDim.x) {
                const int r = ((base + e / kRB) * n_workers + wb) * kRB + e % kRB;
                const int j = r < p.k ? sel[r] : -1;
                j_s[e] = j;
                h_s[e] = j >= 0 ? p.h[j] : 0.f;
            }
            __syncthreads();
            for (int i = 0; i < nr; ++i) {
                load_round<V, PER, false, true>(buf_a, w, nvec, j_s + i * kRB, col, ok);
#pragma unroll
                for (int t = 0; t < kRB; ++t)
#pragma unroll
                    for (int q = 0; q < PER; ++q) V::axpy(h_s[i * kRB + t], buf_a.dn[t][q], acc[q]);
            }
            __syncthreads();
        }
    }

    // ---- partial y of this workgroup
    POP_STAMP(5);
    float *dst = p.partial + (size_t)b * p.d;
#pragma unroll
    for (int q = 0; q < PER; ++q)
        if (ok[q]) {
#pragma unroll
            for (int e = 0; e < E; e += 4)
                *reinterpret_cast<float4 *>(dst + (size_t)col[q] * E + e) =
                    make_float4(acc[q][e], acc[q][e + 1], acc[q][e + 2], acc[q][e + 3]);
        }
    POP_STAMP(6);
}

// y[o] = sum over workgroups 1..n_wg-1 (in order) of partial[b][o], plus shares a workgroup deferred.
// A workgroup owns 64 outputs; its 4 waves sum contiguous quarters of the partial rows and combine in wave order.
__global__ __launch_bounds__(256) void decode_tail_kernel(const float *__restrict__ partial, int n_wg, int d,
                                                          const int *__restrict__ deferred, const int *sync,
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
        const bool any_deferred = sync[3] != 0;  // set only when some workgroup gave up waiting in this step
        for (int b = 1; any_deferred && b < n_wg; ++b) {
            if (!deferred[b]) continue;
            // the workgroup's phase D share: rows (i * n_workers + b - 1) * kRB + t, as in the fused kernel
            for (int i = 0; (i * (n_wg - 1) + b - 1) * kRB < k; ++i)
                for (int t = 0; t < kRB; ++t) {
                    const int r = (i * (n_wg - 1) + b - 1) * kRB + t;
                    if (r >= k) break;
                    const int j = sel[r];
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
template <class V, int PER>
static hipError_t fused_launch(const FusedPlan &pl, FusedParams &p, hipStream_t s)
{
    hipLaunchKernelGGL((decode_fused_kernel<V, PER>), dim3(pl.n_wg), dim3(pl.block), 0, s, p);
    return hipGetLastError();
}

template <class V, int PER>
static hipError_t fused_occupancy(int block, int *blocks_per_cu)
{
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, decode_fused_kernel<V, PER>, block, 0);
}

int fused_max_workgroups() { return 1024; }

// Chooses the launch shape; returns false when this d is not supported by the fused kernel.
bool fused_plan(int d, int is_bf16, int n_ret, int n_cand, int wg_target, FusedPlan *pl)
{
    const int E = is_bf16 ? 8 : 4, nvec = d / E;
    int per = 1;
    if (nvec > 1024) per = 2;
    if (nvec > 2048) return false;
    pl->per = per;
    pl->block = ((nvec + per * kWave - 1) / (per * kWave)) * kWave;
    int workers = (n_ret + kRB - 1) / kRB;
    const int by_cand = (n_cand + kRB - 1) / kRB;
    if (by_cand > workers) workers = by_cand;
    if (workers < 1) workers = 1;
    if (workers > wg_target - 1) workers = wg_target - 1;
    pl->n_wg = workers + 1;
    return true;
}

hipError_t fused_resident_limit(int is_bf16, const FusedPlan &pl, int n_cu, int *max_wg)
{
    int per_cu = 0;
    hipError_t e;
    if (is_bf16)
        e = pl.per == 1 ? fused_occupancy<VecBF16, 1>(pl.block, &per_cu) : fused_occupancy<VecBF16, 2>(pl.block, &per_cu);
    else
        e = pl.per == 1 ? fused_occupancy<VecF32, 1>(pl.block, &per_cu) : fused_occupancy<VecF32, 2>(pl.block, &per_cu);
    if (e != hipSuccess) return e;
    *max_wg = per_cu * n_cu;
    return hipSuccess;
}

hipError_t launch_decode_fused(const FusedPlan &pl, int is_bf16, FusedParams &p, hipStream_t s)
{
    if (is_bf16) return pl.per == 1 ? fused_launch<VecBF16, 1>(pl, p, s) : fused_launch<VecBF16, 2>(pl, p, s);
    return pl.per == 1 ? fused_launch<VecF32, 1>(pl, p, s) : fused_launch<VecF32, 2>(pl, p, s);
}

hipError_t launch_decode_tail(const float *partial, int n_wg, int d, const int *deferred, const int *sync,
                              const int *sel, int k, const float *h, const void *w, int m, int is_bf16, void *y,
                              int y_bf16, hipStream_t s)
{
    hipLaunchKernelGGL(decode_tail_kernel, dim3((d + kWave - 1) / kWave), dim3(256), 0, s, partial, n_wg, d, deferred,
                       sync, sel, k, h, w, m, is_bf16, y, y_bf16);
    return hipGetLastError();
}

}  // namespace pop
