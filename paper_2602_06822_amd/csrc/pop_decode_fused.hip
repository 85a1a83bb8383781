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
//            results (bounded spin on a counter; nobody waits for anything before that point), runs the top-k
//            selection and hands every workgroup one word: a valid bit plus one bit per candidate slot of that
//            workgroup that was selected.  Mask and active list for the caller are written afterwards.
//   phase B  retained rounds, dealt round-robin to workgroups 1..: gate+up dot products -> h, then the down
//            rows of the same round, already in registers, are multiplied by h into the partial y.
//   phase D  down rows of the workgroup's own selected candidates (their h is still in LDS).  The workgroup's
//            word is polled during phase B without ever stalling it; if it has not arrived by the end of
//            phase B the workgroup waits, bounded.  If the bound is ever hit, the workgroup marks its share as
//            deferred (and raises sync[3]) and the tail kernel adds it, so every wave still exits.
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
#ifndef POP_PREFETCH_EARLY
#define POP_PREFETCH_EARLY 0
#endif
constexpr bool kPrefetchEarly = POP_PREFETCH_EARLY != 0;
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

constexpr int kMaxRounds = 64;  // rounds per phase per workgroup (the host plan guarantees it)
constexpr int kKeep = kMaxRounds * kRB;

template <class V, int PER>
struct RoundBuf {
    typename V::vec_t g[kRB][PER], u[kRB][PER], dn[kRB][PER];
    int j[kRB];  // channel of each slot, -1 when the slot is empty
};

// Loads the rows of one round; js points at the round's kRB staged channel indices (LDS), -1 = empty slot.
// Every load is issued unconditionally (an empty slot or an out-of-range column reads the 16 bytes at `dummy`,
// one cached transaction per wave): with no branch around a load the compiler knows exactly how many loads are
// in flight and can wait for the older buffer alone instead of draining the prefetched one as well.
template <class V, int PER, bool GU, bool DN>
__device__ __forceinline__ void load_round(RoundBuf<V, PER> &rb, const typename V::vec_t *__restrict__ w, int nvec,
                                           const int *js, const int (&col)[PER], const bool (&ok)[PER],
                                           const typename V::vec_t *__restrict__ dummy)
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
                rb.g[t][q] = *(ld ? row + col[q] : dummy);
                rb.u[t][q] = *(ld ? row + nvec + col[q] : dummy);
            }
            if (DN) rb.dn[t][q] = *(ld ? row + 2 * nvec + col[q] : dummy);
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
// `after_dots` runs once the round's gate/up data has been consumed: the place to issue the next loads when the
// memory pipeline should hold about one round at a time (see kPrefetchEarly).
template <class V, int PER, class AfterDots>
__device__ __forceinline__ void round_hidden(const RoundBuf<V, PER> &rb, const typename V::vec_t (&xv)[PER],
                                             typename V::acc_t (*part)[kSelMaxWaves], int wave, int lane, int nw,
                                             float (&hv)[kRB], AfterDots after_dots)
{
    typedef typename V::acc_t acc_t;
    static_assert(2 * kRB * kSelMaxWaves == kWave, "one LDS word per lane in the cross-wave step");
    acc_t ag[kRB], au[kRB];
#pragma unroll
    for (int t = 0; t < kRB; ++t) {
        ag[t] = 0;
        au[t] = 0;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            ag[t] = V::dot(rb.g[t][q], xv[q], ag[t]);
            au[t] = V::dot(rb.u[t][q], xv[q], au[t]);
        }
    }
    asm volatile("" ::: "memory");  // keep the loads below behind the uses above
    after_dots();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int t = 0; t < kRB; ++t) {
        const acc_t gt = wave_total(ag[t]), ut = wave_total(au[t]);
        if (lane == 0) {
            part[2 * t][wave] = gt;
            part[2 * t + 1][wave] = ut;
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

__device__ __forceinline__ int coherent_load(const int *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void coherent_store(int *p, int v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void coherent_store(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 16-byte write-through store (device scope), p 16-byte aligned.  Not tracked by the compiler's wait counting:
// follow with an explicit wait before relying on it.
__device__ __forceinline__ void coherent_store4(float *p, float4 v)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 t = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(t) : "memory");
}
constexpr int kStage = 4096;  // floats of a partial output row staged in LDS at a time

constexpr int kBitsStride = 1024;                   // ints between the selection words of two workgroups
constexpr int kGoWord = 64;                          // offset of a workgroup's end-of-step "go" word from its selection word
constexpr int kBitsValid = 1 << 31;                  // set in selbits[b] once the selection of this step is known
constexpr int kMaxCandRounds = 30 / kRB;             // candidate slots of a workgroup must fit the other 31 bits

template <class V, int PER>
__global__ __launch_bounds__(1024) void decode_fused_kernel(FusedParams p)
{
    typedef typename V::vec_t vec_t;
    typedef typename V::acc_t acc_t;
    constexpr int E = V::kElems;
    __shared__ SelShared sh;
    __shared__ int s_flag, s_bits[2];
    __shared__ acc_t part[2][2 * kRB][kSelMaxWaves];
    __shared__ int j_a[kKeep + 2 * kRB], j_b[kKeep + 2 * kRB], j_d[kKeep + 2 * kRB];  // staged channel indices
    __shared__ float h_a[kKeep + 2 * kRB], h_b[kKeep + 2 * kRB];                      // their hidden activations
    __shared__ __attribute__((aligned(16))) float y_stage[kStage];  // single-launch step: partial row on its way out
    __shared__ int wg_bits[1024];                       // selector only: selected candidate slots per workgroup

    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int nw = blockDim.x / kWave;
    const int b = blockIdx.x, n_wg = gridDim.x, n_workers = n_wg - 1, wb = b - 1;
    const int nvec = p.nvec;
    const vec_t *w = reinterpret_cast<const vec_t *>(p.w);

    POP_STAMP(0);
    // end-of-step "go" word of this workgroup: all go words hold the same value between launches, and change once,
    // together, when the last workgroup of a single-launch step has delivered its partial output row
    int *const go = p.selbits + (size_t)b * kBitsStride + kGoWord;
    const int go_before = p.y ? coherent_load(go) : 0;
    if (b == 0 && tid == 0) coherent_store(&p.sync[3], 0);  // "some workgroup deferred its phase D share" flag of this step
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

    // rounds of this workgroup: round i of a list dealt to n_sh sharers = rows (i*n_sh + me)*kRB + t
    auto rounds_of = [](int n_list, int n_sh, int me) {
        return (me >= 0 && me * kRB < n_list) ? (n_list - me * kRB + n_sh * kRB - 1) / (n_sh * kRB) : 0;
    };
    const int n_a = rounds_of(p.n_cand, n_wg, b);
    const int n_a2 = (n_a + 1) & ~1;  // padded to even with an empty round (simplifies the ping-pong)
    const int n_b = rounds_of(p.n_ret, n_workers, wb);
    // staged with empty rounds (-1) behind the real ones, so the streaming loops can prefetch unconditionally
    const int n_b2 = (n_b + 1) & ~1;
    for (int e = tid; e < (n_a2 + 1) * kRB; e += blockDim.x) {
        const int r = ((e / kRB) * n_wg + b) * kRB + e % kRB;
        j_a[e] = (e / kRB < n_a && r < p.n_cand) ? p.cand_idx[r] : -1;
    }
    for (int e = tid; e < (n_b2 + 1) * kRB; e += blockDim.x) {
        const int r = ((e / kRB) * n_workers + wb) * kRB + e % kRB;
        j_b[e] = (e / kRB < n_b && r < p.n_ret) ? p.ret_idx[r] : -1;
    }
    const vec_t *dummy = reinterpret_cast<const vec_t *>(p.x);
    __syncthreads();

    RoundBuf<V, PER> buf_a, buf_b;  // ping-pong: one is reduced while the other's loads are in flight

    // No global store happens inside the streaming loops: a store would make the next wait drain every load
    // in flight, prefetched ones included.  Hidden activations are staged in LDS and written out later.

    // ---- phase A: this workgroup's candidate rounds (gate+up only)
    auto finish_a = [&](const RoundBuf<V, PER> &rb, int i, acc_t(*pt)[kSelMaxWaves]) {
        float hv[kRB];
        round_hidden<V, PER>(rb, xv, pt, wave, lane, nw, hv, [] {});
        if (tid == 0)
#pragma unroll
            for (int t = 0; t < kRB; ++t) h_a[i * kRB + t] = hv[t];
    };
    if (n_a2 > 0) load_round<V, PER, true, false>(buf_a, w, nvec, j_a, col, ok, dummy);
    for (int i = 0; i < n_a2; i += 2) {
        load_round<V, PER, true, false>(buf_b, w, nvec, j_a + (i + 1) * kRB, col, ok, dummy);
        finish_a(buf_a, i, part[0]);
        load_round<V, PER, true, false>(buf_a, w, nvec, j_a + (i + 2) * kRB, col, ok, dummy);  // maybe an empty round
        finish_a(buf_b, i + 1, part[1]);
    }
    __syncthreads();
    for (int e = tid; e < n_a * kRB; e += blockDim.x) {
        const int j = j_a[e];
        if (j >= 0) {
            // write-through stores: visible device-wide once acknowledged, so the hand-over below needs no
            // cache write-back (a full release fence also invalidates this XCD's L2 under the other workgroups'
            // streams; with one per workgroup that stalled the start of phase B for microseconds)
            const float hv = h_a[e];
            coherent_store(&p.h[j], hv);
            coherent_store(&p.cscore[((e / kRB) * n_wg + b) * kRB + e % kRB], p.nrm[j] * fabsf(hv));
        }
    }
    // Phase B's first round goes out now, behind the stores, so its latency overlaps the hand-over; the wait
    // below leaves exactly those loads outstanding (the counter retires in order), i.e. the stores are acknowledged.
    asm volatile("" ::: "memory");
    load_round<V, PER, true, true>(buf_a, w, nvec, j_b, col, ok, dummy);
    asm volatile("" ::: "memory");
    static_assert(kRB * 3 * PER == 6 || kRB * 3 * PER == 12, "literal in the wait below");
    if (PER == 1)
        asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    else
        asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
    __syncthreads();
    POP_STAMP(1);

    float acc[PER][8];
#pragma unroll
    for (int q = 0; q < PER; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[q][e] = 0.f;

    // Phase D of a workgroup: the down rows of those of its own candidates (slots of phase A, h still in LDS)
    // that the selection kept; `bits` has one bit per slot.
    auto phase_d = [&](int bits) {
        for (int e = tid; e < n_a2 * kRB; e += blockDim.x) j_d[e] = ((bits >> e) & 1) ? j_a[e] : -1;
        __syncthreads();
        for (int i = 0; i < n_a2; i += 2) {
            load_round<V, PER, false, true>(buf_a, w, nvec, j_d + i * kRB, col, ok, dummy);
            load_round<V, PER, false, true>(buf_b, w, nvec, j_d + (i + 1) * kRB, col, ok, dummy);
#pragma unroll
            for (int t = 0; t < kRB; ++t)
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    // an unselected slot read the dummy vector: its weight is zero
                    V::axpy(buf_a.j[t] >= 0 ? h_a[i * kRB + t] : 0.f, buf_a.dn[t][q], acc[q]);
                    V::axpy(buf_b.j[t] >= 0 ? h_a[(i + 1) * kRB + t] : 0.f, buf_b.dn[t][q], acc[q]);
                }
        }
    };
    auto store_partial = [&]() __attribute__((always_inline)) {
        float *dst = p.partial + (size_t)b * p.d;
        if (p.y) {
            // single-launch step: other workgroups read these rows in this launch, so write them through; staged
            // in LDS first so that each store instruction covers whole contiguous lines (a write-through store of
            // a few bytes per lane is one memory transaction per lane)
            for (int c0 = 0; c0 < p.d; c0 += kStage) {
#pragma unroll
                for (int q = 0; q < PER; ++q) {
                    const int o = col[q] * E - c0;
                    if (ok[q] && o >= 0 && o < kStage)
#pragma unroll
                        for (int e = 0; e < E; ++e) y_stage[o + e] = acc[q][e];
                }
                __syncthreads();
                const int n = min(kStage, p.d - c0);
                for (int v = tid * 4; v < n; v += blockDim.x * 4)
                    coherent_store4(dst + c0 + v, *reinterpret_cast<const float4 *>(&y_stage[v]));
                __syncthreads();
            }
            return;
        }
#pragma unroll
        for (int q = 0; q < PER; ++q)
            if (ok[q]) {
#pragma unroll
                for (int e = 0; e < E; e += 4)
                    *reinterpret_cast<float4 *>(dst + (size_t)col[q] * E + e) =
                        make_float4(acc[q][e], acc[q][e + 1], acc[q][e + 2], acc[q][e + 3]);
            }
    };
    // Single-launch step: once every workgroup's partial row is acknowledged device-wide (write-through stores,
    // counter wait, barrier, then one arrival per workgroup), each workgroup sums a slice of the d outputs over
    // all rows in a fixed order: 16 lanes take 16 adjacent outputs, the block's blockDim/16 lane groups take the
    // rows round robin, then a fixed tree over the groups.  The wait is bounded like the others; if it expires
    // the sticky error flag is raised and y is left unwritten.
    auto final_reduce = [&]() __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        // Arrival counter + one "go" word per workgroup (each in its own 4 KiB, next to its selection word): the
        // last workgroup to arrive rewinds the counter and changes all the go words, and every workgroup polls
        // only its own.  Hundreds of workgroups polling the one counter would queue up at a single memory
        // channel, in front of the last arrivals.  Nothing here depends on host-side state, so a captured launch
        // can be replayed.
        if (tid == 0) s_flag = atomicAdd(&p.sync[6], 1) == n_wg - 1 ? 1 : 0;
        __syncthreads();
        if (s_flag) {
            if (tid == 0) coherent_store(&p.sync[6], 0);
            for (int i = tid; i < n_wg; i += blockDim.x)
                coherent_store(p.selbits + (size_t)i * kBitsStride + kGoWord, go_before + 1);
        }
        __syncthreads();
        if (tid == 0) {
            bool all_in = false;
            for (int it = 0; !all_in && it < kSpinLimit; ++it) {
                all_in = coherent_load(go) != go_before;
                if (!all_in) __builtin_amdgcn_s_sleep(2);
            }
            if (!all_in) p.sync[2] = 1;
            s_flag = all_in ? 1 : 0;
        }
        __syncthreads();
        POP_STAMP(5);
        if (!s_flag) return;
        const bool whole = coherent_load(&p.sync[3]) == 0;  // some workgroup gave up waiting for the selection: y would miss its share
        float *red = reinterpret_cast<float *>(&sh.hist[0]);  // [waves][16]
        const int cpw = (p.d + n_wg - 1) / n_wg;
        const int c_lo = min(p.d, b * cpw), c_hi = min(p.d, c_lo + cpw);
        const int cc = tid % 16, g = tid / 16, ng = blockDim.x / 16;
        for (int c0 = c_lo; c0 < c_hi; c0 += 16) {
            const int c = c0 + cc;
            const bool in = c < c_hi;
            const float *src = p.partial + (in ? c : c_lo);
            float s = 0.f;
            int r = g;
            for (; r + 15 * ng < n_wg; r += 16 * ng) {  // all of a 256-row grid in one batch of independent loads
                float v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    v[u] = __hip_atomic_load(src + (size_t)(r + u * ng) * p.d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (int u = 0; u < 16; ++u) s += v[u];
            }
            for (; r < n_wg; r += ng)
                s += __hip_atomic_load(src + (size_t)r * p.d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s += __shfl_xor(s, 16, kWave);
            s += __shfl_xor(s, 32, kWave);
            if (lane < 16) red[wave * 16 + lane] = s;
            __syncthreads();
            if (tid < 16 && in && whole) {
                float v = 0.f;
                for (int wv = 0; wv < nw; ++wv) v += red[wv * 16 + tid];
                if (p.y_bf16)
                    reinterpret_cast<uint16_t *>(p.y)[c] = f32_to_bf16(v);
                else
                    reinterpret_cast<float *>(p.y)[c] = v;
            }
            __syncthreads();
        }
    };

    if (b == 0) {
        // ---- select (workgroup 0 only): wait for every other workgroup's phase A, then top-k
        if (tid == 0) {
            bool ok_a = spin_until(&p.sync[0], n_workers);
            if (!ok_a) p.sync[2] = 1;
            coherent_store(&p.sync[0], 0);  // all arrivals are in
            s_flag = ok_a ? 1 : 0;
        }
        for (int i = tid; i < n_wg; i += blockDim.x) wg_bits[i] = 0;
        __syncthreads();
        POP_STAMP(2);
        if (s_flag) {
            block_select_candidates<true>(
                p.cscore, p.cand_idx, p.n_cand, p.k, p.mask, p.active_idx + p.n_ret, sh,
                [&](int c) {  // candidate c was handled by workgroup (c/kRB) % n_wg in its round (c/kRB) / n_wg
                    const int rd = c / kRB;
                    atomicOr(&wg_bits[rd % n_wg], 1 << ((rd / n_wg) * kRB + c % kRB));
                },
                [&]() {  // publish the per-workgroup slot masks first: they are all the other workgroups wait for
                    __syncthreads();
                    for (int i = 1 + tid; i < n_wg; i += blockDim.x) coherent_store(&p.selbits[(size_t)i * kBitsStride], wg_bits[i] | kBitsValid);
                });
            if (tid == 0 && p.n_active) *p.n_active = p.n_ret + p.k;
            POP_STAMP(3);
            phase_d(wg_bits[0]);
        }
        store_partial();
        if (p.y) final_reduce();
        return;
    }

    if (tid == 0) atomicAdd(&p.sync[0], 1);  // every wave's results were acknowledged before the barrier above

    // ---- phase B: retained rounds (gate+up -> h, then the round's down rows).  Thread 0 polls this workgroup's
    // word of selbits along the way; a value is looked at two rounds after its load was issued, when it has
    // certainly arrived, so polling never stalls the stream.
    int pv0 = 0, pv1 = 0, pv2 = 0, my_bits = 0, hk = 0;
    auto finish_b = [&](const RoundBuf<V, PER> &rb, int i, acc_t(*pt)[kSelMaxWaves], auto poll_tag, auto late_load) {
        constexpr bool poll = decltype(poll_tag)::value;
        if (tid == 0) s_bits[hk & 1] = pv2;  // loaded at least two full rounds ago: certainly arrived, never a stall
        pv2 = pv1;
        pv1 = pv0;
        // every thread, no branch around the load; one poll per pair of rounds, each workgroup's word in its own
        // 4 KiB so that the polls of all workgroups do not queue up at one memory channel
        if (poll) pv0 = coherent_load(&p.selbits[(size_t)b * kBitsStride]);
        float hv[kRB];
        round_hidden<V, PER>(rb, xv, pt, wave, lane, nw, hv, late_load);
        // read after the round's barrier: every thread sees the same value; the slot is rewritten two rounds later
        if (!my_bits && (s_bits[hk & 1] & kBitsValid)) my_bits = s_bits[hk & 1];
        ++hk;
        if (tid == 0)
#pragma unroll
            for (int t = 0; t < kRB; ++t) h_b[i * kRB + t] = hv[t];
#pragma unroll
        for (int t = 0; t < kRB; ++t)
#pragma unroll
            for (int q = 0; q < PER; ++q) V::axpy(hv[t], rb.dn[t][q], acc[q]);
    };
    // kPrefetchEarly: the next round's loads go out before the current round's data is waited for (two rounds in
    // flight).  Otherwise they go out right after the current round's data has been consumed (about one round in
    // flight, the reduction and the barrier still overlap the load latency): measured faster on MI355X, whose
    // memory system loses throughput when the request queues get deeper.
    for (int i = 0; i < n_b2; i += 2) {  // buf_a already holds round 0 (loaded during the hand-over)
        if (i == 4) POP_STAMP(5);
        if (i == 8) POP_STAMP(7);
        if (kPrefetchEarly) {
            load_round<V, PER, true, true>(buf_b, w, nvec, j_b + (i + 1) * kRB, col, ok, dummy);
            finish_b(buf_a, i, part[0], std::true_type{}, [] {});
            load_round<V, PER, true, true>(buf_a, w, nvec, j_b + (i + 2) * kRB, col, ok, dummy);
            finish_b(buf_b, i + 1, part[1], std::false_type{}, [] {});
        } else {
            finish_b(buf_a, i, part[0], std::true_type{},
                     [&] { load_round<V, PER, true, true>(buf_b, w, nvec, j_b + (i + 1) * kRB, col, ok, dummy); });
            finish_b(buf_b, i + 1, part[1], std::false_type{},
                     [&] { load_round<V, PER, true, true>(buf_a, w, nvec, j_b + (i + 2) * kRB, col, ok, dummy); });
        }
    }
    POP_STAMP(2);

    // ---- phase D: needs the selection; normally my_bits arrived during phase B, else wait (bounded)
    int bits_final = my_bits;
    if (!my_bits) {
        if (tid == 0) {
            int v = pv2 < 0 ? pv2 : (pv1 < 0 ? pv1 : pv0);  // values still in the polling pipeline
            for (int it = 0; v >= 0 && it < kSpinLimit; ++it) {
                v = coherent_load(&p.selbits[(size_t)b * kBitsStride]);
                if (v >= 0) __builtin_amdgcn_s_sleep(2);
            }
            s_flag = v;
        }
        __syncthreads();
        bits_final = s_flag;
    }
    const bool d_ok = bits_final < 0;  // kBitsValid is the sign bit
    POP_STAMP(3);
    if (d_ok) phase_d(bits_final);
    POP_STAMP(4);
    store_partial();
    if (tid == 0) {
        p.deferred[b] = d_ok ? 0 : 1;
        if (d_ok) {
            coherent_store(&p.selbits[(size_t)b * kBitsStride], 0);  // rearmed for the next launch
        } else {
            p.sync[2] = 1;
            coherent_store(&p.sync[3], 1);
        }
    }
    for (int e = tid; e < n_b * kRB; e += blockDim.x)
        if (j_b[e] >= 0) p.h[j_b[e]] = h_b[e];
    if (p.y) final_reduce();
    POP_STAMP(6);
}

// y[o] = sum over workgroups (in order) of partial[b][o], plus shares a workgroup deferred.  A workgroup owns 64
// outputs; its 16 waves each sum a contiguous sixteenth of the partial rows (independent loads, fixed order)
// and wave 0 combines them in wave order, so y does not depend on scheduling.
constexpr int kTailWaves = 16;
__global__ __launch_bounds__(1024) void decode_tail_kernel(const float *__restrict__ partial, int n_wg, int d,
                                                           const int *__restrict__ deferred, const int *sync,
                                                           const int *__restrict__ selbits,
                                                           const int *__restrict__ cand_idx, int n_cand,
                                                           const float *__restrict__ h, const void *__restrict__ w,
                                                           int m, int is_bf16, void *__restrict__ y, int y_bf16)
{
    __shared__ float part[kTailWaves][kWave];
    const int lane = threadIdx.x % kWave, q = threadIdx.x / kWave;
    const int o = blockIdx.x * kWave + lane;
    const int per = (n_wg + kTailWaves - 1) / kTailWaves;
    const int s0 = min(n_wg, q * per), s1 = min(n_wg, q * per + per);
    float acc = 0.f;
    if (o < d) {
        int s = s0;
        for (; s + 16 <= s1; s += 16) {
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = partial[(size_t)(s + u) * d + o];
#pragma unroll
            for (int u = 0; u < 16; ++u) acc += v[u];
        }
        for (; s < s1; ++s) acc += partial[(size_t)s * d + o];
    }
    part[q][lane] = acc;
    __syncthreads();
    if (q == 0 && o < d) {
        float v = 0.f;
#pragma unroll
        for (int u = 0; u < kTailWaves; ++u) v += part[u][lane];
        const bool any_deferred = sync[3] != 0;  // set only when some workgroup gave up waiting in this step
        for (int b = 1; any_deferred && b < n_wg; ++b) {
            if (!deferred[b]) continue;
            // the workgroup's phase D share: its own candidate slots that the selection kept
            const int bits = selbits[(size_t)b * kBitsStride];
            if (bits >= 0) continue;  // the selection never ran: the step is flagged invalid
            for (int e = 0; e < 31; ++e) {
                if (!((bits >> e) & 1)) continue;
                const int c = ((e / kRB) * n_wg + b) * kRB + e % kRB;
                if (c >= n_cand) continue;
                const int j = cand_idx[c];
                if (j < 0 || j >= m) continue;
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
int fused_selbits_ints() { return 1024 * kBitsStride; }

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
    // the kernel stages at most kMaxRounds rounds per phase (the last candidate round may be padding)
    if ((n_ret + workers * kRB - 1) / (workers * kRB) > kMaxRounds) return false;
    if ((n_cand + (workers + 1) * kRB - 1) / ((workers + 1) * kRB) + 1 > kMaxCandRounds) return false;
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
                              const int *selbits, const int *cand_idx, int n_cand, const float *h, const void *w,
                              int m, int is_bf16, void *y, int y_bf16, hipStream_t s)
{
    hipLaunchKernelGGL(decode_tail_kernel, dim3((d + kWave - 1) / kWave), dim3(kTailWaves * kWave), 0, s, partial, n_wg, d, deferred,
                       sync, selbits, cand_idx, n_cand, h, w, m, is_bf16, y, y_bf16);
    return hipGetLastError();
}

}  // namespace pop
