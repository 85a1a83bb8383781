// Decode-step GEMVs over gathered channel rows (Sec. 3.4 two-step decoding), batch-general form.  Both are
// HBM-bandwidth bound: every weight byte of an active channel is read exactly once per step with 128-bit
// loads, contiguous per channel thanks to the channel-major layout w[j] = [gate | up | down].  The single-
// sequence decode step uses the fused kernel in pop_decode_fused.hip instead.
//
//   gateup: for each listed channel j and each of the B sequences,
//           h[b][j] = silu(x_b . W_gate[j,:]) * (x_b . W_up[j,:]); the first n_score listed channels (the
//           candidates) also get their step score I_j(t) = n_j * |h[b][j]| (Eq. 3 with a single token).
//   down:   y[b][:] = sum over listed j of h[b][j] * W_down[:, j], optionally masked per sequence.
//
// A wave owns a whole row at a time (gateup) or a 64-vector column chunk of a slab of rows (down); lanes
// stride the row in 16-byte vectors, so each wave-level load instruction fetches 1 KiB of contiguous HBM.
#include "pop_select_dev.h"
#include "pop_vec.h"

namespace pop {

// ---------------------------------------------------------------- gate/up GEMV
constexpr int kGuUnroll = 8;  // 16-byte loads per matrix in flight per lane within one group

// One listed channel j (list position p), one wave: h[b][j] = silu(x_b . gate_j) * (x_b . up_j) for the B sequences
// whose x is staged in LDS (xs [B][nvec]); positions p < n_score also get their step score.  kCoherent: the scores
// are written through, for workgroups of the same launch to read.
template <class V, int B, bool kCoherent>
__device__ __forceinline__ void gateup_row(const typename V::vec_t *__restrict__ w, int nvec,
                                           const typename V::vec_t *xs, int j, int p, int lane, float *__restrict__ h,
                                           int m, const float *__restrict__ nrm, float *cscore, int cs_stride,
                                           int n_score)
{
    typedef typename V::vec_t vec_t;
    // (many sequences: fewer row vectors in flight per lane, so that the sequences' accumulators stay in registers)
    constexpr int U = B >= 5 ? kGuUnroll / 2 : kGuUnroll;
    const int group = kWave * U;
    const int nvec_full = nvec / group * group;
    const vec_t *g = w + (size_t)j * 3 * nvec;
    const vec_t *u = g + nvec;
    // Two 16-byte vectors' products (sixteen exact products for bf16 rows) are summed in the row's accumulator type,
    // the pairs of a lane and then the lanes in double: a long float32 chain would round every add at the magnitude
    // of the largest product met so far, and so would a float32 tree over the lanes.
    static_assert(U % 2 == 0, "vectors are taken in pairs");
    double ag[B], au[B];
#pragma unroll
    for (int b = 0; b < B; ++b) ag[b] = au[b] = 0.0;

    for (int c0 = 0; c0 < nvec_full; c0 += group) {
        vec_t wg[U], wu[U];
#pragma unroll
        for (int q = 0; q < U; ++q) {
            wg[q] = g[c0 + q * kWave + lane];
            wu[q] = u[c0 + q * kWave + lane];
        }
#pragma unroll
        for (int q = 0; q < U; q += 2) {
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const vec_t x0 = xs[b * nvec + c0 + q * kWave + lane], x1 = xs[b * nvec + c0 + (q + 1) * kWave + lane];
                ag[b] += (double)V::dot(wg[q + 1], x1, V::dot(wg[q], x0, (typename V::acc_t)0));
                au[b] += (double)V::dot(wu[q + 1], x1, V::dot(wu[q], x0, (typename V::acc_t)0));
            }
        }
    }
    for (int c = nvec_full + lane; c < nvec; c += kWave) {
        vec_t wg = g[c], wu = u[c];
#pragma unroll
        for (int b = 0; b < B; ++b) {
            vec_t xv = xs[b * nvec + c];
            ag[b] += (double)V::dot(wg, xv, (typename V::acc_t)0);
            au[b] += (double)V::dot(wu, xv, (typename V::acc_t)0);
        }
    }
    // Lanes: four values at a time (gate and up sums of two sequences) through halving exchanges inside the rows of
    // 16 lanes, then across the four rows; lanes 0 and 1 end up with the gate sums of the two sequences and fetch
    // the matching up sums from lanes 2 and 3.
#pragma unroll
    for (int b0 = 0; b0 < B; b0 += 2) {
        const double v4[4] = {ag[b0], au[b0], b0 + 1 < B ? ag[b0 + 1] : 0.0, b0 + 1 < B ? au[b0 + 1] : 0.0};
        double z = butterfly4_row_sum(v4, lane);
        z += __shfl_xor(z, 16, kWave);
        z += __shfl_xor(z, 32, kWave);
        const double zu = dpp_move<0x4E>(z);  // quad_perm 2,3,0,1
        const int b = b0 + lane;
        if (lane < 2 && b < B) {
            const float hv = silu_mul((float)z, (float)zu);
            h[(size_t)b * m + j] = hv;
            if (p < n_score) {
                const float sc = nrm[j] * fabsf(hv);
                if (kCoherent)
                    coherent_store(&cscore[(size_t)b * cs_stride + p], sc);
                else
                    cscore[(size_t)b * cs_stride + p] = sc;
            }
        }
    }
}

template <class V, int B>
__global__ __launch_bounds__(1024) void gateup_kernel(const typename V::vec_t *__restrict__ w, int nvec,
                                                     const typename V::vec_t *__restrict__ x,
                                                     const int *__restrict__ rows, int n_rows,
                                                     const int *__restrict__ n_rows_dev, float *__restrict__ h, int m,
                                                     const float *__restrict__ nrm, float *__restrict__ cscore,
                                                     int cs_stride, int n_score)
{
    typedef typename V::vec_t vec_t;
    extern __shared__ uint4 xs_raw[];
    vec_t *xs = reinterpret_cast<vec_t *>(xs_raw);  // [B][nvec]
    for (int i = threadIdx.x; i < B * nvec; i += blockDim.x) xs[i] = x[i];
    __syncthreads();

    const int n = n_rows_dev ? *n_rows_dev : n_rows;
    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int n_waves = gridDim.x * (blockDim.x / kWave);

    for (int p = blockIdx.x * (blockDim.x / kWave) + wave; p < n; p += n_waves)
        gateup_row<V, B, false>(w, nvec, xs, rows[p], p, lane, h, m, nrm, cscore, cs_stride, n_score);
}

// Batched decode with the selection inside: rows = candidates (n_cand) then retained channels (n_ret).  All but
// the last B workgroups evaluate the rows, candidates first, and signal an arrival once their candidate scores are
// acknowledged.  The last B workgroups wait, bounded, for all arrivals and run one sequence's top-k each, the last of
// them also the union of the selections, while the others go on with the retained channels: the selection costs
// no time of its own.  All workgroups are resident (at most one per compute unit is launched), so the wait ends;
// if it ever expires the error flag is raised and the step's selection is not made.
// The arrival counter is never rewound: a second word holds the arrivals expected before this launch, the selectors
// wait for that plus this launch's workers, and the last selector moves the word on.  Every worker arrives exactly
// once before the launch ends, whether or not a selector was still waiting for it, so the two words agree again
// at the start of the next launch whatever happened in this one.
struct GateupSelectArgs {
    const int *cand_idx;
    int n_cand, n_ret;
    BatchK k;
    int act_stride;
    unsigned char *mask;
    int *active_idx, *n_active;
    unsigned char *selflag;
    int *union_list, *n_union;
    int *counters;  // [0] arrivals (ever growing), [1] selectors done, [2] arrivals expected before this launch
    int *err_flag;
    int spin_limit;  // looks a selector's wait takes before it gives up
};

template <class V, int B>
__global__ __launch_bounds__(1024) void gateup_select_kernel(const typename V::vec_t *__restrict__ w, int nvec,
                                                            const typename V::vec_t *__restrict__ x,
                                                            const int *__restrict__ rows, float *__restrict__ h, int m,
                                                            const float *__restrict__ nrm, float *cscore, int cs_stride,
                                                            GateupSelectArgs sa)
{
    typedef typename V::vec_t vec_t;
    extern __shared__ uint4 xs_raw[];
    __shared__ SelShared sh;
    __shared__ int s_flag;
    vec_t *xs = reinterpret_cast<vec_t *>(xs_raw);  // [B][nvec]
    for (int i = threadIdx.x; i < B * nvec; i += blockDim.x) xs[i] = x[i];
    __syncthreads();

    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int wpb = blockDim.x / kWave, n_wg = gridDim.x;
    const int n_cand = sa.n_cand, n = sa.n_cand + sa.n_ret;

    const int n_work = n_wg - B;  // workgroups that evaluate rows; the last B select
    if ((int)blockIdx.x < n_work) {
        // Rows are dealt to the waves of the working workgroups in list order, candidates first.  A workgroup
        // signals its arrival after its last round that holds a candidate (at once if it has none): its scores are
        // then acknowledged (write-through stores, counter wait, barrier).
        const int wg = blockIdx.x, stride = n_work * wpb;
        const int cand_rounds = wg * wpb < n_cand ? (n_cand - wg * wpb + stride - 1) / stride : 0;
        if (cand_rounds == 0 && threadIdx.x == 0) atomicAdd(&sa.counters[0], 1);
        for (int it = 0; it * stride + wg * wpb < n; ++it) {
            const int p = it * stride + wg * wpb + wave;
            if (p < n_cand)
                gateup_row<V, B, true>(w, nvec, xs, rows[p], p, lane, h, m, nrm, cscore, cs_stride, n_cand);
            else if (p < n)
                gateup_row<V, B, false>(w, nvec, xs, rows[p], p, lane, h, m, nrm, cscore, cs_stride, n_cand);
            if (it == cand_rounds - 1) {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's scores are acknowledged
                __syncthreads();
                if (threadIdx.x == 0) atomicAdd(&sa.counters[0], 1);
            }
        }
        return;
    }

    const int b = blockIdx.x - n_work;  // this workgroup selects for sequence b
    const int target = sa.counters[2] + n_work;  // (written by the previous launch: an ordinary load)
    if (threadIdx.x == 0) {
        const bool ok = spin_until(&sa.counters[0], target, sa.spin_limit);
        if (!ok) *sa.err_flag = 1;
        s_flag = ok ? 1 : 0;
    }
    __syncthreads();
    if (s_flag) {
        block_select_candidates<true, SelectNoHook, SelectNoHook, true>(
            cscore + (size_t)b * cs_stride, sa.cand_idx, n_cand, sa.k.k[b], sa.mask + (size_t)b * m,
            sa.active_idx + (size_t)b * sa.act_stride + sa.n_ret, sh, SelectNoHook(), SelectNoHook(), nullptr,
            sa.selflag + b, POP_MAX_BATCH);
        if (threadIdx.x == 0) sa.n_active[b] = sa.n_ret + sa.k.k[b];
    }
    // The flags went out as write-through stores; once they are acknowledged the selector signs off.  The last
    // selector to do so reads every sequence's flags (coherent loads): union of the selections, counters rewound.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) s_flag = atomicAdd(&sa.counters[1], 1) == B - 1;
    __syncthreads();
    if (!s_flag) return;
    static_assert(POP_MAX_BATCH == 8, "one 64-bit word of flags per candidate position");
    const unsigned long long live = B >= 8 ? ~0ull : ((1ull << (8 * B)) - 1ull);
    const unsigned long long *flags = reinterpret_cast<const unsigned long long *>(sa.selflag);
    // this thread's candidate positions: flags and channel numbers requested together
    constexpr int kPre = 4;
    const int E = (n_cand + blockDim.x - 1) / blockDim.x;
    const int lo = min(n_cand, (int)threadIdx.x * E), hi = min(n_cand, lo + E);
    unsigned long long fpre[kPre];
    int jpre[kPre];
#pragma unroll
    for (int u = 0; u < kPre; ++u) {
        fpre[u] = lo + u < hi ? coherent_load(&flags[lo + u]) & live : 0ull;
        jpre[u] = lo + u < hi ? sa.cand_idx[lo + u] : 0;
    }
    int c[1] = {0}, tot[1];
#pragma unroll
    for (int u = 0; u < kPre; ++u) c[0] += fpre[u] != 0;
    for (int i = lo + kPre; i < hi; ++i) c[0] += (coherent_load(&flags[i]) & live) != 0;
    block_excl_scan<1>(c, tot, sh);
    int pos = sa.n_ret + c[0];
#pragma unroll
    for (int u = 0; u < kPre; ++u)
        if (fpre[u] != 0) sa.union_list[pos++] = jpre[u];
    for (int i = lo + kPre; i < hi; ++i)
        if ((coherent_load(&flags[i]) & live) != 0) sa.union_list[pos++] = sa.cand_idx[i];
    if (threadIdx.x == 0) {
        *sa.n_union = sa.n_ret + tot[0];
        sa.counters[1] = 0;
        sa.counters[2] = target;
    }
}

template <class V>
static hipError_t gateup_dispatch(const void *w, int nvec, const void *x, int B, const int *rows, int n_rows,
                                  const int *n_rows_dev, float *h, int m, const float *nrm, float *cscore, int cs_stride,
                                  int n_score, int n_cu, hipStream_t s)
{
    typedef typename V::vec_t vec_t;
    if (n_rows <= 0) return hipSuccess;
    // x is staged in LDS by every workgroup: with several sequences it fills most of it, so one large workgroup
    // per compute unit (16 waves sharing the copy) takes the place of many small ones
    size_t lds = (size_t)B * nvec * sizeof(vec_t);
    const int threads = lds > 16 * 1024 ? 1024 : 256;
    const int wpb = threads / kWave;
    int blocks = (n_rows + wpb - 1) / wpb;
    const int cap = threads == 1024 ? n_cu : 1024;
    if (blocks > cap) blocks = cap;
#define POP_GU(BB)                                                                                                  \
    case BB:                                                                                                        \
        if (lds > 48 * 1024) {                                                                                      \
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gateup_kernel<V, BB>),               \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);               \
            if (e != hipSuccess) return e;                                                                          \
        }                                                                                                           \
        hipLaunchKernelGGL((gateup_kernel<V, BB>), dim3(blocks), dim3(threads), lds, s, (const vec_t *)w, nvec,          \
                           (const vec_t *)x, rows, n_rows, n_rows_dev, h, m, nrm, cscore, cs_stride, n_score);       \
        break;
    switch (B) {
        POP_GU(1) POP_GU(2) POP_GU(3) POP_GU(4) POP_GU(5) POP_GU(6) POP_GU(7) POP_GU(8)
        default: return hipErrorInvalidValue;
    }
#undef POP_GU
    return hipGetLastError();
}

hipError_t launch_gateup(const void *w, int is_bf16, int d, int m, const void *x, int B, const int *rows, int n_rows,
                         const int *n_rows_dev, float *h, const float *nrm, float *cscore, int cs_stride, int n_score,
                         int n_cu, hipStream_t s)
{
    if (is_bf16)
        return gateup_dispatch<VecBF16>(w, d / 8, x, B, rows, n_rows, n_rows_dev, h, m, nrm, cscore, cs_stride,
                                        n_score, n_cu, s);
    return gateup_dispatch<VecF32>(w, d / 4, x, B, rows, n_rows, n_rows_dev, h, m, nrm, cscore, cs_stride, n_score,
                                   n_cu, s);
}

template <class V>
static hipError_t gateup_select_dispatch(const void *w, int nvec, const void *x, int B, const int *rows, float *h, int m,
                                         const float *nrm, float *cscore, int cs_stride, const GateupSelectArgs &sa,
                                         int n_cu, bool *fused, hipStream_t s)
{
    typedef typename V::vec_t vec_t;
    *fused = false;
    const int n_rows = sa.n_cand + sa.n_ret, threads = 1024, wpb = threads / kWave;
    const size_t lds = (size_t)B * nvec * sizeof(vec_t);
    int blocks = (n_rows + wpb - 1) / wpb;
    if (blocks > n_cu) blocks = n_cu;
    if (B < 2 || blocks < 2 * B || sa.n_cand < 1) return hipSuccess;  // too small to set workgroups aside
#define POP_GS(BB)                                                                                                  \
    case BB: {                                                                                                      \
        const void *fn = reinterpret_cast<const void *>(&gateup_select_kernel<V, BB>);                               \
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                \
        if (e != hipSuccess) return e;                                                                               \
        int per_cu = 0;                                                                                              \
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, gateup_select_kernel<V, BB>, threads, lds);        \
        if (e != hipSuccess) return e;                                                                               \
        if (per_cu < 1) return hipSuccess; /* not resident: the caller uses the two-launch form */                   \
        hipLaunchKernelGGL((gateup_select_kernel<V, BB>), dim3(blocks), dim3(threads), lds, s, (const vec_t *)w,     \
                           nvec, (const vec_t *)x, rows, h, m, nrm, cscore, cs_stride, sa);                          \
        break;                                                                                                       \
    }
    switch (B) {
        POP_GS(2) POP_GS(3) POP_GS(4) POP_GS(5) POP_GS(6) POP_GS(7) POP_GS(8)
        default: return hipErrorInvalidValue;
    }
#undef POP_GS
    *fused = true;
    return hipGetLastError();
}

hipError_t launch_gateup_select(const void *w, int is_bf16, int d, int m, const void *x, int B, const int *rows,
                                float *h, const float *nrm, float *cscore, int cs_stride, const int *cand_idx,
                                int n_cand, int n_ret, BatchK k, int act_stride, unsigned char *mask, int *active_idx,
                                int *n_active, unsigned char *selflag, int *union_list, int *n_union, int *counters,
                                int *err_flag, int spin_limit, int n_cu, bool *fused, hipStream_t s)
{
    GateupSelectArgs sa = {cand_idx, n_cand, n_ret, k, act_stride, mask, active_idx, n_active, selflag,
                           union_list, n_union, counters, err_flag, spin_limit};
    if (is_bf16)
        return gateup_select_dispatch<VecBF16>(w, d / 8, x, B, rows, h, m, nrm, cscore, cs_stride, sa, n_cu, fused, s);
    return gateup_select_dispatch<VecF32>(w, d / 4, x, B, rows, h, m, nrm, cscore, cs_stride, sa, n_cu, fused, s);
}

// ---------------------------------------------------------------- down projection
// grid = (column chunks of 64 vectors, slabs).  A workgroup first stages its slab's channel list and the B
// sequences' hidden activations of those channels (zeroed where a sequence's mask excludes the channel) in LDS,
// with independent loads, so that the streaming loop touches global memory for weight rows only.  The 4 waves
// then split the slab's rows, keep float32 accumulators for their 64-vector column chunk, and are combined
// through LDS in wave order; the slab partials are then summed in slab order by down_reduce_kernel, so y does
// not depend on scheduling.
constexpr int kDownUnroll = 8;
constexpr int kDownSlabRows = 256;  // rows of a slab staged at a time

template <class V, int B>
__global__ __launch_bounds__(256) void down_kernel(const typename V::vec_t *__restrict__ w, int nvec,
                                                   const int *__restrict__ list, int n_host,
                                                   const int *__restrict__ n_dev, const float *__restrict__ h, int m,
                                                   const unsigned char *__restrict__ mask, int mask_stride,
                                                   float *__restrict__ partial, int d)
{
    typedef typename V::vec_t vec_t;
    constexpr int E = V::kElems;
    __shared__ float red[3][kWave * 8];
    __shared__ int js[kDownSlabRows];
    __shared__ float hs[B][kDownSlabRows];
    const int n = n_dev ? *n_dev : n_host;
    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int n_slabs = gridDim.y, slab = blockIdx.y;
    const int col = blockIdx.x * kWave + lane;  // vector column
    const bool col_ok = col < nvec;
    const int per_slab = (n + n_slabs - 1) / n_slabs;
    const int s0 = min(n, slab * per_slab), s1 = min(n, s0 + per_slab);

    float acc[B][8];
#pragma unroll
    for (int b = 0; b < B; ++b)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[b][e] = 0.f;

    for (int c0 = s0; c0 < s1; c0 += kDownSlabRows) {
        const int nc = min(kDownSlabRows, s1 - c0);
        __syncthreads();  // the previous chunk's readers are done
        for (int i = threadIdx.x; i < nc; i += blockDim.x) {
            const int j = list[c0 + i];
            js[i] = j;
            float hv[B];
            unsigned char mk[B];
#pragma unroll
            for (int b = 0; b < B; ++b) {
                hv[b] = h[(size_t)b * m + j];
                mk[b] = mask ? mask[(size_t)b * mask_stride + j] : (unsigned char)1;
            }
#pragma unroll
            for (int b = 0; b < B; ++b) hs[b][i] = mk[b] ? hv[b] : 0.f;
        }
        __syncthreads();
        // rows of this wave within the chunk
        const int per_wave = (nc + 3) / 4;
        const int r0 = min(nc, wave * per_wave), r1 = min(nc, r0 + per_wave);
        int i = r0;
        for (; i + kDownUnroll <= r1; i += kDownUnroll) {
            vec_t wv[kDownUnroll];
#pragma unroll
            for (int q = 0; q < kDownUnroll; ++q)
                wv[q] = col_ok ? w[((size_t)js[i + q] * 3 + 2) * nvec + col] : V::zero();
#pragma unroll
            for (int q = 0; q < kDownUnroll; ++q)
#pragma unroll
                for (int b = 0; b < B; ++b) V::axpy(hs[b][i + q], wv[q], acc[b]);
        }
        for (; i < r1; ++i) {
            const vec_t wv1 = col_ok ? w[((size_t)js[i] * 3 + 2) * nvec + col] : V::zero();
#pragma unroll
            for (int b = 0; b < B; ++b) V::axpy(hs[b][i], wv1, acc[b]);
        }
    }

    // combine the 4 waves in wave order, one sequence at a time
#pragma unroll
    for (int b = 0; b < B; ++b) {
        __syncthreads();
        if (wave > 0) {
#pragma unroll
            for (int e = 0; e < E; ++e) red[wave - 1][e * kWave + lane] = acc[b][e];
        }
        __syncthreads();
        if (wave == 0 && col_ok) {
            float *dst = partial + ((size_t)slab * B + b) * d + (size_t)col * E;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                float v = acc[b][e];
                v += red[0][e * kWave + lane];
                v += red[1][e * kWave + lane];
                v += red[2][e * kWave + lane];
                dst[e] = v;
            }
        }
    }
}

// y[b][o] = sum over slabs of partial[slab][b][o]; total = B*d outputs.  A workgroup owns 64 outputs; its 4
// waves each sum a contiguous quarter of the slabs (independent loads, added in slab order) and are combined in
// wave order, so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void down_reduce_kernel(const float *__restrict__ partial, int n_slabs, int total,
                                                          void *__restrict__ y, int y_bf16)
{
    __shared__ float part[4][kWave];
    const int lane = threadIdx.x % kWave, q = threadIdx.x / kWave;
    const int i = blockIdx.x * kWave + lane;
    const int per = (n_slabs + 3) / 4, s0 = min(n_slabs, q * per), s1 = min(n_slabs, s0 + per);
    float acc = 0.f;
    if (i < total) {
        int s = s0;
        for (; s + 8 <= s1; s += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = partial[(size_t)(s + u) * total + i];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; s < s1; ++s) acc += partial[(size_t)s * total + i];
    }
    part[q][lane] = acc;
    __syncthreads();
    if (q == 0 && i < total) {
        float v = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
        if (y_bf16)
            ((uint16_t *)y)[i] = f32_to_bf16(v);
        else
            ((float *)y)[i] = v;
    }
}

template <class V>
static hipError_t down_dispatch(const void *w, int nvec, int d, int m, const int *list, const int *n_dev, int n_host,
                                const float *h, const unsigned char *mask, int mask_stride, int B, float *partial,
                                int n_slabs, void *y, int y_bf16, hipStream_t s)
{
    typedef typename V::vec_t vec_t;
    dim3 grid((nvec + kWave - 1) / kWave, n_slabs);
#define POP_DN(BB)                                                                                                  \
    case BB:                                                                                                        \
        hipLaunchKernelGGL((down_kernel<V, BB>), grid, dim3(256), 0, s, (const vec_t *)w, nvec, list, n_host,        \
                           n_dev, h, m, mask, mask_stride, partial, d);                                              \
        break;
    switch (B) {
        POP_DN(1) POP_DN(2) POP_DN(3) POP_DN(4) POP_DN(5) POP_DN(6) POP_DN(7) POP_DN(8)
        default: return hipErrorInvalidValue;
    }
#undef POP_DN
    int total = B * d;
    hipLaunchKernelGGL(down_reduce_kernel, dim3((total + kWave - 1) / kWave), dim3(256), 0, s, partial, n_slabs, total,
                       y, y_bf16);
    return hipGetLastError();
}

int down_num_slabs(int d, int is_bf16)
{
    int nvec = d / (is_bf16 ? 8 : 4);
    int chunks = (nvec + kWave - 1) / kWave;
    int slabs = (512 + chunks - 1) / chunks;  // about 512 workgroups = 2048 waves
    if (slabs < 1) slabs = 1;
    if (slabs > 256) slabs = 256;
    return slabs;
}

hipError_t launch_down(const void *w, int is_bf16, int d, int m, const int *list, const int *n_dev, int n_host,
                       const float *h, const unsigned char *mask, int mask_stride, int B, float *partial, int n_slabs,
                       void *y, int y_bf16, hipStream_t s)
{
    if (is_bf16)
        return down_dispatch<VecBF16>(w, d / 8, d, m, list, n_dev, n_host, h, mask, mask_stride, B, partial, n_slabs,
                                      y, y_bf16, s);
    return down_dispatch<VecF32>(w, d / 4, d, m, list, n_dev, n_host, h, mask, mask_stride, B, partial, n_slabs, y,
                                 y_bf16, s);
}

}  // namespace pop
