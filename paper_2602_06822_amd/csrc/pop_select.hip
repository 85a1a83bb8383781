// Rank-based selection kernels: the three-region partition at prefill (Sec. 3.3 "Prefilling Stage"), the
// per-step candidate top-k (Sec. 3.3 "Decoding Stage") and the index-list compactions around them.
//
// All selections use one strict total order on channels: higher score first, equal scores by lower channel
// index.  Scores are mapped to order-preserving 32-bit keys; an MSB-first radix select over four 8-bit digits
// finds the key of the n-th best element, and a block scan in index order admits elements equal to that key
// until the count is exact.  One workgroup handles one selection, so the result is deterministic.
#include "pop_select_dev.h"

namespace pop {

// ---------------------------------------------------------------- three-region partition
// The keys are staged in LDS once (eight independent loads in flight per thread), so the radix passes and the
// index-ordered passes never go back to memory; beyond kPartLdsKeys channels they are read from global memory.
constexpr int kPartLdsKeys = 24576;  // 96 KiB of keys

// Index-ordered passes of the partition: thread t owns channels [t*E, (t+1)*E).  A channel above a threshold key is
// in; one equal to it is in while fewer than `take` equal ones precede it.  So with the numbers of greater and of
// equal channels before a thread's range (one scan of 2 NT streams) every channel's region and list position follow
// directly.  NT = 3 also emits the channels within the third threshold: a byte mask, their ascending list, its length.
template <int NT, class KeyFn>
__device__ __forceinline__ void partition_emit(KeyFn key, int m, const uint32_t (&kth)[3], const int (&take)[3],
                                               unsigned char *__restrict__ region, int *__restrict__ ret_idx,
                                               int *__restrict__ cand_idx, const PartitionExtra &ex, SelShared &sh)
{
    const int E = (m + blockDim.x - 1) / blockDim.x;
    const int lo = min(m, (int)threadIdx.x * E), hi = min(m, lo + E);
    int cnt[2 * NT], tot[2 * NT];  // per threshold: greater than its key, equal to it
#pragma unroll
    for (int q = 0; q < 2 * NT; ++q) cnt[q] = 0;
    for (int j = lo; j < hi; ++j) {
        const uint32_t k = key(j);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            cnt[2 * t] += (k > kth[t]);
            cnt[2 * t + 1] += (k == kth[t]);
        }
    }
    block_excl_scan<2 * NT>(cnt, tot, sh);
    for (int j = lo; j < hi; ++j) {
        const uint32_t k = key(j);
        bool in[NT];
        int before[NT];  // channels within threshold t before this one
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            in[t] = (k > kth[t]) || (k == kth[t] && cnt[2 * t + 1] < take[t]);
            before[t] = cnt[2 * t] + min(cnt[2 * t + 1], take[t]);
            cnt[2 * t] += (k > kth[t]);
            cnt[2 * t + 1] += (k == kth[t]);
        }
        if (region) region[j] = in[0] ? POP_REGION_RETAINED : (in[1] ? POP_REGION_CANDIDATE : POP_REGION_PRUNED);
        if (in[0]) {
            if (ret_idx) ret_idx[before[0]] = j;
        } else if (in[1]) {
            if (cand_idx) cand_idx[before[1] - before[0]] = j;
        }
        if (NT == 3) {
            if (ex.top_mask) ex.top_mask[j] = in[NT - 1] ? 1 : 0;
            if (in[NT - 1]) ex.top_list[before[NT - 1]] = j;
        }
    }
    if (NT == 3 && threadIdx.x == 0 && ex.top_count) *ex.top_count = ex.n_top;
}

__global__ __launch_bounds__(1024) void partition_kernel(const float *__restrict__ scores, int m, int n_ret, int n_cand,
                                                         unsigned char *__restrict__ region, int *__restrict__ ret_idx,
                                                         int *__restrict__ cand_idx, PartitionExtra ex)
{
    __shared__ SelShared sh;
    extern __shared__ uint32_t part_keys[];  // [m] when m <= kPartLdsKeys
    const bool in_lds = m <= kPartLdsKeys;
#ifdef POP_TRACE
#define POP_PSTAMP(slot)                                                          \
    do {                                                                          \
        if (ex.trace && threadIdx.x == 0) ex.trace[slot] = wall_clock64();        \
    } while (0)
#else
#define POP_PSTAMP(slot) \
    do {                 \
    } while (0)
#endif
    POP_PSTAMP(0);
    if (ex.sync && threadIdx.x < ex.n_sync) ex.sync[threadIdx.x] = 0;
    // while the keys pass through registers: the bits set in any key and the bits clear in any key (the radix select
    // starts below the leading bits that all keys share)
    __shared__ uint32_t key_or, key_nand;
    uint32_t my_or = 0, my_nand = 0;
    if (in_lds) {
        if (threadIdx.x == 0) key_or = key_nand = 0;
        __syncthreads();
    }
    if (in_lds && ex.s2_part) {
        // scores straight from the prefill kernel's partial rows (Eq. 3), kept for the caller as well
        for (int base = 0; base < m; base += 4 * blockDim.x) {
            double acc[4] = {0.0, 0.0, 0.0, 0.0};
            float nr[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + u * blockDim.x + threadIdx.x;
                nr[u] = ex.nrm[i < m ? i : 0];
            }
            for (int t = 0; t < ex.n_tiles; ++t) {
                float v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = base + u * blockDim.x + threadIdx.x;
                    v[u] = ex.s2_part[(size_t)t * m + (i < m ? i : 0)];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) acc[u] += (double)v[u];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = base + u * blockDim.x + threadIdx.x;
                if (i < m) {
                    const float sc = (float)((double)nr[u] * sqrt(acc[u]));
                    ex.scores_out[i] = sc;
                    const uint32_t k = score_key(sc);
                    part_keys[i] = k;
                    my_or |= k, my_nand |= ~k;
                }
            }
        }
    } else if (in_lds) {
        constexpr int kLoads = 12;  // scores requested together per thread (11008 channels: one pass)
        for (int base = 0; base < m; base += kLoads * blockDim.x) {
            float v[kLoads];
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int i = base + u * blockDim.x + threadIdx.x;
                v[u] = scores[i < m ? i : 0];
            }
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int i = base + u * blockDim.x + threadIdx.x;
                if (i < m) {
                    const uint32_t k = score_key(v[u]);
                    part_keys[i] = k;
                    my_or |= k, my_nand |= ~k;
                }
            }
        }
    }
    if (in_lds) {
        my_or = wave_or_rows(my_or), my_nand = wave_or_rows(my_nand);
        if (threadIdx.x % 16 == 0) {
            atomicOr(&key_or, my_or);
            atomicOr(&key_nand, my_nand);
        }
        __syncthreads();
    }
    POP_PSTAMP(1);
    auto key = [&](int i) { return in_lds ? part_keys[i] : score_key(scores[i]); };
    // thresholds: retained (rank n_ret), retained + candidate (rank n_ret + n_cand) and, on request, the n_top best
    // channels.  An empty set is sought as a set of one and then closed (key above all keys, nothing taken).
    const bool top = ex.top_list != nullptr;
    uint32_t kth[3] = {0xffffffffu, 0xffffffffu, 0xffffffffu};
    int take[3] = {0, 0, 0};
    const uint32_t diff = in_lds ? key_or & key_nand : 0u;
    if (top) {
        const int cnt[3] = {max(n_ret, 1), max(n_ret + n_cand, 1), max(ex.n_top, 1)};
        radix_thresholds_lists<3>(key, m, cnt, sh, kth, take, in_lds, diff);
    } else {
        const int cnt[2] = {max(n_ret, 1), max(n_ret + n_cand, 1)};
        uint32_t kth2[2];
        int take2[2];
#ifdef POP_TRACE
        radix_thresholds_lists<2>(key, m, cnt, sh, kth2, take2, in_lds, diff, ex.trace ? ex.trace + 4 : nullptr);
#else
        radix_thresholds_lists<2>(key, m, cnt, sh, kth2, take2, in_lds, diff);
#endif
        kth[0] = kth2[0], kth[1] = kth2[1], take[0] = take2[0], take[1] = take2[1];
    }
    if (n_ret == 0) kth[0] = 0xffffffffu, take[0] = 0;
    if (n_ret + n_cand == 0) kth[1] = 0xffffffffu, take[1] = 0;
    if (!top || ex.n_top == 0) kth[2] = 0xffffffffu, take[2] = 0;
    POP_PSTAMP(2);
    if (top)
        partition_emit<3>(key, m, kth, take, region, ret_idx, cand_idx, ex, sh);
    else
        partition_emit<2>(key, m, kth, take, region, ret_idx, cand_idx, ex, sh);
    POP_PSTAMP(3);
}

bool partition_takes_partials(int m) { return m <= kPartLdsKeys; }

hipError_t launch_partition(const float *scores, int m, int n_ret, int n_cand, unsigned char *region, int *ret_idx,
                            int *cand_idx, hipStream_t s, const PartitionExtra *extra)
{
    PartitionExtra ex = extra ? *extra : PartitionExtra{};
    if (ex.s2_part && !partition_takes_partials(m)) return hipErrorInvalidValue;
    const size_t lds = m <= kPartLdsKeys ? (size_t)m * 4 : 0;
    if (lds > 32 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&partition_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(partition_kernel, dim3(1), dim3(1024), lds, s, scores, m, n_ret, n_cand, region, ret_idx, cand_idx,
                       ex);
    return hipGetLastError();
}

// ---------------------------------------------------------------- per-step candidate top-k
unsigned long long *g_select_trace = nullptr;  // profiling builds: where topk_kernel stamps its phases (else null)
void set_select_trace(unsigned long long *p) { g_select_trace = p; }

// One workgroup per sequence b.  Only candidate-dependent state is written: the candidate bytes of mask[b][:]
// and the selected suffix of active_idx[b][:]; the retained / pruned bytes and the retained prefix are constant
// for a partition (step_state_init_kernel).
// With a union request (B > 1) every workgroup also leaves one byte per candidate position, and the workgroup
// that finishes last (an arrival counter; nobody waits) compacts the candidates selected by any sequence into
// list[n_ret..] and rewinds the counter.
__global__ __launch_bounds__(1024) void topk_kernel(const float *__restrict__ cscore, int cs_stride,
                                                    const int *__restrict__ cand_idx, int n_cand, int n_ret, int m,
                                                    BatchK kk, int act_stride, unsigned char *__restrict__ mask,
                                                    int *__restrict__ active_idx, int *__restrict__ n_active,
                                                    int *__restrict__ sel_idx, unsigned char *selflag,
                                                    int *union_ctr, int *__restrict__ union_list,
                                                    int *__restrict__ n_union, int keys_in_ext,
                                                    unsigned long long *tr)
{
    __shared__ SelShared sh;
    __shared__ int s_last;
    extern __shared__ uint32_t topk_keys[];  // [2 n_cand] when the launch gave it: candidate sets beyond sh.keys
    const int b = blockIdx.x, B = gridDim.x, k = kk.k[b];
    unsigned char *mk = mask ? mask + (size_t)b * m : nullptr;
    int *act = active_idx ? active_idx + (size_t)b * act_stride + n_ret : (b == 0 ? sel_idx : nullptr);
    // selflag: [n_cand][POP_MAX_BATCH], one 8-byte word per candidate position
    block_select_candidates(cscore + (size_t)b * cs_stride, cand_idx, n_cand, k, mk, act, sh, SelectNoHook(),
                            SelectNoHook(), b == 0 ? tr : nullptr, selflag ? selflag + b : nullptr, POP_MAX_BATCH, false,
                            keys_in_ext ? topk_keys : nullptr, keys_in_ext ? n_cand : 0);
    if (tr && b == 0 && threadIdx.x == 0) tr[6] = wall_clock64();
    if (n_active && threadIdx.x == 0) n_active[b] = n_ret + k;
    if (!union_list) return;
    // the flags of this sequence are written; the last workgroup to get here sees every sequence's flags
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) s_last = atomicAdd(union_ctr, 1) == B - 1;
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    static_assert(POP_MAX_BATCH == 8, "one 64-bit word of flags per candidate position");
    const unsigned long long live = B >= 8 ? ~0ull : ((1ull << (8 * B)) - 1ull);  // bytes of sequences >= B are stale
    const unsigned long long *flags = reinterpret_cast<const unsigned long long *>(selflag);
    int E = (n_cand + blockDim.x - 1) / blockDim.x;
    int lo = min(n_cand, (int)threadIdx.x * E), hi = min(n_cand, lo + E);
    int c[1] = {0}, tot[1];
    for (int i = lo; i < hi; ++i) c[0] += (flags[i] & live) != 0;
    block_excl_scan<1>(c, tot, sh);
    int p = n_ret + c[0];
    for (int i = lo; i < hi; ++i)
        if ((flags[i] & live) != 0) union_list[p++] = cand_idx[i];
    if (threadIdx.x == 0) {
        *n_union = n_ret + tot[0];
        *union_ctr = 0;
    }
}

hipError_t launch_topk(const float *cscore, int cs_stride, const int *cand_idx, int n_cand, int n_ret, int m, int B,
                       BatchK k, int act_stride, unsigned char *mask, int *active_idx, int *n_active, int *sel_idx,
                       unsigned char *selflag, int *union_ctr, int *union_list, int *n_union, hipStream_t s)
{
    int threads = n_cand <= 2048 ? 256 : 1024;
    // candidate sets beyond the select's own key buffer (re-scoring all channels of a layer) get theirs from the launch
    const bool ext = n_cand > kSelLdsKeys && n_cand <= 16384;  // (keys and staged decisions: 8 bytes per candidate)
    const size_t lds = ext ? (size_t)n_cand * 8 : 0;
    if (lds > 32 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&topk_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(topk_kernel, dim3(B), dim3(threads), lds, s, cscore, cs_stride, cand_idx, n_cand, n_ret, m, k,
                       act_stride, mask, active_idx, n_active, sel_idx, selflag, union_ctr, union_list, n_union,
                       ext ? 1 : 0, g_select_trace);
    return hipGetLastError();
}

// Partition-constant part of the step state, for `rows` sequences: mask[b][j] = 1 for retained channels, 0 for
// pruned and (until a step selects them) candidate channels; active_idx[b][0..n_ret) = ret_idx.  Row 0's workgroups
// also write the candidate-then-retained list rc_idx and the retained prefix of the union list, when given.  One
// more row of workgroups zeroes a strided word buffer (clr.n slots of clr.words ints, clr.stride ints apart), and
// further rows gather the columns of a channel list (job), which saves the partition and the prompt's forward pass a
// launch of their own for each.
__global__ __launch_bounds__(256) void step_state_init_kernel(const unsigned char *__restrict__ region, int m,
                                                              const int *__restrict__ ret_idx, int n_ret, int rows,
                                                              int act_stride, unsigned char *__restrict__ mask,
                                                              int *__restrict__ active_idx,
                                                              const int *__restrict__ cand_idx, int n_cand,
                                                              int *__restrict__ rc_idx, int *__restrict__ ulist,
                                                              StridedClear clr, CompactJob job)
{
    const int b = blockIdx.y;
    if (b > rows) {
        compact_hidden_block(job, blockIdx.x, b - rows - 1);
        return;
    }
    if (b == rows) {
        if (!clr.p) return;
        const int per = blockDim.x / clr.words;  // slots a workgroup clears at once
        for (int q = blockIdx.x * per + threadIdx.x / clr.words; q < clr.n && (int)threadIdx.x < per * clr.words;
             q += gridDim.x * per)
            clr.p[(size_t)q * clr.stride + threadIdx.x % clr.words] = 0;
        return;
    }
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < m; j += gridDim.x * blockDim.x) {
        if (mask) mask[(size_t)b * m + j] = region[j] == POP_REGION_RETAINED ? 1 : 0;
        if (j < n_ret) {
            const int r = ret_idx[j];
            if (active_idx) active_idx[(size_t)b * act_stride + j] = r;
            if (b == 0 && rc_idx) rc_idx[n_cand + j] = r;
            if (b == 0 && ulist) ulist[j] = r;
        }
        if (b == 0 && rc_idx && j < n_cand) rc_idx[j] = cand_idx[j];
    }
}

hipError_t launch_step_state_init(const unsigned char *region, int m, const int *ret_idx, int n_ret, int rows,
                                  int act_stride, unsigned char *mask, int *active_idx, hipStream_t s,
                                  const int *cand_idx, int n_cand, int *rc_idx, int *ulist, const StridedClear *clear,
                                  const CompactJob *compact)
{
    StridedClear clr = clear ? *clear : StridedClear{};
    CompactJob job = compact ? *compact : CompactJob{};
    if (clr.p && (clr.words < 1 || clr.words > 256)) return hipErrorInvalidValue;
    // rows of workgroups: `rows` of state, one that clears (idle without a buffer, present whenever a later row is),
    // then the compaction's (its 512 positions per workgroup cover any list of up to m channels in this grid's width)
    const int job_rows = job.hc ? (job.T + kCompactRows - 1) / kCompactRows : 0;
    dim3 grid((m + 255) / 256, rows + ((clr.p || job_rows) ? 1 : 0) + job_rows);
    hipLaunchKernelGGL(step_state_init_kernel, grid, dim3(256), 0, s, region, m, ret_idx, n_ret, rows, act_stride, mask,
                       active_idx, cand_idx, n_cand, rc_idx, ulist, clr, job);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_int_kernel(int *__restrict__ p, int n, int value)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

hipError_t launch_fill_int(int *p, int n, int value, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_int_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p, n, value);
    return hipGetLastError();
}

// ---------------------------------------------------------------- list compaction
// list = ascending channels j with mask[r][j] != 0 for some row r < rows.
__global__ __launch_bounds__(1024) void mask_to_list_kernel(const unsigned char *__restrict__ mask, int rows, int m,
                                                            int *__restrict__ list, int *__restrict__ n_list,
                                                            uint16_t *__restrict__ pad_hc, int pad_ld, int pad_T)
{
    __shared__ SelShared sh;
    int E = (m + blockDim.x - 1) / blockDim.x;
    int lo = min(m, (int)threadIdx.x * E), hi = min(m, lo + E);
    int c[1] = {0}, tot[1];
    for (int j = lo; j < hi; ++j) {
        int any = 0;
        for (int r = 0; r < rows; ++r) any |= mask[(size_t)r * m + j];
        c[0] += (any != 0);
    }
    block_excl_scan<1>(c, tot, sh);
    int p = c[0];
    for (int j = lo; j < hi; ++j) {
        int any = 0;
        for (int r = 0; r < rows; ++r) any |= mask[(size_t)r * m + j];
        if (any) list[p++] = j;
    }
    if (threadIdx.x == 0) *n_list = tot[0];
    if (pad_hc) {
        const int a = tot[0], a_end = min((a + 63) / 64 * 64, pad_ld), w = a_end - a;
        for (int e = threadIdx.x; e < w * pad_T; e += blockDim.x) pad_hc[(size_t)(e / w) * pad_ld + a + e % w] = 0;
    }
}

hipError_t launch_mask_to_list(const unsigned char *mask, int rows, int m, int *list, int *n_list, hipStream_t s,
                               uint16_t *pad_hc, int pad_ld, int pad_T)
{
    hipLaunchKernelGGL(mask_to_list_kernel, dim3(1), dim3(1024), 0, s, mask, rows, m, list, n_list, pad_hc, pad_ld,
                       pad_T);
    return hipGetLastError();
}

// any[j] = 1 where mask[r][j] != 0 for some row r.  any is cleared first; a thread owns 4 adjacent channels and a
// group of 32 rows and writes 1 where it saw a set byte (writers of one byte all write the same value).
constexpr int kAnyRows = 32;
__global__ __launch_bounds__(256) void mask_any_kernel(const unsigned char *__restrict__ mask, int rows, int m,
                                                       unsigned char *__restrict__ any)
{
    const int j = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (j >= m) return;
    const int n = min(4, m - j);
    const int r0 = blockIdx.y * kAnyRows, r1 = min(rows, r0 + kAnyRows);
    unsigned char acc[4] = {0, 0, 0, 0};
    for (int r = r0; r < r1; ++r)
        for (int q = 0; q < n; ++q) acc[q] |= mask[(size_t)r * m + j + q];
    for (int q = 0; q < n; ++q)
        if (acc[q]) any[j + q] = 1;
}

// any must have room for m rounded up to a multiple of 4 bytes.
hipError_t launch_mask_any(const unsigned char *mask, int rows, int m, unsigned char *any, hipStream_t s)
{
    hipError_t e = launch_fill_int((int *)any, (m + 3) / 4, 0, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mask_any_kernel, dim3((m + 1023) / 1024, (rows + kAnyRows - 1) / kAnyRows), dim3(256), 0, s, mask,
                       rows, m, any);
    return hipGetLastError();
}

// Scores of one batch step aggregated over its B sequences (Eq. 3 with the step's tokens and samples):
// cs[b][p] = n_j |h_bj| on entry; on exit every row holds sqrt(sum_b cs[b][p]^2) = n_j * ||h_{:,j}||_2.
__global__ __launch_bounds__(256) void aggregate_scores_kernel(float *__restrict__ cs, int cs_stride, int B, int n)
{
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n) return;
    double acc = 0.0;
    for (int b = 0; b < B; ++b) {
        const double v = (double)cs[(size_t)b * cs_stride + p];
        acc += v * v;
    }
    const float r = (float)sqrt(acc);
    for (int b = 0; b < B; ++b) cs[(size_t)b * cs_stride + p] = r;
}

hipError_t launch_aggregate_scores(float *cs, int cs_stride, int B, int n, hipStream_t s)
{
    if (n < 1) return hipSuccess;
    hipLaunchKernelGGL(aggregate_scores_kernel, dim3((n + 255) / 256), dim3(256), 0, s, cs, cs_stride, B, n);
    return hipGetLastError();
}

}  // namespace pop
