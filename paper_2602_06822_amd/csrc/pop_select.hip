// Rank-based selection kernels: the three-region partition at prefill (Sec. 3.3 "Prefilling Stage"), the
// per-step candidate top-k (Sec. 3.3 "Decoding Stage") and the index-list compactions around them.
//
// All selections use one strict total order on channels: higher score first, equal scores by lower channel
// index.  Scores are mapped to order-preserving 32-bit keys; an MSB-first radix select over four 8-bit digits
// finds the key of the n-th best element, and a block scan in index order admits elements equal to that key
// until the count is exact.  One workgroup handles one selection, so the result is deterministic.
#include "pop_internal.h"

namespace pop {

constexpr int kSelMaxWaves = 16;

struct SelShared {
    unsigned int hist[256];
    int wave_tot[4][kSelMaxWaves];
    int digit;
    int remaining;
};

// Exclusive block scan of up to 4 integer streams at once (N streams).  Returns exclusive prefix in v[],
// block totals in tot[].  All threads of the block must call.
template <int N>
__device__ void block_excl_scan(int (&v)[N], int (&tot)[N], SelShared &sh)
{
    int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
    int inc[N];
#pragma unroll
    for (int q = 0; q < N; ++q) {
        int x = v[q];
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            int y = __shfl_up(x, off, kWave);
            if (lane >= off) x += y;
        }
        inc[q] = x;
        if (lane == kWave - 1) sh.wave_tot[q][wave] = x;
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < N; ++q) {
        int base = 0, total = 0;
        for (int w = 0; w < nw; ++w) {
            int t = sh.wave_tot[q][w];
            if (w < wave) base += t;
            total += t;
        }
        v[q] = base + inc[q] - v[q];
        tot[q] = total;
    }
    __syncthreads();
}

// Key of the n_top-th best element among key(0..n), and how many elements equal to that key belong to the
// top n_top (taken in index order).  n_top == 0 gives take_eq = 0 with kth = 0xffffffff.
template <class KeyFn>
__device__ void radix_threshold(KeyFn key, int n, int n_top, SelShared &sh, uint32_t &kth, int &take_eq)
{
    if (n_top <= 0) {
        kth = 0xffffffffu;
        take_eq = 0;
        return;
    }
    uint32_t prefix = 0, known = 0;
    int remaining = n_top;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (threadIdx.x < 256) sh.hist[threadIdx.x] = 0;
        __syncthreads();
        for (int i = threadIdx.x; i < n; i += blockDim.x) {
            uint32_t k = key(i);
            if ((k & known) == prefix) atomicAdd(&sh.hist[(k >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (threadIdx.x < kWave) {
            // lane l owns the four digits 255-4l .. 252-4l, scanned from the largest digit down
            int l = threadIdx.x;
            int c[4], lane_tot = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                c[q] = (int)sh.hist[255 - (4 * l + q)];
                lane_tot += c[q];
            }
            int x = lane_tot;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                int y = __shfl_up(x, off, kWave);
                if (l >= off) x += y;
            }
            int before = x - lane_tot;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (before < remaining && remaining <= before + c[q]) {
                    sh.digit = 255 - (4 * l + q);
                    sh.remaining = remaining - before;
                }
                before += c[q];
            }
        }
        __syncthreads();
        prefix |= ((uint32_t)sh.digit) << shift;
        known |= 255u << shift;
        remaining = sh.remaining;
        __syncthreads();
    }
    kth = prefix;
    take_eq = remaining;
}

// ---------------------------------------------------------------- three-region partition
__global__ __launch_bounds__(1024) void partition_kernel(const float *__restrict__ scores, int m, int n_ret, int n_cand,
                                                         unsigned char *__restrict__ region, int *__restrict__ ret_idx,
                                                         int *__restrict__ cand_idx)
{
    __shared__ SelShared sh;
    auto key = [&](int i) { return score_key(scores[i]); };
    uint32_t kth_a, kth_b;
    int take_a, take_b;
    radix_threshold(key, m, n_ret, sh, kth_a, take_a);
    radix_threshold(key, m, n_ret + n_cand, sh, kth_b, take_b);

    // index-ordered pass: thread t owns channels [t*E, (t+1)*E)
    int E = (m + blockDim.x - 1) / blockDim.x;
    int lo = threadIdx.x * E, hi = min(m, lo + E);
    int cnt[2] = {0, 0}, tot[2];
    for (int j = lo; j < hi; ++j) {
        uint32_t k = key(j);
        cnt[0] += (k == kth_a);
        cnt[1] += (k == kth_b);
    }
    block_excl_scan<2>(cnt, tot, sh);
    int eq_a = cnt[0], eq_b = cnt[1];
    int nr[2] = {0, 0};
    for (int j = lo; j < hi; ++j) {
        uint32_t k = key(j);
        bool in_r = (k > kth_a) || (k == kth_a && eq_a < take_a);
        bool in_rc = (k > kth_b) || (k == kth_b && eq_b < take_b);
        eq_a += (k == kth_a);
        eq_b += (k == kth_b);
        nr[0] += in_r;
        nr[1] += (!in_r && in_rc);
    }
    block_excl_scan<2>(nr, tot, sh);
    int pr = nr[0], pc = nr[1];
    eq_a = cnt[0];
    eq_b = cnt[1];
    for (int j = lo; j < hi; ++j) {
        uint32_t k = key(j);
        bool in_r = (k > kth_a) || (k == kth_a && eq_a < take_a);
        bool in_rc = (k > kth_b) || (k == kth_b && eq_b < take_b);
        eq_a += (k == kth_a);
        eq_b += (k == kth_b);
        if (region) region[j] = in_r ? POP_REGION_RETAINED : (in_rc ? POP_REGION_CANDIDATE : POP_REGION_PRUNED);
        if (in_r) {
            if (ret_idx) ret_idx[pr] = j;
            ++pr;
        } else if (in_rc) {
            if (cand_idx) cand_idx[pc] = j;
            ++pc;
        }
    }
}

hipError_t launch_partition(const float *scores, int m, int n_ret, int n_cand, unsigned char *region, int *ret_idx,
                            int *cand_idx, hipStream_t s)
{
    hipLaunchKernelGGL(partition_kernel, dim3(1), dim3(1024), 0, s, scores, m, n_ret, n_cand, region, ret_idx, cand_idx);
    return hipGetLastError();
}

// ---------------------------------------------------------------- per-step candidate top-k
// One workgroup per sequence b.  Writes mask[b][:], active_idx[b][:], n_active[b] (and sel_idx for b == 0).
__global__ __launch_bounds__(1024) void topk_kernel(const float *__restrict__ cscore, int cs_stride,
                                                    const int *__restrict__ cand_idx, int n_cand,
                                                    const int *__restrict__ ret_idx, int n_ret,
                                                    const unsigned char *__restrict__ region, int m, BatchK kk,
                                                    int act_stride, unsigned char *__restrict__ mask,
                                                    int *__restrict__ active_idx, int *__restrict__ n_active,
                                                    int *__restrict__ sel_idx)
{
    __shared__ SelShared sh;
    int b = blockIdx.x;
    int k = kk.k[b];
    const float *cs = cscore + (size_t)b * cs_stride;
    auto key = [&](int i) { return score_key(cs[i]); };
    uint32_t kth;
    int take;
    radix_threshold(key, n_cand, k, sh, kth, take);

    int E = (n_cand + blockDim.x - 1) / blockDim.x;
    int lo = min(n_cand, (int)threadIdx.x * E), hi = min(n_cand, lo + E);
    int cnt[1] = {0}, tot[1];
    for (int i = lo; i < hi; ++i) cnt[0] += (key(i) == kth);
    block_excl_scan<1>(cnt, tot, sh);
    int eq0 = cnt[0];
    int ns[1] = {0};
    int eq = eq0;
    for (int i = lo; i < hi; ++i) {
        uint32_t kv = key(i);
        bool sel = (kv > kth) || (kv == kth && eq < take);
        eq += (kv == kth);
        ns[0] += sel;
    }
    block_excl_scan<1>(ns, tot, sh);
    int ps = ns[0];
    eq = eq0;
    unsigned char *mk = mask ? mask + (size_t)b * m : nullptr;
    int *act = active_idx ? active_idx + (size_t)b * act_stride : nullptr;
    for (int i = lo; i < hi; ++i) {
        uint32_t kv = key(i);
        bool sel = (kv > kth) || (kv == kth && eq < take);
        eq += (kv == kth);
        int j = cand_idx[i];
        if (mk) mk[j] = sel ? 1 : 0;
        if (sel) {
            if (act) act[n_ret + ps] = j;
            if (sel_idx && b == 0) sel_idx[ps] = j;
            ++ps;
        }
    }
    // retained and pruned channels of the mask; retained prefix of the active list
    if (mk)
        for (int j = threadIdx.x; j < m; j += blockDim.x) {
            unsigned char r = region[j];
            if (r != POP_REGION_CANDIDATE) mk[j] = (r == POP_REGION_RETAINED) ? 1 : 0;
        }
    if (act)
        for (int i = threadIdx.x; i < n_ret; i += blockDim.x) act[i] = ret_idx[i];
    if (n_active && threadIdx.x == 0) n_active[b] = n_ret + k;
}

hipError_t launch_topk(const float *cscore, int cs_stride, const int *cand_idx, int n_cand, const int *ret_idx,
                       int n_ret, const unsigned char *region, int m, int B, BatchK k, int act_stride,
                       unsigned char *mask, int *active_idx, int *n_active, int *sel_idx, hipStream_t s)
{
    int threads = n_cand <= 2048 ? 256 : 1024;
    hipLaunchKernelGGL(topk_kernel, dim3(B), dim3(threads), 0, s, cscore, cs_stride, cand_idx, n_cand, ret_idx, n_ret,
                       region, m, k, act_stride, mask, active_idx, n_active, sel_idx);
    return hipGetLastError();
}

// ---------------------------------------------------------------- list compactions
// list = ret_idx ++ { cand_idx[i] : mask[b][cand_idx[i]] for some b }, n_list = its length.
__global__ __launch_bounds__(1024) void union_kernel(const unsigned char *__restrict__ mask, int m, int B,
                                                     const int *__restrict__ ret_idx, int n_ret,
                                                     const int *__restrict__ cand_idx, int n_cand,
                                                     int *__restrict__ list, int *__restrict__ n_list)
{
    __shared__ SelShared sh;
    int E = (n_cand + blockDim.x - 1) / blockDim.x;
    int lo = min(n_cand, (int)threadIdx.x * E), hi = min(n_cand, lo + E);
    int c[1] = {0}, tot[1];
    for (int i = lo; i < hi; ++i) {
        int j = cand_idx[i];
        int any = 0;
        for (int b = 0; b < B; ++b) any |= mask[(size_t)b * m + j];
        c[0] += (any != 0);
    }
    block_excl_scan<1>(c, tot, sh);
    int p = n_ret + c[0];
    for (int i = lo; i < hi; ++i) {
        int j = cand_idx[i];
        int any = 0;
        for (int b = 0; b < B; ++b) any |= mask[(size_t)b * m + j];
        if (any) list[p++] = j;
    }
    for (int i = threadIdx.x; i < n_ret; i += blockDim.x) list[i] = ret_idx[i];
    if (threadIdx.x == 0) *n_list = n_ret + tot[0];
}

hipError_t launch_union(const unsigned char *mask, int m, int B, const int *ret_idx, int n_ret, const int *cand_idx,
                        int n_cand, int *list, int *n_list, hipStream_t s)
{
    int threads = n_cand <= 2048 ? 256 : 1024;
    hipLaunchKernelGGL(union_kernel, dim3(1), dim3(threads), 0, s, mask, m, B, ret_idx, n_ret, cand_idx, n_cand, list,
                       n_list);
    return hipGetLastError();
}

// list = ascending channels j with mask[r][j] != 0 for some row r < rows.
__global__ __launch_bounds__(1024) void mask_to_list_kernel(const unsigned char *__restrict__ mask, int rows, int m,
                                                            int *__restrict__ list, int *__restrict__ n_list)
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
}

hipError_t launch_mask_to_list(const unsigned char *mask, int rows, int m, int *list, int *n_list, hipStream_t s)
{
    hipLaunchKernelGGL(mask_to_list_kernel, dim3(1), dim3(1024), 0, s, mask, rows, m, list, n_list);
    return hipGetLastError();
}

}  // namespace pop
