// Workgroup-level rank selection shared by the selection kernels and the fused decode kernel.
//
// One strict total order on channels: higher score first, equal scores by lower channel index.  Scores are
// mapped to order-preserving 32-bit keys; an MSB-first radix select over four 8-bit digits finds the key of
// the n-th best element, and a block scan in index order admits elements equal to that key until the count
// is exact.  One workgroup handles one selection, so the result is deterministic.
#pragma once
#include "pop_internal.h"

namespace pop {

constexpr int kSelMaxWaves = 16;
constexpr int kSelLdsKeys = 4096;  // candidate keys staged in LDS when they fit (16 KiB)

struct SelShared {
    unsigned int hist[256];
    int wave_tot[4][kSelMaxWaves];
    int digit;
    int remaining;
    uint32_t keys[kSelLdsKeys];
};

// Exclusive block scan of N integer streams at once.  Returns the exclusive prefix in v[], block totals in
// tot[].  All threads of the block must call.
template <int N>
__device__ __forceinline__ void block_excl_scan(int (&v)[N], int (&tot)[N], SelShared &sh)
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
__device__ __forceinline__ void radix_threshold(KeyFn key, int n, int n_top, SelShared &sh, uint32_t &kth,
                                                int &take_eq)
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
        if (blockDim.x < 256)
            for (int i = threadIdx.x + blockDim.x; i < 256; i += blockDim.x) sh.hist[i] = 0;
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

struct SelectNoHook {
    __device__ __forceinline__ void operator()(int) const {}
    __device__ __forceinline__ void operator()() const {}
};

// Select the best k of n_cand candidates (cs[i] is the score of channel cand_idx[i], cand_idx ascending).
// Writes, each if non-null: mk[cand_idx[i]] = selected (candidate bytes only; the bytes of retained and pruned
// channels are constant for a partition and written when the partition is made), act_sel[0..k) = selected
// channels ascending.  on_selected(i) is called for every selected position before any of those global writes,
// then after_selected() by every thread (it may contain barriers): callers that only need the positions get
// them without waiting for the index loads.  All threads of the block must call.
// kCoherentScores: the scores were just written by other workgroups of the same kernel with write-through stores;
// read them with device-coherent loads (no cache invalidation needed).
template <bool kCoherentScores = false, class OnSelected = SelectNoHook, class AfterSelected = SelectNoHook>
__device__ __forceinline__ void block_select_candidates(const float *__restrict__ cs, const int *__restrict__ cand_idx,
                                                        int n_cand, int k, unsigned char *__restrict__ mk,
                                                        int *__restrict__ act_sel, SelShared &sh,
                                                        OnSelected on_selected = OnSelected(),
                                                        AfterSelected after_selected = AfterSelected())
{
    auto score = [&](int i) -> float {
        return kCoherentScores ? __hip_atomic_load(&cs[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : cs[i];
    };
    const bool in_lds = n_cand <= kSelLdsKeys;
    if (in_lds) {
        for (int i = threadIdx.x; i < n_cand; i += blockDim.x) sh.keys[i] = score_key(score(i));
        __syncthreads();
    }
    auto key = [&](int i) -> uint32_t { return in_lds ? sh.keys[i] : score_key(score(i)); };
    uint32_t kth;
    int take;
    radix_threshold(key, n_cand, k, sh, kth, take);

    const int E = (n_cand + blockDim.x - 1) / blockDim.x;
    const int lo = min(n_cand, (int)threadIdx.x * E), hi = min(n_cand, lo + E);
    int cnt[2] = {0, 0}, tot[2];
    for (int i = lo; i < hi; ++i) {
        uint32_t kv = key(i);
        cnt[0] += (kv == kth);
        cnt[1] += (kv > kth);
    }
    block_excl_scan<2>(cnt, tot, sh);
    {
        int eq = cnt[0];
        for (int i = lo; i < hi; ++i) {
            uint32_t kv = key(i);
            if ((kv > kth) || (kv == kth && eq < take)) on_selected(i);
            eq += (kv == kth);
        }
    }
    after_selected();
    // position of a selected element = (# greater before it) + (# admitted equal before it)
    int eq = cnt[0], gt = cnt[1];
    for (int i = lo; i < hi; ++i) {
        uint32_t kv = key(i);
        bool sel = (kv > kth) || (kv == kth && eq < take);
        int pos = gt + min(eq, take);
        eq += (kv == kth);
        gt += (kv > kth);
        int j = cand_idx[i];
        if (mk) mk[j] = sel ? 1 : 0;
        if (sel && act_sel) act_sel[pos] = j;
    }
}

}  // namespace pop
