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
    unsigned int hist[3][256];  // digit histograms of three consecutive radix passes (see radix_threshold)
    unsigned int hist2[3][256]; // the second threshold's histograms when several are sought in one sweep
    unsigned int hist3[3][256]; // the third threshold's
    int wave_tot[6][kSelMaxWaves];
    int digit;
    int remaining;
    int list_len[3];            // lengths of the key lists of radix_thresholds_lists
    uint32_t keys[kSelLdsKeys];
};

// Inclusive prefix sum over the 64 lanes of a wave with DPP moves (register-to-register: a few cycles per step,
// where a shuffle through the LDS crossbar costs a full LDS round trip per step).
__device__ __forceinline__ int wave_incl_scan(int v)
{
    // within each row of 16 lanes: shifts by 1, 2, 4, 8 (lanes without a source keep 0)
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);  // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);  // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);  // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);  // row_shr:8
    // across rows: last lane of row 0 -> row 1, of row 2 -> row 3; then last lane of row 1 -> rows 2 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31
    return v;
}

// Exclusive block scan of N integer streams at once.  Returns the exclusive prefix in v[], block totals in
// tot[].  All threads of the block must call.
template <int N>
__device__ __forceinline__ void block_excl_scan(int (&v)[N], int (&tot)[N], SelShared &sh)
{
    int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave, nw = (blockDim.x + kWave - 1) / kWave;
    int inc[N];
#pragma unroll
    for (int q = 0; q < N; ++q) {
        inc[q] = wave_incl_scan(v[q]);
        if (lane == kWave - 1) sh.wave_tot[q][wave] = inc[q];
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < N; ++q) {
        // lane l < nw reads the total of wave l; a second in-wave scan gives every wave's base
        const int t = lane < nw ? sh.wave_tot[q][lane] : 0;
        const int ts = wave_incl_scan(t);
        const int base = wave > 0 ? __builtin_amdgcn_readlane(ts, wave - 1) : 0;
        const int total = __builtin_amdgcn_readlane(ts, kWave - 1);
        v[q] = base + inc[q] - v[q];
        tot[q] = total;
    }
    __syncthreads();
}

// OR over each row of 16 lanes (every lane of the row gets it).
__device__ __forceinline__ uint32_t wave_or_rows(uint32_t v)
{
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true);   // quad_perm 1,0,3,2
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, true);   // quad_perm 2,3,0,1
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, true);  // row_half_mirror
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, true);  // row_mirror
    return v;
}

// hist[d] += 1 for every lane with valid set, d < 256.  Lanes of a wave that hold the same digit as its first
// valid lane are counted by that lane, and again for the rest as long as such a group covers a quarter of the wave;
// whatever is left adds on its own.  Scores of one layer share their exponent bits, so without this the leading
// digit of every key would hit one LDS word, one lane at a time; for well-spread digits the loop ends after one try.
__device__ __forceinline__ void wave_hist_add(unsigned int *hist, uint32_t d, bool valid)
{
    unsigned long long todo = __ballot(valid);
    const int lane = threadIdx.x % kWave;
#pragma unroll 1
    for (int it = 0; it < 4 && todo; ++it) {
        const int leader = __builtin_ctzll(todo);
        const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)d, leader);
        const unsigned long long same = __ballot(valid && d == d0) & todo;
        const int n_same = __popcll(same);
        if (lane == leader) atomicAdd(&hist[d0], (unsigned int)n_same);
        todo &= ~same;
        if (n_same < kWave / 4) break;
    }
    if ((todo >> lane) & 1ull) atomicAdd(&hist[d], 1u);
}

// Key of the n_top-th best element among key(0..n), and how many elements equal to that key belong to the
// top n_top (taken in index order).  n_top == 0 gives take_eq = 0 with kth = 0xffffffff.
// MSB-first radix select over 8-bit digits, starting below the bits that all keys have in common.
template <class KeyFn>
__device__ __forceinline__ void radix_threshold(KeyFn key, int n, int n_top, SelShared &sh, uint32_t &kth,
                                                int &take_eq)
{
    if (n_top <= 0) {
        kth = 0xffffffffu;
        take_eq = 0;
        return;
    }
    // bits in which any two keys differ: OR over all keys of (key ^ key(0))
    unsigned int *scratch = &sh.hist[2][0];
    if (threadIdx.x == 0) scratch[0] = 0;
    if (threadIdx.x < 256) sh.hist[0][threadIdx.x] = 0;
    if (blockDim.x < 256)
        for (int i = threadIdx.x + blockDim.x; i < 256; i += blockDim.x) sh.hist[0][i] = 0;
    __syncthreads();
    const uint32_t k0 = key(0);
    uint32_t diff = 0;
    for (int i = threadIdx.x; i < n; i += blockDim.x) diff |= key(i) ^ k0;
    diff |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)diff, 0xB1, 0xf, 0xf, true);   // quad_perm 1,0,3,2
    diff |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)diff, 0x4E, 0xf, 0xf, true);   // quad_perm 2,3,0,1
    diff |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)diff, 0x141, 0xf, 0xf, true);  // row_half_mirror
    diff |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)diff, 0x140, 0xf, 0xf, true);  // row_mirror
    if (threadIdx.x % 16 == 0 && diff) atomicOr(&scratch[0], diff);  // one lane per row of 16
    __syncthreads();
    diff = scratch[0];
    if (diff == 0) {  // all keys equal
        __syncthreads();
        kth = k0;
        take_eq = n_top;
        return;
    }
    const int top_bit = 31 - __builtin_clz(diff);          // highest bit in which keys differ
    const int n_pass = top_bit / 8 + 1;                     // digits below and including that bit
    uint32_t known = top_bit == 31 ? 0u : ~((2u << top_bit) - 1u);  // the common leading bits
    uint32_t prefix = k0 & known;
    int remaining = n_top;
    const int lane = threadIdx.x % kWave;
    // Pass p counts into hist[p % 3], and clears hist[(p + 1) % 3] for the next pass: that one was last read in
    // pass p - 2, which every wave had finished before any wave could pass the barrier of pass p - 1.  Every wave
    // then finds the digit for itself, so a pass has a single barrier.
    int pass = 0;
    for (int shift = (n_pass - 1) * 8; shift >= 0; shift -= 8, ++pass) {
        unsigned int *hist = sh.hist[pass % 3], *next = sh.hist[(pass + 1) % 3];
        if (threadIdx.x < 256) next[threadIdx.x] = 0;
        if (blockDim.x < 256)
            for (int i = threadIdx.x + blockDim.x; i < 256; i += blockDim.x) next[i] = 0;
        const int n_round = (n + blockDim.x - 1) / blockDim.x * blockDim.x;  // whole waves take part in the ballots
        if (pass == 0) {
            // leading digit: scores of one layer crowd into a few values of it
            for (int i = threadIdx.x; i < n_round; i += blockDim.x) {
                const uint32_t k = i < n ? key(i) : 0u;
                wave_hist_add(hist, (k >> shift) & 255u, i < n && (k & known) == prefix);
            }
        } else {
            // later digits are spread out (and few keys are left): one atomic each
            for (int i = threadIdx.x; i < n; i += blockDim.x) {
                const uint32_t k = key(i);
                if ((k & known) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1u);
            }
        }
        __syncthreads();
        // lane l owns the four digits 255-4l .. 252-4l, scanned from the largest digit down
        int c[4], lane_tot = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            c[q] = (int)hist[255 - (4 * lane + q)];
            lane_tot += c[q];
        }
        int before = wave_incl_scan(lane_tot) - lane_tot;
        int digit = -1, rem_new = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (before < remaining && remaining <= before + c[q]) {
                digit = 255 - (4 * lane + q);
                rem_new = remaining - before;
            }
            before += c[q];
        }
        const int owner = __builtin_ctzll(__ballot(digit >= 0));  // exactly one lane holds the digit
        digit = __builtin_amdgcn_readlane(digit, owner);
        remaining = __builtin_amdgcn_readlane(rem_new, owner);
        prefix |= ((uint32_t)digit) << shift;
        known |= 255u << shift;
    }
    __syncthreads();  // the caller may reuse the histograms
    kth = prefix;
    take_eq = remaining;
}

// NT (2 or 3) thresholds in the same sweeps: kth[t] = key of the n_top[t]-th best element, 1 <= n_top[t] <= n, with
// its take count, as NT calls of radix_threshold would give them.  The common leading bits and the leading digit's
// histogram serve all; from the second digit on a key is counted for the threshold(s) whose prefix it matches.
// Made for a large key set: digits are cut from the highest differing bit down (so the leading digit spreads the
// keys over all its values even when that bit is not at a byte boundary), and the sweep for the second digit also
// copies the keys that share a threshold's leading digit into a short list in sh.keys (one NT-th of it per
// threshold; thresholds under one leading digit share a list), which the sweeps for the remaining digits read
// instead of all n keys.  A threshold whose leading digit holds more keys than its list can take keeps sweeping all
// keys.  Must not be used while sh.keys holds data.  have_diff: diff_in holds the bits in which any two keys differ.
template <int NT, class KeyFn>
__device__ __forceinline__ void radix_thresholds_lists(KeyFn key, int n, const int (&n_top)[NT], SelShared &sh,
                                                       uint32_t (&kth)[NT], int (&take)[NT], bool have_diff = false,
                                                       uint32_t diff_in = 0, unsigned long long *tr = nullptr)
{
    static_assert(NT == 2 || NT == 3, "two or three thresholds");
    constexpr int kCap = kSelLdsKeys / NT;
    unsigned int *scratch = &sh.hist[2][0];
    if (threadIdx.x == 0) {
        scratch[0] = 0;
#pragma unroll
        for (int t = 0; t < NT; ++t) sh.list_len[t] = 0;
    }
    if (threadIdx.x < 256) sh.hist[0][threadIdx.x] = 0;
    if (blockDim.x < 256)
        for (int i = threadIdx.x + blockDim.x; i < 256; i += blockDim.x) sh.hist[0][i] = 0;
    __syncthreads();
    const uint32_t k0 = key(0);
    // bits in which any two keys differ: from the caller (who had every key in hand), else one sweep
    uint32_t diff = diff_in;
    if (!have_diff) {
        diff = 0;
        for (int i = threadIdx.x; i < n; i += blockDim.x) diff |= key(i) ^ k0;
        diff = wave_or_rows(diff);
        if (threadIdx.x % 16 == 0 && diff) atomicOr(&scratch[0], diff);
        __syncthreads();
        diff = scratch[0];
    }
    if (diff == 0) {  // all keys equal
        __syncthreads();
#pragma unroll
        for (int t = 0; t < NT; ++t) kth[t] = k0, take[t] = n_top[t];
        return;
    }
    const int top_bit = 31 - __builtin_clz(diff);
    const int n_pass = top_bit / 8 + 1;
    uint32_t known = top_bit == 31 ? 0u : ~((2u << top_bit) - 1u);
    uint32_t prefix[NT];
    int remaining[NT], matching[NT], list_of[NT];  // list_of[t]: the list threshold t reads (-1: sweeps all keys)
#pragma unroll
    for (int t = 0; t < NT; ++t) prefix[t] = k0 & known, remaining[t] = n_top[t], matching[t] = n, list_of[t] = -1;
    const int lane = threadIdx.x % kWave;
    for (int pass = 0; pass < n_pass; ++pass) {
        const int hi = top_bit - 8 * pass, lo = hi >= 7 ? hi - 7 : 0;
        const uint32_t dmask = (1u << (hi - lo + 1)) - 1u;
        // pass p counts into set p % 3 and clears set (p + 1) % 3, last read in pass p - 2 (one barrier per pass); the
        // leading digit's histogram is shared
        unsigned int *hist[3] = {sh.hist[pass % 3], pass == 0 ? sh.hist[0] : sh.hist2[pass % 3],
                                 pass == 0 ? sh.hist[0] : sh.hist3[pass % 3]};
        for (int i = threadIdx.x; i < 256; i += blockDim.x) {
            sh.hist[(pass + 1) % 3][i] = 0;
            sh.hist2[(pass + 1) % 3][i] = 0;
            if (NT > 2) sh.hist3[(pass + 1) % 3][i] = 0;
        }
        if (pass == 0) {
            const int n_round = (n + blockDim.x - 1) / blockDim.x * blockDim.x;
            for (int i = threadIdx.x; i < n_round; i += blockDim.x) {
                const uint32_t k = i < n ? key(i) : 0u;
                wave_hist_add(hist[0], (k >> lo) & dmask, i < n);
            }
        } else if (pass == 1) {
            // the one sweep that also fills the lists; a threshold under the same leading digit as an earlier one
            // reads that one's list
            bool fill[NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                int same_as = -1;
#pragma unroll
                for (int u = 0; u < t; ++u)
                    if (same_as < 0 && prefix[u] == prefix[t]) same_as = u;
                fill[t] = same_as < 0 && matching[t] <= kCap;
                list_of[t] = same_as >= 0 ? list_of[same_as] : (fill[t] ? t : -1);
            }
            for (int i = threadIdx.x; i < n; i += blockDim.x) {
                const uint32_t k = key(i);
                const uint32_t kk = k & known, dg = (k >> lo) & dmask;
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    if (kk == prefix[t]) {
                        atomicAdd(&hist[t][dg], 1u);
                        if (fill[t]) sh.keys[t * kCap + atomicAdd(&sh.list_len[t], 1)] = k;
                    }
            }
        } else {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (list_of[t] >= 0) {
                    // (the list holds the keys that matched after the leading digit: a superset of the current matches)
                    const uint32_t *lst = sh.keys + list_of[t] * kCap;
                    const int len = sh.list_len[list_of[t]];
                    for (int i = threadIdx.x; i < len; i += blockDim.x) {
                        const uint32_t k = lst[i];
                        if ((k & known) == prefix[t]) atomicAdd(&hist[t][(k >> lo) & dmask], 1u);
                    }
                } else {
                    for (int i = threadIdx.x; i < n; i += blockDim.x) {
                        const uint32_t k = key(i);
                        if ((k & known) == prefix[t]) atomicAdd(&hist[t][(k >> lo) & dmask], 1u);
                    }
                }
            }
        }
        __syncthreads();
        if (tr && threadIdx.x == 0 && pass < 4) tr[pass] = wall_clock64();  // (profiling builds: the sweep is done)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            int c[4], lane_tot = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                c[q] = (int)hist[t][255 - (4 * lane + q)];
                lane_tot += c[q];
            }
            int before = wave_incl_scan(lane_tot) - lane_tot;
            int digit = -1, rem_new = 0, in_digit = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (before < remaining[t] && remaining[t] <= before + c[q]) {
                    digit = 255 - (4 * lane + q);
                    rem_new = remaining[t] - before;
                    in_digit = c[q];
                }
                before += c[q];
            }
            const int owner = __builtin_ctzll(__ballot(digit >= 0));
            digit = __builtin_amdgcn_readlane(digit, owner);
            remaining[t] = __builtin_amdgcn_readlane(rem_new, owner);
            matching[t] = __builtin_amdgcn_readlane(in_digit, owner);
            prefix[t] |= ((uint32_t)digit) << lo;
        }
        known |= dmask << lo;
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < NT; ++t) kth[t] = prefix[t], take[t] = remaining[t];
}

struct SelectNoHook {
    __device__ __forceinline__ void operator()(int) const {}
    __device__ __forceinline__ void operator()() const {}
};

// Select the best k of n_cand candidates (cs[i] is the score of channel cand_idx[i], cand_idx ascending).
// Writes, each if non-null: mk[cand_idx[i]] = selected (candidate bytes only; the bytes of retained and pruned
// channels are constant for a partition and written when the partition is made), act_sel[0..k) = selected
// channels ascending, selpos[i] = selected (by position in cand_idx).  on_selected(i) is called for every selected position before any of those global writes,
// then after_selected() by every thread (it may contain barriers): callers that only need the positions get
// them without waiting for the index loads.  All threads of the block must call.
// kCoherentScores: the scores were just written by other workgroups of the same kernel with write-through stores;
// read them with device-coherent loads (no cache invalidation needed).  kCoherentFlags: selpos is written through,
// for another workgroup of the same kernel to read.
template <bool kCoherentScores = false, class OnSelected = SelectNoHook, class AfterSelected = SelectNoHook,
          bool kCoherentFlags = false>
__device__ __forceinline__ void block_select_candidates(const float *__restrict__ cs, const int *__restrict__ cand_idx,
                                                        int n_cand, int k, unsigned char *__restrict__ mk,
                                                        int *__restrict__ act_sel, SelShared &sh,
                                                        OnSelected on_selected = OnSelected(),
                                                        AfterSelected after_selected = AfterSelected(),
                                                        unsigned long long *tr = nullptr,
                                                        unsigned char *__restrict__ selpos = nullptr,
                                                        int selpos_stride = 1, bool keys_ready = false,
                                                        uint32_t *keys_ext = nullptr, int keys_cap = 0)
{
#define SEL_STAMP(k) do { if (tr && threadIdx.x == 0) tr[k] = wall_clock64(); } while (0)
    SEL_STAMP(0);
    auto score = [&](int i) -> float {
        return kCoherentScores ? __hip_atomic_load(&cs[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : cs[i];
    };
    // keys_ready: the caller has put score_key(score) of every candidate into sh.keys (n_cand <= kSelLdsKeys) and
    // synchronised the block.  keys_ext: LDS of the caller's, 2 * keys_cap words, used instead of sh.keys (a large
    // candidate set then stays out of global memory after the first sweep as well; the second half stages the
    // decisions for the output pass)
    uint32_t *const keys = keys_ext ? keys_ext : sh.keys;
    const bool in_lds = n_cand <= (keys_ext ? keys_cap : kSelLdsKeys);
    // (large sets: the channel numbers the output pass needs are requested now, so that they are there by then)
    constexpr int kAhead = 12;
    int jj[kAhead];
    if (keys_ext && in_lds) {
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int i = u * blockDim.x + threadIdx.x;
            jj[u] = i < n_cand ? cand_idx[i] : 0;
        }
    }
    if (in_lds && !keys_ready) {
        // twelve independent loads in flight per thread: under a streaming load a trip to memory takes microseconds
        constexpr int kLoads = 12;
        for (int base = 0; base < n_cand; base += kLoads * blockDim.x) {
            float v[kLoads];
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int i = base + u * blockDim.x + threadIdx.x;
                v[u] = score(i < n_cand ? i : 0);
            }
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int i = base + u * blockDim.x + threadIdx.x;
                if (i < n_cand) keys[i] = score_key(v[u]);
            }
        }
        __syncthreads();
    }
    auto key = [&](int i) -> uint32_t { return in_lds ? keys[i] : score_key(score(i)); };
    uint32_t kth;
    int take;
    SEL_STAMP(1);
    if (keys_ext && in_lds && k > 0) {
        // a large key set in the caller's LDS: sh.keys is free for the short lists of the sweeps after the second
        // digit (the two-threshold form, asked for the same rank twice)
        const int cnt2[2] = {k, k};
        uint32_t kth2[2];
        int take2[2];
        radix_thresholds_lists<2>(key, n_cand, cnt2, sh, kth2, take2);
        kth = kth2[0], take = take2[0];
    } else {
        radix_threshold(key, n_cand, k, sh, kth, take);
    }
    SEL_STAMP(2);

    const int E = (n_cand + blockDim.x - 1) / blockDim.x;
    const int lo = min(n_cand, (int)threadIdx.x * E), hi = min(n_cand, lo + E);
    int cnt[2] = {0, 0}, tot[2];
    for (int i = lo; i < hi; ++i) {
        uint32_t kv = key(i);
        cnt[0] += (kv == kth);
        cnt[1] += (kv > kth);
    }
    block_excl_scan<2>(cnt, tot, sh);
    SEL_STAMP(3);
    {
        int eq = cnt[0];
        for (int i = lo; i < hi; ++i) {
            uint32_t kv = key(i);
            if ((kv > kth) || (kv == kth && eq < take)) on_selected(i);
            eq += (kv == kth);
        }
    }
    SEL_STAMP(4);
    after_selected();
    SEL_STAMP(5);
    // position of a selected element = (# greater before it) + (# admitted equal before it)
    if (keys_ext && in_lds) {
        // Large sets (the caller's LDS holds n_cand more words behind the keys): every thread leaves the decisions of
        // its contiguous range in LDS - the position among the selected, or -1 - and the outputs are then written
        // by consecutive threads for consecutive candidates: whole cache lines instead of one byte per lane 11 apart.
        int *code = reinterpret_cast<int *>(keys_ext + n_cand);
        int eq = cnt[0], gt = cnt[1];
        for (int i = lo; i < hi; ++i) {
            const uint32_t kv = key(i);
            const bool sel = (kv > kth) || (kv == kth && eq < take);
            code[i] = sel ? gt + min(eq, take) : -1;
            eq += (kv == kth);
            gt += (kv > kth);
        }
        __syncthreads();
        for (int base = 0; base < n_cand; base += kAhead * blockDim.x) {
            if (base > 0) {  // (beyond what was requested at the start)
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    const int i = base + u * blockDim.x + threadIdx.x;
                    jj[u] = i < n_cand ? cand_idx[i] : 0;
                }
            }
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                const int i = base + u * blockDim.x + threadIdx.x;
                if (i < n_cand) {
                    const int c = code[i];
                    if (mk) mk[jj[u]] = c >= 0 ? 1 : 0;
                    if (selpos) {
                        if (kCoherentFlags)
                            coherent_store(&selpos[(size_t)i * selpos_stride], (unsigned char)(c >= 0 ? 1 : 0));
                        else
                            selpos[(size_t)i * selpos_stride] = c >= 0 ? 1 : 0;
                    }
                    if (c >= 0 && act_sel) act_sel[c] = jj[u];
                }
            }
        }
        return;
    }
    // the channel numbers of this thread's range are requested together, not one trip to memory per element
    constexpr int kPre = 12;
    int jpre[kPre];
#pragma unroll
    for (int u = 0; u < kPre; ++u) jpre[u] = lo + u < hi ? cand_idx[lo + u] : 0;
    int eq = cnt[0], gt = cnt[1];
#pragma unroll
    for (int u = 0; u < kPre; ++u) {
        const int i = lo + u;
        if (i < hi) {
            uint32_t kv = key(i);
            bool sel = (kv > kth) || (kv == kth && eq < take);
            int pos = gt + min(eq, take);
            eq += (kv == kth);
            gt += (kv > kth);
            const int j = jpre[u];
            if (mk) mk[j] = sel ? 1 : 0;
            if (selpos) {  // the same decision by candidate position
                if (kCoherentFlags)
                    coherent_store(&selpos[(size_t)i * selpos_stride], (unsigned char)(sel ? 1 : 0));
                else
                    selpos[(size_t)i * selpos_stride] = sel ? 1 : 0;
            }
            if (sel && act_sel) act_sel[pos] = j;
        }
    }
    for (int i = lo + kPre; i < hi; ++i) {
        uint32_t kv = key(i);
        bool sel = (kv > kth) || (kv == kth && eq < take);
        int pos = gt + min(eq, take);
        eq += (kv == kth);
        gt += (kv > kth);
        int j = cand_idx[i];
        if (mk) mk[j] = sel ? 1 : 0;
        if (selpos) {
            if (kCoherentFlags)
                coherent_store(&selpos[(size_t)i * selpos_stride], (unsigned char)(sel ? 1 : 0));
            else
                selpos[(size_t)i * selpos_stride] = sel ? 1 : 0;
        }
        if (sel && act_sel) act_sel[pos] = j;
    }
}

}  // namespace pop
