// Internal declarations shared by the HIP translation units of the POP library.
// Each .hip file defines its kernels and a host launcher; pop_api.hip holds the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "pop.h"

namespace pop {

constexpr int kWave = 64;

// Order-preserving key of a float32 score: larger score <=> larger key; -0.0 maps to the key of +0.0.
__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t b = __float_as_uint(s);
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// round-to-nearest-even float32 -> bf16 bits (finite inputs)
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.0f + expf(-g)) * u; }

template <typename T>
__device__ __forceinline__ T wave_sum(T v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

struct BatchK {
    int k[POP_MAX_BATCH];
};

// Device-coherent (agent scope) accesses for values that workgroups of one kernel hand to each other: the
// loads bypass stale cache lines, the stores write through, so no cache write-back or invalidation is needed.
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
__device__ __forceinline__ void coherent_store(unsigned char *p, unsigned char v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float coherent_load(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long coherent_load(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Bounded wait until the counter *addr, which only ever grows (and may wrap), has reached target: at most `limit`
// looks, at least one (a launch that waits is sized so that all its workgroups are resident).
__device__ __forceinline__ bool spin_until(const int *addr, int target, int limit)
{
    for (int it = 0;; ++it) {
        if (coherent_load(addr) - target >= 0) return true;
        if (it >= limit) return false;
        __builtin_amdgcn_s_sleep(2);
    }
}

// ---- setup (pop_setup.hip) ----
// w[j][0][:] = w_gate[j][:], w[j][1][:] = w_up[j][:], w[j][2][o] = w_down[o][j];  nrm[j] = ||w_down[:,j]||.
hipError_t launch_repack(const void *w_gate, const void *w_up, const void *w_down, int d, int m, int esize,
                         void *w, float *nrm, int is_bf16, hipStream_t s);

// ---- selection (pop_select.hip) ----
// Regions by rank of scores[m]; outputs may be null.  Two things the prefill call needs can ride in the same
// launch: the scores themselves from the prefill kernel's partial rows (scores[j] = nrm[j] * sqrt(sum over tiles,
// in order, of s2_part[tile][j]), written to scores_out and used instead of the scores argument; only when
// partition_takes_partials(m)), and n_sync <= 1024 counters to clear.
struct PartitionExtra {
    const float *s2_part = nullptr;
    int n_tiles = 0;
    const float *nrm = nullptr;
    float *scores_out = nullptr;
    int *sync = nullptr;
    int n_sync = 0;
    // with top_list given: the n_top best channels of the same order as well (the prompt's own mask, Sec. 3.4: the
    // retained channels plus the best candidates by prefill score are the n_top best overall) - top_mask[m] bytes
    // (optional), their ascending list, *top_count = n_top
    int n_top = 0;
    unsigned char *top_mask = nullptr;
    int *top_list = nullptr;
    int *top_count = nullptr;
    unsigned long long *trace = nullptr;  // profiling builds only: timestamps of the kernel's phases, else null
};
bool partition_takes_partials(int m);
void set_select_trace(unsigned long long *p);  // profiling builds: phase stamps of topk_kernel (8 words), or null
hipError_t launch_partition(const float *scores, int m, int n_ret, int n_cand, unsigned char *region, int *ret_idx,
                            int *cand_idx, hipStream_t s, const PartitionExtra *extra = nullptr);
// Per sequence b (grid = B): select k.k[b] of n_cand candidates by cscore[b*cs_stride + i]; writes the candidate
// bytes of mask[b][m], active_idx[b*act_stride + n_ret .. n_ret+k), n_active[b], sel_idx (sequence 0, only when
// active_idx is null), each if non-null.  With union_list non-null also: selflag [B][n_cand] (scratch), and the
// union of the B selections: union_list[n_ret..] = candidates selected by any b (ascending), *n_union = n_ret +
// their number; the prefix union_list[0..n_ret) = ret_idx is written by the caller once per partition.  union_ctr
// is a zeroed counter that the kernel leaves at zero.
hipError_t launch_topk(const float *cscore, int cs_stride, const int *cand_idx, int n_cand, int n_ret, int m, int B,
                       BatchK k, int act_stride, unsigned char *mask, int *active_idx, int *n_active, int *sel_idx,
                       unsigned char *selflag, int *union_ctr, int *union_list, int *n_union, hipStream_t s);
// Partition-constant step state: mask[b][j] = (region[j] == retained), active_idx[b][0..n_ret) = ret_idx.
// With cand_idx / rc_idx / ulist given it also writes rc_idx = cand_idx ++ ret_idx and ulist[0..n_ret) = ret_idx.
// With `clear` given the same launch zeroes that buffer's words.
struct StridedClear {
    int *p = nullptr;  // n slots of `words` ints (<= 256), `stride` ints apart
    int n = 0, stride = 0, words = 0;
};
// hc[t][c] = h_all[t][list[c]] for c < *n_list, t < T (bf16 bits): the columns of the listed channels moved next to
// each other.  With `compact` given the same launch does this as well (the list must be final when it starts).
struct CompactJob {
    const uint16_t *h_all = nullptr;
    int ldh = 0, T = 0;
    const int *list = nullptr, *n_list = nullptr;
    uint16_t *hc = nullptr;
    int ldhc = 0;  // even
};
constexpr int kCompactRows = 8;  // tokens a workgroup of the compaction walks
// The compaction's workgroup (bx, by) of 256 threads: positions 512 bx .. + 511, tokens kCompactRows by .. + 7.
__device__ __forceinline__ void compact_hidden_block(const CompactJob &job, int bx, int by)
{
    const int a = *job.n_list;
    const int c = (bx * 256 + (int)threadIdx.x) * 2;  // a thread owns two adjacent positions (one 32-bit store)
    const int t0 = by * kCompactRows, t1 = min(job.T, t0 + kCompactRows);
    if (c >= a) {
        // the columns between the list's end and the end of its last 64-channel k-step are read by the direct-load
        // GEMM (against rows of zeros): they must not keep what an earlier, longer list left there
        if (c < min((a + 63) / 64 * 64, job.ldhc))
            for (int t = t0; t < t1; ++t) *reinterpret_cast<uint32_t *>(job.hc + (size_t)t * job.ldhc + c) = 0u;
        return;
    }
    const int j0 = job.list[c], j1 = c + 1 < a ? job.list[c + 1] : -1;
    for (int t = t0; t < t1; ++t) {
        const uint16_t *row = job.h_all + (size_t)t * job.ldh;
        const uint32_t v = (uint32_t)row[j0] | (j1 >= 0 ? (uint32_t)row[j1] << 16 : 0u);
        *reinterpret_cast<uint32_t *>(job.hc + (size_t)t * job.ldhc + c) = v;
    }
}
hipError_t launch_step_state_init(const unsigned char *region, int m, const int *ret_idx, int n_ret, int rows,
                                  int act_stride, unsigned char *mask, int *active_idx, hipStream_t s,
                                  const int *cand_idx = nullptr, int n_cand = 0, int *rc_idx = nullptr,
                                  int *ulist = nullptr, const StridedClear *clear = nullptr,
                                  const CompactJob *compact = nullptr);
// mask rows -> ascending list of channels active in any row.  With pad_hc given ([pad_T][pad_ld] bf16, pad_ld a
// multiple of 64) the launch also zeroes its columns from the list's length up to the next multiple of 64 (what the
// direct-load GEMM reads beyond a compact H's last column).
hipError_t launch_mask_to_list(const unsigned char *mask, int rows, int m, int *list, int *n_list, hipStream_t s,
                               uint16_t *pad_hc = nullptr, int pad_ld = 0, int pad_T = 0);

// ---- decode GEMVs (pop_gemv.hip) ----
// h[b][j] = silu(x_b . gate_j) * (x_b . up_j) for j in rows[0..n_rows); if cscore != null, rows [0, n_score)
// also get cscore[b][pos] = nrm[j] * |h|.  n_rows_dev (optional) overrides n_rows with a device-side count.
hipError_t launch_gateup(const void *w, int is_bf16, int d, int m, const void *x, int B, const int *rows, int n_rows,
                         const int *n_rows_dev, float *h, const float *nrm, float *cscore, int cs_stride, int n_score,
                         int n_cu, hipStream_t s);
// y[b][:] = sum_{i<n} hm(b, list[i]) * w[list[i]][2][:], hm = h[b][j] (masked by mask[b][j] when mask != null).
// Two stages: slab partials then a fixed-order reduction; y written as float32 or bf16.
hipError_t launch_down(const void *w, int is_bf16, int d, int m, const int *list, const int *n_dev, int n_host,
                       const float *h, const unsigned char *mask, int mask_stride, int B, float *partial, int n_slabs,
                       void *y, int y_bf16, hipStream_t s);
int down_num_slabs(int d, int is_bf16);
// Batched decode (2 <= B <= POP_MAX_BATCH) with the per-sequence selection inside the gate/up kernel: the listed
// rows are the n_cand candidates followed by the n_ret retained channels; all workgroups evaluate the candidates
// first, then the last B workgroups wait (bounded) for everybody's candidate scores and select for one sequence
// each while the others evaluate the retained channels.  Outputs as launch_gateup + launch_topk with a union
// request.  counters: [0] arrivals, [1] selectors done (both zero between launches); err_flag is set if a wait
// expired.  *fused = false (and nothing launched) when the shape does not allow it: use the two launches.
hipError_t launch_gateup_select(const void *w, int is_bf16, int d, int m, const void *x, int B, const int *rows,
                                float *h, const float *nrm, float *cscore, int cs_stride, const int *cand_idx,
                                int n_cand, int n_ret, BatchK k, int act_stride, unsigned char *mask, int *active_idx,
                                int *n_active, unsigned char *selflag, int *union_list, int *n_union, int *counters,
                                int *err_flag, int spin_limit, int n_cu, bool *fused, hipStream_t s);

// ---- fused single-sequence decode step (pop_decode_fused.hip) ----
struct FusedParams {
    const void *w;
    const void *x;
    int nvec, d, m;
    const int *ret_idx;
    int n_ret;
    const int *cand_idx;
    int n_cand, k;
    const float *nrm;
    float *h;                   // [m]
    float *cscore;              // [n_cand]
    unsigned char *mask;        // [m]
    int *active_idx;            // [>= n_ret + k]
    int *n_active;              // [1]
    // what the workgroups hand to each other: 64-bit words {value, epoch}
    unsigned long long *hc;     // [n_cand] a candidate's h (input-side reading: its step score), by candidate position
    unsigned long long *selw;   // [n_wg] per-workgroup selection word (selected candidate slots), 128 bytes apart
    float *partial;             // [n_wg][d] partial output rows (summed by decode_tail_kernel)
    int *ctr;                   // [0] epoch (>= 1), [1] workgroups that finished (back at zero when the kernel ends),
                                // [2] sticky error flag: a bounded wait gave up
    int spin_limit;             // looks a bounded wait takes before it gives up
    int input_side;             // candidates are ranked by || [gate_j, up_j] * |x_t| ||_2 instead of n_j |h_j|
    int n_static;               // retained rounds per worker
    unsigned long long *trace;  // profiling builds only: 8 timestamps per workgroup, else null
};

struct FusedPlan {
    int n_wg, block, per;
    int n_static;  // retained rounds per worker
};
int fused_max_workgroups();
size_t fused_selw_words();  // 64-bit words of the selection-word buffer (one per workgroup, spaced apart)
// Launch shape for (d, dtype, region sizes); false when the fused kernel does not support the shape.
bool fused_plan(int d, int is_bf16, int n_ret, int n_cand, int wg_target, FusedPlan *pl);
// Largest grid of this shape that is co-resident on n_cu compute units.
hipError_t fused_resident_limit(int is_bf16, const FusedPlan &pl, int n_cu, int *max_wg);
hipError_t launch_decode_fused(const FusedPlan &pl, int is_bf16, FusedParams &p, hipStream_t s);
hipError_t launch_decode_tail(const float *partial, int n_wg, int d, void *y, int y_bf16, hipStream_t s);
hipError_t launch_fill_int(int *p, int n, int value, hipStream_t s);

// ---- measurement aids (pop_probe.hip): bare reads, nothing of the method ----
hipError_t launch_probe_read(const void *buf, size_t bytes, int workgroups, unsigned int *sink, hipStream_t s);
hipError_t launch_probe_step_read(const void *w, int nvec, const int *gu_list, int n_gu, const int *dn_ret,
                                  int n_dn_ret, const int *dn_sel, int n_dn_sel, int workgroups, unsigned int *sink,
                                  hipStream_t s);

// ---- prefill (pop_prefill.hip) ----
// s2_part[tile][j] = sum over the tile's tokens of H[t][j]^2, one row per token tile.
int prefill_num_tiles(int T, int is_bf16);  // upper bound on the rows used, for sizing s2_part
int prefill_rows_used(int T, int is_bf16, int m, int n_cu);  // rows the launch below writes for this T
// With `fin`, launches for which prefill_forms_scores holds (bf16 layers, prompts of one tile per compute unit) also leave scores[j] = nrm[j] * sqrt(sum over the token tiles, in tile
// order and in double, of s2_part[tile][j]) (Eq. 3): the token tile of a channel chunk that finishes last does the sum.
// chunk_ctr: one int per channel chunk (m of them suffice), zero before the launch and zero again after it.
struct PrefillScores {
    int *chunk_ctr;
    const float *nrm;
    float *scores;
};
bool prefill_forms_scores(int is_bf16, int T, int m, int n_cu);
hipError_t launch_prefill_gateup(const void *w, int is_bf16, int d, int m, const void *x, int T, float *s2_part,
                                 int n_cu, hipStream_t s, const PrefillScores *fin = nullptr);
// bf16 layers: gate/up over the channels of a device-resident list (n_list: its length, on the device);
// hc[t][c] = bf16(H[t][list[c]]), times tmask[t][list[c]] if tmask ([T][m]) is given.  ldh % 8 == 0.
hipError_t launch_gateup_list_bf16(const void *w, int d, int m, const void *x, int T, const int *list, const int *n_list,
                                   const unsigned char *tmask, uint16_t *hc, int ldh, int n_cu, hipStream_t s);
// y[t][n] = sum_c hc[t][c] * w[list[c]][2][n] on the matrix cores; part (float32 [n_split][T][d]) is needed when
// n_split = down_gemm_splits(...) > 1.  With zero_row (256 bytes of zeros), d % 128 == 0 and ldh % 64 == 0 the
// operands go straight into LDS; that form reads hc columns up to the list length rounded up to 64, which must hold
// finite values.
int down_gemm_splits(int T, int d, int n_cu);
hipError_t launch_down_gemm_bf16(const void *w, int d, const int *list, const int *n_list, const uint16_t *hc, int ldh,
                                 int T, int n_split, float *part, void *y, int y_bf16, hipStream_t s,
                                 const uint16_t *zero_row = nullptr);
// bf16 layers: the prefill contraction (s2_part as in launch_prefill_gateup) that also keeps H:
// h_all[t][j] = bf16(H[t][j]), row stride ldh.
hipError_t launch_prefill_gateup_keep_bf16(const void *w, int d, int m, const void *x, int T, float *s2_part,
                                           uint16_t *h_all, int ldh, int n_cu, hipStream_t s,
                                           const PrefillScores *fin = nullptr);
// ---- input-side importance (pop_input_side.hip) ----
int input_side_groups(int T);  // row groups of a T-token prompt (sizes part below: [groups][d] doubles)
// s2[k] = sum_t x[t][k]^2 over the T rows (fixed summation order)
hipError_t launch_input_norms(const void *x, int is_bf16, int T, int d, double *part, float *s2, hipStream_t s);
// s2[b][k] = x[b][k]^2
hipError_t launch_input_squares(const void *x, int is_bf16, int B, int d, float *s2, hipStream_t s);
// out[q][p] = sqrt(sum_k (w_gate[j][k]^2 + w_up[j][k]^2) s2[q][k]), j = rows ? rows[p] : p, q < S, p < n_rows
hipError_t launch_input_side_scores(const void *w, int is_bf16, int d, const float *s2, int S, const int *rows,
                                    int n_rows, float *out, int out_stride, hipStream_t s);
// cs[b][p] <- sqrt(sum over b' < B of cs[b'][p]^2) for every b < B, p < n
hipError_t launch_aggregate_scores(float *cs, int cs_stride, int B, int n, hipStream_t s);
// any[j] = 1 if mask[t][j] != 0 for some t < rows, else 0
hipError_t launch_mask_any(const unsigned char *mask, int rows, int m, unsigned char *any, hipStream_t s);
// scores[j] = nrm[j] * sqrt(sum_tile s2_part[tile][j])
hipError_t launch_scores_from_partials(const float *s2_part, int n_tiles, int m, const float *nrm, float *scores,
                                       hipStream_t s);
// stand-alone column reduction of a materialised H[T][m] (pop_importance.hip); scratch: device memory of
// importance_reduce_scratch_bytes(T, m) bytes, 8-byte aligned, for the per-chunk partial sums
size_t importance_reduce_scratch_bytes(int T, int m);
hipError_t launch_importance_reduce(const void *h, int is_bf16, int T, int m, const float *nrm, float *scores,
                                    void *scratch, hipStream_t s);

}  // namespace pop
