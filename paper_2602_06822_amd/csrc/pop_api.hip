// C ABI of the POP pruned-FFN library: argument validation, layer state and kernel sequencing.
// Every step of the path runs in the HIP kernels of the sibling files; nothing here computes on the host
// except the integer region counts.
#include <stddef.h>
#include <stdint.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "pop_internal.h"

using namespace pop;

namespace {

thread_local char g_hip_err[256] = "";

int hip_fail(hipError_t e, const char *what)
{
    snprintf(g_hip_err, sizeof g_hip_err, "%s: %s", what, hipGetErrorString(e));
    return POP_EHIP;
}

#define POP_HIP(call)                                      \
    do {                                                   \
        hipError_t e__ = (call);                           \
        if (e__ != hipSuccess) return hip_fail(e__, #call); \
    } while (0)

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

// The kernels read activations and weights, and write y, with 16-byte accesses.
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#ifdef POP_TRACE
unsigned long long *g_trace = nullptr;  // profiling builds: device buffer the fused kernel stamps into
#endif

}  // namespace

struct pop_layer {
    int d = 0, m = 0, esize = 0, is_bf16 = 0, max_tokens = 0, max_batch = 0;
    void *w = nullptr;     // [m][3][d]: gate row, up row, down column of each channel
    float *nrm = nullptr;  // [m]
    int n_cu = 0, wg_target = 0;
    bool shared_mask = false;    // B > 1: one selection for the batch from scores aggregated over its sequences
    bool input_side = false;     // importance from the first projections and the FFN input (pop_layer_set_importance)
    float *in_s2 = nullptr;      // [max_batch][d]: squared input norms (input-side importance)
    double *in_part = nullptr;   // [row groups][d]: their partial sums over a prompt
    // partition
    bool has_partition = false;
    int n_ret = 0, n_cand = 0;
    float *scores = nullptr;           // [m]
    float *s2_part = nullptr;          // [tiles][m]
    int *pf_ctr = nullptr;             // [m] arrival counters of the prefill kernel's channel chunks (zero at rest)
    int tiles_cap = 0;
    unsigned char *region = nullptr;   // [m]
    int *ret_idx = nullptr;            // [m]
    int *cand_idx = nullptr;           // [m]
    int *rc_idx = nullptr;             // [m]: candidates then retained
    // decode step
    bool has_step = false, step_fused = false, ulist_prefix_ok = false;
    int strat_n_ret = -1, strat_n_cand = -1, strat_k = -1;  // decode strategy of the layer (pop_layer_set_strategy)
    int step_B = 0;
    bool fused_ok = false;             // the fused kernel supports this partition
    FusedPlan plan = {};
    int *sync = nullptr;               // [16]: [2] error flag of the batched kernels, [8..9] and [10..12] their counters
    // what the fused kernel's workgroups hand to each other: 64-bit words {value, epoch}
    unsigned long long *hc = nullptr;     // [m] a candidate's h, by candidate position
    unsigned long long *selw = nullptr;   // per-workgroup selection words
    int *fctr = nullptr;                  // [16]: [0] epoch, [1] finished workgroups, [2] sticky error flag
    int spin_limit = 1 << 16;             // looks a bounded in-kernel wait takes before it gives up
    BatchK step_k = {};
    float *h = nullptr;                // [max_batch][m]
    float *cscore = nullptr;           // [max_batch][m]
    unsigned char *mask = nullptr;     // [max_batch][m]
    unsigned char *selflag = nullptr;  // [m][POP_MAX_BATCH]: per-sequence selection by candidate position (B > 1)
    int *active_idx = nullptr;         // [max_batch][m]
    int *n_active = nullptr;           // [max_batch]
    int *ulist = nullptr;              // [m]
    int *n_ulist = nullptr;            // [1]
    float *partial = nullptr;          // max([n_slabs][max_batch][d], [fused workgroups][d])
    int n_slabs = 0;
    // whole-prompt pruned FFN on the matrix cores (bf16 layers), allocated at its first use
    uint16_t *ffn_hc = nullptr;        // [tokens][ldh] bf16: H of the active channels, compact
    size_t ffn_hc_cap = 0;             // elements
    uint16_t *ffn_hall = nullptr;      // [tokens][ldh] bf16: H of all channels, kept by pop_prefill_forward
    size_t ffn_hall_cap = 0;           // elements
    float *ffn_part = nullptr;         // [splits][tokens][d]: partial outputs of the split contraction
    size_t ffn_part_cap = 0;           // elements
    unsigned char *ffn_any = nullptr;  // [m]: channels active in any row of a per-token mask
    int *top_list = nullptr;           // [m] + 1: the prompt's own active channels (ascending), then their number
    uint16_t *zero_row = nullptr;      // 256 bytes of zeros: stands in for weight rows beyond a channel list
};

namespace {

// Launch shape of the fused single-sequence step for the layer's current region sizes, sized to be co-resident.
int plan_fused_step(pop_layer *L)
{
    L->fused_ok = fused_plan(L->d, L->is_bf16, L->n_ret, L->n_cand, L->wg_target, &L->plan);
    if (L->fused_ok) {
        int max_wg = 0;
        POP_HIP(fused_resident_limit(L->is_bf16, L->plan, L->n_cu, &max_wg));
        if (max_wg < 2) {
            L->fused_ok = false;
        } else if (L->plan.n_wg > max_wg) {
            L->fused_ok = fused_plan(L->d, L->is_bf16, L->n_ret, L->n_cand, max_wg, &L->plan) && L->plan.n_wg <= max_wg;
        }
    }
    return POP_OK;
}

// Copies the step's selection results from the layer's state to the caller's buffers (each may be null).
int copy_step_outputs(pop_layer *L, int B, float *cand_scores, unsigned char *mask, int *active_idx, int *n_active,
                      hipStream_t s)
{
    const int m = L->m, n_ret = L->n_ret, n_cand = L->n_cand;
    if (cand_scores && n_cand)
        POP_HIP(hipMemcpy2DAsync(cand_scores, (size_t)n_cand * 4, L->cscore, (size_t)m * 4, (size_t)n_cand * 4, B,
                                 hipMemcpyDeviceToDevice, s));
    if (mask) POP_HIP(hipMemcpyAsync(mask, L->mask, (size_t)B * m, hipMemcpyDeviceToDevice, s));
    if (active_idx && n_ret + n_cand)
        POP_HIP(hipMemcpy2DAsync(active_idx, (size_t)(n_ret + n_cand) * 4, L->active_idx, (size_t)m * 4,
                                 (size_t)(n_ret + n_cand) * 4, B, hipMemcpyDeviceToDevice, s));
    if (n_active) POP_HIP(hipMemcpyAsync(n_active, L->n_active, (size_t)B * 4, hipMemcpyDeviceToDevice, s));
    return POP_OK;
}

// From this many tokens on a bf16 layer's stand-alone pruned FFN runs on the matrix cores (below it, the decode
// kernels take the tokens eight at a time).
constexpr int kFfnMfmaMinTokens = 32;

// hipMalloc that leaves no pending error behind when it fails (a later launch check would report it as its own).
bool dev_alloc(void **p, size_t bytes)
{
    if (hipMalloc(p, bytes) == hipSuccess) return true;
    (void)hipGetLastError();
    *p = nullptr;
    return false;
}

// Makes *p hold at least `need` elements of esize bytes; the old contents are dropped.  Growing frees first, which
// synchronises the device.
int grow(void **p, size_t *cap, size_t need, size_t esize)
{
    if (need <= *cap) return POP_OK;
    if (*p) POP_HIP(hipFree(*p));
    *p = nullptr, *cap = 0;
    if (!dev_alloc(p, need * esize)) return POP_ENOMEM;
    *cap = need;
    return POP_OK;
}

// Scratch of the prompt-sized forward pass for T tokens: compact H, split partials, the byte mask; with keep_all
// also H of all channels.  Returns the row stride of the H buffers and the number of contraction splits.
int ffn_scratch(pop_layer *L, int T, bool keep_all, int *ldh, int *n_split, hipStream_t s, bool shorter_too = false)
{
    // rows are whole 64-channel k-steps long: the direct-load GEMM reads the columns between a list's end and the end
    // of its last k-step (times rows of zeros, so they only have to be finite; every writer of compact H zeroes them).
    // New buffers are cleared by a kernel on the caller's stream, ahead of the kernels that read them.
    *ldh = (L->m + 63) / 64 * 64;
    *n_split = down_gemm_splits(T, L->d, L->n_cu);
    const size_t hc_before = L->ffn_hc_cap;
    int rc = grow((void **)&L->ffn_hc, &L->ffn_hc_cap, (size_t)T * *ldh, sizeof(uint16_t));
    if (rc == POP_OK && L->ffn_hc_cap != hc_before)
        POP_HIP(launch_fill_int((int *)L->ffn_hc, (int)(L->ffn_hc_cap / 2), 0, s));
    if (rc == POP_OK && !L->zero_row) {
        if (!dev_alloc((void **)&L->zero_row, 256)) return POP_ENOMEM;
        POP_HIP(launch_fill_int((int *)L->zero_row, 64, 0, s));
    }
    size_t part_rows = *n_split > 1 ? (size_t)*n_split * T : 0;
    if (shorter_too)  // a shorter prompt is split more ways: room for every prompt length up to T
        for (int t = 1; t < T; ++t) {
            const size_t r = (size_t)down_gemm_splits(t, L->d, L->n_cu) * t;
            if (r > part_rows) part_rows = r;
        }
    if (rc == POP_OK && part_rows)
        rc = grow((void **)&L->ffn_part, &L->ffn_part_cap, part_rows * L->d, sizeof(float));
    if (rc == POP_OK && keep_all) rc = grow((void **)&L->ffn_hall, &L->ffn_hall_cap, (size_t)T * *ldh, sizeof(uint16_t));
    if (rc == POP_OK && !L->ffn_any && !dev_alloc((void **)&L->ffn_any, ((size_t)L->m + 3) / 4 * 4))
        rc = POP_ENOMEM;
    return rc;
}

// Whole-prompt pruned FFN (Sec. 3.4: forward pass under the pruning structure): active list from the mask(s),
// gate/up over the listed channels with H written in compact bf16 form, then the K-gathered down-projection GEMM.
int pruned_ffn_mfma(pop_layer *L, const void *x, int T, const unsigned char *mask, int mask_rows, void *y, int y_bf16,
                    hipStream_t s)
{
    const int m = L->m, d = L->d;
    int ldh, n_split;
    { int rc = ffn_scratch(L, T, false, &ldh, &n_split, s); if (rc != POP_OK) return rc; }
    const unsigned char *tmask = nullptr;
    if (mask_rows == 1) {
        POP_HIP(launch_mask_to_list(mask, 1, m, L->ulist, L->n_ulist, s, L->ffn_hc, ldh, T));
    } else {
        POP_HIP(launch_mask_any(mask, T, m, L->ffn_any, s));
        POP_HIP(launch_mask_to_list(L->ffn_any, 1, m, L->ulist, L->n_ulist, s, L->ffn_hc, ldh, T));
        tmask = mask;
    }
    POP_HIP(launch_gateup_list_bf16(L->w, d, m, x, T, L->ulist, L->n_ulist, tmask, L->ffn_hc, ldh, L->n_cu, s));
    POP_HIP(launch_down_gemm_bf16(L->w, d, L->ulist, L->n_ulist, L->ffn_hc, ldh, T, n_split, L->ffn_part, y, y_bf16, s,
                                  L->zero_row));
    return POP_OK;
}

// Scores, partition and partition-constant step state from s2_part (the second half of the prefilling stage).
// n_top >= 0: the same launch also leaves the n_top best channels as an ascending list with its length in top_list
// and, with top_mask, as a byte mask in ffn_any; compact: a column gather that the state launch takes along.
int finish_partition(pop_layer *L, int T, int n_ret, int n_cand, float *scores, unsigned char *region, int *ret_idx,
                     int *cand_idx, hipStream_t s, bool scores_ready, int n_top = -1, bool top_mask = true,
                     const CompactJob *compact = nullptr)
{
    const int m = L->m;
    // the partition launch also forms the scores from the contraction's partial rows (the input-side scores are
    // already in place) and clears the step counters; one more launch writes everything that is constant per
    // partition (retained bytes of every mask row, retained prefix of every active list and of the union list, the
    // candidate-then-retained list)
    PartitionExtra ex;
    const bool from_partials = !scores_ready && partition_takes_partials(m);
    if (!scores_ready && !from_partials)
        POP_HIP(launch_scores_from_partials(L->s2_part, prefill_rows_used(T, L->is_bf16, m, L->n_cu), m, L->nrm, L->scores, s));
    if (from_partials) {
        ex.s2_part = L->s2_part, ex.n_tiles = prefill_rows_used(T, L->is_bf16, m, L->n_cu), ex.nrm = L->nrm;
        ex.scores_out = L->scores;
    }
    ex.sync = L->sync, ex.n_sync = 16;
#ifdef POP_TRACE
    ex.trace = g_trace ? g_trace + 1000 * 8 : nullptr;
#endif
    if (n_top >= 0) {
        ex.n_top = n_top, ex.top_list = L->top_list, ex.top_count = L->top_list + m;
        ex.top_mask = top_mask ? L->ffn_any : nullptr;
    }
    POP_HIP(launch_partition(L->scores, m, n_ret, n_cand, L->region, L->ret_idx, L->cand_idx, s, &ex));
    POP_HIP(launch_step_state_init(L->region, m, L->ret_idx, n_ret, L->max_batch, m, L->mask, L->active_idx, s,
                                   L->cand_idx, n_cand, L->rc_idx, L->ulist, nullptr, compact));
    L->ulist_prefix_ok = true;
    L->n_ret = n_ret;
    L->n_cand = n_cand;
    { int rc = plan_fused_step(L); if (rc != POP_OK) return rc; }
    if (scores) POP_HIP(hipMemcpyAsync(scores, L->scores, (size_t)m * 4, hipMemcpyDeviceToDevice, s));
    if (region) POP_HIP(hipMemcpyAsync(region, L->region, (size_t)m, hipMemcpyDeviceToDevice, s));
    if (ret_idx && n_ret) POP_HIP(hipMemcpyAsync(ret_idx, L->ret_idx, (size_t)n_ret * 4, hipMemcpyDeviceToDevice, s));
    if (cand_idx && n_cand)
        POP_HIP(hipMemcpyAsync(cand_idx, L->cand_idx, (size_t)n_cand * 4, hipMemcpyDeviceToDevice, s));
    L->has_partition = true;
    return POP_OK;
}

// Arguments of the fused single-sequence kernel for the layer's current partition.
FusedParams fused_params(pop_layer *L, const void *x_t, int k)
{
    FusedParams p = {};
    p.w = L->w;
    p.x = x_t;
    p.nvec = L->d / (L->is_bf16 ? 8 : 4);
    p.d = L->d;
    p.m = L->m;
    p.ret_idx = L->ret_idx;
    p.n_ret = L->n_ret;
    p.cand_idx = L->cand_idx;
    p.n_cand = L->n_cand;
    p.k = k;
    p.nrm = L->nrm;
    p.h = L->h;
    p.cscore = L->cscore;
    p.mask = L->mask;
    p.active_idx = L->active_idx;
    p.n_active = L->n_active;
    p.hc = L->hc;
    p.selw = L->selw;
    p.partial = L->partial;
    p.ctr = L->fctr;
    p.spin_limit = L->spin_limit;
    p.input_side = L->input_side ? 1 : 0;
#ifdef POP_TRACE
    p.trace = g_trace;
#endif
    return p;
}

}  // namespace

extern "C" {

int pop_version(void) { return 100; }

const char *pop_strerror(int status)
{
    switch (status) {
        case POP_OK: return "ok";
        case POP_EINVAL: return "invalid argument";
        case POP_ESHAPE: return "inconsistent sizes";
        case POP_ENOMEM: return "out of device memory";
        case POP_EHIP: return "HIP call failed";
        case POP_ESTATE: return "call order violated";
        case POP_EUNSUPPORTED: return "unsupported configuration";
        case POP_EDEVICE: return "a kernel gave up a bounded wait";
        default: return "unknown status";
    }
}

const char *pop_last_hip_error(void) { return g_hip_err; }

int pop_region_counts(int m, double f_ret, double f_cand, int *n_ret, int *n_cand, int *n_prn)
{
    if (!n_ret || !n_cand || !n_prn) return POP_EINVAL;
    if (m <= 0 || !(f_ret >= 0.0) || !(f_cand >= 0.0) || !(f_ret + f_cand <= 1.0 + 1e-12)) return POP_EINVAL;
    long long a = (long long)floor(f_ret * (double)m + 0.5);
    long long b = (long long)floor((f_ret + f_cand) * (double)m + 0.5);
    if (a > m) a = m;
    if (b > m) b = m;
    if (b < a) b = a;
    *n_ret = (int)a;
    *n_cand = (int)(b - a);
    *n_prn = (int)(m - b);
    return POP_OK;
}

int pop_k_for_ratio(int m, double r, int n_ret, int n_cand, int *k)
{
    if (!k) return POP_EINVAL;
    if (m <= 0 || !(r >= 0.0) || !(r <= 1.0) || n_ret < 0 || n_cand < 0 || n_ret + n_cand > m) return POP_EINVAL;
    long long a = (long long)floor((1.0 - r) * (double)m + 0.5);
    long long kk = a - n_ret;
    if (kk < 0) kk = 0;
    if (kk > n_cand) kk = n_cand;
    *k = (int)kk;
    return POP_OK;
}

int pop_strategy_counts(int strategy, int m, double r, double gamma, int *n_ret, int *n_cand, int *k)
{
    if (!n_ret || !n_cand || !k) return POP_EINVAL;
    if (m <= 0 || !(r >= 0.0) || !(r <= 1.0) || !(gamma >= 0.0) || !(gamma <= 1.0)) return POP_EINVAL;
    const int a = (int)floor((1.0 - r) * (double)m + 0.5);  // active channels per token
    switch (strategy) {
    case POP_STRATEGY_STATIC_MASK:
        *n_ret = a, *n_cand = 0, *k = 0;
        return POP_OK;
    case POP_STRATEGY_RESCORE_ALL:
        *n_ret = 0, *n_cand = m, *k = a;
        return POP_OK;
    case POP_STRATEGY_POP: {
        if (1.0 - r - gamma / 2 < 0.0 || 1.0 - r + gamma / 2 > 1.0) return POP_EINVAL;
        int n_prn = 0;
        int rc = pop_region_counts(m, 1.0 - r - gamma / 2, gamma, n_ret, n_cand, &n_prn);
        if (rc != POP_OK) return rc;
        return pop_k_for_ratio(m, r, *n_ret, *n_cand, k);
    }
    default:
        return POP_EINVAL;
    }
}

int pop_layer_destroy(pop_layer_t *L)
{
    if (!L) return POP_EINVAL;
    void *ptrs[] = {L->w,      L->nrm, L->scores, L->s2_part, L->region,     L->ret_idx,  L->cand_idx, L->rc_idx,
                    L->h,      L->cscore, L->mask, L->selflag, L->active_idx, L->n_active, L->ulist, L->n_ulist,  L->partial,
                    L->sync,   L->hc, L->selw, L->fctr, L->pf_ctr, L->ffn_hc, L->ffn_part, L->ffn_any, L->ffn_hall, L->in_s2, L->in_part, L->top_list, L->zero_row};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    delete L;
    return POP_OK;
}

int pop_layer_create(pop_layer_t **out, int d, int m, pop_dtype_t wdtype, const void *w_gate, const void *w_up,
                     const void *w_down, int max_tokens, int max_batch, void *stream)
{
    if (!out) return POP_EINVAL;
    *out = nullptr;
    if (!w_gate || !w_up || !w_down) return POP_EINVAL;
    if (!aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down)) return POP_EINVAL;
    if (wdtype != POP_F32 && wdtype != POP_BF16) return POP_EINVAL;
    if (d <= 0 || m <= 0 || max_tokens < 1) return POP_ESHAPE;
    if (max_batch < 1 || max_batch > POP_MAX_BATCH) return POP_ESHAPE;
    const int is_bf16 = wdtype == POP_BF16, esize = is_bf16 ? 2 : 4;
    if ((d * esize) % 16 != 0) return POP_EUNSUPPORTED;
    if ((long long)m * 3 * d >= (1LL << 34)) return POP_EUNSUPPORTED;  // 16-byte vectors of w are indexed with 32 bits

    int dev = 0, lds_max = 0, n_cu = 0;
    POP_HIP(hipGetDevice(&dev));
    POP_HIP(hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev));
    POP_HIP(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    if ((long long)max_batch * d * esize > lds_max) return POP_EUNSUPPORTED;  // x_t is staged in LDS

    pop_layer *L = new (std::nothrow) pop_layer;
    if (!L) return POP_ENOMEM;
    L->d = d;
    L->m = m;
    L->esize = esize;
    L->is_bf16 = is_bf16;
    L->max_tokens = max_tokens;
    L->max_batch = max_batch;
    L->tiles_cap = prefill_num_tiles(max_tokens, is_bf16);
    L->n_slabs = down_num_slabs(d, is_bf16);
    L->n_cu = n_cu;
    L->wg_target = n_cu;  // one workgroup per compute unit; POP_FUSED_WGS overrides (tuning)
    if (const char *e = getenv("POP_FUSED_WGS")) {
        int v = atoi(e);
        if (v >= 2 && v <= fused_max_workgroups()) L->wg_target = v;
    }
    if (L->wg_target > fused_max_workgroups()) L->wg_target = fused_max_workgroups();
    if (const char *e = getenv("POP_WAIT_LIMIT")) L->spin_limit = atoi(e) < 0 ? 0 : atoi(e);  // (tuning, tests)

    const size_t mm = (size_t)m, B = (size_t)max_batch;
    struct Req { void **p; size_t bytes; };
    Req reqs[] = {
        {&L->w, mm * 3 * d * esize},
        {(void **)&L->nrm, mm * 4},
        {(void **)&L->scores, mm * 4},
        {(void **)&L->s2_part, (size_t)L->tiles_cap * mm * 4},
        {(void **)&L->region, mm},
        {(void **)&L->ret_idx, mm * 4},
        {(void **)&L->cand_idx, mm * 4},
        {(void **)&L->rc_idx, mm * 4},
        {(void **)&L->h, B * mm * 4},
        {(void **)&L->cscore, B * mm * 4},
        {(void **)&L->mask, B * mm},
        {(void **)&L->selflag, (size_t)POP_MAX_BATCH * mm},
        {(void **)&L->active_idx, B * mm * 4},
        {(void **)&L->n_active, B * 4},
        {(void **)&L->ulist, mm * 4},
        {(void **)&L->n_ulist, 4},
        {(void **)&L->partial, ((size_t)L->n_slabs * B > (size_t)fused_max_workgroups() ? (size_t)L->n_slabs * B
                                                                                        : (size_t)fused_max_workgroups()) * d * 4},
        {(void **)&L->sync, 64},
        {(void **)&L->hc, mm * 8},
        {(void **)&L->selw, fused_selw_words() * 8},
        {(void **)&L->fctr, 64},
        {(void **)&L->pf_ctr, mm * 4},
    };
    for (const Req &r : reqs) {
        hipError_t e = hipMalloc(r.p, r.bytes);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            pop_layer_destroy(L);
            return e == hipErrorOutOfMemory ? POP_ENOMEM : hip_fail(e, "hipMalloc");
        }
    }
    hipStream_t s = as_stream(stream);
    hipError_t e = launch_repack(w_gate, w_up, w_down, d, m, esize, L->w, L->nrm, is_bf16, s);
    if (e == hipSuccess) e = launch_fill_int(L->sync, 16, 0, s);
    // the words the fused kernel's workgroups exchange start out with epoch 0, the counter at 1: nothing stale can
    // ever look valid
    if (e == hipSuccess) e = hipMemsetAsync(L->hc, 0, mm * 8, s);
    if (e == hipSuccess) e = hipMemsetAsync(L->selw, 0, fused_selw_words() * 8, s);
    if (e == hipSuccess) e = launch_fill_int(L->fctr, 16, 0, s);
    if (e == hipSuccess) e = launch_fill_int(L->pf_ctr, m, 0, s);
    if (e == hipSuccess) e = launch_fill_int(L->fctr, 1, 1, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) {
        pop_layer_destroy(L);
        return hip_fail(e, "layer repack");
    }
    *out = L;
    return POP_OK;
}

int pop_prefill_partition(pop_layer_t *L, const void *x, int T, int n_ret, int n_cand, float *scores,
                          unsigned char *region, int *ret_idx, int *cand_idx, void *stream)
{
    if (!L) return POP_EINVAL;
    if (T < 0 || T > L->max_tokens) return POP_ESHAPE;
    if (T > 0 && (!x || !aligned16(x))) return POP_EINVAL;
    if (n_ret == POP_FROM_STRATEGY && n_cand == POP_FROM_STRATEGY) {
        if (L->strat_n_ret < 0) return POP_ESTATE;
        n_ret = L->strat_n_ret, n_cand = L->strat_n_cand;
    }
    if (n_ret < 0 || n_cand < 0 || (long long)n_ret + n_cand > L->m) return POP_ESHAPE;
    hipStream_t s = as_stream(stream);
    const int m = L->m;
    L->has_partition = false;
    L->has_step = false;
    if (T == 0) {
        // no tokens: every importance is zero under either reading, and the order falls back on the channel index
        POP_HIP(launch_fill_int((int *)L->scores, m, 0, s));
    } else if (L->input_side) {
        POP_HIP(launch_input_norms(x, L->is_bf16, T, L->d, L->in_part, L->in_s2, s));
        POP_HIP(launch_input_side_scores(L->w, L->is_bf16, L->d, L->in_s2, 1, nullptr, m, L->scores, m, s));
    } else {
        const PrefillScores fin{L->pf_ctr, L->nrm, L->scores};
        POP_HIP(launch_prefill_gateup(L->w, L->is_bf16, L->d, m, x, T, L->s2_part, L->n_cu, s, &fin));
    }
    return finish_partition(L, T, n_ret, n_cand, scores, region, ret_idx, cand_idx, s,
                            T == 0 || L->input_side || prefill_forms_scores(L->is_bf16, T, m, L->n_cu));
}

int pop_prefill_forward(pop_layer_t *L, const void *x, int T, int n_ret, int n_cand, int k0, void *y, pop_dtype_t ydtype,
                        float *scores, unsigned char *region, int *ret_idx, int *cand_idx, unsigned char *mask,
                        void *stream)
{
    if (!L) return POP_EINVAL;
    if (T < 0 || T > L->max_tokens) return POP_ESHAPE;
    if (T > 0 && (!x || !y || !aligned16(x) || !aligned16(y))) return POP_EINVAL;
    if (ydtype != POP_F32 && ydtype != POP_BF16) return POP_EINVAL;
    if (n_ret == POP_FROM_STRATEGY && n_cand == POP_FROM_STRATEGY) {
        if (L->strat_n_ret < 0) return POP_ESTATE;
        n_ret = L->strat_n_ret, n_cand = L->strat_n_cand;
        if (k0 == POP_FROM_STRATEGY) k0 = L->strat_k;
    }
    if (n_ret < 0 || n_cand < 0 || (long long)n_ret + n_cand > L->m) return POP_ESHAPE;
    if (k0 < 0 || k0 > n_cand) return POP_ESHAPE;
    hipStream_t s = as_stream(stream);
    const int m = L->m, d = L->d;
    // H of the importance contraction is kept and the output runs on the matrix cores (the input-side importance
    // has no such contraction: partition first, then the masked FFN)
    const bool keep = L->is_bf16 && T >= kFfnMfmaMinTokens && !L->input_side;
    L->has_partition = false;
    L->has_step = false;
    int ldh = 0, n_split = 1;
    if (keep) {
        int rc = ffn_scratch(L, T, true, &ldh, &n_split, s);
        if (rc != POP_OK) return rc;
        const PrefillScores fin{L->pf_ctr, L->nrm, L->scores};
        POP_HIP(launch_prefill_gateup_keep_bf16(L->w, d, m, x, T, L->s2_part, L->ffn_hall, ldh, L->n_cu, s, &fin));
    } else {
        if (!L->ffn_any && !dev_alloc((void **)&L->ffn_any, ((size_t)m + 3) / 4 * 4)) return POP_ENOMEM;
        if (T == 0) {
            POP_HIP(launch_fill_int((int *)L->scores, m, 0, s));  // no tokens: all importances zero
        } else if (L->input_side) {
            POP_HIP(launch_input_norms(x, L->is_bf16, T, d, L->in_part, L->in_s2, s));
            POP_HIP(launch_input_side_scores(L->w, L->is_bf16, d, L->in_s2, 1, nullptr, m, L->scores, m, s));
        } else {
            const PrefillScores fin{L->pf_ctr, L->nrm, L->scores};
            POP_HIP(launch_prefill_gateup(L->w, L->is_bf16, d, m, x, T, L->s2_part, L->n_cu, s, &fin));
        }
    }
    // prefill mask: retained channels plus the best k0 candidates by prefill score, i.e. the n_ret + k0 best channels
    // of the partition's own order: the partition launch emits them as well (mask bytes and ascending list)
    if (!L->top_list && !dev_alloc((void **)&L->top_list, ((size_t)m + 1) * sizeof(int))) return POP_ENOMEM;
    // (the byte mask only where somebody reads it: the caller, or the path below that works from a mask; the gather of
    // the active columns of H into compact form rides along with the partition's state launch)
    CompactJob gather;
    if (keep) {
        gather.h_all = L->ffn_hall, gather.ldh = ldh, gather.T = T, gather.list = L->top_list;
        gather.n_list = L->top_list + m, gather.hc = L->ffn_hc, gather.ldhc = ldh;
    }
    {
        int rc = finish_partition(L, T, n_ret, n_cand, scores, region, ret_idx, cand_idx, s,
                                  T == 0 || L->input_side || prefill_forms_scores(L->is_bf16, T, m, L->n_cu), n_ret + k0, mask || !keep, keep ? &gather : nullptr);
        if (rc != POP_OK) return rc;
    }
    unsigned char *pm = L->ffn_any;
    if (mask) POP_HIP(hipMemcpyAsync(mask, pm, (size_t)m, hipMemcpyDeviceToDevice, s));
    if (T == 0) return POP_OK;  // no token rows to produce
    if (keep) {
        POP_HIP(launch_down_gemm_bf16(L->w, d, L->top_list, L->top_list + m, L->ffn_hc, ldh, T, n_split, L->ffn_part, y,
                                      ydtype == POP_BF16, s, L->zero_row));
        return POP_OK;
    }
    const int rc = pop_pruned_ffn(L, x, T, pm, 1, y, ydtype, stream);
    return rc;
}

int pop_decode_mask(pop_layer_t *L, const void *x_t, int B, const int *k, float *cand_scores, unsigned char *mask,
                    int *active_idx, int *n_active, void *stream)
{
    if (!L || !x_t || !aligned16(x_t)) return POP_EINVAL;
    if (!L->has_partition) return POP_ESTATE;
    if (!k && L->strat_k < 0) return POP_EINVAL;  // no per-sequence counts and no strategy to take them from
    if (B < 1 || B > L->max_batch) return POP_ESHAPE;
    BatchK kk = {};
    for (int b = 0; b < B; ++b) {
        const int kb = k ? k[b] : L->strat_k;
        if (kb < 0 || kb > L->n_cand) return POP_ESHAPE;
        kk.k[b] = kb;
    }
    hipStream_t s = as_stream(stream);
    const int m = L->m, n_ret = L->n_ret, n_cand = L->n_cand;
    L->has_step = false;
    if (B == 1 && L->fused_ok) {
        FusedParams p = fused_params(L, x_t, kk.k[0]);
        POP_HIP(launch_decode_fused(L->plan, L->is_bf16, p, s));
        L->step_fused = true;
    } else {
        if (B > 1) {
            if (!L->ulist_prefix_ok && n_ret)
                POP_HIP(hipMemcpyAsync(L->ulist, L->ret_idx, (size_t)n_ret * 4, hipMemcpyDeviceToDevice, s));
            L->ulist_prefix_ok = true;
        }
        if (L->input_side) {
            // (a single sequence on a shape the fused kernel takes went there: it scores the candidates from the same
            // rows it reads for h.)  Here candidates are scored from their gate and up rows and |x_t| alone, so the
            // selection comes first and the forward pass runs over retained and selected channels only
            const bool shared = B > 1 && L->shared_mask;
            if (shared)
                for (int b = 1; b < B; ++b)
                    if (kk.k[b] != kk.k[0]) return POP_ESHAPE;
            POP_HIP(launch_input_squares(x_t, L->is_bf16, B, L->d, L->in_s2, s));
            POP_HIP(launch_input_side_scores(L->w, L->is_bf16, L->d, L->in_s2, B, L->cand_idx, n_cand, L->cscore, m, s));
            // one mask for the batch: the root of the sum of the sequences' squared scores is this reading's importance
            // over the step's B rows (Eq. 1-2 with s_k over tokens and samples); every row gets it
            if (shared) POP_HIP(launch_aggregate_scores(L->cscore, m, B, n_cand, s));
            POP_HIP(launch_topk(L->cscore, m, L->cand_idx, n_cand, n_ret, m, B, kk, m, L->mask, L->active_idx,
                                L->n_active, nullptr, B > 1 ? L->selflag : nullptr, L->sync + 8, B > 1 ? L->ulist : nullptr, L->n_ulist,
                                s));
            if (B == 1)
                POP_HIP(launch_gateup(L->w, L->is_bf16, L->d, m, x_t, 1, L->active_idx, n_ret + kk.k[0], nullptr, L->h,
                                      nullptr, nullptr, 0, 0, L->n_cu, s));
            else
                POP_HIP(launch_gateup(L->w, L->is_bf16, L->d, m, x_t, B, L->ulist, m, L->n_ulist, L->h, nullptr, nullptr,
                                      0, 0, L->n_cu, s));
            L->step_fused = false;
            { int rc = copy_step_outputs(L, B, cand_scores, mask, active_idx, n_active, s); if (rc != POP_OK) return rc; }
            L->step_B = B;
            L->step_k = kk;
            L->has_step = true;
            return POP_OK;
        }
        bool sel_inside = false;
        const bool shared = B > 1 && L->shared_mask;
        if (shared)
            for (int b = 1; b < B; ++b)
                if (kk.k[b] != kk.k[0]) return POP_ESHAPE;
        if (B > 1 && !shared)  // per-sequence top-k and their union inside the gate/up kernel, behind the retained channels
            POP_HIP(launch_gateup_select(L->w, L->is_bf16, L->d, m, x_t, B, L->rc_idx, L->h, L->nrm, L->cscore, m,
                                         L->cand_idx, n_cand, n_ret, kk, m, L->mask, L->active_idx, L->n_active,
                                         L->selflag, L->ulist, L->n_ulist, L->sync + 10, L->sync + 2, L->spin_limit,
                                         L->n_cu, &sel_inside, s));
        if (!sel_inside) {
            POP_HIP(launch_gateup(L->w, L->is_bf16, L->d, m, x_t, B, L->rc_idx, n_ret + n_cand, nullptr, L->h, L->nrm,
                                  L->cscore, m, n_cand, L->n_cu, s));
            // one mask for the batch: every sequence's row gets the scores aggregated over the batch, so the B
            // selections below come out identical
            if (shared) POP_HIP(launch_aggregate_scores(L->cscore, m, B, n_cand, s));
            // B > 1: the kernel also builds the union of the B selections for the batched down projection
            POP_HIP(launch_topk(L->cscore, m, L->cand_idx, n_cand, n_ret, m, B, kk, m, L->mask, L->active_idx,
                                L->n_active, nullptr, B > 1 ? L->selflag : nullptr, L->sync + 8, B > 1 ? L->ulist : nullptr, L->n_ulist,
                                s));
        }
        L->step_fused = false;
    }
    { int rc = copy_step_outputs(L, B, cand_scores, mask, active_idx, n_active, s); if (rc != POP_OK) return rc; }
    L->step_B = B;
    L->step_k = kk;
    L->has_step = true;
    return POP_OK;
}

int pop_decode_step(pop_layer_t *L, const void *x_t, int B, const int *k, void *y, pop_dtype_t ydtype,
                    float *cand_scores, unsigned char *mask, int *active_idx, int *n_active, void *stream)
{
    if (!L || !x_t || !y || !aligned16(x_t) || !aligned16(y)) return POP_EINVAL;
    if (ydtype != POP_F32 && ydtype != POP_BF16) return POP_EINVAL;
    if (!L->has_partition) return POP_ESTATE;
    if (!k && L->strat_k < 0) return POP_EINVAL;
    if (B < 1 || B > L->max_batch) return POP_ESHAPE;
    for (int b = 0; b < B; ++b) {
        const int kb = k ? k[b] : L->strat_k;
        if (kb < 0 || kb > L->n_cand) return POP_ESHAPE;
    }
    // the launches of the two calls (a single-sequence step on a shape the fused kernel takes: that kernel, then the
    // small kernel that sums its workgroups' partial outputs)
    int rc = pop_decode_mask(L, x_t, B, k, cand_scores, mask, active_idx, n_active, stream);
    if (rc != POP_OK) return rc;
    return pop_pruned_ffn(L, nullptr, B, nullptr, 0, y, ydtype, stream);
}

int pop_pruned_ffn(pop_layer_t *L, const void *x, int T, const unsigned char *mask, int mask_rows, void *y,
                   pop_dtype_t ydtype, void *stream)
{
    if (!L || !y || !aligned16(y)) return POP_EINVAL;
    if (ydtype != POP_F32 && ydtype != POP_BF16) return POP_EINVAL;
    hipStream_t s = as_stream(stream);
    const int m = L->m, d = L->d, y_bf16 = ydtype == POP_BF16, ysize = y_bf16 ? 2 : 4;
    if (!mask) {
        if (!L->has_step) return POP_ESTATE;
        if (T != L->step_B) return POP_ESHAPE;
        if (L->step_fused)
            POP_HIP(launch_decode_tail(L->partial, L->plan.n_wg, d, y, y_bf16, s));
        else if (T == 1)
            POP_HIP(launch_down(L->w, L->is_bf16, d, m, L->active_idx, nullptr, L->n_ret + L->step_k.k[0], L->h,
                                nullptr, 0, 1, L->partial, L->n_slabs, y, y_bf16, s));
        else
            POP_HIP(launch_down(L->w, L->is_bf16, d, m, L->ulist, L->n_ulist, 0, L->h, L->mask, m, T, L->partial,
                                L->n_slabs, y, y_bf16, s));
        return POP_OK;
    }
    if (!x || !aligned16(x)) return POP_EINVAL;
    if (T < 1) return POP_ESHAPE;
    if (mask_rows != 1 && mask_rows != T) return POP_ESHAPE;
    L->has_step = false;  // the step scratch is reused below
    L->ulist_prefix_ok = false;
    if (L->is_bf16 && T >= kFfnMfmaMinTokens) return pruned_ffn_mfma(L, x, T, mask, mask_rows, y, y_bf16, s);
    if (mask_rows == 1) POP_HIP(launch_mask_to_list(mask, 1, m, L->ulist, L->n_ulist, s));
    for (int t0 = 0; t0 < T; t0 += L->max_batch) {
        const int Bc = (T - t0 < L->max_batch) ? T - t0 : L->max_batch;
        const unsigned char *mk = mask_rows == 1 ? nullptr : mask + (size_t)t0 * m;
        if (mk) POP_HIP(launch_mask_to_list(mk, Bc, m, L->ulist, L->n_ulist, s));
        const char *xc = (const char *)x + (size_t)t0 * d * L->esize;
        POP_HIP(launch_gateup(L->w, L->is_bf16, d, m, xc, Bc, L->ulist, m, L->n_ulist, L->h, nullptr, nullptr, 0, 0,
                              L->n_cu, s));
        POP_HIP(launch_down(L->w, L->is_bf16, d, m, L->ulist, L->n_ulist, 0, L->h, mk, m, Bc, L->partial, L->n_slabs,
                            (char *)y + (size_t)t0 * d * ysize, y_bf16, s));
    }
    return POP_OK;
}

int pop_partition_from_scores(const float *scores, int m, int n_ret, int n_cand, unsigned char *region, int *ret_idx,
                              int *cand_idx, void *stream)
{
    if (!scores) return POP_EINVAL;
    if (m <= 0 || n_ret < 0 || n_cand < 0 || (long long)n_ret + n_cand > m) return POP_ESHAPE;
    POP_HIP(launch_partition(scores, m, n_ret, n_cand, region, ret_idx, cand_idx, as_stream(stream)));
    return POP_OK;
}

int pop_partition_top_from_scores(const float *scores, int m, int n_ret, int n_cand, int n_top, unsigned char *region,
                                  int *ret_idx, int *cand_idx, unsigned char *top_mask, int *top_list, void *stream)
{
    if (!scores || !top_list) return POP_EINVAL;
    if (m <= 0 || n_ret < 0 || n_cand < 0 || (long long)n_ret + n_cand > m) return POP_ESHAPE;
    if (n_top < 0 || n_top > m) return POP_ESHAPE;
    PartitionExtra ex;
    ex.n_top = n_top, ex.top_mask = top_mask, ex.top_list = top_list;
    POP_HIP(launch_partition(scores, m, n_ret, n_cand, region, ret_idx, cand_idx, as_stream(stream), &ex));
    return POP_OK;
}

int pop_topk_from_scores(const float *cand_scores, const int *cand_idx, int n_cand, int k, const unsigned char *region,
                         int m, unsigned char *mask, int *sel_idx, void *stream)
{
    if (m <= 0 || n_cand < 0 || n_cand > m || k < 0 || k > n_cand) return POP_ESHAPE;
    if (n_cand > 0 && (!cand_scores || !cand_idx)) return POP_EINVAL;
    if (mask && !region) return POP_EINVAL;
    BatchK kk = {};
    kk.k[0] = k;
    if (mask) POP_HIP(launch_step_state_init(region, m, nullptr, 0, 1, 0, mask, nullptr, as_stream(stream)));
    POP_HIP(launch_topk(cand_scores, n_cand, cand_idx, n_cand, 0, m, 1, kk, 0, mask, nullptr, nullptr, sel_idx,
                        nullptr, nullptr, nullptr, nullptr, as_stream(stream)));
    return POP_OK;
}

int pop_importance_reduce(const void *h, pop_dtype_t hdtype, int T, int m, const float *nrm, float *scores,
                          void *stream)
{
    if (!h || !nrm || !scores) return POP_EINVAL;
    if (hdtype != POP_F32 && hdtype != POP_BF16) return POP_EINVAL;
    if (T < 1 || m < 1) return POP_ESHAPE;
    // the per-chunk partial sums live in stream-ordered scratch: allocated and freed on the caller's stream
    hipStream_t s = as_stream(stream);
    void *scratch = nullptr;
    hipError_t e = hipMallocAsync(&scratch, importance_reduce_scratch_bytes(T, m), s);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return e == hipErrorOutOfMemory ? POP_ENOMEM : hip_fail(e, "hipMallocAsync");
    }
    e = launch_importance_reduce(h, hdtype == POP_BF16, T, m, nrm, scores, scratch, s);
    const hipError_t ef = hipFreeAsync(scratch, s);
    if (e != hipSuccess) return hip_fail(e, "importance reduction");
    if (ef != hipSuccess) return hip_fail(ef, "hipFreeAsync");
    return POP_OK;
}

int pop_layer_reserve_prompt(pop_layer_t *L, int T, void *stream)
{
    if (!L) return POP_EINVAL;
    if (T < 1 || T > L->max_tokens) return POP_ESHAPE;
    if (!L->is_bf16 || T < kFfnMfmaMinTokens) return POP_OK;  // those forward passes use the layer's fixed scratch
    int ldh = 0, n_split = 1;
    { int rc = ffn_scratch(L, T, true, &ldh, &n_split, as_stream(stream), true); if (rc != POP_OK) return rc; }
    if (!L->top_list && !dev_alloc((void **)&L->top_list, ((size_t)L->m + 1) * sizeof(int))) return POP_ENOMEM;
    return POP_OK;
}

int pop_probe_read(const void *buf, size_t bytes, int workgroups, unsigned int *sink, void *stream)
{
    if (!buf || !sink || !aligned16(buf)) return POP_EINVAL;
    if (bytes < 16 || workgroups < 1 || workgroups > 65535) return POP_ESHAPE;
    POP_HIP(launch_probe_read(buf, bytes, workgroups, sink, as_stream(stream)));
    return POP_OK;
}

int pop_probe_step_read(pop_layer_t *L, int k, int workgroups, unsigned int *sink, void *stream)
{
    if (!L || !sink) return POP_EINVAL;
    if (!L->has_partition) return POP_ESTATE;
    if (k < 0 || k > L->n_cand || workgroups < 1 || workgroups > 65535) return POP_ESHAPE;
    if (L->n_ret + L->n_cand == 0) return POP_OK;
    POP_HIP(launch_probe_step_read(L->w, L->d / (L->is_bf16 ? 8 : 4), L->rc_idx, L->n_ret + L->n_cand, L->ret_idx,
                                   L->n_ret, L->cand_idx, k, workgroups, sink, as_stream(stream)));
    return POP_OK;
}

int pop_layer_get_norms(pop_layer_t *L, float *nrm, void *stream)
{
    if (!L) return POP_EINVAL;
    if (nrm) POP_HIP(hipMemcpyAsync(nrm, L->nrm, (size_t)L->m * 4, hipMemcpyDeviceToDevice, as_stream(stream)));
    return POP_OK;
}

#ifdef POP_TRACE
void pop_trace_set_buffer(void *dev_ptr)
{
    g_trace = (unsigned long long *)dev_ptr;
    set_select_trace(g_trace ? g_trace + 1010 * 8 : nullptr);
}
#endif

int pop_layer_sync_status(pop_layer_t *L, void *stream)
{
    if (!L) return POP_EINVAL;
    int flag = 0, flag_fused = 0;
    POP_HIP(hipMemcpyAsync(&flag, L->sync + 2, 4, hipMemcpyDeviceToHost, as_stream(stream)));
    POP_HIP(hipMemcpyAsync(&flag_fused, L->fctr + 2, 4, hipMemcpyDeviceToHost, as_stream(stream)));
    POP_HIP(hipStreamSynchronize(as_stream(stream)));
    if (flag) POP_HIP(launch_fill_int(L->sync + 2, 1, 0, as_stream(stream)));  // reported once
    if (flag_fused) POP_HIP(launch_fill_int(L->fctr + 2, 1, 0, as_stream(stream)));
    return (flag || flag_fused) ? POP_EDEVICE : POP_OK;
}

int pop_layer_set_importance(pop_layer_t *L, int reading)
{
    if (!L) return POP_EINVAL;
    if (reading != POP_IMPORTANCE_OUTPUT_SIDE && reading != POP_IMPORTANCE_INPUT_SIDE) return POP_EINVAL;
    if (reading == POP_IMPORTANCE_INPUT_SIDE) {
        const size_t groups = (size_t)input_side_groups(L->max_tokens);
        if (!L->in_s2 && !dev_alloc((void **)&L->in_s2, (size_t)L->max_batch * L->d * sizeof(float)))
            return POP_ENOMEM;
        if (!L->in_part && !dev_alloc((void **)&L->in_part, groups * L->d * sizeof(double)))
            return POP_ENOMEM;
    }
    L->input_side = reading == POP_IMPORTANCE_INPUT_SIDE;
    L->has_partition = false;
    L->has_step = false;
    return POP_OK;
}

int pop_layer_set_shared_batch_mask(pop_layer_t *L, int on)
{
    if (!L) return POP_EINVAL;
    L->shared_mask = on != 0;
    L->has_step = false;
    return POP_OK;
}

int pop_layer_set_strategy(pop_layer_t *L, int strategy, double r, double gamma)
{
    if (!L) return POP_EINVAL;
    int n_ret = 0, n_cand = 0, k = 0;
    const int rc = pop_strategy_counts(strategy, L->m, r, gamma, &n_ret, &n_cand, &k);
    if (rc != POP_OK) return rc;
    L->strat_n_ret = n_ret, L->strat_n_cand = n_cand, L->strat_k = k;
    return POP_OK;
}

int pop_layer_set_wait_limit(pop_layer_t *L, int looks)
{
    if (!L || looks < 0) return POP_EINVAL;
    L->spin_limit = looks;
    return POP_OK;
}

int pop_layer_step_kind(pop_layer_t *L, int *workgroups)
{
    if (!L) return POP_EINVAL;
    if (workgroups) *workgroups = (L->has_partition && L->fused_ok) ? L->plan.n_wg : 0;
    return !L->has_step ? 0 : (L->step_fused ? 1 : 2);
}

int pop_layer_get_hidden(pop_layer_t *L, float *h, int B, void *stream)
{
    if (!L) return POP_EINVAL;
    if (B < 1 || B > L->max_batch) return POP_ESHAPE;
    if (h) POP_HIP(hipMemcpyAsync(h, L->h, (size_t)B * L->m * 4, hipMemcpyDeviceToDevice, as_stream(stream)));
    return POP_OK;
}

}  // extern "C"
