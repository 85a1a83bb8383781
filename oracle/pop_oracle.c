/*
 * POP (Partition-guided Online Pruning) -- CPU oracle, double precision.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * pruned-FFN path computes.  It is used by the tests, by the smoke check and by
 * the benchmark's cpu_baseline leg, and by nothing else; it shares no code with
 * the HIP library and the HIP library never calls it.
 *
 * What it follows (paper sections / equations):
 *   - Sec. 3.1 Eq. 1-2 and Sec. 3.4 Eq. 3: activation-aware channel importance.
 *     Reading used here: the linear map W is the FFN's down projection
 *     W_down[d][m], its input activations are the intermediate activations
 *     H[T][m] = silu(X W_gate^T) * (X W_up^T); the importance of intermediate
 *     channel j aggregates the element scores |W_down[o][j]| * ||H[:,j]||_2 over
 *     o with an l2 norm.  With T = 1 this is the decode-step score taken from
 *     H_t (Sec. 3.4, two-step decoding).  The alternative reading (Eq. 1-2
 *     literally on the first projections and the FFN input) is
 *     pop_oracle_importance_input_side.
 *   - Sec. 3.3 "Prefilling Stage": retained / candidate / pruned regions.  The
 *     quantile thresholds are realised as exact rank counts (n_ret, n_cand) in
 *     the total order (score descending, channel index ascending).
 *   - Sec. 3.3 "Decoding Stage", Sec. 3.4: retained and candidate channels run
 *     the forward pass, candidates are re-scored from H_t, k of them are
 *     selected, the output uses retained + selected channels only.
 *
 * All tensors are host pointers.  Stored tensors (x, weights) are passed in
 * their storage dtype (0 = float32, 1 = bf16 bit patterns in uint16) and widened
 * exactly to double; all arithmetic is double.  No blocking, no fusion.
 *
 * Pins (tests/test_oracle_pins.py): dense SwiGLU from a library routine at 0 %
 * pruning, brute-force enumeration of partition / top-k on tiny inputs, the
 * threshold form of the regions on tie-free scores, literal vs factorised
 * importance, T = 1 special case, the two ablation variants, equivariance and
 * directed scaling tests.  Accuracy / perplexity / latency tables of the paper:
 * parity unpinned (they need trained checkpoints and benchmark data).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_EINVAL (-1)

static double load_elem(const void *p, int dtype, size_t i)
{
    if (dtype == 0)
        return (double)((const float *)p)[i];
    uint32_t bits = ((uint32_t)((const uint16_t *)p)[i]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

int pop_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Region sizes from fractions: n_ret = floor(f_ret*m + 1/2),
 * n_ret + n_cand = floor((f_ret+f_cand)*m + 1/2), the rest is pruned.
 * (Sec. 3.3: quantile levels r-delta and r+delta turned into rank counts.) */
int pop_oracle_region_counts(int m, double f_ret, double f_cand, int *n_ret, int *n_cand, int *n_prn)
{
    if (m <= 0 || f_ret < 0 || f_cand < 0 || f_ret + f_cand > 1.0 + 1e-12)
        return ORACLE_EINVAL;
    long a = (long)floor(f_ret * m + 0.5);
    long b = (long)floor((f_ret + f_cand) * m + 0.5);
    if (a > m) a = m;
    if (b > m) b = m;
    if (b < a) b = a;
    *n_ret = (int)a;
    *n_cand = (int)(b - a);
    *n_prn = (int)(m - b);
    return ORACLE_OK;
}

/* Number of candidates to select so that the active count is floor((1-r)*m + 1/2)
 * (Sec. 3.3 "Decoding Stage": active channels match the target ratio r). */
int pop_oracle_k_for_ratio(int m, double r, int n_ret, int n_cand)
{
    long a = (long)floor((1.0 - r) * m + 0.5);
    long k = a - n_ret;
    if (k < 0) k = 0;
    if (k > n_cand) k = n_cand;
    return (int)k;
}

/* SwiGLU hidden activations for the listed channels (chan == NULL: all m):
 *   H[t][j] = silu(x_t . W_gate[j,:]) * (x_t . W_up[j,:]),  silu(z) = z / (1 + exp(-z)).
 * H is [T][m]; entries of channels not listed are left untouched. */
int pop_oracle_hidden(const void *x, const void *w_gate, const void *w_up, int dtype,
                      int T, int d, int m, const int *chan, int n_chan, double *H)
{
    if (T < 0 || d <= 0 || m <= 0) return ORACLE_EINVAL;
    int n = chan ? n_chan : m;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < n; ++c) {
        int j = chan ? chan[c] : c;
        for (int t = 0; t < T; ++t) {
            double g = 0.0, u = 0.0;
            for (int k = 0; k < d; ++k) {
                double xv = load_elem(x, dtype, (size_t)t * d + k);
                g += xv * load_elem(w_gate, dtype, (size_t)j * d + k);
                u += xv * load_elem(w_up, dtype, (size_t)j * d + k);
            }
            double silu = g / (1.0 + exp(-g));
            H[(size_t)t * m + j] = silu * u;
        }
    }
    return ORACLE_OK;
}

/* Channel importance, written out from Eq. 1 -> Eq. 2 with the l2 aggregator of Eq. 3:
 *   s_j     = sqrt(sum_t H[t][j]^2)                  (activation norm over tokens and samples)
 *   I_{o,j} = |W_down[o][j]| * s_j                    (element score)
 *   I_j     = sqrt(sum_o I_{o,j}^2)                   (aggregate over the channel's weights)
 * Only the listed channels are written (chan == NULL: all). */
int pop_oracle_importance(const void *w_down, int dtype, int d, int m, const double *H, int T,
                          const int *chan, int n_chan, double *I)
{
    if (T < 0 || d <= 0 || m <= 0) return ORACLE_EINVAL;
    int n = chan ? n_chan : m;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < n; ++c) {
        int j = chan ? chan[c] : c;
        double s2 = 0.0;
        for (int t = 0; t < T; ++t) {
            double h = H[(size_t)t * m + j];
            s2 += h * h;
        }
        double s = sqrt(s2);
        double acc = 0.0;
        for (int o = 0; o < d; ++o) {
            double e = fabs(load_elem(w_down, dtype, (size_t)o * m + j)) * s;
            acc += e * e;
        }
        I[j] = sqrt(acc);
    }
    return ORACLE_OK;
}

/* The other reading of Sec. 3.1 (Eq. 1-2 taken literally for the FFN's first projections): the linear maps are
 * W_gate and W_up [m][d], their input is the FFN input X[T][d], intermediate channel j is output channel j of both:
 *   s_k       = sqrt(sum_t X[t][k]^2)                 (input activation norm over tokens and samples)
 *   I^g_{j,k} = |W_gate[j][k]| * s_k,  I^u_{j,k} = |W_up[j][k]| * s_k      (element scores, Eq. 1)
 *   I_j       = sqrt(sum_k (I^g_{j,k})^2 + (I^u_{j,k})^2)                  (l2 aggregate over the channel's weights)
 * A channel is removed from both matrices at once, so its weights are both rows.  With T = 1, s_k = |x_k|: the
 * decode-step score under this reading.  Only the listed channels are written (chan == NULL: all). */
int pop_oracle_importance_input_side(const void *x, const void *w_gate, const void *w_up, int dtype, int T, int d,
                                     int m, const int *chan, int n_chan, double *I)
{
    if (T < 0 || d <= 0 || m <= 0) return ORACLE_EINVAL;
    double *s = (double *)malloc(sizeof(double) * (size_t)d);
    if (!s) return ORACLE_EINVAL;
    for (int k = 0; k < d; ++k) {
        double s2 = 0.0;
        for (int t = 0; t < T; ++t) {
            double v = load_elem(x, dtype, (size_t)t * d + k);
            s2 += v * v;
        }
        s[k] = sqrt(s2);
    }
    int n = chan ? n_chan : m;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < n; ++c) {
        int j = chan ? chan[c] : c;
        double acc = 0.0;
        for (int k = 0; k < d; ++k) {
            double eg = fabs(load_elem(w_gate, dtype, (size_t)j * d + k)) * s[k];
            double eu = fabs(load_elem(w_up, dtype, (size_t)j * d + k)) * s[k];
            acc += eg * eg + eu * eu;
        }
        I[j] = sqrt(acc);
    }
    free(s);
    return ORACLE_OK;
}

/* Column norms of the down projection, n_j = ||W_down[:,j]||_2 (the weight factor of Eq. 3). */
int pop_oracle_down_norms(const void *w_down, int dtype, int d, int m, double *n)
{
    if (d <= 0 || m <= 0) return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (int j = 0; j < m; ++j) {
        double acc = 0.0;
        for (int o = 0; o < d; ++o) {
            double w = load_elem(w_down, dtype, (size_t)o * m + j);
            acc += w * w;
        }
        n[j] = sqrt(acc);
    }
    return ORACLE_OK;
}

/* ---- selection: one strict total order, (score descending, index ascending) ---- */

typedef struct { double s; int j; } ranked_t;

static int ranked_before(const void *pa, const void *pb)
{
    const ranked_t *a = (const ranked_t *)pa, *b = (const ranked_t *)pb;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;          /* -0.0 and +0.0 compare equal here */
    return (a->j > b->j) - (a->j < b->j);
}

static int int_ascending(const void *pa, const void *pb)
{
    int a = *(const int *)pa, b = *(const int *)pb;
    return (a > b) - (a < b);
}

/* Sec. 3.3 regions by rank: the n_ret best channels are retained (code 0), the next
 * n_cand are candidates (code 1), the rest are pruned (code 2).  Index lists ascending. */
int pop_oracle_partition(const double *scores, int m, int n_ret, int n_cand,
                         uint8_t *region, int *ret_idx, int *cand_idx)
{
    if (m <= 0 || n_ret < 0 || n_cand < 0 || n_ret + n_cand > m) return ORACLE_EINVAL;
    ranked_t *r = (ranked_t *)malloc(sizeof(ranked_t) * (size_t)m);
    if (!r) return ORACLE_EINVAL;
    for (int j = 0; j < m; ++j) { r[j].s = scores[j]; r[j].j = j; }
    qsort(r, (size_t)m, sizeof(ranked_t), ranked_before);
    for (int p = 0; p < m; ++p)
        region[r[p].j] = (uint8_t)(p < n_ret ? 0 : (p < n_ret + n_cand ? 1 : 2));
    free(r);
    int a = 0, b = 0;
    for (int j = 0; j < m; ++j) {
        if (region[j] == 0 && ret_idx) ret_idx[a++] = j;
        if (region[j] == 1 && cand_idx) cand_idx[b++] = j;
    }
    return ORACLE_OK;
}

/* Decode-step selection (Sec. 3.3 "Decoding Stage"): among the candidates, listed by
 * channel in cand_idx with scores cscore[i] for cand_idx[i], take the k best.
 * mask[j] = 1 for retained and selected channels, else 0.
 * active_idx = retained channels ascending, then selected channels ascending. */
int pop_oracle_select(const uint8_t *region, int m, const double *cscore, const int *cand_idx,
                      int n_cand, int k, uint8_t *mask, int *sel_idx, int *active_idx, int *n_active)
{
    if (k < 0 || k > n_cand) return ORACLE_EINVAL;
    ranked_t *r = (ranked_t *)malloc(sizeof(ranked_t) * (size_t)(n_cand > 0 ? n_cand : 1));
    int *sel = (int *)malloc(sizeof(int) * (size_t)(k > 0 ? k : 1));
    if (!r || !sel) { free(r); free(sel); return ORACLE_EINVAL; }
    for (int i = 0; i < n_cand; ++i) {
        if (region[cand_idx[i]] != 1) { free(r); free(sel); return ORACLE_EINVAL; }
        r[i].s = cscore[i];
        r[i].j = cand_idx[i];
    }
    qsort(r, (size_t)n_cand, sizeof(ranked_t), ranked_before);
    for (int i = 0; i < k; ++i) sel[i] = r[i].j;
    qsort(sel, (size_t)k, sizeof(int), int_ascending);
    int a = 0;
    for (int j = 0; j < m; ++j) {
        mask[j] = (uint8_t)(region[j] == 0);
        if (region[j] == 0 && active_idx) active_idx[a] = j;
        a += (region[j] == 0);
    }
    for (int i = 0; i < k; ++i) {
        mask[sel[i]] = 1;
        if (sel_idx) sel_idx[i] = sel[i];
        if (active_idx) active_idx[a + i] = sel[i];
    }
    if (n_active) *n_active = a + k;
    free(r);
    free(sel);
    return ORACLE_OK;
}

/* Down projection over the active channels of each token:
 *   y[t][o] = sum_{j : mask_t[j] != 0} H[t][j] * W_down[o][j]
 * mask is [mask_rows][m] with mask_rows == 1 (shared) or == T (one row per token). */
int pop_oracle_down(const double *H, const void *w_down, int dtype, int T, int d, int m,
                    const uint8_t *mask, int mask_rows, double *y)
{
    if (mask_rows != 1 && mask_rows != T) return ORACLE_EINVAL;
#pragma omp parallel for schedule(static)
    for (int o = 0; o < d; ++o) {
        for (int t = 0; t < T; ++t) {
            const uint8_t *mk = mask + (mask_rows == 1 ? 0 : (size_t)t * m);
            double acc = 0.0;
            for (int j = 0; j < m; ++j)
                if (mk[j]) acc += H[(size_t)t * m + j] * load_elem(w_down, dtype, (size_t)o * m + j);
            y[(size_t)t * d + o] = acc;
        }
    }
    return ORACLE_OK;
}

/* Pruned SwiGLU FFN under a given mask: hidden activations of the masked channels, then
 * the down projection over them.  With an all-ones mask this is the dense FFN. */
int pop_oracle_pruned_ffn(const void *x, const void *w_gate, const void *w_up, const void *w_down,
                          int dtype, int T, int d, int m, const uint8_t *mask, int mask_rows, double *y)
{
    if (mask_rows != 1 && mask_rows != T) return ORACLE_EINVAL;
    double *H = (double *)calloc((size_t)T * m, sizeof(double));
    int *chan = (int *)malloc(sizeof(int) * (size_t)m);
    if (!H || !chan) { free(H); free(chan); return ORACLE_EINVAL; }
    int n = 0;
    for (int j = 0; j < m; ++j) {
        int any = 0;
        for (int t = 0; t < mask_rows; ++t) any |= mask[(size_t)t * m + j];
        if (any) chan[n++] = j;
    }
    int rc = pop_oracle_hidden(x, w_gate, w_up, dtype, T, d, m, chan, n, H);
    if (rc == ORACLE_OK) rc = pop_oracle_down(H, w_down, dtype, T, d, m, mask, mask_rows, y);
    free(H);
    free(chan);
    return rc;
}

/* Prefill (Sec. 3.3 "Prefilling Stage"): hidden activations of all channels for all T prompt
 * tokens, importance of every channel, regions by rank. */
int pop_oracle_prefill(const void *x, const void *w_gate, const void *w_up, const void *w_down,
                       int dtype, int T, int d, int m, int n_ret, int n_cand,
                       double *scores, uint8_t *region, int *ret_idx, int *cand_idx)
{
    double *H = (double *)malloc(sizeof(double) * (size_t)T * m);
    if (!H) return ORACLE_EINVAL;
    int rc = pop_oracle_hidden(x, w_gate, w_up, dtype, T, d, m, NULL, 0, H);
    if (rc == ORACLE_OK) rc = pop_oracle_importance(w_down, dtype, d, m, H, T, NULL, 0, scores);
    if (rc == ORACLE_OK) rc = pop_oracle_partition(scores, m, n_ret, n_cand, region, ret_idx, cand_idx);
    free(H);
    return rc;
}

/* One decode step for one token (Sec. 3.4 two-step decoding):
 *   1. h_j for j in retained + candidate (pass 1), h_j = 0 elsewhere in the output array;
 *   2. I_j(t) for candidates from h (Eq. 3 with a single token);
 *   3. select k candidates; 4. y over retained + selected.
 * cscore is [n_cand] in cand_idx order. */
int pop_oracle_decode(const void *x_t, const void *w_gate, const void *w_up, const void *w_down,
                      int dtype, int d, int m, const uint8_t *region, const int *cand_idx, int n_cand,
                      int k, double *h, double *cscore, uint8_t *mask, int *sel_idx,
                      int *active_idx, int *n_active, double *y)
{
    int *rc_list = (int *)malloc(sizeof(int) * (size_t)m);
    double *I = (double *)calloc((size_t)m, sizeof(double));
    if (!rc_list || !I) { free(rc_list); free(I); return ORACLE_EINVAL; }
    int n = 0;
    for (int j = 0; j < m; ++j) {
        h[j] = 0.0;
        if (region[j] != 2) rc_list[n++] = j;
    }
    int rc = pop_oracle_hidden(x_t, w_gate, w_up, dtype, 1, d, m, rc_list, n, h);
    if (rc == ORACLE_OK) rc = pop_oracle_importance(w_down, dtype, d, m, h, 1, cand_idx, n_cand, I);
    if (rc == ORACLE_OK) {
        for (int i = 0; i < n_cand; ++i) cscore[i] = I[cand_idx[i]];
        rc = pop_oracle_select(region, m, cscore, cand_idx, n_cand, k, mask, sel_idx, active_idx, n_active);
    }
    if (rc == ORACLE_OK && y) rc = pop_oracle_down(h, w_down, dtype, 1, d, m, mask, 1, y);
    free(rc_list);
    free(I);
    return rc;
}
