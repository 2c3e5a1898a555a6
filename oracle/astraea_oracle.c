/*
 * CPU oracle for the token-wise attention path of Astraea (arXiv 2506.05096).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP
 * kernels are checked against.  It shares no code, header, table or helper
 * with the HIP path and must never be called from the product path.
 *
 * What it computes (paper, Sec. 3.2 and supplementary Algorithm 1):
 *   oracle_score        S_token = w_a * (S_LSE * Delta) + w_b * e^{n_i}      (selection metric equations)
 *   oracle_topk         I_sel, I_remain = TopK(S_token, theta)               (Algorithm 1, TopK step)
 *   oracle_sparse_attn  X_out[I_sel] = Softmax(Q_sel K^T / sqrt(d)) V        (Algorithm 1, attention step;
 *                                                                             softmax as in the Self-Attention equations)
 *   oracle_scatter      X_out,t[I_sel] <- fresh rows, X_out,t[I_remain] kept (Algorithm 1, cache reuse step)
 *   oracle_gather       X[I_sel]                                             (Algorithm 1, query selection)
 *   oracle_lse_weight_update  per-token S_LSE carried to the next step          (selection metric, S_sig equation)
 *   oracle_sparse_linear  act(X[I_sel] W^T + b): the per-token layers on the selected rows only
 *                                                                             (Algorithm 1, "Q = X_in[I_sel] W_Q";
 *                                                                             FLOPs appendix: projections and MLP)
 *
 * Precision.  Attention accumulates in fp64 (acc_mode 0) or in fp32 (acc_mode 1,
 * the "naive fp32" form); its outputs are returned as fp64.  The score is a
 * value that decides integers (the selected indices), so it is taken in the
 * kernel's precision: fp32, channels visited strictly in ascending order with
 * one accumulator.  oracle_score_f64 is the same formula in fp64 and exists to
 * pin the fp32 one.
 *
 * Every loop is the definition written out: no blocking, no fusion, no
 * reordering.  OpenMP only distributes independent rows over threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_DELTA_L2 = 0, ORACLE_DELTA_MEAN_ABS = 1, ORACLE_DELTA_MEAN_SQ = 2 };

/* bfloat16 is the upper half of an IEEE binary32 (format definition). */
static float bf16_bits_to_float(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static float load_elem(const void *base, int dtype, int64_t i)
{
    if (dtype == ORACLE_F32)
        return ((const float *)base)[i];
    return bf16_bits_to_float(((const uint16_t *)base)[i]);
}

/* Round a double to bfloat16, ties to even, in one rounding. */
static uint16_t double_to_bf16_bits(double x)
{
    float f = (float)x; /* RNE to binary32 */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7f800000u) == 0x7f800000u) { /* inf / nan */
        if (u & 0x007fffffu)
            return (uint16_t)((u >> 16) | 0x0040u);
        return (uint16_t)(u >> 16);
    }
    uint32_t low = u & 0xffffu;
    uint32_t hi = u >> 16;
    int up;
    if (low > 0x8000u)
        up = 1;
    else if (low < 0x8000u)
        up = 0;
    else {
        /* binary32 value sits on a bf16 midpoint: the first rounding may have
         * put it there, so decide from the exact double. */
        double fd = (double)f;
        double ax = fabs(x), af = fabs(fd);
        if (ax > af)
            up = 1;
        else if (ax < af)
            up = 0;
        else
            up = (int)(hi & 1u);
    }
    return (uint16_t)(hi + (uint32_t)up);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- score -- */

/*
 * Selection metric (paper Sec. 3.2 "Selection Metric"; Algorithm 1 steps 1-2).
 *   d_c     = x_cur[i,c] - x_prev[i,c]                       (one fp32 subtraction)
 *   Delta_i = sqrt(sum_c d_c^2) | mean_c |d_c| | mean_c d_c^2 (mode)
 *   sig_i   = Delta_i * lse_weight[i]      (lse_weight == NULL: weight 1, no multiply)
 *   S_i     = w_alpha * sig_i              (skip_count == NULL: no penalty term)
 *   S_i     = fma(w_beta, table[min(n_i, table_len-1)], w_alpha * sig_i)   otherwise
 * The sum runs over c = 0..C-1 in order with a single fp32 accumulator and a
 * fused multiply-add per squared term.
 */
int oracle_score(const void *x_cur, const void *x_prev, int dtype, int64_t N, int64_t C,
                 int64_t row_stride, int mode, const float *lse_weight, const int32_t *skip_count,
                 const float *penalty_table, int32_t table_len, float w_alpha, float w_beta,
                 float *score_out)
{
    if (N < 0 || C <= 0)
        return -1;
    if (skip_count && (!penalty_table || table_len <= 0))
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        float acc = 0.0f;
        for (int64_t c = 0; c < C; ++c) {
            float d = load_elem(x_cur, dtype, i * row_stride + c) - load_elem(x_prev, dtype, i * row_stride + c);
            if (mode == ORACLE_DELTA_MEAN_ABS)
                acc = acc + fabsf(d);
            else
                acc = fmaf(d, d, acc);
        }
        float delta;
        if (mode == ORACLE_DELTA_L2)
            delta = sqrtf(acc);
        else
            delta = acc / (float)C;
        float sig = lse_weight ? delta * lse_weight[i] : delta;
        float s = w_alpha * sig;
        if (skip_count) {
            int32_t n = skip_count[i];
            if (n < 0)
                n = 0;
            if (n > table_len - 1)
                n = table_len - 1;
            s = fmaf(w_beta, penalty_table[n], s);
        }
        score_out[i] = s;
    }
    return 0;
}

/* Same formula in fp64 (penalty = exp(n) evaluated directly). */
int oracle_score_f64(const void *x_cur, const void *x_prev, int dtype, int64_t N, int64_t C,
                     int64_t row_stride, int mode, const float *lse_weight, const int32_t *skip_count,
                     double w_alpha, double w_beta, double *score_out)
{
    if (N < 0 || C <= 0)
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        double acc = 0.0;
        for (int64_t c = 0; c < C; ++c) {
            double d = (double)load_elem(x_cur, dtype, i * row_stride + c) -
                       (double)load_elem(x_prev, dtype, i * row_stride + c);
            if (mode == ORACLE_DELTA_MEAN_ABS)
                acc += fabs(d);
            else
                acc += d * d;
        }
        double delta = (mode == ORACLE_DELTA_L2) ? sqrt(acc) : acc / (double)C;
        double s = w_alpha * delta * (lse_weight ? (double)lse_weight[i] : 1.0);
        if (skip_count)
            s += w_beta * exp((double)(skip_count[i] < 0 ? 0 : skip_count[i]));
        score_out[i] = s;
    }
    return 0;
}

/* ---------------------------------------------------------------- top-k -- */

typedef struct {
    float s;
    int32_t i;
} scored_t;

/* Total order: larger score first; NaN after every number; equal -> lower index first. */
static int cmp_scored(const void *pa, const void *pb)
{
    const scored_t *a = (const scored_t *)pa, *b = (const scored_t *)pb;
    int an = isnan(a->s), bn = isnan(b->s);
    if (an != bn)
        return an ? 1 : -1;
    if (!an) {
        if (a->s > b->s)
            return -1;
        if (a->s < b->s)
            return 1;
    }
    return (a->i > b->i) - (a->i < b->i);
}

static int cmp_i32(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

/*
 * TopK(S_token, theta) (Algorithm 1, TopK step): sort all tokens by
 * (score descending, index ascending), keep the first k, then list the kept
 * and the remaining indices in ascending order.
 */
int oracle_topk(const float *score, int64_t N, int64_t k, int32_t *idx_sel, int32_t *idx_remain,
                uint8_t *sel_mask)
{
    if (N < 0 || k < 0 || k > N || N > 2147483647LL)
        return -1;
    scored_t *a = (scored_t *)malloc(sizeof(scored_t) * (size_t)(N > 0 ? N : 1));
    uint8_t *m = (uint8_t *)calloc((size_t)(N > 0 ? N : 1), 1);
    if (!a || !m) {
        free(a);
        free(m);
        return -2;
    }
    for (int64_t i = 0; i < N; ++i) {
        a[i].s = score[i];
        a[i].i = (int32_t)i;
    }
    qsort(a, (size_t)N, sizeof(scored_t), cmp_scored);
    for (int64_t r = 0; r < k; ++r) {
        idx_sel[r] = a[r].i;
        m[a[r].i] = 1;
    }
    qsort(idx_sel, (size_t)k, sizeof(int32_t), cmp_i32);
    if (idx_remain) {
        int64_t w = 0;
        for (int64_t i = 0; i < N; ++i)
            if (!m[i])
                idx_remain[w++] = (int32_t)i;
    }
    if (sel_mask)
        memcpy(sel_mask, m, (size_t)N);
    free(a);
    free(m);
    return 0;
}

/* Consecutive non-selection counter n_i of the penalty term: 0 when selected, +1 otherwise. */
int oracle_update_skip_count(int32_t *skip_count, const uint8_t *sel_mask, int64_t N)
{
    for (int64_t i = 0; i < N; ++i)
        skip_count[i] = sel_mask[i] ? 0 : skip_count[i] + 1;
    return 0;
}

/* ------------------------------------------------------------ attention -- */

/*
 * Attention of the selected queries over all N keys and values
 * (Algorithm 1, attention step; Softmax as defined in the Self-Attention
 * paragraph, evaluated with the row maximum subtracted, which is the same
 * function).  For selected row r (token i = idx_sel[r], or r itself when q is
 * compact) and head h:
 *     s_j   = scale * sum_c q[i,h,c] * k[j,h,c]          j = 0..N-1
 *     m     = max_j s_j
 *     p_j   = exp(s_j - m),   l = sum_j p_j
 *     o_c   = (sum_j p_j * v[j,h,c]) / l
 *     lse   = m + ln l
 * o_out is [k_sel, H, D] fp64, lse_out (optional) is [k_sel, H] fp64.
 * Strides are in elements; the head-dim index is contiguous.
 */
int oracle_sparse_attn(const void *q, const void *k, const void *v, int dtype, int64_t N, int32_t H,
                       int32_t D, int64_t q_stride_n, int64_t q_stride_h, int64_t kv_stride_n,
                       int64_t kv_stride_h, const int32_t *idx_sel, int64_t k_sel, int q_is_compact,
                       float softmax_scale, int acc_mode, double *o_out, double *lse_out)
{
    if (N <= 0 || H <= 0 || D <= 0 || k_sel < 0)
        return -1;
    int64_t pairs = k_sel * (int64_t)H;
    int bad = 0;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)N);
        double *acc = (double *)malloc(sizeof(double) * (size_t)D);
        float *pf = (float *)malloc(sizeof(float) * (size_t)N);
        float *accf = (float *)malloc(sizeof(float) * (size_t)D);
        if (!p || !acc || !pf || !accf) {
#pragma omp atomic write
            bad = 1;
        } else {
#pragma omp for schedule(dynamic, 4)
            for (int64_t rh = 0; rh < pairs; ++rh) {
                int64_t r = rh / H;
                int32_t h = (int32_t)(rh % H);
                int64_t qi = q_is_compact ? r : (int64_t)idx_sel[r];
                int64_t qoff = qi * q_stride_n + (int64_t)h * q_stride_h;
                if (acc_mode == 0) {
                    double m = -INFINITY;
                    for (int64_t j = 0; j < N; ++j) {
                        int64_t koff = j * kv_stride_n + (int64_t)h * kv_stride_h;
                        double dot = 0.0;
                        for (int32_t c = 0; c < D; ++c)
                            dot += (double)load_elem(q, dtype, qoff + c) * (double)load_elem(k, dtype, koff + c);
                        p[j] = (double)softmax_scale * dot;
                        if (p[j] > m)
                            m = p[j];
                    }
                    double l = 0.0;
                    for (int64_t j = 0; j < N; ++j) {
                        p[j] = exp(p[j] - m);
                        l += p[j];
                    }
                    for (int32_t c = 0; c < D; ++c)
                        acc[c] = 0.0;
                    for (int64_t j = 0; j < N; ++j) {
                        int64_t voff = j * kv_stride_n + (int64_t)h * kv_stride_h;
                        for (int32_t c = 0; c < D; ++c)
                            acc[c] += p[j] * (double)load_elem(v, dtype, voff + c);
                    }
                    for (int32_t c = 0; c < D; ++c)
                        o_out[(r * H + h) * (int64_t)D + c] = acc[c] / l;
                    if (lse_out)
                        lse_out[r * H + h] = m + log(l);
                } else {
                    float m = -INFINITY;
                    for (int64_t j = 0; j < N; ++j) {
                        int64_t koff = j * kv_stride_n + (int64_t)h * kv_stride_h;
                        float dot = 0.0f;
                        for (int32_t c = 0; c < D; ++c)
                            dot += load_elem(q, dtype, qoff + c) * load_elem(k, dtype, koff + c);
                        pf[j] = softmax_scale * dot;
                        if (pf[j] > m)
                            m = pf[j];
                    }
                    float l = 0.0f;
                    for (int64_t j = 0; j < N; ++j) {
                        pf[j] = expf(pf[j] - m);
                        l += pf[j];
                    }
                    for (int32_t c = 0; c < D; ++c)
                        accf[c] = 0.0f;
                    for (int64_t j = 0; j < N; ++j) {
                        int64_t voff = j * kv_stride_n + (int64_t)h * kv_stride_h;
                        for (int32_t c = 0; c < D; ++c)
                            accf[c] += pf[j] * load_elem(v, dtype, voff + c);
                    }
                    for (int32_t c = 0; c < D; ++c)
                        o_out[(r * H + h) * (int64_t)D + c] = (double)(accf[c] / l);
                    if (lse_out)
                        lse_out[r * H + h] = (double)(m + logf(l));
                }
            }
        }
        free(p);
        free(acc);
        free(pf);
        free(accf);
    }
    return bad ? -2 : 0;
}

/* Round an fp64 array to the storage dtype (fp32: RNE cast; bf16: RNE, single rounding). */
int oracle_round_to_dtype(const double *src, int64_t n, int dtype, void *dst)
{
    if (dtype == ORACLE_F32) {
        for (int64_t i = 0; i < n; ++i)
            ((float *)dst)[i] = (float)src[i];
    } else {
        for (int64_t i = 0; i < n; ++i)
            ((uint16_t *)dst)[i] = double_to_bf16_bits(src[i]);
    }
    return 0;
}

/*
 * Per-token S_LSE carried to the next step (Sec. 3.2 "Selection Metric"; the softmax row sum is the
 * by-product the paper reuses).  Reading taken for H heads: the mean over heads of the mean
 * exponential, weight[idx[r]] = (1/H) sum_h exp(min(lse[r,h] - ln N, 64)); evaluated in fp64, stored as
 * fp32.  The paper's S_LSE is a plain sum of exponentials, which has no finite fp32 value once a logit
 * passes ~88; the exponent is therefore capped at 64 (a head's mean exponential saturates at e^64), so
 * that the weight, and the score it multiplies, stay finite and ordered.
 */
int oracle_lse_weight_update(const double *lse_sel, int32_t H, int64_t N, const int32_t *idx_sel, int64_t k_sel,
                             float *lse_weight)
{
    if (N <= 0 || H <= 0 || k_sel < 0)
        return -1;
    for (int64_t r = 0; r < k_sel; ++r) {
        double acc = 0.0;
        for (int32_t h = 0; h < H; ++h)
            acc += exp(fmin(lse_sel[r * H + h] - log((double)N), 64.0));
        if (idx_sel[r] < 0 || idx_sel[r] >= N)
            return -1;
        lse_weight[idx_sel[r]] = (float)(acc / (double)H);
    }
    return 0;
}

/* ------------------------------------------------------- gather / scatter -- */

static size_t elem_size(int dtype) { return dtype == ORACLE_F32 ? 4u : 2u; }

/*
 * Cache update (Algorithm 1, last two steps): rows listed in idx_sel are
 * overwritten, every other row keeps the value cached at the earlier step.
 * src_is_full == 0: src row r      -> cache row idx_sel[r]
 * src_is_full == 1: src row idx[r] -> cache row idx_sel[r]
 */
int oracle_scatter(void *cache, const void *src, int dtype, int64_t N, int64_t row_elems,
                   int64_t cache_row_stride, int64_t src_row_stride, const int32_t *idx_sel, int64_t k_sel,
                   int src_is_full)
{
    size_t es = elem_size(dtype);
    for (int64_t r = 0; r < k_sel; ++r) {
        int64_t i = idx_sel[r];
        if (i < 0 || i >= N)
            return -1;
        int64_t s = src_is_full ? i : r;
        memcpy((char *)cache + (size_t)(i * cache_row_stride) * es, (const char *)src + (size_t)(s * src_row_stride) * es,
               (size_t)row_elems * es);
    }
    return 0;
}

/* Row gather: dst row r <- src row idx_sel[r] (Algorithm 1, X_in[I_sel]). */
int oracle_gather(const void *src, void *dst, int dtype, int64_t N, int64_t row_elems, int64_t src_row_stride,
                  int64_t dst_row_stride, const int32_t *idx_sel, int64_t k_sel)
{
    size_t es = elem_size(dtype);
    for (int64_t r = 0; r < k_sel; ++r) {
        int64_t i = idx_sel[r];
        if (i < 0 || i >= N)
            return -1;
        memcpy((char *)dst + (size_t)(r * dst_row_stride) * es, (const char *)src + (size_t)(i * src_row_stride) * es,
               (size_t)row_elems * es);
    }
    return 0;
}

/*
 * Per-token linear layer evaluated for the selected tokens only (Algorithm 1: Q = X_in[I_sel] W_Q, and in the
 * same way every projection and MLP layer of the block, which act on each token by itself; FLOPs appendix,
 * the 2*N*D*D' terms with N replaced by the number of selected tokens):
 *     y[r, o] = act( sum_c x[row(r), c] * w[o, c] + bias[o] ),   row(r) = idx_sel[r], or r if x_is_compact
 * w is [c_out, c_in] (one output feature's weights contiguous), bias may be NULL, everything in fp64.
 * act 0: identity; act 1: GELU in its tanh form, 0.5 t (1 + tanh( sqrt(2/pi) (t + 0.044715 t^3) )).
 * (The paper does not name the MLP's activation; this is the one the video DiTs it evaluates use.)
 */
enum { ORACLE_ACT_NONE = 0, ORACLE_ACT_GELU_TANH = 1 };
int oracle_sparse_linear(const void *x, int dtype, int64_t N, int64_t c_in, int64_t x_row_stride, const void *w,
                         int64_t c_out, const void *bias, int act, const int32_t *idx_sel, int64_t k_sel,
                         int x_is_compact, double *y)
{
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16)
        return -1;
    if (act != ORACLE_ACT_NONE && act != ORACLE_ACT_GELU_TANH)
        return -1;
    if (!x_is_compact)
        for (int64_t r = 0; r < k_sel; ++r)
            if (idx_sel[r] < 0 || idx_sel[r] >= N)
                return -1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < k_sel; ++r) {
        int64_t row = x_is_compact ? r : (int64_t)idx_sel[r];
        for (int64_t o = 0; o < c_out; ++o) {
            double t = 0.0;
            for (int64_t c = 0; c < c_in; ++c)
                t += (double)load_elem(x, dtype, row * x_row_stride + c) * (double)load_elem(w, dtype, o * c_in + c);
            if (bias)
                t += (double)load_elem(bias, dtype, o);
            if (act == ORACLE_ACT_GELU_TANH)
                t = 0.5 * t * (1.0 + tanh(0.79788456080286535588 * (t + 0.044715 * t * t * t)));
            y[r * c_out + o] = t;
        }
    }
    return 0;
}

/* k = round-half-up(N * pct / 100): number of tokens a percent budget selects. */
int64_t oracle_budget_to_k(int64_t N, int32_t budget_percent)
{
    return (N * (int64_t)budget_percent + 50) / 100;
}
