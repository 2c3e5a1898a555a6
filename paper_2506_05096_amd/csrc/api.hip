// C ABI of libastraea: host-side argument validation and dispatch.  Every check happens here,
// before the first HIP call, so a rejected call enqueues nothing.
#include <cmath>
#include <cstdarg>
#include <cstdio>

#include "common.h"

namespace astraea {

static thread_local char g_err[512] = "";

int fail(int status, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return status;
}

int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ASTRAEA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return ASTRAEA_OK;
}

static bool dtype_ok(int dt) { return dt == ASTRAEA_F32 || dt == ASTRAEA_BF16; }
static size_t esize(int dt) { return dt == ASTRAEA_F32 ? 4 : 2; }
static const int64_t kMaxTokens = 2147483647LL;

}  // namespace astraea

using namespace astraea;

extern "C" {

int astraea_score(const void *x_cur, const void *x_prev, astraea_dtype dt, int64_t N, int64_t C,
                  int64_t row_stride_elems, astraea_delta_mode mode, const float *lse_weight,
                  const int32_t *skip_count, const float *penalty_table, int32_t table_len, float w_alpha,
                  float w_beta, float *score_out, void *stream)
{
    if (!dtype_ok(dt)) return fail(ASTRAEA_ERR_UNSUPPORTED, "astraea_score: unknown dtype %d", (int)dt);
    if (mode != ASTRAEA_DELTA_L2 && mode != ASTRAEA_DELTA_MEAN_ABS && mode != ASTRAEA_DELTA_MEAN_SQ)
        return fail(ASTRAEA_ERR_INVALID, "astraea_score: unknown delta mode %d", (int)mode);
    if (N < 0 || N > kMaxTokens) return fail(ASTRAEA_ERR_INVALID, "astraea_score: N=%lld out of range", (long long)N);
    if (C <= 0) return fail(ASTRAEA_ERR_INVALID, "astraea_score: C=%lld must be positive", (long long)C);
    if (row_stride_elems < C)
        return fail(ASTRAEA_ERR_INVALID, "astraea_score: row stride %lld < C=%lld", (long long)row_stride_elems,
                    (long long)C);
    if (N > 0 && (!x_cur || !x_prev || !score_out)) return fail(ASTRAEA_ERR_INVALID, "astraea_score: NULL tensor");
    if (((uintptr_t)x_cur | (uintptr_t)x_prev) % esize(dt) != 0 || (uintptr_t)score_out % 4 != 0)
        return fail(ASTRAEA_ERR_INVALID, "astraea_score: pointer not aligned to its element size");
    if (skip_count && (!penalty_table || table_len <= 0))
        return fail(ASTRAEA_ERR_INVALID, "astraea_score: skip_count needs a penalty table");
    return launch_score(x_cur, x_prev, dt, N, C, row_stride_elems, mode, lse_weight, skip_count, penalty_table,
                        table_len, w_alpha, w_beta, score_out, (hipStream_t)stream);
}

static int check_topk(const char *fn, const float *score, int64_t N, int64_t k, const int32_t *idx_sel,
                      const int32_t *idx_remain, const int32_t *skip_count)
{
    if (N < 0 || N > kMaxTokens) return fail(ASTRAEA_ERR_INVALID, "%s: N=%lld out of range", fn, (long long)N);
    if (k < 0 || k > N) return fail(ASTRAEA_ERR_INVALID, "%s: k=%lld not in [0, N=%lld]", fn, (long long)k, (long long)N);
    if (N == 0) return ASTRAEA_OK;
    if (!score) return fail(ASTRAEA_ERR_INVALID, "%s: NULL score", fn);
    if (k > 0 && !idx_sel) return fail(ASTRAEA_ERR_INVALID, "%s: NULL idx_sel", fn);
    if (((uintptr_t)score | (uintptr_t)idx_sel | (uintptr_t)idx_remain | (uintptr_t)skip_count) % 4 != 0)
        return fail(ASTRAEA_ERR_INVALID, "%s: pointer not 4-byte aligned", fn);
    return ASTRAEA_OK;
}

int astraea_select_topk(const float *score, int64_t N, int64_t k, int32_t *idx_sel, int32_t *idx_remain,
                        uint8_t *sel_mask, int32_t *skip_count, void *workspace, size_t workspace_bytes,
                        void *stream)
{
    const int rc = check_topk("astraea_select_topk", score, N, k, idx_sel, idx_remain, skip_count);
    if (rc != ASTRAEA_OK || N == 0) return rc;
    const size_t need = topk_workspace_bytes(N);
    if (!workspace || (uintptr_t)workspace % 256 != 0 || workspace_bytes < need)
        return fail(ASTRAEA_ERR_WORKSPACE, "astraea_select_topk: workspace must be 256-byte aligned and >= %zu bytes",
                    need);
    return launch_select_topk(score, N, k, idx_sel, idx_remain, sel_mask, skip_count, workspace, (hipStream_t)stream);
}

int astraea_select_topk_static(const float *score, int64_t N, int64_t k, int32_t *idx_sel, int32_t *idx_remain,
                               uint8_t *sel_mask, int32_t *skip_count, void *stream)
{
    const int rc = check_topk("astraea_select_topk_static", score, N, k, idx_sel, idx_remain, skip_count);
    if (rc != ASTRAEA_OK || N == 0) return rc;
    if (N > topk_static_max_n())
        return fail(ASTRAEA_ERR_UNSUPPORTED,
                    "astraea_select_topk_static: N=%lld exceeds the %lld scores the built-in scratch array holds; use "
                    "astraea_select_topk with a workspace", (long long)N, (long long)topk_static_max_n());
    void *scratch_ptr = nullptr;
    const int rs = topk_static_scratch(&scratch_ptr);
    if (rs != ASTRAEA_OK) return rs;
    return launch_select_topk(score, N, k, idx_sel, idx_remain, sel_mask, skip_count, scratch_ptr, (hipStream_t)stream);
}

// Shared body of the two attention entry points: `out` is either the compact [k_sel, H, D] result
// (scatter == 0, row stride H*D) or the cached per-token buffer [N, out_stride_n] whose rows idx_sel
// names are overwritten (scatter == 1).
static int sparse_attn_common(const char *fn, const void *q, const void *k, const void *v, astraea_dtype dt, int64_t N,
                              int32_t H, int32_t D, int64_t q_stride_n, int64_t q_stride_h, int64_t kv_stride_n,
                              int64_t kv_stride_h, const int32_t *idx_sel, int64_t k_sel, int q_is_compact,
                              float softmax_scale, void *out, int64_t out_stride_n, int scatter, float *lse_sel,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    if (!dtype_ok(dt)) return fail(ASTRAEA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, (int)dt);
    if (N <= 0 || N > kMaxTokens) return fail(ASTRAEA_ERR_INVALID, "%s: N=%lld out of range", fn, (long long)N);
    if (H <= 0 || H > 65535) return fail(ASTRAEA_ERR_INVALID, "%s: H=%d out of range", fn, (int)H);
    if (k_sel < 0 || k_sel > kMaxTokens || ((!q_is_compact || scatter) && k_sel > N))
        return fail(ASTRAEA_ERR_INVALID, "%s: k_sel=%lld out of range", fn, (long long)k_sel);
    if (!(dt == ASTRAEA_BF16 && D == 128) && !(dt == ASTRAEA_F32 && (D == 64 || D == 128)))
        return fail(ASTRAEA_ERR_UNSUPPORTED, "%s: no kernel for dtype %d with head_dim %d", fn, (int)dt, (int)D);
    if (!(softmax_scale > 0.0f) || !std::isfinite(softmax_scale))
        return fail(ASTRAEA_ERR_INVALID, "%s: softmax_scale must be positive and finite", fn);
    if (scatter && (out_stride_n < (int64_t)H * D || out_stride_n % 8 != 0))
        return fail(ASTRAEA_ERR_INVALID, "%s: cache_row_stride must be a multiple of 8 and at least H*D", fn);
    if (k_sel == 0) return ASTRAEA_OK;
    if (!q || !k || !v || !out) return fail(ASTRAEA_ERR_INVALID, "%s: NULL tensor", fn);
    if ((!q_is_compact || scatter) && !idx_sel)
        return fail(ASTRAEA_ERR_INVALID, "%s: idx_sel is required to gather queries or to place rows", fn);
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) % 16 != 0)
        return fail(ASTRAEA_ERR_INVALID, "%s: q, k, v and the output must be 16-byte aligned", fn);
    if (((uintptr_t)idx_sel | (uintptr_t)lse_sel) % 4 != 0)
        return fail(ASTRAEA_ERR_INVALID, "%s: idx_sel / lse_sel must be 4-byte aligned", fn);
    if (q_stride_h < D || kv_stride_h < D || q_stride_n < D || kv_stride_n < D)
        return fail(ASTRAEA_ERR_INVALID, "%s: strides must be at least head_dim", fn);
    if ((q_stride_n | q_stride_h | kv_stride_n | kv_stride_h) % 8 != 0)
        return fail(ASTRAEA_ERR_INVALID, "%s: strides must be multiples of 8 elements", fn);
    const size_t need = dt == ASTRAEA_BF16 ? attn_bf16_workspace_bytes(N, H) : 0;
    if (need > 0 && (!workspace || (uintptr_t)workspace % 256 != 0 || workspace_bytes < need))
        return fail(ASTRAEA_ERR_WORKSPACE, "%s: workspace must be 256-byte aligned and >= %zu bytes", fn, need);
    if (dt == ASTRAEA_BF16)
        return launch_attn_bf16_d128(q, k, v, N, H, q_stride_n, q_stride_h, kv_stride_n, kv_stride_h, idx_sel, k_sel,
                                     q_is_compact, softmax_scale, out, out_stride_n, scatter, lse_sel, workspace,
                                     (hipStream_t)stream);
    return launch_attn_f32(q, k, v, N, H, D, q_stride_n, q_stride_h, kv_stride_n, kv_stride_h, idx_sel, k_sel,
                           q_is_compact, softmax_scale, out, out_stride_n, scatter, lse_sel,
                           (uintptr_t)workspace % 256 == 0 ? workspace : nullptr, workspace_bytes, (hipStream_t)stream);
}

int astraea_sparse_attn_fwd(const void *q, const void *k, const void *v, astraea_dtype dt, int64_t N, int32_t H,
                            int32_t D, int64_t q_stride_n, int64_t q_stride_h, int64_t kv_stride_n,
                            int64_t kv_stride_h, const int32_t *idx_sel, int64_t k_sel, int q_is_compact,
                            float softmax_scale, void *o_sel, float *lse_sel, void *workspace,
                            size_t workspace_bytes, void *stream)
{
    return sparse_attn_common("astraea_sparse_attn_fwd", q, k, v, dt, N, H, D, q_stride_n, q_stride_h, kv_stride_n,
                              kv_stride_h, idx_sel, k_sel, q_is_compact, softmax_scale, o_sel, (int64_t)H * D, 0,
                              lse_sel, workspace, workspace_bytes, stream);
}

int astraea_sparse_attn_update_fwd(const void *q, const void *k, const void *v, astraea_dtype dt, int64_t N, int32_t H,
                                   int32_t D, int64_t q_stride_n, int64_t q_stride_h, int64_t kv_stride_n,
                                   int64_t kv_stride_h, const int32_t *idx_sel, int64_t k_sel, int q_is_compact,
                                   float softmax_scale, void *out_cache, int64_t cache_row_stride, float *lse_sel,
                                   void *workspace, size_t workspace_bytes, void *stream)
{
    return sparse_attn_common("astraea_sparse_attn_update_fwd", q, k, v, dt, N, H, D, q_stride_n, q_stride_h,
                              kv_stride_n, kv_stride_h, idx_sel, k_sel, q_is_compact, softmax_scale, out_cache,
                              cache_row_stride, 1, lse_sel, workspace, workspace_bytes, stream);
}

int astraea_sparse_linear(const void *x, const void *w, const void *bias, astraea_dtype dt, int64_t N, int64_t c_in,
                          int64_t c_out, int64_t x_row_stride, const int32_t *idx_sel, int64_t k_sel,
                          int x_is_compact, astraea_activation act, void *y, int64_t y_row_stride, int y_is_compact,
                          void *stream)
{
    const char *fn = "astraea_sparse_linear";
    if (!dtype_ok(dt)) return fail(ASTRAEA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, (int)dt);
    if (act != ASTRAEA_ACT_NONE && act != ASTRAEA_ACT_GELU_TANH)
        return fail(ASTRAEA_ERR_UNSUPPORTED, "%s: unknown activation %d", fn, (int)act);
    if (N <= 0 || N > kMaxTokens) return fail(ASTRAEA_ERR_INVALID, "%s: N=%lld out of range", fn, (long long)N);
    const bool indexed = !x_is_compact || !y_is_compact;
    if (k_sel < 0 || k_sel > kMaxTokens || (indexed && k_sel > N))
        return fail(ASTRAEA_ERR_INVALID, "%s: k_sel=%lld out of range", fn, (long long)k_sel);
    if (c_in <= 0 || c_out <= 0 || c_in > (1 << 24) || c_out > (1 << 24))
        return fail(ASTRAEA_ERR_INVALID, "%s: c_in=%lld, c_out=%lld out of range", fn, (long long)c_in, (long long)c_out);
    if (c_in % 64 != 0 || c_out % 8 != 0)
        return fail(ASTRAEA_ERR_UNSUPPORTED, "%s: c_in must be a multiple of 64 and c_out of 8", fn);
    if (x_row_stride < c_in || y_row_stride < c_out || x_row_stride % 8 != 0 || y_row_stride % 8 != 0)
        return fail(ASTRAEA_ERR_INVALID, "%s: row strides must cover a row and be multiples of 8 elements", fn);
    // the bf16 kernel's tile copies address x and w with 32-bit byte offsets
    const int64_t x_rows = x_is_compact ? k_sel : N;
    if (dt == ASTRAEA_BF16 && (x_rows * x_row_stride * 2 >= ((int64_t)1 << 32) || c_out * c_in * 2 >= ((int64_t)1 << 32)))
        return fail(ASTRAEA_ERR_UNSUPPORTED, "%s: x and w must each span less than 4 GiB", fn);
    if (k_sel == 0) return ASTRAEA_OK;
    if (!x || !w || !y) return fail(ASTRAEA_ERR_INVALID, "%s: NULL tensor", fn);
    if (indexed && !idx_sel) return fail(ASTRAEA_ERR_INVALID, "%s: idx_sel is required to gather or place rows", fn);
    if (((uintptr_t)x | (uintptr_t)w | (uintptr_t)y | (uintptr_t)bias) % 16 != 0)
        return fail(ASTRAEA_ERR_INVALID, "%s: x, w, bias and y must be 16-byte aligned", fn);
    if ((uintptr_t)idx_sel % 4 != 0) return fail(ASTRAEA_ERR_INVALID, "%s: idx_sel must be 4-byte aligned", fn);
    if (dt == ASTRAEA_F32)
        return launch_linear_f32(x, w, bias, y, idx_sel, k_sel, N, (int32_t)c_in, (int32_t)c_out, x_row_stride,
                                 y_row_stride, x_is_compact ? 0 : 1, y_is_compact ? 0 : 1, (int)act, (hipStream_t)stream);
    return launch_linear_bf16(x, w, bias, y, idx_sel, k_sel, N, (int32_t)c_in, (int32_t)c_out, x_row_stride, y_row_stride,
                              x_is_compact ? 0 : 1, y_is_compact ? 0 : 1, (int)act, (hipStream_t)stream);
}

static int check_rows(const char *fn, const void *a, const void *b, astraea_dtype dt, int64_t N, int64_t row_elems,
                      int64_t stride_a, int64_t stride_b, const int32_t *idx_sel, int64_t k_sel)
{
    if (!dtype_ok(dt)) return fail(ASTRAEA_ERR_UNSUPPORTED, "%s: unknown dtype %d", fn, (int)dt);
    if (N < 0 || N > kMaxTokens) return fail(ASTRAEA_ERR_INVALID, "%s: N=%lld out of range", fn, (long long)N);
    if (k_sel < 0 || k_sel > N)
        return fail(ASTRAEA_ERR_INVALID, "%s: k_sel=%lld not in [0, N=%lld]", fn, (long long)k_sel, (long long)N);
    if (row_elems < 0 || stride_a < row_elems || stride_b < row_elems)
        return fail(ASTRAEA_ERR_INVALID, "%s: row strides must be at least row_elems", fn);
    if (k_sel == 0) return ASTRAEA_OK;
    if (!a || !b || !idx_sel) return fail(ASTRAEA_ERR_INVALID, "%s: NULL tensor", fn);
    if (((uintptr_t)a | (uintptr_t)b) % esize(dt) != 0 || (uintptr_t)idx_sel % 4 != 0)
        return fail(ASTRAEA_ERR_INVALID, "%s: pointer not aligned to its element size", fn);
    return ASTRAEA_OK;
}

int astraea_scatter_update(void *cache, const void *src, astraea_dtype dt, int64_t N, int64_t row_elems,
                           int64_t cache_row_stride, int64_t src_row_stride, const int32_t *idx_sel,
                           int64_t k_sel, int src_is_full, void *stream)
{
    int rc = check_rows("astraea_scatter_update", cache, src, dt, N, row_elems, cache_row_stride, src_row_stride,
                        idx_sel, k_sel);
    if (rc != ASTRAEA_OK || k_sel == 0) return rc;
    const int64_t es = (int64_t)esize(dt);
    return launch_move_rows(cache, src, row_elems * es, cache_row_stride * es, src_row_stride * es, idx_sel, k_sel,
                            N, true, src_is_full != 0, (hipStream_t)stream);
}

int astraea_kv_refresh(void *k_cache, void *v_cache, const void *k_new, const void *v_new, astraea_dtype dt, int64_t N,
                       int64_t row_elems, int64_t cache_row_stride, int64_t src_row_stride, const int32_t *idx_sel,
                       int64_t k_sel, void *stream)
{
    int rc = check_rows("astraea_kv_refresh", k_cache, k_new, dt, N, row_elems, cache_row_stride, src_row_stride, idx_sel,
                        k_sel);
    if (rc == ASTRAEA_OK)
        rc = check_rows("astraea_kv_refresh", v_cache, v_new, dt, N, row_elems, cache_row_stride, src_row_stride, idx_sel,
                        k_sel);
    if (rc != ASTRAEA_OK || k_sel == 0) return rc;
    const int64_t es = (int64_t)esize(dt);
    return launch_move_rows(k_cache, k_new, row_elems * es, cache_row_stride * es, src_row_stride * es, idx_sel, k_sel, N,
                            true, true, (hipStream_t)stream, v_cache, v_new);
}

int astraea_gather_rows(const void *src, void *dst, astraea_dtype dt, int64_t N, int64_t row_elems,
                        int64_t src_row_stride, int64_t dst_row_stride, const int32_t *idx_sel, int64_t k_sel,
                        void *stream)
{
    int rc = check_rows("astraea_gather_rows", src, dst, dt, N, row_elems, src_row_stride, dst_row_stride, idx_sel,
                        k_sel);
    if (rc != ASTRAEA_OK || k_sel == 0) return rc;
    const int64_t es = (int64_t)esize(dt);
    return launch_move_rows(dst, src, row_elems * es, dst_row_stride * es, src_row_stride * es, idx_sel, k_sel, N,
                            false, true, (hipStream_t)stream);
}

int astraea_lse_weight_update(const float *lse_sel, int32_t H, int64_t N, const int32_t *idx_sel, int64_t k_sel,
                              float *lse_weight, void *stream)
{
    const char *fn = "astraea_lse_weight_update";
    if (N <= 0 || N > kMaxTokens) return fail(ASTRAEA_ERR_INVALID, "%s: N=%lld out of range", fn, (long long)N);
    if (H <= 0) return fail(ASTRAEA_ERR_INVALID, "%s: H=%d out of range", fn, (int)H);
    if (k_sel < 0 || k_sel > N)
        return fail(ASTRAEA_ERR_INVALID, "%s: k_sel=%lld not in [0, N=%lld]", fn, (long long)k_sel, (long long)N);
    if (k_sel == 0) return ASTRAEA_OK;
    if (!lse_sel || !idx_sel || !lse_weight) return fail(ASTRAEA_ERR_INVALID, "%s: NULL tensor", fn);
    if (((uintptr_t)lse_sel | (uintptr_t)idx_sel | (uintptr_t)lse_weight) % 4 != 0)
        return fail(ASTRAEA_ERR_INVALID, "%s: pointer not 4-byte aligned", fn);
    return launch_lse_weight_update(lse_sel, H, N, idx_sel, k_sel, lse_weight, (hipStream_t)stream);
}

size_t astraea_workspace_bytes(int op, int64_t N, int64_t k_sel, int32_t H, int32_t D)
{
    if (N < 0) return 0;
    if (op == ASTRAEA_OP_SELECT_TOPK) return topk_workspace_bytes(N);
    // enough for either dtype: the bf16 path (head_dim 128) stages V and partial results, the fp32 path
    // partial results when a small selection is cut along the keys
    if (op == ASTRAEA_OP_SPARSE_ATTN) {
        const size_t f32 = (D == 64 || D == 128) ? attn_f32_workspace_bytes(N, H, D, k_sel) : 0;
        const size_t bf16 = D == 128 ? attn_bf16_workspace_bytes(N, H) : 0;
        return f32 > bf16 ? f32 : bf16;
    }
    return 0;
}

int64_t astraea_budget_to_k(int64_t N, int32_t budget_percent)
{
    if (N < 0 || budget_percent < 0 || budget_percent > 100) return -1;
    return (N * (int64_t)budget_percent + 50) / 100;
}

double astraea_attn_flops(int64_t N, int64_t k_sel, int32_t H, int32_t D)
{
    return 4.0 * (double)k_sel * (double)N * (double)D * (double)H;
}

int astraea_check_indices(const int32_t *idx_sel, int64_t k_sel, int64_t N, int32_t *counts_out, void *stream)
{
    if (N <= 0 || N > kMaxTokens || k_sel < 0 || k_sel > kMaxTokens)
        return fail(ASTRAEA_ERR_INVALID, "astraea_check_indices: N=%lld, k_sel=%lld out of range", (long long)N,
                    (long long)k_sel);
    if (!counts_out || (k_sel > 0 && !idx_sel)) return fail(ASTRAEA_ERR_INVALID, "astraea_check_indices: NULL pointer");
    if (((uintptr_t)idx_sel | (uintptr_t)counts_out) % 4 != 0)
        return fail(ASTRAEA_ERR_INVALID, "astraea_check_indices: pointers must be 4-byte aligned");
    return launch_check_indices(idx_sel, k_sel, N, counts_out, (hipStream_t)stream);
}

int astraea_attn_plan(int64_t N, int32_t H, int64_t k_sel, int64_t plan_out[8])
{
    if (!plan_out) return fail(ASTRAEA_ERR_INVALID, "astraea_attn_plan: NULL output");
    if (N <= 0 || N > kMaxTokens || H <= 0 || H > 65535 || k_sel <= 0 || k_sel > kMaxTokens)
        return fail(ASTRAEA_ERR_INVALID, "astraea_attn_plan: N=%lld, H=%d, k_sel=%lld out of range", (long long)N, (int)H,
                    (long long)k_sel);
    return attn_bf16_plan(N, H, k_sel, plan_out);
}

const char *astraea_status_string(int status)
{
    switch (status) {
    case ASTRAEA_OK: return "ok";
    case ASTRAEA_ERR_INVALID: return "invalid argument";
    case ASTRAEA_ERR_UNSUPPORTED: return "unsupported dtype or head dimension";
    case ASTRAEA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case ASTRAEA_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

const char *astraea_last_error(void) { return g_err; }

}  // extern "C"
