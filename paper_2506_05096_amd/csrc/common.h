// Internal declarations shared by the HIP translation units of libastraea (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "astraea.h"

namespace astraea {

constexpr int kWave = 64;

// Records a message for astraea_last_error() and returns `status`.
int fail(int status, const char *fmt, ...);
// Checks hipGetLastError() after a launch.
int check_launch(const char *what);

// Measurement aid: while the kernel timer is on, the attention launchers bracket their main kernel with a
// pair of HIP events on the caller's stream (astraea_probe_kernel_timer / astraea_probe_kernel_ms).
void kernel_timer_begin(hipStream_t stream);
void kernel_timer_end(hipStream_t stream);

// ---- launchers (each enqueues on `stream`, arguments already validated) ----
int launch_score(const void *x_cur, const void *x_prev, astraea_dtype dt, int64_t N, int64_t C, int64_t row_stride,
                 astraea_delta_mode mode, const float *lse_weight, const int32_t *skip_count,
                 const float *penalty_table, int32_t table_len, float w_alpha, float w_beta, float *score_out,
                 hipStream_t stream);

size_t topk_workspace_bytes(int64_t N);
int64_t topk_static_max_n();
int topk_static_scratch(void **ptr_out);      // the library's own per-device scratch array, for astraea_select_topk_static
int launch_select_topk(const float *score, int64_t N, int64_t k, int32_t *idx_sel, int32_t *idx_remain,
                       uint8_t *sel_mask, int32_t *skip_count, void *workspace, hipStream_t stream);

// dst_b / src_b: an optional second buffer pair of the same shape and strides, moved by the same launch
int launch_move_rows(void *dst, const void *src, int64_t row_bytes, int64_t dst_stride_bytes,
                     int64_t src_stride_bytes, const int32_t *idx, int64_t k_sel, int64_t n_rows, bool index_dst,
                     bool index_src, hipStream_t stream, void *dst_b = nullptr, const void *src_b = nullptr);

int launch_check_indices(const int32_t *idx_sel, int64_t k_sel, int64_t N, int32_t *counts, hipStream_t stream);

int launch_lse_weight_update(const float *lse_sel, int32_t H, int64_t N, const int32_t *idx_sel, int64_t k_sel,
                             float *lse_weight, hipStream_t stream);

int launch_linear_bf16(const void *x, const void *w, const void *bias, void *y, const int32_t *idx_sel, int64_t k_sel,
                       int64_t n_rows, int32_t c_in, int32_t c_out, int64_t ldx, int64_t ldy, int x_indexed,
                       int y_indexed, int act, hipStream_t stream);

int launch_linear_f32(const void *x, const void *w, const void *bias, void *y, const int32_t *idx_sel, int64_t k_sel,
                      int64_t n_rows, int32_t c_in, int32_t c_out, int64_t ldx, int64_t ldy, int x_indexed,
                      int y_indexed, int act, hipStream_t stream);

size_t attn_bf16_workspace_bytes(int64_t N, int32_t H);
int attn_bf16_plan(int64_t N, int32_t H, int64_t k_sel, int64_t plan[8]);
int launch_attn_bf16_d128(const void *q, const void *k, const void *v, int64_t N, int32_t H, int64_t q_stride_n,
                          int64_t q_stride_h, int64_t kv_stride_n, int64_t kv_stride_h, const int32_t *idx_sel,
                          int64_t k_sel, int q_is_compact, float scale, void *o_sel, int64_t o_stride_n, int o_scatter,
                          float *lse_sel, void *workspace,
                          hipStream_t stream);
int launch_attn_f32(const void *q, const void *k, const void *v, int64_t N, int32_t H, int32_t D, int64_t q_stride_n,
                    int64_t q_stride_h, int64_t kv_stride_n, int64_t kv_stride_h, const int32_t *idx_sel,
                    int64_t k_sel, int q_is_compact, float scale, void *o_sel, int64_t o_stride_n, int o_scatter,
                    float *lse_sel, void *workspace, size_t workspace_bytes, hipStream_t stream);
size_t attn_f32_workspace_bytes(int64_t N, int32_t H, int32_t D, int64_t k_sel);

}  // namespace astraea
