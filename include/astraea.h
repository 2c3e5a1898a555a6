/*
 * astraea.h - C ABI of the token-wise attention hot path of Astraea
 * (arXiv 2506.05096) for AMD MI355X (gfx950).
 *
 * One layer-step of the method (paper Sec. 3.2; supplementary Algorithm 1) is
 *     score -> select top-k -> [gather] -> attention of the selected queries
 *     over all keys/values -> scatter into the cached per-token outputs.
 * Each call below is one of those steps.  Conventions shared by all calls:
 *
 *  - Every tensor pointer is DEVICE memory owned by the caller; the library
 *    keeps no state between calls and never allocates or frees device memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work on it; they never synchronise and never copy to
 *    the host.
 *  - Batch is 1: a batch of B sequences is B calls.  0 <= k <= N < 2^31.
 *  - All argument checks run on the host before the first HIP call.  On
 *    failure nothing is enqueued, a negative status is returned and
 *    astraea_last_error() holds a message (thread-local).
 *  - bf16 is the upper half of IEEE binary32; conversions to bf16 round to
 *    nearest even.
 *  - idx_sel is device data, so the host cannot check it.  It must hold
 *    distinct indices in [0, N) (what astraea_select_topk writes).  An index
 *    outside that range never becomes an access outside the buffers: a row
 *    read through it reads some valid row instead, a row written through it
 *    is dropped; no error is reported.  Duplicates make the writes race.
 */
#ifndef ASTRAEA_H
#define ASTRAEA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { ASTRAEA_F32 = 0, ASTRAEA_BF16 = 1 } astraea_dtype;

/* How the per-token change Delta is reduced over the C feature channels.
 * The paper describes it three ways (equation text: "value difference";
 * Algorithm 1 step 1: a mean over channels, commented as a squared
 * difference; procedure text: absolute difference).  L2 is what the benchmark
 * configurations use. */
typedef enum {
    ASTRAEA_DELTA_L2 = 0,       /* sqrt(sum_c d_c^2) */
    ASTRAEA_DELTA_MEAN_ABS = 1, /* (sum_c |d_c|) / C */
    ASTRAEA_DELTA_MEAN_SQ = 2   /* (sum_c d_c^2) / C */
} astraea_delta_mode;

enum {
    ASTRAEA_OK = 0,
    ASTRAEA_ERR_INVALID = -1,     /* NULL pointer, negative size, k > N, bad stride ... */
    ASTRAEA_ERR_UNSUPPORTED = -2, /* dtype / head_dim combination without a kernel */
    ASTRAEA_ERR_WORKSPACE = -3,   /* workspace missing, misaligned or too small */
    ASTRAEA_ERR_HIP = -4          /* a HIP launch reported an error */
};

/* Operation ids for astraea_workspace_bytes. */
typedef enum { ASTRAEA_ACT_NONE = 0, ASTRAEA_ACT_GELU_TANH = 1 } astraea_activation;
enum { ASTRAEA_OP_SELECT_TOPK = 1, ASTRAEA_OP_SPARSE_ATTN = 2 };

/*
 * astraea_score - selection metric S_token (paper Sec. 3.2 "Selection Metric":
 * S_token = w_alpha * S_sig + w_beta * S_penalty, S_sig = S_LSE,t-1 * Delta_token,t,
 * S_penalty = e^{n_i}; Algorithm 1 steps 1-2).
 *
 *   x_cur, x_prev  [N, C] rows `row_stride_elems` apart, dtype `dt`: token features of
 *                  this step and of the last computed step.
 *   lse_weight     [N] fp32 per-token S_LSE,t-1, or NULL for weight 1.
 *   skip_count     [N] int32 n_i (consecutive non-selections), or NULL: then the
 *                  penalty term is left out altogether (w_beta is ignored).
 *   penalty_table  [table_len] fp32, entry n = e^n as the caller rounded it; the
 *                  counter is clamped to [0, table_len-1].  Required with skip_count.
 *   score_out      [N] fp32.
 *
 * Arithmetic (fp32, defined to the bit so that selection is reproducible):
 * d_c = x_cur[i,c] - x_prev[i,c]; one accumulator runs over c = 0..C-1 in order with
 * acc = fma(d_c, d_c, acc) (or acc + |d_c|); Delta = sqrt(acc) correctly rounded, or
 * acc / (float)C; sig = Delta * lse_weight[i]; S = w_alpha * sig, and with counters
 * S = fma(w_beta, table[n], w_alpha * sig).
 */
int astraea_score(const void *x_cur, const void *x_prev, astraea_dtype dt, int64_t N, int64_t C,
                  int64_t row_stride_elems, astraea_delta_mode mode, const float *lse_weight,
                  const int32_t *skip_count, const float *penalty_table, int32_t table_len, float w_alpha,
                  float w_beta, float *score_out, void *stream);

/*
 * astraea_select_topk - I_sel, I_remain = TopK(S_token, theta) (Algorithm 1 step 3).
 * Selects the k tokens with the largest score; equal scores are won by the lower
 * index; -0 equals +0; NaN ranks below every number.  The result is unique.
 *
 *   score       [N] fp32.
 *   idx_sel     [k] int32 out, ascending token indices.
 *   idx_remain  [N-k] int32 out, ascending, or NULL.
 *   sel_mask    [N] uint8 out (1 = selected), or NULL.
 *   skip_count  [N] int32 in/out, or NULL: set to 0 for selected tokens and
 *               incremented for the others (the n_i of the penalty term).
 *   workspace   at least astraea_workspace_bytes(ASTRAEA_OP_SELECT_TOPK, N, k, 0, 0)
 *               bytes, 256-byte aligned; contents need not be initialised and are
 *               clobbered.  Calls sharing a workspace must not overlap in time.
 * k == 0 and k == N are valid.
 */
int astraea_select_topk(const float *score, int64_t N, int64_t k, int32_t *idx_sel, int32_t *idx_remain,
                        uint8_t *sel_mask, int32_t *skip_count, void *workspace, size_t workspace_bytes,
                        void *stream);

/*
 * astraea_select_topk_static - astraea_select_topk for callers that cannot allocate device memory or
 * hand over a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments without the workspace, same result to the bit.  The selection state, the
 * digit histogram and the per-workgroup counts live in a device array built into the library
 * (24.25 KiB per GPU, held until the process ends); the call allocates and frees nothing.
 *   N           at most 4194304 (2^22) scores; more returns ASTRAEA_ERR_UNSUPPORTED and enqueues nothing.
 * The GPU that `stream` belongs to must be the current device.  The array's address on that device is
 * looked up at the first call made with it current (hipGetSymbolAddress; make that first call outside
 * a graph capture).  All calls on one GPU share the one array, whatever their stream: two calls
 * that overlap in time on the same GPU race, so order them on one stream or with events.  Every
 * call clears what it needs at its start, with a kernel, so calls of any sizes may follow each other.
 */
int astraea_select_topk_static(const float *score, int64_t N, int64_t k, int32_t *idx_sel, int32_t *idx_remain,
                               uint8_t *sel_mask, int32_t *skip_count, void *stream);

/*
 * astraea_sparse_attn_fwd - attention of the selected queries over the full-length
 * keys and values (Algorithm 1 step 6; Sec. 3.2 "Sparse Attention"):
 *     o_sel[r, h, :] = sum_j softmax_j(scale * <q_r,h , k_j,h>) * v_j,h      j = 0..N-1
 * with no mask.  Row r of the result is exactly row idx_sel[r] of dense attention.
 *
 *   q           q_is_compact == 0: [N, H, D], the row of selected query r is
 *               q + idx_sel[r]*q_stride_n (gathered inside the kernel);
 *               q_is_compact == 1: [k_sel, H, D], row r is used and idx_sel may be NULL.
 *   k, v        [N, H, D]; K/V of unselected tokens are whatever the caller cached.
 *   strides     in elements; the head-dim index is contiguous.
 *   o_sel       [k_sel, H, D] contiguous, dtype `dt`.
 *   lse_sel     [k_sel, H] fp32 natural-log sum of exponentials of the scaled logits, or NULL.
 *   workspace   at least astraea_workspace_bytes(ASTRAEA_OP_SPARSE_ATTN, N, k_sel, H, D) bytes,
 *               256-byte aligned (may be NULL when that is 0).  The bf16 path stages a re-tiled
 *               copy of V there (N rounded up to 64, times H*D*2 bytes) plus 68 MB of partial
 *               results and 4 bytes per workgroup of the largest launch (flags of the workgroups
 *               a second launch redoes, see below) on every call; contents need not be
 *               initialised and are clobbered.
 *               The fp32 path uses it only for a selection too small to fill the chip, which
 *               it then cuts into key ranges (up to 8 x k_sel x H x (D + 4) floats of partial
 *               results); there the workspace is optional: with NULL, or fewer bytes than
 *               named, every work item sweeps all keys itself and the result is the same up
 *               to summation order.
 * The bf16 path runs its main kernel with each row's exponent offset fixed at the row max over the
 * first key tile, which is exact as long as no later logit exceeds that max by more than 80 powers of
 * two; workgroups with a row that does are redone by a second launch that takes a max per key tile.
 * The result does not depend on which of the two served a row beyond rounding.
 * Supported: (BF16, D = 128) on bf16 MFMA with fp32 softmax and accumulation;
 * (F32, D = 64 or 128) on fp32 MFMA.  k_sel == 0 enqueues nothing.
 * Pointers must be 16-byte aligned and strides multiples of 8 elements.
 */
int astraea_sparse_attn_fwd(const void *q, const void *k, const void *v, astraea_dtype dt, int64_t N, int32_t H,
                            int32_t D, int64_t q_stride_n, int64_t q_stride_h, int64_t kv_stride_n,
                            int64_t kv_stride_h, const int32_t *idx_sel, int64_t k_sel, int q_is_compact,
                            float softmax_scale, void *o_sel, float *lse_sel, void *workspace,
                            size_t workspace_bytes, void *stream);

/*
 * astraea_sparse_attn_update_fwd - the same attention with the cache merge fused into its last
 * step (Algorithm 1 steps 6-7 as one operation: X_out,t[I_sel] = Softmax(Q_sel K^T / sqrt(d)) V while
 * X_out,t[I_remain] keeps the cached rows): result row r is written straight to
 *     out_cache[idx_sel[r], h*D : (h+1)*D]
 * of the caller's per-token output buffer instead of to a compact array, which saves one write and one
 * read of k_sel*H*D elements and the astraea_scatter_update call.  Bit-identical to
 * astraea_sparse_attn_fwd followed by astraea_scatter_update(src_is_full = 0).
 *   out_cache         [N, cache_row_stride] elements of dtype `dt`, rows not in idx_sel untouched;
 *                     cache_row_stride >= H*D and a multiple of 8.
 *   idx_sel           required (distinct, in [0, N)), also when q_is_compact == 1.
 * All other arguments, limits and the workspace are those of astraea_sparse_attn_fwd.
 */
int astraea_sparse_attn_update_fwd(const void *q, const void *k, const void *v, astraea_dtype dt, int64_t N, int32_t H,
                                   int32_t D, int64_t q_stride_n, int64_t q_stride_h, int64_t kv_stride_n,
                                   int64_t kv_stride_h, const int32_t *idx_sel, int64_t k_sel, int q_is_compact,
                                   float softmax_scale, void *out_cache, int64_t cache_row_stride, float *lse_sel,
                                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * astraea_scatter_update - cache merge (Algorithm 1 steps 6-7): rows listed in idx_sel
 * are overwritten, every other row keeps what it held (the reuse of cached results).
 *   src_is_full == 0: cache[idx_sel[r], :] = src[r, :]            (src is [k_sel, row_elems])
 *   src_is_full == 1: cache[idx_sel[r], :] = src[idx_sel[r], :]   (src is [N, row_elems])
 * The second form refreshes cached K/V rows or the stored features of the last
 * computed step.  idx_sel must hold distinct indices in [0, N); duplicates race.
 * Row strides are in elements.  k_sel == 0 enqueues nothing.
 */
int astraea_scatter_update(void *cache, const void *src, astraea_dtype dt, int64_t N, int64_t row_elems,
                           int64_t cache_row_stride, int64_t src_row_stride, const int32_t *idx_sel,
                           int64_t k_sel, int src_is_full, void *stream);

/*
 * astraea_kv_refresh - the cached keys and values of the selected tokens are replaced by this step's, the
 * others keep what they hold (the configurations' "unselected tokens reuse cached K/V"; Algorithm 1 computes K
 * and V before its attention step):
 *     k_cache[idx_sel[r], :] = k_new[idx_sel[r], :],   v_cache[idx_sel[r], :] = v_new[idx_sel[r], :]
 * The same as two astraea_scatter_update calls with src_is_full = 1, in one launch.  The four buffers are
 * [N, row_elems] with a common row stride per side (elements); k_sel == 0 enqueues nothing.
 */
int astraea_kv_refresh(void *k_cache, void *v_cache, const void *k_new, const void *v_new, astraea_dtype dt, int64_t N,
                       int64_t row_elems, int64_t cache_row_stride, int64_t src_row_stride, const int32_t *idx_sel,
                       int64_t k_sel, void *stream);

/*
 * astraea_sparse_linear - a layer that acts on each token by itself, evaluated for the selected
 * tokens only (Algorithm 1: Q = X_in[I_sel] W_Q; Sec. 3.2: such layers are computed for the selected
 * tokens and taken from the cache for the rest; FLOPs appendix: the projection and MLP terms, whose
 * cost 2*N*c_in*c_out becomes 2*k_sel*c_in*c_out):
 *     y[row_out(r), o] = act( sum_c x[row_in(r), c] * w[o, c] + bias[o] ),   r = 0..k_sel-1, o = 0..c_out-1
 *   x        x_is_compact == 0: [N, x_row_stride], row_in(r) = idx_sel[r] (gathered inside the kernel);
 *            x_is_compact == 1: [k_sel, x_row_stride], row_in(r) = r.
 *   w        [c_out, c_in] contiguous: the weights of one output feature are contiguous.
 *   bias     [c_out] or NULL.
 *   y        y_is_compact == 1: [k_sel, y_row_stride], row_out(r) = r;
 *            y_is_compact == 0: [N, y_row_stride], row_out(r) = idx_sel[r] and every other row keeps
 *            what it held: with a cached K, V or output buffer as y this is the projection fused
 *            with the cache refresh.
 *   act      ASTRAEA_ACT_NONE, or ASTRAEA_ACT_GELU_TANH: 0.5 t (1 + tanh(sqrt(2/pi) (t + 0.044715 t^3))).
 * BF16: bf16 MFMA, fp32 accumulation, bias and activation in fp32, one rounding to bf16; x and w must
 * each span less than 4 GiB.  F32: fp32 MFMA, everything in fp32.  Both: c_in a multiple of 64, c_out a
 * multiple of 8, strides multiples of 8 elements, pointers 16-byte aligned.
 * idx_sel (distinct, in [0, N)) is required unless both sides are compact.  No workspace.
 * k_sel == 0 enqueues nothing.
 */
int astraea_sparse_linear(const void *x, const void *w, const void *bias, astraea_dtype dt, int64_t N, int64_t c_in,
                          int64_t c_out, int64_t x_row_stride, const int32_t *idx_sel, int64_t k_sel,
                          int x_is_compact, astraea_activation act, void *y, int64_t y_row_stride, int y_is_compact,
                          void *stream);

/*
 * Token-budget search (Sec. 3.3 "Algorithm"; supplementary algorithm "Evolutionary Search for Token
 * Scheduling").  Host-only: no GPU work, every pointer is host memory.  A schedule is T int32 levels in
 * tenths, theta_i in 0..10 for 0 %..100 % of the tokens at timestep i; budget_tenths is the target sum and
 * [ceil(0.9 B), floor(1.1 B)] the accepted range.  Random draws come from SplitMix64 seeded by the caller
 * (below(n) = floor(next*n / 2^64), unit() = (next >> 11) * 2^-53), so a seed fixes the result.
 *
 * astraea_budget_search: `population` random schedules are repaired into the range; per generation g = 1..G
 * `children` new ones are made, each from a random pair of distinct parents of the current population by
 * crossover (uniform or block, chosen with equal probability), mutation with probability
 * P(g) = p_mutation_start - (g/G)(p_mutation_start - p_mutation_final) per timestep, and repair, dropped
 * if already present (at most 64*children draws per generation); all are evaluated with `fitness` (lower is
 * better; called once per new candidate) and the best `population` survive, ties keeping the earlier one.
 *   best_theta [T] out; best_fitness out or NULL; population_out [population*T] and fitness_out
 *   [population] (best first) out or NULL; population_size_out (<= population) out or NULL.
 * The operator entry points apply one step to caller-held schedules and advance *rng_state (the SplitMix64
 * state): crossover kind ASTRAEA_CROSSOVER_UNIFORM takes each level from either parent with equal
 * probability; _BLOCK takes a contiguous range [min(a,b), max(a,b)), a and b drawn from 0..T, from parent0
 * and the rest from parent1; mutate redraws a level from 0..10 with probability p_mutation; repair lowers
 * (raises) random levels one tenth at a time, drawn among those that can still move, until the sum is in
 * range, and draws nothing if it already is.  Errors: ASTRAEA_ERR_INVALID for NULL, sizes, probabilities or
 * levels out of range.
 */
typedef double (*astraea_fitness_fn)(const int32_t *theta_tenths, int32_t T, void *user);
typedef struct {
    int32_t T;                 /* timesteps */
    int32_t population;        /* K: candidates kept per generation (the paper uses 50) */
    int32_t children;          /* P: new candidates per generation (30) */
    int32_t generations;       /* G (30) */
    int64_t budget_tenths;     /* target sum of the levels */
    double p_mutation_start;   /* P_0 */
    double p_mutation_final;   /* P_final */
    uint64_t seed;
} astraea_search_config;
enum { ASTRAEA_CROSSOVER_UNIFORM = 0, ASTRAEA_CROSSOVER_BLOCK = 1 };
int astraea_budget_search(const astraea_search_config *cfg, astraea_fitness_fn fitness, void *user,
                          int32_t *best_theta, double *best_fitness, int32_t *population_out, double *fitness_out,
                          int32_t *population_size_out);
int astraea_search_crossover(const int32_t *parent0, const int32_t *parent1, int32_t T, int kind, uint64_t *rng_state,
                             int32_t *child);
int astraea_search_mutate(int32_t *theta, int32_t T, double p_mutation, uint64_t *rng_state);
int astraea_search_repair(int32_t *theta, int32_t T, int64_t budget_tenths, uint64_t *rng_state);

/*
 * astraea_lse_weight_update - carries the softmax by-product S_LSE of the selection metric to the
 * next timestep (Sec. 3.2 "Selection Metric": S_sig = S_LSE,t-1 * Delta_token,t, where S_LSE is the
 * row sum of exponentials the softmax computes anyway).  For every selected token
 *     lse_weight[idx_sel[r]] = (1/H) * sum_h exp(min(lse_sel[r, h] - ln N, 64)),
 * the mean over heads of the row's mean exponential (the paper does not say how heads combine).  The
 * 1/N keeps the value near 1; it is the same as dividing w_alpha by N, so it changes no ranking while
 * the score is w_alpha * S_sig alone and does weigh S_sig against the penalty term w_beta * e^{n_i}
 * once counters are used: choose w_alpha for this scaling.  The exponent is capped at 64: a head whose
 * logits leave the range of the fp32 exponential contributes e^64 instead of infinity, so the weight
 * and the score it multiplies stay finite (beyond that point heads are no longer told apart).
 * Tokens not selected keep the weight of the last step they were computed in.  The sum runs over h
 * ascending in fp32.
 *   lse_sel     [k_sel, H] fp32, as written by astraea_sparse_attn_fwd.
 *   lse_weight  [N] fp32 in/out, the array astraea_score reads.
 */
int astraea_lse_weight_update(const float *lse_sel, int32_t H, int64_t N, const int32_t *idx_sel, int64_t k_sel,
                              float *lse_weight, void *stream);

/*
 * astraea_gather_rows - dst[r, :] = src[idx_sel[r], :] (Algorithm 1 step 5, X_in[I_sel]).
 */
int astraea_gather_rows(const void *src, void *dst, astraea_dtype dt, int64_t N, int64_t row_elems,
                        int64_t src_row_stride, int64_t dst_row_stride, const int32_t *idx_sel, int64_t k_sel,
                        void *stream);

/* Bytes of device workspace an operation needs for these sizes, valid for either dtype (host only). */
size_t astraea_workspace_bytes(int op, int64_t N, int64_t k_sel, int32_t H, int32_t D);

/* Tokens selected by a percent budget (Sec. 3.3: theta in {0, 10%, ..., 100%}):
 * (N * pct + 50) / 100, i.e. rounded half up.  Host only. */
int64_t astraea_budget_to_k(int64_t N, int32_t budget_percent);

/* Multiply-add count of the selected-query attention, 4*k_sel*N*D*H (the QK^T and AV terms
 * of the paper's FLOPs appendix with one N replaced by k_sel).  Host only. */
double astraea_attn_flops(int64_t N, int64_t k_sel, int32_t H, int32_t D);

/*
 * Debugging aid for callers that build idx_sel themselves: counts, on the device, the entries that
 * break the contract of the calls above.  counts_out (device, 2 x int32, overwritten):
 *   [0] entries outside [0, N);
 *   [1] positions r >= 1 with idx_sel[r] <= idx_sel[r-1], i.e. where the list is not strictly
 *       ascending, the form astraea_select_topk emits (a list with [1] == 0 has no duplicates;
 *       a list with [1] > 0 may still be duplicate-free, only not in that form).
 * Asynchronous on `stream` like every other call; the caller reads the counts when it chooses.
 */
int astraea_check_indices(const int32_t *idx_sel, int64_t k_sel, int64_t N, int32_t *counts_out, void *stream);

/*
 * How the bf16 attention would spread k_sel selected queries of H heads over the chip (the
 * budget-aware launch: time proportional to the selected-token count, paper Sec. 3.2 "linear
 * speedup").  Host only, nothing is enqueued; for inspection and tests.  A work item is one head
 * times one tile of 256 selected queries, head-major; XCD x (of 8) owns items
 * [x*items_per_xcd, (x+1)*items_per_xcd).  The first full_items of each XCD sweep all key tiles
 * (64 keys each); every later item is cut into `splits` consecutive key ranges of tiles_per_split
 * tiles, each run by its own workgroup, whose partial results a second kernel combines.
 * plan_out (host, 8 entries): q_tiles, items_per_xcd, full_items, splits, tiles_per_split,
 * workgroups launched, key tiles, partial-result slots the workspace holds.
 */
int astraea_attn_plan(int64_t N, int32_t H, int64_t k_sel, int64_t plan_out[8]);

/*
 * Measurement aids for the benchmark; neither is a step of the method.
 *
 * astraea_probe_mfma_bf16 runs a register-resident loop of v_mfma_f32_32x32x16_bf16
 * (`workgroups` workgroups of 4 waves, `iters` iterations of 4 independent MFMAs per wave) with
 * constant or pseudo-random operands and writes one float per thread to `sink` (device,
 * >= workgroups*256 floats).  *flops_out (host, may be NULL) receives the flops enqueued.
 *
 * astraea_probe_copy copies `bytes` (multiple of 16) from src to dst (device) with a plain
 * 16-byte-per-lane kernel: a transfer of known size against which the profiler's memory
 * counters are scaled.
 */
int astraea_probe_mfma_bf16(int32_t workgroups, int32_t iters, int32_t randomize, float *sink, int64_t sink_elems,
                            double *flops_out, void *stream);
int astraea_probe_copy(const void *src, void *dst, int64_t bytes, void *stream);
/*
 * Kernel timer, also a measurement aid.  astraea_probe_kernel_timer(1) makes every following
 * astraea_sparse_attn_fwd / astraea_sparse_attn_update_fwd call of this thread record a pair of HIP
 * events on its stream around its main kernel alone (not the V re-tiling pre-pass, not the launch that
 * redoes flagged workgroups, not the merge of partial results), for up to 64 calls; (0) stops it; either resets the count.  The events are created
 * on the first enable and kept.  astraea_probe_kernel_count returns how many launches were timed,
 * astraea_probe_kernel_ms(i, &ms) waits for launch i to finish and returns its duration (host pointer).
 */
int astraea_probe_kernel_timer(int enable);
int32_t astraea_probe_kernel_count(void);
int astraea_probe_kernel_ms(int32_t index, double *ms_out);

const char *astraea_status_string(int status);
const char *astraea_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ASTRAEA_H */
