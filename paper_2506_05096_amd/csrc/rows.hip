// Row movers behind astraea_gather_rows, astraea_scatter_update and astraea_kv_refresh, and the per-token
// S_LSE update (paper, Algorithm 1: X_in[I_sel] in step 5, and the cache merge of steps 6-7).
//
// A token row (H*D elements, 6 KiB for 24 heads x 128 x bf16) is contiguous, so the copy is fully
// coalesced without staging.  Shape: one 16-byte vector per thread and one wavefront per workgroup, i.e. a
// workgroup moves 1 KiB of one row and ends; consecutive workgroups take consecutive pieces of a row, then
// the next row.  Measured at N = 118800, k = 35640, caches flushed before each call, against the earlier
// shape (one wavefront per whole row, 6 vectors per lane): scatter 88 -> 74 us, K/V refresh 185 -> 147 us,
// gather 86 -> 72 us; the same holds for a dense 1 GiB copy (one vector per thread 6.2 - 6.6 TB/s, a
// grid-stride loop 4.6, eight vectors per thread 5.4).  Pieces of 128 or 384 threads: 5 - 10 % slower; 256: worse
// than the earlier shape.  Unselected rows are never touched, which is exactly the "reuse the cached result"
// half of the merge.  HBM-bound: 2 * row_bytes per selected token.
// A source row is read once, so its loads carry the streaming hint (not kept in L2).  Stores carry it when
// both sides are rows of full-size buffers (the K/V refresh, the copy of the selected tokens' features): 172 ->
// 148 us for the refresh.  Stores of compact rows stay plain (the next kernel reads them), and so do the
// scatter's: its source was written by the kernel before it and is still in the caches, and with streaming
// stores that case is slower (64 -> 70 us inside a layer-step).
#include "common.h"

namespace astraea {
namespace {

typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

template <typename V> __device__ __forceinline__ V load_once(const V *p) { return __builtin_nontemporal_load(p); }

// blockIdx.x = row * pieces + piece; blockIdx.y picks one of up to two (destination, source) buffer pairs that
// share shape, strides and index list: the K and the V cache of a layer are refreshed by one launch.
// STREAM_DST is a template parameter because a run-time choice between the two kinds of store is merged by
// the compiler into one plain store.
template <typename V, bool STREAM_DST>
__global__ __launch_bounds__(kWave) void move_rows_kernel(
    char *__restrict__ dst0, const char *__restrict__ src0, char *__restrict__ dst1, const char *__restrict__ src1,
    int64_t row_bytes, int64_t dst_stride, int64_t src_stride,
    const int32_t *__restrict__ idx, int64_t k_sel, int64_t n_rows, int index_dst, int index_src, int32_t pieces)
{
    char *__restrict__ dst = blockIdx.y ? dst1 : dst0;
    const char *__restrict__ src = blockIdx.y ? src1 : src0;
    const int64_t r = blockIdx.x / (uint32_t)pieces;
    const int64_t p = (int64_t)(blockIdx.x % (uint32_t)pieces) * kWave + threadIdx.x;
    if (r >= k_sel || p >= row_bytes / (int64_t)sizeof(V)) return;
    const int64_t tok = idx[r];
    if ((uint64_t)tok >= (uint64_t)n_rows) return;      // an index outside the buffer moves nothing
    const V *s = reinterpret_cast<const V *>(src + (index_src ? tok : r) * src_stride);
    V *d = reinterpret_cast<V *>(dst + (index_dst ? tok : r) * dst_stride);
    const V v = load_once(s + p);
    if (STREAM_DST) __builtin_nontemporal_store(v, d + p);
    else d[p] = v;
}

// lse_weight[idx[r]] = mean over heads of exp(min(lse[r, h] - ln N, 64)); one thread per selected token.
// The cap keeps the weight finite when a head's logits leave the range of the fp32 exponential.
__global__ __launch_bounds__(256) void lse_weight_kernel(const float *__restrict__ lse_sel, int32_t H, float log_n,
                                                         const int32_t *__restrict__ idx, int64_t k_sel, int64_t n_rows,
                                                         float *__restrict__ lse_weight)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= k_sel) return;
    float acc = 0.0f;
    for (int h = 0; h < H; ++h) acc += expf(fminf(lse_sel[r * H + h] - log_n, 64.0f));
    const int64_t tok = idx[r];
    if ((uint64_t)tok < (uint64_t)n_rows) lse_weight[tok] = acc / (float)H;
}

// counts[0] += entries outside [0, n_rows); counts[1] += positions r >= 1 with idx[r] <= idx[r-1].
__global__ __launch_bounds__(256) void check_indices_kernel(const int32_t *__restrict__ idx, int64_t k_sel,
                                                            int64_t n_rows, int32_t *__restrict__ counts)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= k_sel) return;
    const int32_t ix = idx[r];
    if ((uint64_t)(int64_t)ix >= (uint64_t)n_rows) atomicAdd(&counts[0], 1);
    if (r > 0 && ix <= idx[r - 1]) atomicAdd(&counts[1], 1);
}

__global__ void clear_counts_kernel(int32_t *counts)
{
    if (threadIdx.x < 2) counts[threadIdx.x] = 0;
}

}  // namespace

int launch_check_indices(const int32_t *idx_sel, int64_t k_sel, int64_t N, int32_t *counts, hipStream_t stream)
{
    // a fill kernel, not a memset: the call may be recorded into a graph
    hipLaunchKernelGGL(clear_counts_kernel, dim3(1), dim3(64), 0, stream, counts);
    if (k_sel > 0)
        hipLaunchKernelGGL(check_indices_kernel, dim3((unsigned)((k_sel + 255) / 256)), dim3(256), 0, stream, idx_sel,
                           k_sel, N, counts);
    return check_launch("astraea_check_indices");
}

int launch_lse_weight_update(const float *lse_sel, int32_t H, int64_t N, const int32_t *idx_sel, int64_t k_sel,
                             float *lse_weight, hipStream_t stream)
{
    if (k_sel == 0) return ASTRAEA_OK;
    hipLaunchKernelGGL(lse_weight_kernel, dim3((unsigned)((k_sel + 255) / 256)), dim3(256), 0, stream, lse_sel, H,
                       logf((float)N), idx_sel, k_sel, N, lse_weight);
    return check_launch("astraea_lse_weight_update");
}

int launch_move_rows(void *dst, const void *src, int64_t row_bytes, int64_t dst_stride_bytes,
                     int64_t src_stride_bytes, const int32_t *idx, int64_t k_sel, int64_t n_rows, bool index_dst,
                     bool index_src, hipStream_t stream, void *dst_b, const void *src_b)
{
    if (k_sel == 0 || row_bytes == 0) return ASTRAEA_OK;
    const uintptr_t all = (uintptr_t)dst | (uintptr_t)src | (uintptr_t)dst_b | (uintptr_t)src_b | (uintptr_t)row_bytes |
                          (uintptr_t)dst_stride_bytes | (uintptr_t)src_stride_bytes;
    const int vec = all % 16 == 0 ? 16 : (all % 4 == 0 ? 4 : 2);
    const int64_t pieces = (row_bytes / vec + kWave - 1) / kWave;
    if (pieces > 2147483647LL / k_sel) return fail(ASTRAEA_ERR_INVALID, "astraea row move: k_sel * row pieces exceeds the grid limit");
    dim3 grid((unsigned)(k_sel * pieces), dst_b ? 2u : 1u), block(kWave);
#define ASTRAEA_MOVE(V, S)                                                                                              \
    hipLaunchKernelGGL((move_rows_kernel<V, S>), grid, block, 0, stream, (char *)dst, (const char *)src, (char *)dst_b, \
                       (const char *)src_b, row_bytes, dst_stride_bytes, src_stride_bytes, idx, k_sel, n_rows,         \
                       (int)index_dst, (int)index_src, (int32_t)pieces)
    // cache rows refreshed from rows of another full-size buffer: both sides come from and go to HBM
    const bool stream_dst = index_dst && index_src;
    if (vec == 16) {
        if (stream_dst) ASTRAEA_MOVE(uint4v, true);
        else ASTRAEA_MOVE(uint4v, false);
    } else if (vec == 4) {
        if (stream_dst) ASTRAEA_MOVE(uint32_t, true);
        else ASTRAEA_MOVE(uint32_t, false);
    } else {
        if (stream_dst) ASTRAEA_MOVE(uint16_t, true);
        else ASTRAEA_MOVE(uint16_t, false);
    }
#undef ASTRAEA_MOVE
    return check_launch("astraea row move");
}

}  // namespace astraea
