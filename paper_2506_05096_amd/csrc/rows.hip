// Row movers behind astraea_gather_rows and astraea_scatter_update, and the per-token S_LSE update
// (paper, Algorithm 1: X_in[I_sel] in step 5, and the cache merge of steps 6-7).
//
// A token row (H*D elements, 6 KiB for 24 heads x 128 x bf16) is contiguous, so the copy is fully
// coalesced without staging: one wavefront moves one row, each lane 16 bytes per step, all of a
// lane's loads issued before its stores.  Unselected rows are never touched, which is exactly the
// "reuse the cached result" half of the merge.  HBM-bound: 2 * row_bytes per selected token.
// A source row is read once, so its loads carry the streaming hint (not kept in L2): 112 -> 88 us for
// the 219 MB scatter at N = 118800 with cold caches, no worse with warm ones.  Stores stay plain: the
// destination rows are read again by the next kernel.
#include "common.h"

namespace astraea {
namespace {

typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

constexpr int kRowsPerBlock = 4;      // one wave per row

template <typename V> __device__ __forceinline__ V load_once(const V *p) { return __builtin_nontemporal_load(p); }

// blockIdx.y picks one of up to two (destination, source) buffer pairs that share shape, strides and index list:
// the K and the V cache of a layer are refreshed by one launch.
template <typename V>
__global__ __launch_bounds__(kRowsPerBlock *kWave) void move_rows_kernel(
    char *__restrict__ dst0, const char *__restrict__ src0, char *__restrict__ dst1, const char *__restrict__ src1,
    int64_t row_bytes, int64_t dst_stride, int64_t src_stride,
    const int32_t *__restrict__ idx, int64_t k_sel, int64_t n_rows, int index_dst, int index_src)
{
    char *__restrict__ dst = blockIdx.y ? dst1 : dst0;
    const char *__restrict__ src = blockIdx.y ? src1 : src0;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = (int64_t)blockIdx.x * kRowsPerBlock + threadIdx.x / kWave;
    if (r >= k_sel) return;
    const int64_t tok = idx[r];
    if ((uint64_t)tok >= (uint64_t)n_rows) return;      // an index outside the buffer moves nothing
    const V *s = reinterpret_cast<const V *>(src + (index_src ? tok : r) * src_stride);
    V *d = reinterpret_cast<V *>(dst + (index_dst ? tok : r) * dst_stride);
    const int64_t nvec = row_bytes / (int64_t)sizeof(V);
    // groups of 4, then 2, then 1 vectors per lane: every group's loads are issued before its stores
    int64_t p = lane;
#pragma unroll 1
    for (; p + 3 * kWave < nvec; p += 4 * kWave) {
        const V b0 = load_once(s + p), b1 = load_once(s + p + kWave), b2 = load_once(s + p + 2 * kWave),
                b3 = load_once(s + p + 3 * kWave);
        d[p] = b0;
        d[p + kWave] = b1;
        d[p + 2 * kWave] = b2;
        d[p + 3 * kWave] = b3;
    }
    if (p + kWave < nvec) {
        const V b0 = load_once(s + p), b1 = load_once(s + p + kWave);
        d[p] = b0;
        d[p + kWave] = b1;
        p += 2 * kWave;
    }
    if (p < nvec) d[p] = load_once(s + p);
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
    dim3 grid((unsigned)((k_sel + kRowsPerBlock - 1) / kRowsPerBlock), dst_b ? 2u : 1u), block(kRowsPerBlock * kWave);
    const uintptr_t all = (uintptr_t)dst | (uintptr_t)src | (uintptr_t)dst_b | (uintptr_t)src_b | (uintptr_t)row_bytes |
                          (uintptr_t)dst_stride_bytes | (uintptr_t)src_stride_bytes;
    if (all % 16 == 0)
        hipLaunchKernelGGL(move_rows_kernel<uint4v>, grid, block, 0, stream, (char *)dst, (const char *)src, (char *)dst_b,
                           (const char *)src_b, row_bytes, dst_stride_bytes, src_stride_bytes, idx, k_sel, n_rows,
                           (int)index_dst, (int)index_src);
    else if (all % 4 == 0)
        hipLaunchKernelGGL(move_rows_kernel<uint32_t>, grid, block, 0, stream, (char *)dst, (const char *)src, (char *)dst_b,
                           (const char *)src_b, row_bytes, dst_stride_bytes, src_stride_bytes, idx, k_sel, n_rows,
                           (int)index_dst, (int)index_src);
    else
        hipLaunchKernelGGL(move_rows_kernel<uint16_t>, grid, block, 0, stream, (char *)dst, (const char *)src, (char *)dst_b,
                           (const char *)src_b, row_bytes, dst_stride_bytes, src_stride_bytes, idx, k_sel, n_rows,
                           (int)index_dst, (int)index_src);
    return check_launch("astraea row move");
}

}  // namespace astraea
