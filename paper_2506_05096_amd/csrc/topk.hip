// astraea_select_topk: I_sel, I_remain = TopK(S_token, theta) (paper, Algorithm 1 step 3).
//
// Exact, deterministic selection of the k largest fp32 scores with lowest-index tie-break:
//   1. scores map to order-preserving 32-bit keys (-0 -> +0, NaN -> lowest key);
//   2. a 3-pass radix select (11 + 11 + 10 bits, most significant first) finds the key T of the
//      k-th largest element and `need`, the number of elements equal to T that are still selected;
//      each pass is a histogram over the elements that match the prefix found so far, built with
//      wavefront match-free LDS atomics and merged by integer global atomics (order-independent);
//      the workgroup that finishes last (atomic ticket) resolves the digit, so no host round trip
//      and no spinning is involved;
//   3. a count kernel + an emit kernel compact the selected indices in ascending index order:
//      an element is selected iff key > T, or key == T and fewer than `need` equal elements
//      precede it.  Ranks come from wavefront ballots and prefix popcounts.
// The score array (4N bytes) stays in L2 across the five small launches; the step is latency-bound.
// Up to 32768 scores take a single-workgroup kernel instead (one launch, keys held in LDS).  (A single
// workgroup that streams more scores than LDS holds from L2 in every pass was measured too: one launch, but
// one compute unit's loads are latency-bound, 129 us against 43 us at 118800 scores.)
#include <mutex>

#include "common.h"

namespace astraea {
namespace {

constexpr int kThreads = 256;
constexpr int kItems = 8;                       // consecutive elements per thread
constexpr int kChunk = kThreads * kItems;       // elements per workgroup
constexpr int kBins = 2048;
constexpr int kNumPass = 3;
__constant__ const int kShift[kNumPass] = {21, 10, 0};
__constant__ const int kBits[kNumPass] = {11, 11, 10};

struct SelectState {
    uint32_t prefix;      // key bits decided so far
    uint32_t mask;        // which bits those are
    uint32_t k_rem;       // how many elements are still to be taken among those matching the prefix
    uint32_t ticket;      // workgroups finished in the current launch
    uint32_t pad[60];
};
static_assert(sizeof(SelectState) == 256, "state block is one 256-byte line");

// workspace layout: [SelectState][hist kBins u32][cnt_gt nb u32][cnt_eq nb u32]
__host__ __device__ inline size_t ws_hist_off() { return sizeof(SelectState); }
__host__ __device__ inline size_t ws_cnt_off() { return sizeof(SelectState) + kBins * sizeof(uint32_t); }

__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t b = __float_as_uint(s);
    if ((b & 0x7fffffffu) > 0x7f800000u) return 0u;        // NaN: below every number
    if (b == 0x80000000u) b = 0u;                           // -0 == +0
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// k > 0: empty prefix, the passes refine it.  k == 0: the passes are skipped and the threshold is
// the key no score maps to (all ones), so nothing compares above or equal to it with need = 0.
__global__ void topk_init_kernel(SelectState *st, uint32_t *hist, uint32_t k)
{
    for (int i = threadIdx.x; i < kBins; i += blockDim.x) hist[i] = 0;
    if (threadIdx.x == 0) {
        st->prefix = k ? 0u : 0xffffffffu;
        st->mask = 0;
        st->k_rem = k;
        st->ticket = 0;
    }
}

// One radix pass.  PASS is the digit position (0 = most significant).
template <int PASS>
__global__ __launch_bounds__(kThreads) void topk_hist_kernel(const float *__restrict__ score, int64_t N,
                                                             SelectState *st, uint32_t *hist)
{
    __shared__ uint32_t lh[kBins];
    __shared__ uint32_t wave_tot[kThreads / kWave];
    __shared__ uint32_t is_last;
    const int shift = kShift[PASS];
    const uint32_t nb = 1u << kBits[PASS];
    for (int i = threadIdx.x; i < kBins; i += kThreads) lh[i] = 0;
    __syncthreads();
    const uint32_t prefix = st->prefix, mask = st->mask;
    const int64_t base = (int64_t)blockIdx.x * kChunk;
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        int64_t i = base + it * kThreads + threadIdx.x;       // order is irrelevant for counting
        if (i < N) {
            uint32_t key = score_key(score[i]);
            if ((key & mask) == prefix) atomicAdd(&lh[(key >> shift) & (nb - 1)], 1u);
        }
    }
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < nb; b += kThreads) {
        uint32_t c = lh[b];
        if (c) atomicAdd(&hist[b], c);
    }
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) is_last = (atomicAdd(&st->ticket, 1u) == gridDim.x - 1) ? 1u : 0u;
    __syncthreads();
    if (!is_last) return;
    __threadfence();

    // Last workgroup: walk the bins from the largest digit down until k_rem elements are covered.
    // Thread t owns bins [hi - t*per, hi - (t+1)*per) in descending order.
    const uint32_t per = nb / kThreads;                    // 8 or 4
    const uint32_t k_rem = st->k_rem;
    uint32_t cnt[8];
    uint32_t mine = 0;
    for (uint32_t j = 0; j < per; ++j) {
        uint32_t b = nb - 1 - (threadIdx.x * per + j);
        cnt[j] = __hip_atomic_load(&hist[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        mine += cnt[j];
    }
    // exclusive prefix over threads (descending bins): wave scan, then across waves
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    uint32_t incl = mine;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        uint32_t o = __shfl_up(incl, d);
        if (lane >= d) incl += o;
    }
    if (lane == kWave - 1) wave_tot[wv] = incl;
    __syncthreads();
    uint32_t before = incl - mine;
    for (int w = 0; w < wv; ++w) before += wave_tot[w];
    // the digit is the first bin (descending) whose running count reaches k_rem
    uint32_t run = before;
    for (uint32_t j = 0; j < per; ++j) {
        uint32_t b = nb - 1 - (threadIdx.x * per + j);
        if (run < k_rem && run + cnt[j] >= k_rem) {
            st->prefix = prefix | (b << shift);
            st->mask = mask | ((nb - 1) << shift);
            st->k_rem = k_rem - run;
        }
        run += cnt[j];
    }
    // reset for the next launch
    for (int i = threadIdx.x; i < kBins; i += kThreads) hist[i] = 0;
    if (threadIdx.x == 0) st->ticket = 0;
}

// Per-workgroup counts of keys above / equal to the threshold; the last workgroup turns them into
// exclusive offsets over workgroups (ascending index order).
__global__ __launch_bounds__(kThreads) void topk_count_kernel(const float *__restrict__ score, int64_t N,
                                                              SelectState *st, uint32_t *cnt_gt, uint32_t *cnt_eq)
{
    __shared__ uint32_t red_gt[kThreads / kWave], red_eq[kThreads / kWave];
    __shared__ uint32_t is_last;
    const uint32_t T = st->prefix;
    const int64_t base = (int64_t)blockIdx.x * kChunk;
    uint32_t g = 0, e = 0;
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        int64_t i = base + it * kThreads + threadIdx.x;
        if (i < N) {
            uint32_t key = score_key(score[i]);
            g += key > T;
            e += key == T;
        }
    }
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) {
        g += __shfl_xor(g, d);
        e += __shfl_xor(e, d);
    }
    if (lane == 0) {
        red_gt[wv] = g;
        red_eq[wv] = e;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t sg = 0, se = 0;
        for (int w = 0; w < kThreads / kWave; ++w) {
            sg += red_gt[w];
            se += red_eq[w];
        }
        cnt_gt[blockIdx.x] = sg;
        cnt_eq[blockIdx.x] = se;
        __threadfence();
        is_last = (atomicAdd(&st->ticket, 1u) == gridDim.x - 1) ? 1u : 0u;
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();

    // exclusive scan of both count arrays over workgroups, by this one workgroup
    __shared__ uint32_t carry_g, carry_e;
    __shared__ uint32_t wt_g[kThreads / kWave], wt_e[kThreads / kWave];
    if (threadIdx.x == 0) {
        carry_g = 0;
        carry_e = 0;
    }
    __syncthreads();
    const uint32_t nblk = gridDim.x;
    for (uint32_t b0 = 0; b0 < nblk; b0 += kThreads) {
        uint32_t b = b0 + threadIdx.x;
        uint32_t vg = 0, ve = 0;
        if (b < nblk) {
            vg = __hip_atomic_load(&cnt_gt[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ve = __hip_atomic_load(&cnt_eq[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        uint32_t ig = vg, ie = ve;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            uint32_t og = __shfl_up(ig, d), oe = __shfl_up(ie, d);
            if (lane >= d) {
                ig += og;
                ie += oe;
            }
        }
        if (lane == kWave - 1) {
            wt_g[wv] = ig;
            wt_e[wv] = ie;
        }
        __syncthreads();
        uint32_t pg = carry_g + ig - vg, pe = carry_e + ie - ve;
        for (int w = 0; w < wv; ++w) {
            pg += wt_g[w];
            pe += wt_e[w];
        }
        if (b < nblk) {
            cnt_gt[b] = pg;
            cnt_eq[b] = pe;
        }
        __syncthreads();
        if (threadIdx.x == kThreads - 1) {
            carry_g = pg + vg;
            carry_e = pe + ve;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) st->ticket = 0;
}

// Writes idx_sel / idx_remain / mask / skip counters.  Thread t owns elements
// [base + t*kItems, base + (t+1)*kItems), so ranks follow index order.
__global__ __launch_bounds__(kThreads) void topk_emit_kernel(const float *__restrict__ score, int64_t N,
                                                             const SelectState *st, const uint32_t *off_gt,
                                                             const uint32_t *off_eq, int32_t *__restrict__ idx_sel,
                                                             int32_t *__restrict__ idx_remain,
                                                             uint8_t *__restrict__ sel_mask,
                                                             int32_t *__restrict__ skip_count)
{
    __shared__ uint32_t wt_g[kThreads / kWave], wt_e[kThreads / kWave];
    const uint32_t T = st->prefix, need = st->k_rem;
    const int64_t base = (int64_t)blockIdx.x * kChunk + (int64_t)threadIdx.x * kItems;
    uint32_t gt_bits = 0, eq_bits = 0;
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        int64_t i = base + it;
        if (i < N) {
            uint32_t key = score_key(score[i]);
            gt_bits |= (uint32_t)(key > T) << it;
            eq_bits |= (uint32_t)(key == T) << it;
        }
    }
    const uint32_t mg = __popc(gt_bits), me = __popc(eq_bits);
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    uint32_t ig = mg, ie = me;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        uint32_t og = __shfl_up(ig, d), oe = __shfl_up(ie, d);
        if (lane >= d) {
            ig += og;
            ie += oe;
        }
    }
    if (lane == kWave - 1) {
        wt_g[wv] = ig;
        wt_e[wv] = ie;
    }
    __syncthreads();
    uint32_t g_before = off_gt[blockIdx.x] + ig - mg;     // keys > T before this thread's first element
    uint32_t e_before = off_eq[blockIdx.x] + ie - me;     // keys == T before it
    for (int w = 0; w < wv; ++w) {
        g_before += wt_g[w];
        e_before += wt_e[w];
    }
#pragma unroll
    for (int it = 0; it < kItems; ++it) {
        int64_t i = base + it;
        if (i >= N) break;
        const bool g = (gt_bits >> it) & 1u, e = (eq_bits >> it) & 1u;
        const uint32_t sel_before = g_before + (e_before < need ? e_before : need);
        const bool sel = g || (e && e_before < need);
        if (sel)
            idx_sel[sel_before] = (int32_t)i;
        else if (idx_remain)
            idx_remain[i - sel_before] = (int32_t)i;
        if (sel_mask) sel_mask[i] = sel ? 1 : 0;
        if (skip_count) skip_count[i] = sel ? 0 : skip_count[i] + 1;
        g_before += g;
        e_before += e;
    }
}

// ---- small inputs: the whole selection in one workgroup and one launch.  Up to kSmallMax keys live in LDS
// (128 KiB of the CU's 160); the three radix passes, the digit search and the ordered emit are the steps of
// the kernels above with workgroup barriers where those have launches.  Thread t owns the contiguous
// elements [t*items, (t+1)*items), so ranks follow index order; a thread adds a run of equal digits with one
// LDS atomic, which keeps tightly clustered scores (all of them in one or two bins) from serialising.
constexpr int kSmallMax = 32768;
constexpr int kSmallThreads = 1024;

__global__ __launch_bounds__(kSmallThreads) void topk_small_kernel(const float *__restrict__ score, int32_t N, uint32_t k,
                                                                   int32_t *__restrict__ idx_sel,
                                                                   int32_t *__restrict__ idx_remain,
                                                                   uint8_t *__restrict__ sel_mask,
                                                                   int32_t *__restrict__ skip_count)
{
    __shared__ uint32_t keys[kSmallMax];
    __shared__ uint32_t hist[kBins];
    __shared__ uint32_t wt_a[kSmallThreads / kWave], wt_b[kSmallThreads / kWave];
    __shared__ uint32_t s_prefix, s_mask, s_krem;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int items = ((N + kSmallThreads - 1) / kSmallThreads) | 1;    // odd: a thread's walk through its elements is free of bank conflicts
    const int first = tid * items;
    const int last = first + items < N ? first + items : N;         // this thread's elements: [first, last)
    for (int i = tid; i < N; i += kSmallThreads) keys[i] = score_key(score[i]);
    if (tid == 0) {
        s_prefix = k ? 0u : 0xffffffffu;       // k == 0: a threshold no key reaches, nothing is selected
        s_mask = 0;
        s_krem = k;
    }
    __syncthreads();
    if (k > 0) {
        for (int pass = 0; pass < kNumPass; ++pass) {
            const int shift = kShift[pass];
            const uint32_t nb = 1u << kBits[pass];
            for (int i = tid; i < kBins; i += kSmallThreads) hist[i] = 0;
            __syncthreads();
            const uint32_t prefix = s_prefix, mask = s_mask, k_rem = s_krem;
            uint32_t run_bin = 0, run_len = 0;
            for (int i = first; i < last; ++i) {
                const uint32_t key = keys[i];
                if ((key & mask) != prefix) continue;
                const uint32_t b = (key >> shift) & (nb - 1);
                if (run_len && b != run_bin) {
                    atomicAdd(&hist[run_bin], run_len);
                    run_len = 0;
                }
                run_bin = b;
                ++run_len;
            }
            if (run_len) atomicAdd(&hist[run_bin], run_len);
            __syncthreads();
            // the digit: walking the bins from the largest down, the first whose running count reaches k_rem.
            // Thread t owns bins nb-1 - (t*per + j), j < per (per = 2 or 1).
            const uint32_t per = nb / kSmallThreads;
            uint32_t cnt[2] = {0, 0}, mine = 0;
            for (uint32_t j = 0; j < per; ++j) {
                cnt[j] = hist[nb - 1 - (tid * per + j)];
                mine += cnt[j];
            }
            uint32_t incl = mine;
#pragma unroll
            for (int d = 1; d < kWave; d <<= 1) {
                const uint32_t o = __shfl_up(incl, d);
                if (lane >= d) incl += o;
            }
            if (lane == kWave - 1) wt_a[wv] = incl;
            __syncthreads();
            uint32_t run = incl - mine;
            for (int w = 0; w < wv; ++w) run += wt_a[w];
            for (uint32_t j = 0; j < per; ++j) {
                const uint32_t b = nb - 1 - (tid * per + j);
                if (run < k_rem && run + cnt[j] >= k_rem) {          // true for exactly one bin of one thread
                    s_prefix = prefix | (b << shift);
                    s_mask = mask | ((nb - 1) << shift);
                    s_krem = k_rem - run;
                }
                run += cnt[j];
            }
            __syncthreads();
        }
    }
    // ordered emit, as in topk_emit_kernel
    const uint32_t T = s_prefix, need = s_krem;
    uint32_t mg = 0, me = 0;
    for (int i = first; i < last; ++i) {
        mg += keys[i] > T;
        me += keys[i] == T;
    }
    uint32_t ig = mg, ie = me;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t og = __shfl_up(ig, d), oe = __shfl_up(ie, d);
        if (lane >= d) {
            ig += og;
            ie += oe;
        }
    }
    if (lane == kWave - 1) {
        wt_a[wv] = ig;
        wt_b[wv] = ie;
    }
    __syncthreads();
    uint32_t g_before = ig - mg, e_before = ie - me;
    for (int w = 0; w < wv; ++w) {
        g_before += wt_a[w];
        e_before += wt_b[w];
    }
    for (int i = first; i < last; ++i) {
        const bool g = keys[i] > T, e = keys[i] == T;
        const uint32_t sel_before = g_before + (e_before < need ? e_before : need);
        const bool sel = g || (e && e_before < need);
        if (sel)
            idx_sel[sel_before] = i;
        else if (idx_remain)
            idx_remain[i - sel_before] = i;
        if (sel_mask) sel_mask[i] = sel ? 1 : 0;
        if (skip_count) skip_count[i] = sel ? 0 : skip_count[i] + 1;
        g_before += g;
        e_before += e;
    }
}

// ---- astraea_select_topk_static: the same selection for callers that cannot allocate.  The selection state,
// the histogram and the per-workgroup counts live in this file-scope device array instead of a caller's
// workspace: 256 B of state + 8 KiB of histogram + 8 B per 2048 scores, 24.25 KiB for the largest input
// the entry point takes.  Every GPU the library runs on holds its own copy, at its own address, until the
// process ends.  In host code the array's name only stands for the symbol: the address kernels are given is
// the one hipGetSymbolAddress returns for the device that is current, looked up once per device.
constexpr int64_t kStaticMaxN = (int64_t)1 << 22;
constexpr size_t kStaticBytes = sizeof(SelectState) + kBins * sizeof(uint32_t) + 2 * (size_t)(kStaticMaxN / kChunk) * sizeof(uint32_t);
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxDevices] = {};

}  // namespace

int64_t topk_static_max_n() { return kStaticMaxN; }

// Device address of `scratch` on the current device (first use on a device looks it up and keeps it).
int topk_static_scratch(void **ptr_out)
{
    static_assert(kStaticBytes % 256 == 0, "scratch size keeps the 256-byte granularity of the workspace");
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(ASTRAEA_ERR_HIP, "astraea_select_topk_static: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices)
        return fail(ASTRAEA_ERR_UNSUPPORTED, "astraea_select_topk_static: device ordinal %d not below %d", dev, kMaxDevices);
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(ASTRAEA_ERR_HIP, "astraea_select_topk_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *ptr_out = g_scratch_ptr[dev];
    return ASTRAEA_OK;
}

size_t topk_workspace_bytes(int64_t N)
{
    const int64_t nblk = (N + kChunk - 1) / kChunk;
    size_t b = ws_cnt_off() + 2 * (size_t)(nblk > 0 ? nblk : 1) * sizeof(uint32_t);
    return (b + 255) & ~(size_t)255;
}

int launch_select_topk(const float *score, int64_t N, int64_t k, int32_t *idx_sel, int32_t *idx_remain,
                       uint8_t *sel_mask, int32_t *skip_count, void *workspace, hipStream_t stream)
{
    if (N == 0) return ASTRAEA_OK;
    if (N <= kSmallMax) {
        hipLaunchKernelGGL(topk_small_kernel, dim3(1), dim3(kSmallThreads), 0, stream, score, (int32_t)N, (uint32_t)k,
                           idx_sel, idx_remain, sel_mask, skip_count);
        return check_launch("astraea_select_topk");
    }
    const unsigned nblk = (unsigned)((N + kChunk - 1) / kChunk);
    SelectState *st = reinterpret_cast<SelectState *>(workspace);
    uint32_t *hist = reinterpret_cast<uint32_t *>((char *)workspace + ws_hist_off());
    uint32_t *cnt_gt = reinterpret_cast<uint32_t *>((char *)workspace + ws_cnt_off());
    uint32_t *cnt_eq = cnt_gt + nblk;
    hipLaunchKernelGGL(topk_init_kernel, dim3(1), dim3(kThreads), 0, stream, st, hist, (uint32_t)k);
    if (k > 0) {
        hipLaunchKernelGGL(topk_hist_kernel<0>, dim3(nblk), dim3(kThreads), 0, stream, score, N, st, hist);
        hipLaunchKernelGGL(topk_hist_kernel<1>, dim3(nblk), dim3(kThreads), 0, stream, score, N, st, hist);
        hipLaunchKernelGGL(topk_hist_kernel<2>, dim3(nblk), dim3(kThreads), 0, stream, score, N, st, hist);
    }
    hipLaunchKernelGGL(topk_count_kernel, dim3(nblk), dim3(kThreads), 0, stream, score, N, st, cnt_gt, cnt_eq);
    hipLaunchKernelGGL(topk_emit_kernel, dim3(nblk), dim3(kThreads), 0, stream, score, N, st, cnt_gt, cnt_eq, idx_sel,
                       idx_remain, sel_mask, skip_count);
    return check_launch("astraea_select_topk");
}

}  // namespace astraea
