// astraea_sparse_attn_fwd, fp32 mode (paper, Algorithm 1 step 6: Softmax(Q_sel K^T / sqrt(d)) V over
// all N keys for the selected queries only).
//
// Everything stays in fp32: QK^T and PV run on the fp32 matrix instruction
// v_mfma_f32_32x32x2_f32, the softmax is the online (running max / running sum) form.
// Both products are computed transposed, S^T = K Q^T and O^T = V^T P^T, so that a lane owns one
// query column in every accumulator: row max, row sum and the rescale factor are per-lane values
// (one exchange between lane l and lane l+32), and the S^T accumulator registers feed the second
// product directly as its B operand.
//
// Workgroup = 4 waves x 32 queries; keys are swept in tiles of 32 staged in LDS.  This is the
// accuracy-first path for small layers; the bf16 path carries the throughput.
#include "gfx950.h"

namespace astraea {
namespace {


constexpr int kWaves = 4;
constexpr int kBq = 32 * kWaves;   // queries per workgroup
constexpr int kBk = 32;            // keys per tile

__device__ __forceinline__ float xhalf_max(float x)
{
    // max of lane l and lane l^32
    float o = __shfl_xor(x, 32);
    return fmaxf(x, o);
}
__device__ __forceinline__ float xhalf_sum(float x) { return x + __shfl_xor(x, 32); }

template <int D>
__global__ __launch_bounds__(kWaves *kWave) void attn_f32_kernel(
    const float *__restrict__ q, const float *__restrict__ k, const float *__restrict__ v, int64_t N, int32_t H,
    int64_t q_stride_n, int64_t q_stride_h, int64_t kv_stride_n, int64_t kv_stride_h,
    const int32_t *__restrict__ idx_sel, int64_t k_sel, int q_is_compact, float scale_log2e,
    float *__restrict__ o_sel, int64_t o_stride_n, int o_scatter, float *__restrict__ lse_sel, int32_t splits,
    int64_t tiles_per_split, float *__restrict__ partial)
{
    constexpr int kPartialPitch = D + 4;   // a share's row: D accumulators, running max, row sum (16-byte aligned)
    constexpr int KP = D + 2;      // K tile pitch (floats): lanes (key, d-parity) hit 64 distinct banks
    constexpr int VP = D + 8;      // V tile pitch: rows r and r+4 land 32 banks apart
    constexpr int DB = D / 32;
    __shared__ float k_lds[kBk * KP];
    __shared__ float v_lds[kBk * VP];

    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int qc = lane & 31, hf = lane >> 5;
    const int head = blockIdx.y;
    const int64_t r0 = (int64_t)blockIdx.x * kBq + wave * 32;

    // Q operand: lane holds query column qc, head-dim elements 2s + hf
    int64_t r = r0 + qc;
    if (r > k_sel - 1) r = k_sel - 1;                    // ragged last tile: duplicate a valid row, never stored
    // an index outside [0, N) reads a valid row instead
    const int64_t qrow = q_is_compact ? r : (int64_t)clamp_row(idx_sel[r], (int32_t)N);
    const float *qp = q + qrow * q_stride_n + (int64_t)head * q_stride_h;
    float qreg[D / 2];
#pragma unroll
    for (int s = 0; s < D / 2; ++s) qreg[s] = qp[2 * s + hf];

    floatx16 oacc[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[b][i] = 0.0f;
    float m_run = -INFINITY;   // running max of the scaled logits in log2 units
    float l_run = 0.0f;        // this lane's share of the running sum

    const float *kb = k + (int64_t)head * kv_stride_h;
    const float *vb = v + (int64_t)head * kv_stride_h;
    // blockIdx.z takes one of `splits` consecutive key ranges (the budget-aware launch: a small selection
    // does not fill the chip with whole sweeps)
    const int64_t ntiles = (N + kBk - 1) / kBk;
    const int64_t t_begin = (int64_t)blockIdx.z * tiles_per_split;
    const int64_t t_end = t_begin + tiles_per_split < ntiles ? t_begin + tiles_per_split : ntiles;
    for (int64_t t = t_begin; t < t_end; ++t) {
        const int64_t key0 = t * kBk;
        __syncthreads();
        // stage the tile: 32 rows x D floats each for K and V, 16-byte global loads
        for (int c = threadIdx.x; c < kBk * (D / 4); c += kWaves * kWave) {
            const int row = c / (D / 4), c4 = c % (D / 4);
            int64_t key = key0 + row;
            if (key > N - 1) key = N - 1;
            const float4 kv4 = *reinterpret_cast<const float4 *>(kb + key * kv_stride_n + c4 * 4);
            const float4 vv4 = *reinterpret_cast<const float4 *>(vb + key * kv_stride_n + c4 * 4);
            float *kd = k_lds + row * KP + c4 * 4;
            kd[0] = kv4.x; kd[1] = kv4.y; kd[2] = kv4.z; kd[3] = kv4.w;
            *reinterpret_cast<float4 *>(v_lds + row * VP + c4 * 4) = vv4;
        }
        __syncthreads();

        // S^T[key, q] = sum_d K[key, d] Q[q, d]
        floatx16 sacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = 0.0f;
#pragma unroll
        for (int s = 0; s < D / 2; ++s) {
            const float a = k_lds[qc * KP + 2 * s + hf];      // A: row = key (lane&31), k index = hf
            sacc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, qreg[s], sacc, 0, 0, 0);
        }
        // register i of sacc: key = key0 + (i/4)*8 + hf*4 + i%4, query = qc
        float tmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float sv = sacc[i] * scale_log2e;
            const int64_t key = key0 + (i >> 2) * 8 + hf * 4 + (i & 3);
            if (key >= N) sv = -INFINITY;
            sacc[i] = sv;
            tmax = fmaxf(tmax, sv);
        }
        tmax = xhalf_max(tmax);
        const float m_new = fmaxf(m_run, tmax);
        const float alpha = exp2f(m_run - m_new);          // 0 on the first tile
        float psum = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float p = exp2f(sacc[i] - m_new);
            sacc[i] = p;
            psum += p;
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[b][i] *= alpha;
        // O^T[d, q] += sum_key V[key, d] P^T[key, q]; MFMA i contracts keys (i/4)*8 + i%4 (+4 in the upper half)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int key = (i >> 2) * 8 + hf * 4 + (i & 3);
#pragma unroll
            for (int b = 0; b < DB; ++b) {
                const float a = v_lds[key * VP + b * 32 + qc];   // A: row = d (lane&31), k index = hf
                oacc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, sacc[i], oacc[b], 0, 0, 0);
            }
        }
    }

    const float l_tot = xhalf_sum(l_run);
    const int64_t rr = r0 + qc;
    if (rr >= k_sel) return;
    if (splits > 1) {
        // a key-range share: unnormalised accumulators, running max and row sum go to the workspace
        float *pp = partial + (((int64_t)blockIdx.z * k_sel + rr) * H + head) * kPartialPitch;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *reinterpret_cast<float4 *>(pp + b * 32 + g * 8 + hf * 4) =
                    make_float4(oacc[b][4 * g], oacc[b][4 * g + 1], oacc[b][4 * g + 2], oacc[b][4 * g + 3]);
        if (hf == 0) {
            pp[D] = m_run;
            pp[D + 1] = l_tot;
        }
        return;
    }
    const float inv = 1.0f / l_tot;
    // compact output row rr, or straight into the cached buffer's row of that token
    const int64_t orow = o_scatter ? (int64_t)idx_sel[rr] : rr;
    float *op = o_sel + orow * o_stride_n + (int64_t)head * D;
    if (!o_scatter || (uint64_t)orow < (uint64_t)N)      // a row index outside the cached buffer writes nothing
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            // registers 4g..4g+3: head-dim b*32 + g*8 + hf*4 + 0..3
            float4 o4 = make_float4(oacc[b][4 * g] * inv, oacc[b][4 * g + 1] * inv, oacc[b][4 * g + 2] * inv,
                                    oacc[b][4 * g + 3] * inv);
            *reinterpret_cast<float4 *>(op + b * 32 + g * 8 + hf * 4) = o4;
        }
    if (lse_sel && hf == 0) lse_sel[rr * H + head] = (m_run + log2f(l_tot)) * 0.69314718055994530942f;
}

// Combines the key-range shares: with m* = max_s m_s and w_s = 2^(m_s - m*), O = sum_s w_s O_s / sum_s w_s l_s.
// One thread per (selected row, head, 4 head-dim elements), shares visited in order.
template <int D>
__global__ __launch_bounds__(256) void merge_f32_kernel(const float *__restrict__ partial, int32_t splits, int32_t H,
                                                        int64_t k_sel, int64_t n_rows, const int32_t *__restrict__ idx_sel,
                                                        float *__restrict__ o_sel, int64_t o_stride_n, int o_scatter,
                                                        float *__restrict__ lse_sel)
{
    constexpr int Q4 = D / 4, kPartialPitch = D + 4;
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t rh = id / Q4;
    const int d4 = (int)(id % Q4) * 4;
    if (rh >= k_sel * H) return;
    const int64_t rr = rh / H;
    const int head = (int)(rh % H);
    const int64_t share = k_sel * H * (int64_t)kPartialPitch;
    const float *base = partial + rh * kPartialPitch;
    float m_star = -INFINITY;
    for (int s = 0; s < splits; ++s) m_star = fmaxf(m_star, base[s * share + D]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float l = 0.0f;
    for (int s = 0; s < splits; ++s) {
        const float *ps = base + s * share;
        const float w = exp2f(ps[D] - m_star);
        const float4 o = *reinterpret_cast<const float4 *>(ps + d4);
        acc.x += w * o.x;
        acc.y += w * o.y;
        acc.z += w * o.z;
        acc.w += w * o.w;
        l += w * ps[D + 1];
    }
    const float inv = 1.0f / l;
    const int64_t orow = o_scatter ? (int64_t)idx_sel[rr] : rr;
    if (!o_scatter || (uint64_t)orow < (uint64_t)n_rows)
        *reinterpret_cast<float4 *>(o_sel + orow * o_stride_n + (int64_t)head * D + d4) =
            make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
    if (lse_sel && d4 == 0) lse_sel[rh] = (m_star + log2f(l)) * 0.69314718055994530942f;
}

// Key-range shares per work item: enough workgroups for two waves per SIMD of the chip, shares of at least 8 key
// tiles, at most 8 shares.  Large selections get 1 (no workspace, no merge).
static int32_t f32_splits(int64_t N, int32_t H, int64_t k_sel)
{
    const int64_t waves = ((k_sel + kBq - 1) / kBq) * H * kWaves;
    const int64_t ntiles = (N + kBk - 1) / kBk;
    int64_t s = 2048 / (waves > 0 ? waves : 1);
    if (s > ntiles / 8) s = ntiles / 8;
    if (s > 8) s = 8;
    return s < 2 ? 1 : (int32_t)s;
}

}  // namespace

// Partial-result bytes the key-range split needs at exactly k_sel selected queries (0 when it is not cut).
static size_t f32_partial_bytes(int64_t N, int32_t H, int32_t D, int64_t k_sel)
{
    if (N <= 0 || H <= 0 || k_sel <= 0) return 0;
    const int32_t s = f32_splits(N, H, k_sel);
    return s > 1 ? (size_t)s * (size_t)k_sel * (size_t)H * (size_t)(D + 4) * sizeof(float) : 0;
}

// What astraea_workspace_bytes names: enough for every selection of up to k_sel queries.  The need is not
// monotone in k_sel (fewer queries are cut into more shares), so a buffer sized once for the largest budget
// must cover the smaller ones too: the maximum over k' <= k_sel.  Within one count of query tiles the share
// count is fixed and the need grows with k', so only tile multiples (and k_sel itself) are candidates, and
// past 2048 waves nothing is cut any more.
size_t attn_f32_workspace_bytes(int64_t N, int32_t H, int32_t D, int64_t k_sel)
{
    if (N <= 0 || H <= 0 || k_sel <= 0) return 0;
    size_t need = f32_partial_bytes(N, H, D, k_sel);
    const int64_t t_max = 2048 / ((int64_t)H * kWaves) + 1;
    for (int64_t t = 1; t <= t_max && t * kBq <= k_sel; ++t) {
        const size_t b = f32_partial_bytes(N, H, D, t * kBq);
        if (b > need) need = b;
    }
    return need;
}

int launch_attn_f32(const void *q, const void *k, const void *v, int64_t N, int32_t H, int32_t D, int64_t q_stride_n,
                    int64_t q_stride_h, int64_t kv_stride_n, int64_t kv_stride_h, const int32_t *idx_sel,
                    int64_t k_sel, int q_is_compact, float scale, void *o_sel, int64_t o_stride_n, int o_scatter,
                    float *lse_sel, void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    if (k_sel == 0) return ASTRAEA_OK;
    // the split is an option: without a workspace of the size astraea_workspace_bytes names, every work item
    // sweeps all keys itself
    int32_t splits = f32_splits(N, H, k_sel);
    if (splits > 1 && (!workspace || workspace_bytes < f32_partial_bytes(N, H, D, k_sel))) splits = 1;
    const int64_t ntiles = (N + kBk - 1) / kBk;
    const int64_t tps = (ntiles + splits - 1) / splits;
    if ((int64_t)(splits - 1) * tps >= ntiles) splits = (int32_t)((ntiles + tps - 1) / tps);   // no empty share
    float *partial = (float *)workspace;
    dim3 grid((unsigned)((k_sel + kBq - 1) / kBq), (unsigned)H, (unsigned)splits), block(kWaves * kWave);
    const float c = scale * 1.44269504088896340736f;
    kernel_timer_begin(stream);
    if (D == 64)
        hipLaunchKernelGGL(attn_f32_kernel<64>, grid, block, 0, stream, (const float *)q, (const float *)k,
                           (const float *)v, N, H, q_stride_n, q_stride_h, kv_stride_n, kv_stride_h, idx_sel, k_sel,
                           q_is_compact, c, (float *)o_sel, o_stride_n, o_scatter, lse_sel, splits, tps, partial);
    else
        hipLaunchKernelGGL(attn_f32_kernel<128>, grid, block, 0, stream, (const float *)q, (const float *)k,
                           (const float *)v, N, H, q_stride_n, q_stride_h, kv_stride_n, kv_stride_h, idx_sel, k_sel,
                           q_is_compact, c, (float *)o_sel, o_stride_n, o_scatter, lse_sel, splits, tps, partial);
    kernel_timer_end(stream);
    if (splits > 1) {
        const int64_t threads = k_sel * H * (D / 4);
        const dim3 mgrid((unsigned)((threads + 255) / 256));
        if (D == 64)
            hipLaunchKernelGGL(merge_f32_kernel<64>, mgrid, dim3(256), 0, stream, partial, splits, H, k_sel, N, idx_sel,
                               (float *)o_sel, o_stride_n, o_scatter, lse_sel);
        else
            hipLaunchKernelGGL(merge_f32_kernel<128>, mgrid, dim3(256), 0, stream, partial, splits, H, k_sel, N, idx_sel,
                               (float *)o_sel, o_stride_n, o_scatter, lse_sel);
    }
    return check_launch("astraea_sparse_attn_fwd(f32)");
}

}  // namespace astraea
