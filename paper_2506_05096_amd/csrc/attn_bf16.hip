// astraea_sparse_attn_fwd, bf16 mode, head_dim 128 (paper, Algorithm 1 step 6:
// X_out[I_sel] = Softmax(Q_sel K^T / sqrt(d)) V with every key and value kept, Sec. 3.2
// "Sparse Attention").  Flash-style: K/V are streamed once per query tile, the N x N map is never
// materialised, softmax is the online form in fp32.
//
// Shape of the computation on gfx950:
//  * both products are computed transposed, S^T = K Q^T and O^T = V^T P^T, with
//    v_mfma_f32_32x32x16_bf16.  In every accumulator a lane then owns one query column, so the row
//    max / row sum / rescale factor are per-lane scalars (one exchange between lanes l and l+32),
//    and the S^T accumulator registers, converted to bf16, are the B operand of the second
//    product as they stand: register group 8*(t%2)..+7 of key block t/2 feeds MFMA t, with the key
//    order inside the contraction permuted the same way on the V side.
//  * K/V tiles go from global memory straight into LDS (global_load_lds_dwordx4), double
//    buffered, with no register staging.  Such a load writes 64 x 16 B contiguously, so rows
//    cannot be padded; bank conflicts are avoided by an XOR swizzle of the 16-byte chunks inside
//    each 256-byte row, applied through the per-lane global address.
//  * V^T fragments come from the row-major [key][d] tile through the transposing LDS read
//    ds_read_b64_tr_b16, so neither K nor V is transposed in memory.
//  * queries are gathered by index while loading the Q fragment, which then lives in registers
//    for the whole sweep (the "gather" step of the path is fused here).
//  * the rescale of the O accumulators is lazy: the running max is only raised when some row's
//    max grew by more than 2^kTau, so stale maxima cost range, not accuracy.
//  * workgroup ids are mapped so that the workgroups resident on one XCD work on the same head and
//    sweep the keys together; K/V tiles are then served from that XCD's L2.
#include <type_traits>

#include "common.h"

namespace astraea {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int kWaves = 8;
constexpr int kBq = 32 * kWaves;        // queries per workgroup
constexpr int kBk = 64;                 // keys per LDS tile
constexpr int kRowBytes = D * 2;        // 256 B per key row, unpadded
constexpr int kTileBytes = kBk * kRowBytes;          // 16 KiB
constexpr int kBufBytes = 2 * kTileBytes;            // K tile then V tile
constexpr float kTau = 8.0f;            // lazy-rescale threshold, log2 units
constexpr int kNumXcd = 8;

__device__ __forceinline__ float xhalf_max(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    floatx2 f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));   // v_cvt_pk_bf16_f32, RNE
}

__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr)
{
    return *reinterpret_cast<const bf16x8 __attribute__((address_space(3))) *>((uintptr_t)addr);
}
// Transposing LDS read: within each group of 16 lanes, lane i receives element (i % 4) of the
// 8-byte rows addressed by lanes 4j + i/4, j = 0..3.
__device__ __forceinline__ short4v lds_read_tr(uint32_t addr)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3))) *)(uintptr_t)addr);
}

// 16 bytes per lane from global memory straight into LDS: lane l of the wave lands at
// lds_wave_base + 16*l.  The LDS base travels in M0.  Completion is counted by vmcnt; the kernel
// waits for it explicitly before the barrier that publishes the tile.
__device__ __forceinline__ void dma16(const void *gbase, uint32_t goff, uint32_t lds_wave_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_wave_base), "v"(goff), "s"(gbase)
                 : "memory");
}
__device__ __forceinline__ void wait_dma() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

constexpr int MFMA = 0x008, DSR = 0x100;
#define SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)

__global__ __launch_bounds__(kWaves *kWave, 1) void attn_bf16_kernel(
    const __bf16 *__restrict__ q, const __bf16 *__restrict__ k, const __bf16 *__restrict__ v, int64_t N, int32_t H,
    int64_t q_stride_n, int64_t q_stride_h, int64_t kv_stride_n, int64_t kv_stride_h,
    const int32_t *__restrict__ idx_sel, int64_t k_sel, int q_is_compact, float scale_log2e,
    __bf16 *__restrict__ o_sel, float *__restrict__ lse_sel, int32_t q_tiles, int64_t items_per_xcd)
{
    // [buffer][K tile | V tile]; 64 KiB, one 8-wave workgroup per CU (two waves per SIMD)
    __shared__ __attribute__((aligned(1024))) char lds[2 * kBufBytes];

    // work item = (head, query tile), head-major; XCD x owns the contiguous item range
    // [x * items_per_xcd, (x+1) * items_per_xcd), and workgroups reach XCDs round-robin by id.
    const int64_t total_items = (int64_t)H * q_tiles;
    const int64_t xcd = blockIdx.x % kNumXcd, slot = blockIdx.x / kNumXcd;
    const int64_t item = xcd * items_per_xcd + slot;
    if (slot >= items_per_xcd || item >= total_items) return;
    const int head = (int)(item / q_tiles);
    const int64_t qt = item % q_tiles;

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int qc = lane & 31, hf = lane >> 5;
    const int64_t r0 = qt * kBq + wave * 32;
    const uint32_t lds0 = (uint32_t)(uintptr_t)lds;

    // ---- Q fragment: lane holds query column qc, head-dim 16*s + 8*hf + 0..7 (B operand of K Q^T)
    int64_t r = r0 + qc;
    if (r > k_sel - 1) r = k_sel - 1;               // ragged last tile: duplicate a valid row, never stored
    const int64_t qrow = q_is_compact ? r : (int64_t)idx_sel[r];
    const __bf16 *qp = q + qrow * q_stride_n + (int64_t)head * q_stride_h + 8 * hf;
    bf16x8 qf[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);

    floatx16 oacc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[b][i] = 0.0f;
    float m_c = -INFINITY;     // running max of scale*log2(e)*logit actually used as exponent offset
    float l_run = 0.0f;        // this lane's share of the running sum

    // ---- tile DMA.  A wave instruction fills 4 consecutive rows (1 KiB) of a tile: lane l writes
    // physical chunk l%16 of row l/16.  Wave w issues blocks w, w + kWaves, ... of K and of V.
    // Physical chunk p of row r holds logical chunk p ^ (r & 15) for K and p ^ (4 * (r & 3)) for V.
    constexpr int kDmaPerWave = (kBk / 4) / kWaves;
    const char *kbase = reinterpret_cast<const char *>(k + (int64_t)head * kv_stride_h);
    const char *vbase = reinterpret_cast<const char *>(v + (int64_t)head * kv_stride_h);
    const int64_t row_pitch = kv_stride_n * 2;       // bytes between consecutive keys
    const int d_row = lane >> 4, d_p = lane & 15;
    uint32_t koff[kDmaPerWave], voff[kDmaPerWave];   // lane offsets inside a full tile
#pragma unroll
    for (int i = 0; i < kDmaPerWave; ++i) {
        const int rr = 4 * (kWaves * i + wave) + d_row;
        koff[i] = (uint32_t)(rr * row_pitch) + ((d_p ^ (rr & 15)) << 4);
        voff[i] = (uint32_t)(rr * row_pitch) + ((d_p ^ ((rr & 3) << 2)) << 4);
    }
    auto issue_dma = [&](int64_t key0, int buf) {
        const char *kt = kbase + key0 * row_pitch, *vt = vbase + key0 * row_pitch;
        if (key0 + kBk <= N) {
#pragma unroll
            for (int i = 0; i < kDmaPerWave; ++i) {
                const uint32_t dst = lds0 + buf * kBufBytes + (kWaves * i + wave) * 1024;
                dma16(kt, koff[i], dst);
                dma16(vt, voff[i], dst + kTileBytes);
            }
        } else {
            const int64_t last = N - 1 - key0;       // rows past the last key re-read it (masked later)
#pragma unroll
            for (int i = 0; i < kDmaPerWave; ++i) {
                const int rr = 4 * (kWaves * i + wave) + d_row;
                const int64_t rc = rr < last ? rr : last;
                const uint32_t dst = lds0 + buf * kBufBytes + (kWaves * i + wave) * 1024;
                dma16(kt, (uint32_t)(rc * row_pitch) + ((d_p ^ (rr & 15)) << 4), dst);
                dma16(vt, (uint32_t)(rc * row_pitch) + ((d_p ^ ((rr & 3) << 2)) << 4), dst + kTileBytes);
            }
        }
    };

    // ---- LDS read addresses (lane part; tile, buffer and block offsets are immediates)
    // K fragment (kb, s): row 32*kb + qc, logical chunk 2*s + hf
    uint32_t ka[D / 16];
#pragma unroll
    for (int s = 0; s < D / 16; ++s) ka[s] = lds0 + qc * kRowBytes + (((2 * s + hf) ^ (qc & 15)) << 4);
    // V^T fragment (tt, b, half): lane i of a 16-lane group addresses row 16*tt + 8*half + 4*hf + i/4,
    // head-dim 32*b + 16*(group & 1) + 4*(i % 4) .. +3
    const int li = lane & 15, vr = li >> 2;
    uint32_t va[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
        va[b] = lds0 + kTileBytes + (4 * hf + vr) * kRowBytes +
                ((((4 * b) ^ (vr << 2)) + 2 * ((lane >> 4) & 1) + ((li & 3) >> 1)) << 4) + 8 * (li & 1);

    const int64_t ntiles = (N + kBk - 1) / kBk;
    issue_dma(0, 0);
    // The Q fragment must be resident before the loop starts: a load still counted as pending at the
    // loop header would make the compiler wait on the vector-memory counter inside the loop.
#pragma unroll
    for (int s = 0; s < D / 16; ++s) asm volatile("" ::"v"(qf[s]));
    wait_dma();
    __syncthreads();

    auto tile_step = [&](int64_t t, auto buf_tag) {
        constexpr int BUF = decltype(buf_tag)::value;
        constexpr uint32_t KOFF = BUF * kBufBytes;
        const int64_t key0 = t * kBk;
        if (t + 1 < ntiles) issue_dma(key0 + kBk, BUF ^ 1);

        // ---- S^T[key, q] = sum_d K[key, d] Q[q, d]; two blocks of 32 keys
        floatx16 sacc[2];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            sacc[0][i] = 0.0f;
            sacc[1][i] = 0.0f;
        }
        bf16x8 kf[D / 16], kg[D / 16];
#pragma unroll
        for (int s = 0; s < D / 16; ++s) kf[s] = lds_read_b128(ka[s] + KOFF);
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[s], sacc[0], 0, 0, 0);
            kg[s] = lds_read_b128(ka[s] + KOFF + 32 * kRowBytes);
        }
        // V^T fragments of the first 32 keys are fetched under the second block's MFMAs
        short4v vh[2][4][2];
#pragma unroll
        for (int s = 0; s < D / 16; ++s) {
            sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kg[s], qf[s], sacc[1], 0, 0, 0);
            const int tt = s >> 2, b = s & 3;
            vh[tt][b][0] = lds_read_tr(va[b] + KOFF + (16 * tt) * kRowBytes);
            vh[tt][b][1] = lds_read_tr(va[b] + KOFF + (16 * tt + 8) * kRowBytes);
        }
        SGB(DSR, 8);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            SGB(MFMA, 1);
            SGB(DSR, 1);
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            SGB(MFMA, 1);
            SGB(DSR, 2);
        }

        // register i of sacc[kb]: key = key0 + 32*kb + (i/4)*8 + hf*4 + i%4, query = qc
        if (key0 + kBk > N) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int64_t key = key0 + 32 * kb + (i >> 2) * 8 + hf * 4 + (i & 3);
                    if (key >= N) sacc[kb][i] = -INFINITY;
                }
        }
        float tmax = sacc[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, sacc[kb][i]);
        tmax = xhalf_max(tmax) * scale_log2e;
        // lazy rescale: only when some row's max moved up by more than 2^kTau
        if (__builtin_amdgcn_ballot_w64(tmax > m_c + kTau) != 0) {
            const float m_new = fmaxf(m_c, tmax);
            const float alpha = __builtin_amdgcn_exp2f(m_c - m_new);   // 0 on the first tile
            m_c = m_new;
            l_run *= alpha;
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[b][i] *= alpha;
        }
        float psum = 0.0f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][i], scale_log2e, -m_c));
                sacc[kb][i] = p;
                psum += p;
            }
        l_run += psum;

        // ---- O^T[d, q] += sum_key V[key, d] P^T[key, q]; MFMA tt contracts the 16 keys
        //      16*tt + {0..3, 8..11} (lanes 0-31) and 16*tt + {4..7, 12..15} (lanes 32-63)
        short4v wh[2][4][2];
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            const int kb = tt >> 1, rb = 8 * (tt & 1);
            uint4v pw;
#pragma unroll
            for (int j = 0; j < 4; ++j) pw[j] = pack_bf16(sacc[kb][rb + 2 * j], sacc[kb][rb + 2 * j + 1]);
            const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const short4v h0 = tt < 2 ? vh[tt][b][0] : wh[tt - 2][b][0];
                const short4v h1 = tt < 2 ? vh[tt][b][1] : wh[tt - 2][b][1];
                const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7));
                oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[b], 0, 0, 0);
                if (tt < 2) {   // fetch the fragments of keys 32..63 under the first 8 MFMAs
                    wh[tt][b][0] = lds_read_tr(va[b] + KOFF + (16 * (tt + 2)) * kRowBytes);
                    wh[tt][b][1] = lds_read_tr(va[b] + KOFF + (16 * (tt + 2) + 8) * kRowBytes);
                }
            }
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            SGB(MFMA, 1);
            SGB(DSR, 2);
        }

        wait_dma();
        __syncthreads();
    };

    int64_t t = 0;
    for (; t + 1 < ntiles; t += 2) {
        tile_step(t, std::integral_constant<int, 0>{});
        tile_step(t + 1, std::integral_constant<int, 1>{});
    }
    if (t < ntiles) tile_step(t, std::integral_constant<int, 0>{});

    const float l_tot = xhalf_sum(l_run);
    const float inv = 1.0f / l_tot;
    const int64_t rr = r0 + qc;
    if (rr >= k_sel) return;
    __bf16 *op = o_sel + (rr * H + head) * (int64_t)D;
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            // registers 4g..4g+3: head-dim 32*b + 8*g + 4*hf + 0..3
            uint2v o4;
            o4[0] = pack_bf16(oacc[b][4 * g] * inv, oacc[b][4 * g + 1] * inv);
            o4[1] = pack_bf16(oacc[b][4 * g + 2] * inv, oacc[b][4 * g + 3] * inv);
            *reinterpret_cast<uint2v *>(op + 32 * b + 8 * g + 4 * hf) = o4;
        }
    if (lse_sel && hf == 0) lse_sel[rr * H + head] = (m_c + log2f(l_tot)) * 0.69314718055994530942f;
}

}  // namespace

// The bf16 path stages nothing outside its inputs and outputs.
size_t attn_bf16_workspace_bytes(int64_t, int32_t) { return 0; }

int launch_attn_bf16_d128(const void *q, const void *k, const void *v, int64_t N, int32_t H, int64_t q_stride_n,
                          int64_t q_stride_h, int64_t kv_stride_n, int64_t kv_stride_h, const int32_t *idx_sel,
                          int64_t k_sel, int q_is_compact, float scale, void *o_sel, float *lse_sel, void *,
                          hipStream_t stream)
{
    if (k_sel == 0) return ASTRAEA_OK;
    // a tile's lane offsets are 32-bit: 64 rows must span less than 4 GiB
    if (kv_stride_n * 2 * kBk >= (int64_t)1 << 32)
        return fail(ASTRAEA_ERR_UNSUPPORTED, "astraea_sparse_attn_fwd: K/V token stride too large");
    const int64_t q_tiles = (k_sel + kBq - 1) / kBq;
    const int64_t total = q_tiles * H;
    const int64_t per_xcd = (total + kNumXcd - 1) / kNumXcd;
    if (per_xcd * kNumXcd > 2147483647LL) return fail(ASTRAEA_ERR_INVALID, "astraea_sparse_attn_fwd: grid too large");
    dim3 grid((unsigned)(per_xcd * kNumXcd)), block(kWaves * kWave);
    hipLaunchKernelGGL(attn_bf16_kernel, grid, block, 0, stream, (const __bf16 *)q, (const __bf16 *)k,
                       (const __bf16 *)v, N, H, q_stride_n, q_stride_h, kv_stride_n, kv_stride_h, idx_sel, k_sel,
                       q_is_compact, scale * 1.44269504088896340736f, (__bf16 *)o_sel, lse_sel, (int32_t)q_tiles,
                       per_xcd);
    return check_launch("astraea_sparse_attn_fwd(bf16)");
}

}  // namespace astraea
