// astraea_score: selection metric S_token (paper Sec. 3.2 "Selection Metric"; Algorithm 1 steps 1-2).
//
// The score decides which tokens are selected, so its fp32 value is defined to the bit: per token
// one accumulator walks the channels in ascending order.  To keep that order and still stream HBM
// with coalesced 16-byte loads, a wavefront owns 64 consecutive tokens: it loads a
// [64 tokens x 128 bytes] slab of both feature arrays (8 lanes cover one 128-byte row segment),
// writes the fp32 differences into a wave-private LDS tile, and then lane t walks row t of the tile.
// The next slab's loads are in flight while the current one is reduced.  No workgroup barrier is
// needed: the tile is private to the wave and a wave's LDS operations complete in order.
//
// HBM-bound: 2*C*sizeof(T) bytes read and 4 written per token.
#include "common.h"

#pragma clang fp contract(off)

namespace astraea {
namespace {

typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

constexpr int kWavesPerBlock = 4;
constexpr int kTok = 64;            // tokens per wave (lane == token in the reduce phase)
constexpr int kSegBytes = 128;      // bytes of each row handled per slab
constexpr int kVecPerLane = 8;      // 64 rows * 8 vec16 per row / 64 lanes

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// 16-byte load; with NT the load carries the streaming hint (the line is not kept in L2)
template <bool NT, typename T> __device__ __forceinline__ uint4v load16(const T *p)
{
    if (NT) return __builtin_nontemporal_load(reinterpret_cast<const uint4v *>(p));
    return *reinterpret_cast<const uint4v *>(p);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static constexpr int kPerVec = 4;
    __device__ static float load(const float *p) { return *p; }
    __device__ static void diff(const uint4v &a, const uint4v &b, float *d)
    {
        d[0] = __uint_as_float(a.x) - __uint_as_float(b.x);
        d[1] = __uint_as_float(a.y) - __uint_as_float(b.y);
        d[2] = __uint_as_float(a.z) - __uint_as_float(b.z);
        d[3] = __uint_as_float(a.w) - __uint_as_float(b.w);
    }
};
template <> struct Elem<uint16_t> {
    static constexpr int kPerVec = 8;
    __device__ static float load(const uint16_t *p) { return __uint_as_float(((uint32_t)*p) << 16); }
    __device__ static void diff(const uint4v &a, const uint4v &b, float *d)
    {
        d[0] = bf16_lo(a.x) - bf16_lo(b.x);
        d[1] = bf16_hi(a.x) - bf16_hi(b.x);
        d[2] = bf16_lo(a.y) - bf16_lo(b.y);
        d[3] = bf16_hi(a.y) - bf16_hi(b.y);
        d[4] = bf16_lo(a.z) - bf16_lo(b.z);
        d[5] = bf16_hi(a.z) - bf16_hi(b.z);
        d[6] = bf16_lo(a.w) - bf16_lo(b.w);
        d[7] = bf16_hi(a.w) - bf16_hi(b.w);
    }
};

// Orders this wave's LDS traffic without a workgroup barrier.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <typename T, int MODE, bool VEC, bool NT>
__global__ __launch_bounds__(kWavesPerBlock *kWave) void score_kernel(
    const T *__restrict__ x_cur, const T *__restrict__ x_prev, int64_t N, int64_t C, int64_t row_stride,
    const float *__restrict__ lse_weight, const int32_t *__restrict__ skip_count,
    const float *__restrict__ penalty_table, int32_t table_len, float w_alpha, float w_beta,
    float *__restrict__ score_out)
{
    constexpr int EPV = Elem<T>::kPerVec;              // elements per 16-byte vector
    constexpr int SEG = kSegBytes / (int)sizeof(T);    // channels per slab
    constexpr int PITCH = SEG + 4;                     // floats; keeps b128 row reads conflict-free
    __shared__ float tile_all[kWavesPerBlock][kTok * PITCH];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    float *tile = tile_all[wave];
    const int64_t tok0 = ((int64_t)blockIdx.x * kWavesPerBlock + wave) * kTok;
    if (tok0 >= N) return;

    // load slot j of this lane: row j*8 + lane/8 of the slab, 16-byte vector lane%8 of the segment
    const int vrow = lane >> 3, vcol = lane & 7;
    const T *pc[kVecPerLane];
    const T *pp[kVecPerLane];
#pragma unroll
    for (int j = 0; j < kVecPerLane; ++j) {
        int64_t tok = tok0 + j * 8 + vrow;
        if (tok > N - 1) tok = N - 1;                  // ragged last wave: re-read a valid row, result unused
        pc[j] = x_cur + tok * row_stride + vcol * EPV;
        pp[j] = x_prev + tok * row_stride + vcol * EPV;
    }

    uint4v ra[kVecPerLane], rb[kVecPerLane];
    auto issue = [&](int64_t c0) {
#pragma unroll
        for (int j = 0; j < kVecPerLane; ++j) {
            if (VEC && c0 + SEG <= C) {
                ra[j] = load16<NT>(pc[j] + c0);
                rb[j] = load16<NT>(pp[j] + c0);
            }
        }
    };

    float acc = 0.0f;
    const int64_t nslab = (C + SEG - 1) / SEG;
    issue(0);
    for (int64_t s = 0; s < nslab; ++s) {
        const int64_t c0 = s * SEG;
        const bool fast = VEC && (c0 + SEG <= C);
        // 1. differences of this slab -> LDS tile
#pragma unroll
        for (int j = 0; j < kVecPerLane; ++j) {
            float d[EPV];
            if (fast) {
                Elem<T>::diff(ra[j], rb[j], d);
            } else {
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    int64_t c = c0 + vcol * EPV + e;
                    // channels past C contribute +0, which leaves the accumulator unchanged
                    d[e] = (c < C) ? Elem<T>::load(pc[j] + c0 + e) - Elem<T>::load(pp[j] + c0 + e) : 0.0f;
                }
            }
            float *dst = tile + (j * 8 + vrow) * PITCH + vcol * EPV;
#pragma unroll
            for (int e = 0; e < EPV; e += 4)
                *reinterpret_cast<float4 *>(dst + e) = make_float4(d[e], d[e + 1], d[e + 2], d[e + 3]);
        }
        // 2. next slab's loads go out before the reduce phase
        if (s + 1 < nslab) issue(c0 + SEG);
        wave_lds_sync();
        // 3. lane t reduces row t, channels ascending
        const float *row = tile + lane * PITCH;
#pragma unroll
        for (int e = 0; e < SEG; e += 4) {
            float4 v = *reinterpret_cast<const float4 *>(row + e);
            if (MODE == ASTRAEA_DELTA_MEAN_ABS) {
                acc = acc + fabsf(v.x);
                acc = acc + fabsf(v.y);
                acc = acc + fabsf(v.z);
                acc = acc + fabsf(v.w);
            } else {
                acc = __builtin_fmaf(v.x, v.x, acc);
                acc = __builtin_fmaf(v.y, v.y, acc);
                acc = __builtin_fmaf(v.z, v.z, acc);
                acc = __builtin_fmaf(v.w, v.w, acc);
            }
        }
        wave_lds_sync();
    }

    const int64_t tok = tok0 + lane;
    if (tok >= N) return;
    float delta = (MODE == ASTRAEA_DELTA_L2) ? sqrtf(acc) : acc / (float)C;
    float sig = lse_weight ? delta * lse_weight[tok] : delta;
    float sc = w_alpha * sig;
    if (skip_count) {
        int32_t n = skip_count[tok];
        n = n < 0 ? 0 : n;
        n = n > table_len - 1 ? table_len - 1 : n;
        sc = __builtin_fmaf(w_beta, penalty_table[n], sc);
    }
    score_out[tok] = sc;
}

template <typename T, bool VEC, bool NT>
void launch_mode(astraea_delta_mode mode, dim3 grid, dim3 block, hipStream_t st, const T *xc, const T *xp, int64_t N,
                 int64_t C, int64_t rs, const float *lw, const int32_t *sc, const float *pt, int32_t tl, float wa,
                 float wb, float *out)
{
    switch (mode) {
    case ASTRAEA_DELTA_L2:
        hipLaunchKernelGGL((score_kernel<T, ASTRAEA_DELTA_L2, VEC, NT>), grid, block, 0, st, xc, xp, N, C, rs, lw, sc, pt,
                           tl, wa, wb, out);
        break;
    case ASTRAEA_DELTA_MEAN_ABS:
        hipLaunchKernelGGL((score_kernel<T, ASTRAEA_DELTA_MEAN_ABS, VEC, NT>), grid, block, 0, st, xc, xp, N, C, rs, lw,
                           sc, pt, tl, wa, wb, out);
        break;
    default:
        hipLaunchKernelGGL((score_kernel<T, ASTRAEA_DELTA_MEAN_SQ, VEC, NT>), grid, block, 0, st, xc, xp, N, C, rs, lw,
                           sc, pt, tl, wa, wb, out);
        break;
    }
}

}  // namespace

int launch_score(const void *x_cur, const void *x_prev, astraea_dtype dt, int64_t N, int64_t C, int64_t row_stride,
                 astraea_delta_mode mode, const float *lse_weight, const int32_t *skip_count,
                 const float *penalty_table, int32_t table_len, float w_alpha, float w_beta, float *score_out,
                 hipStream_t stream)
{
    if (N == 0) return ASTRAEA_OK;
    const int64_t tokens_per_block = (int64_t)kWavesPerBlock * kTok;
    const int64_t nblocks = (N + tokens_per_block - 1) / tokens_per_block;
    dim3 grid((unsigned)nblocks), block(kWavesPerBlock * kWave);
    const size_t es = dt == ASTRAEA_F32 ? 4 : 2;
    const bool vec = ((uintptr_t)x_cur % 16 == 0) && ((uintptr_t)x_prev % 16 == 0) && ((row_stride * es) % 16 == 0);
    // Feature arrays larger than the chip's caches (4 MB of L2 per XCD, 256 MB behind them) are read once and
    // gone: their loads then carry the streaming hint, which raises the rate from 5.96 to 6.77 TB/s at
    // N = 118800, C = 3072.  Smaller arrays are often still cached from their producer, and the hint would
    // make them miss (N = 17550: 3.3 TB/s without it, 2.8 with it).
    const bool stream_loads = vec && 2 * N * row_stride * (int64_t)es > ((int64_t)256 << 20);
#define ASTRAEA_SCORE_LAUNCH(T, VEC, NT)                                                                       \
    launch_mode<T, VEC, NT>(mode, grid, block, stream, (const T *)x_cur, (const T *)x_prev, N, C, row_stride,  \
                            lse_weight, skip_count, penalty_table, table_len, w_alpha, w_beta, score_out)
    if (dt == ASTRAEA_F32) {
        if (stream_loads)
            ASTRAEA_SCORE_LAUNCH(float, true, true);
        else if (vec)
            ASTRAEA_SCORE_LAUNCH(float, true, false);
        else
            ASTRAEA_SCORE_LAUNCH(float, false, false);
    } else {
        if (stream_loads)
            ASTRAEA_SCORE_LAUNCH(uint16_t, true, true);
        else if (vec)
            ASTRAEA_SCORE_LAUNCH(uint16_t, true, false);
        else
            ASTRAEA_SCORE_LAUNCH(uint16_t, false, false);
    }
#undef ASTRAEA_SCORE_LAUNCH
    return check_launch("astraea_score");
}

}  // namespace astraea
